"""GPU parity of the adaptive key-precision path (selector, Rung-1 growth, per-group union, FP16-key
gather, attend pass with gated key precision, achieved-tail certificate, ranking check) against
the oracle, through the C ABI.

Integer decisions (K*, the selected blocks, the promoted mask) are compared exactly: the oracle's
selector is run on the very log-masses the scoring pass produced on the GPU, so both sides decide
on identical numbers.  The attend pass is then compared against the oracle's, given that mask,
to the usual floating-point bars (O 1e-3, certificate terms 1e-4, log-masses 1e-4 absolute).
"""
import math

import numpy as np
import pytest

import oracle
import workloads
from oracle import adaptive as ad
from oracle import attention as att
from oracle import quantizer as qz
from helpers import GpuLayerCache, assert_head_matches, load_binding, to_gpu_tol

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def make_case(seed, bt, hq, hkv, n_tokens, student=False, peaked=()):
    rng = np.random.Generator(np.random.Philox(seed))
    shape = (bt, hkv, n_tokens, 128)
    k = workloads.student_t3_f16(rng, shape) if student else workloads.normal_f16(rng, shape)
    v = workloads.normal_f16(rng, shape)
    q = workloads.normal_f16(rng, (bt, hq, 128))
    g = hq // hkv
    for (b, h, pos, c) in peaked:                    # heads aligned with one key
        q[b, h] = (k[b, h // g, pos].astype(np.float32) * c).astype(np.float16)
    return k, v, q


def gpu_adaptive(gc, q, tol, sel, step=False):
    cqa = gc.cqa
    qd = gc.to_dev(q)
    gtol = to_gpu_tol(cqa, tol)
    gsel = cqa.Selector(sel.tau_cov, sel.k_min, sel.k_max, sel.k_limit, sel.v_limit, sel.v_greedy,
                        sel.canary, sel.explore_frac, sel.explore_seed, sel.per_head)
    # the scoring pass on its own first: its certificate (lse, Delta_h, V_max) is what the selector
    # reads inside the adaptive call, bit for bit (same kernel, same inputs)
    gc.cqa.cqa_certified_decode(gc.h, 0, qd, cqa.Tolerances(int8_query=int(tol.int8_query)), gc.O, gc.cert, gc.flags, None)
    _, cert0, _ = gc.results()
    rung = None
    if step == "enqueue":
        cqa.cqa_adaptive_step_enqueue(gc.h, 0, qd, gtol, gsel, gc.O, gc.cert, gc.flags)
    elif step:
        rung = cqa.cqa_adaptive_step(gc.h, 0, qd, gtol, gsel, gc.O, gc.cert, gc.flags)
    else:
        cqa.cqa_adaptive_decode(gc.h, 0, qd, gtol, gsel, gc.O, gc.cert, gc.flags)
    O, cert, flags = gc.results()
    state = cqa.cqa_adaptive_state(gc.h, 0, gc.bt, gc.hq, gc.hkv)
    return dict(O=O, cert=cert, flags=flags, cert0=cert0, rung=rung, k_star=state[0], selected=state[1],
                promoted=(state[2] & 1).astype(bool), v_promoted=(state[2] & 2).astype(bool),
                head_keys=(state[2] >> 4) & 15, head_values=(state[2] >> 8) & 15, l8=state[3],
                lx=state[4], v_count=state[5], v_selected=state[6], contrib=state[7], score_dev=state[8])


def check_against_oracle(oc, q, tol, sel, out, heads=None, served=None):
    """Exact selector decisions on the GPU's log-masses; attend pass vs the oracle given the mask."""
    bt, hq, _ = q.shape
    g = hq // oc.hkv
    nb = oc.n_blocks
    heads = heads or [(b, h) for b in range(bt) for h in range(hq)]
    groups = sorted({(b, h // g) for (b, h) in heads})
    for (b, kh) in groups:
        k_hat = qz.dequantize_keys(oc.k_codes[b, kh], oc.sigma[b, kh], oc.z[b, kh]).reshape(nb * 16, 128)
        v_hat = qz.dequantize_values(oc.v_codes[b, kh], oc.v_scale[b, kh], oc.v_offset[b, kh]).reshape(nb * 16, 128)
        k_tr, v_tr = oc.k16[b, kh, nb * 16:], oc.v16[b, kh, nb * 16:]
        picks = []
        for i in range(g):
            h = kh * g + i
            # ---- selector, on the GPU's own numbers
            c0 = out["cert0"][b, h]
            s = ad.select_blocks(out["l8"][b, h].astype(np.float64), float(c0["lse"]), sel)
            k = ad.rung1_expand(s, float(c0["delta_h"]), float(c0["v_max"]), tol, sel)
            if int(out["k_star"][b, h]) != k:
                # the GPU sums single-precision exponentials for the total mass: a coverage within
                # 3e-7 of tau_cov may fall on either side (decisions away from thresholds are exact)
                alt = [ad.select_blocks(out["l8"][b, h].astype(np.float64), float(c0["lse"]),
                                        ad.SelectorParams(sel.tau_cov + d, sel.k_min, sel.k_max, sel.k_limit))
                       for d in (-3e-7, 3e-7)]
                alt_k = [ad.rung1_expand(x, float(c0["delta_h"]), float(c0["v_max"]), tol, sel) for x in alt]
                assert int(out["k_star"][b, h]) in alt_k, ("K*", b, h, int(out["k_star"][b, h]), k, alt_k)
                k = int(out["k_star"][b, h])
            assert out["selected"][b, h, :k].tolist() == s["order"][:k].tolist(), ("selection", b, h)
            picks.append(s["order"][:k])
        explored = ad.explored_blocks(nb, b * oc.hkv + kh, sel)
        union = ad.group_union(picks, nb) | explored
        assert (out["promoted"][b, kh] == union).all(), ("promoted mask", b, kh)
        # ---- value promotion: decisions on the GPU's own contributions, thresholds as the GPU holds them
        vunion = np.zeros(nb, bool)
        vpicks = [np.zeros(0, np.int64)] * g
        if sel.v_limit > 0:
            tol32 = att.Tolerances(v_tol=float(np.float32(tol.v_tol)), eps_val=float(np.float32(tol.eps_val)))
            vpicks = []
            for i in range(g):
                h = kh * g + i
                c0 = out["cert0"][b, h]
                want_c = ad.value_contributions(out["l8"][b, h].astype(np.float64), float(c0["lse"]), oc.eta[b, kh])
                assert np.allclose(out["contrib"][b, h], want_c, rtol=1e-5, atol=1e-12), ("contributions", b, h)
                vs = ad.select_value_blocks_from(out["contrib"][b, h].astype(np.float64), tol32, sel)
                assert int(out["v_count"][b, h]) == len(vs), ("value count", b, h, int(out["v_count"][b, h]), len(vs))
                assert out["v_selected"][b, h, :len(vs)].tolist() == vs.tolist(), ("value selection", b, h)
                vpicks.append(vs)
            vunion = ad.group_union(vpicks, nb)
        assert (out["v_promoted"][b, kh] == vunion).all(), ("value-promoted mask", b, kh)
        for i in range(g):
            h = kh * g + i
            # the head's own promoted sets: its selections (+ explored blocks), or the group's unions
            fk = (ad.group_union([picks[i]], nb) | explored) if sel.per_head else union
            fv = ad.group_union([vpicks[i]], nb) if sel.per_head else vunion
            assert ((((out["head_keys"][b, kh] >> i) & 1) != 0) == fk).all(), ("head key bits", b, h)
            assert ((((out["head_values"][b, kh] >> i) & 1) != 0) == fv).all(), ("head value bits", b, h)
            if (b, h) not in heads:
                continue
            sc = att.certified_head(q[b, h], k_hat, v_hat, oc.sigma[b, kh], oc.eta[b, kh], oc.nu[b, kh],
                                    k_tr, v_tr, att.Tolerances(int8_query=tol.int8_query),
                                    k_codes=oc.k_codes[b, kh], z=oc.z[b, kh])
            assert np.abs(out["l8"][b, h] - sc["blk_logmass"]).max() <= 1e-4, ("scoring log-masses", b, h)
            ref = ad.mixed_head(q[b, h], k_hat, oc.k16[b, kh, :nb * 16], v_hat, oc.eta[b, kh], oc.nu[b, kh],
                                k_tr, v_tr, fk, sc["blk_logmass"], sc["lse"], sc["delta_h"], tol,
                                v_promoted=fv, v16_sealed=oc.v16[b, kh, :nb * 16], canary=sel.canary,
                                s_scored=sc["scores_sealed"] if tol.int8_query else None)
            if sel.canary:
                assert abs(float(out["score_dev"][b, h]) - ref["score_dev"]) <= 1e-4, ("score deviation", b, h)
            w = ("adaptive", b, h)
            ct = out["cert"][b, h]
            if served and served.get((b, h)):
                dense = oc.dense_head(q, b, h, hq)
                assert np.linalg.norm(out["O"][b, h] - dense) <= 1e-3 * np.linalg.norm(dense) + 1e-6, w
                assert int(ct["served_rung"]) == served[(b, h)] and ct["E_key"] == 0 and ct["E_val"] == 0, w
                assert int(out["flags"][b, h]) == (ref["flags"] | (served[(b, h)] << att.RUNG_SHIFT)), w
                continue
            # O is a convex combination of value rows of norm <= V_max, accumulated in FP32: the
            # absolute floor scales with V_max (it matters for the planted head, whose two
            # dominant values cancel and leave ||O|| ~ 4e-4 V_max)
            err = np.linalg.norm(out["O"][b, h] - ref["O"])
            assert err <= 1e-3 * np.linalg.norm(ref["O"]) + 2e-6 * ref["v_max"], (w, "O", err)
            for name in ("E_key", "E_val", "delta_h", "v_max", "alpha_tail_hat", "max_block_contrib"):
                x, y = float(ct[name]), ref[name]
                assert abs(x - y) <= 1e-4 * abs(y) + 1e-9, (w, name, x, y)
            assert abs(float(ct["lse"]) - ref["lse"]) <= 1e-4 * max(1.0, abs(ref["lse"])), (w, "lse")
            assert np.abs(out["lx"][b, h] - ref["blk_logmass"]).max() <= 1e-4, (w, "attend log-masses")
            if fk.any():
                rk = ref["ranking"]
                top2 = np.sort(ref["blk_logmass"][fk])[::-1]
                if len(top2) < 2 or top2[0] - top2[1] > 1e-3:
                    assert int(ct["top_block"]) == rk["top_fp16"], (w, "top block")
            assert int(out["flags"][b, h]) == ref["flags"], (w, "flags", int(out["flags"][b, h]), ref["flags"])


def test_adaptive_small_all_heads():
    say("adaptive: 2 sequences x 2 KV heads x 8 query heads, 2000 tokens, every head against the oracle")
    k, v, q = make_case(1, 2, 8, 2, 2000, peaked=[(0, 1, 333, 0.8), (1, 6, 1500, 1.2), (1, 7, 1501, 0.5)])
    oc = oracle.OracleLayerCache(2, 2)
    oc.append(k, v)
    with GpuLayerCache(2, 8, 2, 2048) as gc:
        gc.append(k, v)
        for tau, kmin, kmax in ((0.995, 2, 16), (0.5, 0, 4), (0.9, 1, 64)):
            sel = ad.SelectorParams(tau, kmin, kmax, kmax)
            tol = att.Tolerances(rank_depth=1)
            out = gpu_adaptive(gc, q, tol, sel)
            check_against_oracle(oc, q, tol, sel, out)
            say(f"  tau {tau} K in [{kmin},{kmax}]: K* = {out['k_star'].ravel().tolist()}, "
                f"promoted per group {out['promoted'].sum(axis=2).ravel().tolist()}")
            # promotion lowers the key term of a peaked head by orders of magnitude
            if kmax >= 16:
                assert out["cert"]["E_key"][1, 6] < 0.05 * out["cert0"]["E_key"][1, 6]


def test_adaptive_rung1_growth_and_clamps():
    say("adaptive: Rung-1 doubling against a key-term threshold, K_min / K_max / block-count clamps")
    k, v, q = make_case(2, 1, 4, 1, 1024 + 7, peaked=[(0, 2, 100, 0.7)])
    oc = oracle.OracleLayerCache(1, 1)
    oc.append(k, v)
    with GpuLayerCache(1, 4, 1, 1100) as gc:
        gc.append(k, v)
        base = gpu_adaptive(gc, q, att.Tolerances(key_bound_mode=1), ad.SelectorParams(0.3, 1, 2, 64))
        # a threshold between the key terms at K and at 4K of the most diffuse head forces growth
        ek = np.sort(base["cert"]["E_key"].ravel())
        eps = float(0.25 * ek[-1])
        tol = att.Tolerances(key_bound_mode=1, eps_key=eps)
        sel = ad.SelectorParams(0.3, 1, 2, 64)
        out = gpu_adaptive(gc, q, tol, sel)
        check_against_oracle(oc, q, tol, sel, out)
        assert (out["k_star"] > base["k_star"]).any() and out["k_star"].max() <= 64
        say(f"  K* {base['k_star'].ravel().tolist()} -> {out['k_star'].ravel().tolist()} at eps_key {eps:.3g}")
        # K_max above the number of blocks: everything is promoted, the key term vanishes and the
        # output is plain attention over the FP16 keys and the INT4-reconstructed values
        sel = ad.SelectorParams(2.0, 0, 512, 512)
        out = gpu_adaptive(gc, q, att.Tolerances(), sel)
        check_against_oracle(oc, q, att.Tolerances(), sel, out)
        assert out["promoted"].all() and (out["k_star"] == oc.n_blocks).all()
        assert (out["cert"]["E_key"] == 0).all() and (out["cert"]["alpha_tail_hat"] == 0).all()
        # nothing promoted: the one-pass result
        sel = ad.SelectorParams(0.995, 0, 0, 0)
        out = gpu_adaptive(gc, q, att.Tolerances(), sel)
        assert not out["promoted"].any() and (out["k_star"] == 0).all()
        O1, cert1, _ = gc.certified_decode(q)
        assert np.allclose(out["O"], O1, rtol=0, atol=1e-6)
        for name in ("E_key", "E_val", "alpha_tail_hat", "lse"):
            assert np.allclose(out["cert"][name], cert1[name], rtol=1e-6, atol=0)


def test_adaptive_ranking_check_and_ladder():
    say("adaptive: ranking disagreement / boundary failure set RANK, the ladder serves the head by Rung 3")
    # two planted keys in different blocks, FP16 logits 0.002 apart, both far above the rest; with this
    # seed the INT8 scores order the two blocks the other way round (found with the oracle)
    k, v, q = make_case(10, 1, 8, 2, 4096 + 3)
    workloads.plant_near_tie(k, v, q, 0, 5, 8, seed=10, gap=12.0, nudge=0.002)
    oc = oracle.OracleLayerCache(1, 2)
    oc.append(k, v)
    with GpuLayerCache(1, 8, 2, 4200) as gc:
        gc.append(k, v)
        tol = att.Tolerances(rank_depth=1, rank_min_mass=0.25)
        # (i) both tied blocks promoted: the two rankings disagree on the top block
        sel = ad.SelectorParams(0.995, 2, 32, 32)
        out = gpu_adaptive(gc, q, tol, sel)
        check_against_oracle(oc, q, tol, sel, out)
        assert out["flags"][0, 5] & att.FLAG_RANK
        # (ii) room for one block only: the other tied block stays in INT8 and its upper-bounded
        # log-mass reaches the promoted one's, so the boundary test cannot certify the ranking
        sel1 = ad.SelectorParams(0.0, 1, 1, 1)
        out1 = gpu_adaptive(gc, q, tol, sel1)
        check_against_oracle(oc, q, tol, sel1, out1)
        assert out1["flags"][0, 5] & att.FLAG_RANK and out1["cert"]["rank_margin"][0, 5] < 0
        # the ladder
        flagged = {(0, h): 3 for h in range(8) if out["flags"][0, h] & att.FLAG_ANY}
        stepped = gpu_adaptive(gc, q, tol, sel, step=True)
        assert stepped["rung"] == 3 and (0, 5) in flagged
        check_against_oracle(oc, q, tol, sel, stepped, served=flagged)
        say(f"  heads served by Rung 3: {sorted(h for (_, h) in flagged)}")
        # the same step with the ladder resolved on the device
        enq = gpu_adaptive(gc, q, tol, sel, step="enqueue")
        check_against_oracle(oc, q, tol, sel, enq, served=flagged)
        assert (enq["flags"] == stepped["flags"]).all()
        assert (enq["cert"]["served_rung"] == stepped["cert"]["served_rung"]).all()
        sv = enq["cert"]["served_rung"] == 3
        assert (enq["O"][~sv] == stepped["O"][~sv]).all()
        # (two dense passes that split the sequence differently; the planted head's two dominant
        # values nearly cancel, so the bar is absolute: 2e-6 of the largest value magnitude)
        assert np.abs(enq["O"][sv] - stepped["O"][sv]).max() <= 2e-6 * float(np.abs(v.astype(np.float32)).max())


def test_adaptive_value_promotion():
    say("adaptive: value promotion (threshold and hard-budget policies), alone and together with key promotion")
    k, v, q = make_case(5, 2, 8, 2, 3000, peaked=[(0, 2, 700, 0.9), (1, 5, 2100, 1.1)])
    oc = oracle.OracleLayerCache(2, 2)
    oc.append(k, v)
    with GpuLayerCache(2, 8, 2, 3100) as gc:
        gc.append(k, v)
        base = gpu_adaptive(gc, q, att.Tolerances(), ad.SelectorParams(0.995, 0, 0, 0))
        ev = base["cert"]["E_val"]
        # (i) threshold policy only, no key promotion
        sel = ad.SelectorParams(0.995, 0, 0, 0, v_limit=64)
        tol = att.Tolerances(v_tol=0.02)
        out = gpu_adaptive(gc, q, tol, sel)
        check_against_oracle(oc, q, tol, sel, out)
        assert out["v_promoted"].any() and (out["cert"]["E_val"] <= ev + 1e-6).all()
        assert (out["cert"]["max_block_contrib"] <= 0.02 * (1 + 1e-3)).all()
        # (ii) hard budget: half of the one-pass value term of the most demanding head
        sel = ad.SelectorParams(0.995, 0, 0, 0, v_limit=512, v_greedy=True)
        tol = att.Tolerances(eps_val=float(0.5 * ev.max()))
        out = gpu_adaptive(gc, q, tol, sel)
        check_against_oracle(oc, q, tol, sel, out)
        assert (out["cert"]["E_val"] <= tol.eps_val * (1 + 1e-4)).all() and not (out["flags"] & att.FLAG_VAL).any()
        say(f"  budget {tol.eps_val:.3f}: value blocks per head {out['v_count'].ravel().tolist()}")
        # (iii) both rungs together
        sel = ad.SelectorParams(0.995, 2, 32, 32, v_limit=128, v_greedy=True)
        tol = att.Tolerances(eps_val=float(0.7 * ev.max()), v_tol=0.05, rank_depth=1)
        out = gpu_adaptive(gc, q, tol, sel)
        check_against_oracle(oc, q, tol, sel, out)
        both = (out["promoted"] & out["v_promoted"]).sum()
        say(f"  keys and values: {out['promoted'].sum()} key blocks, {out['v_promoted'].sum()} value blocks, {both} both")
        # (iv) every value promoted and every key promoted: the dense result
        sel = ad.SelectorParams(2.0, 0, 512, 512, v_limit=512, v_greedy=True)
        tol = att.Tolerances(eps_val=0.0)
        out = gpu_adaptive(gc, q, tol, sel)
        check_against_oracle(oc, q, tol, sel, out)
        assert out["promoted"].all() and out["v_promoted"].all()
        assert (out["cert"]["E_key"] == 0).all() and (out["cert"]["E_val"] == 0).all()
        for b in range(2):
            for h in range(8):
                dense = oc.dense_head(q, b, h, 8)
                assert np.linalg.norm(out["O"][b, h] - dense) <= 1e-3 * np.linalg.norm(dense) + 1e-6


def test_adaptive_monitors():
    say("adaptive: score-consistency canary and exploration budget")
    k, v, q = make_case(6, 1, 8, 2, 4096 + 9, peaked=[(0, 3, 1000, 1.0)])
    oc = oracle.OracleLayerCache(1, 2)
    oc.append(k, v)
    with GpuLayerCache(1, 8, 2, 4200) as gc:
        gc.append(k, v)
        sel = ad.SelectorParams(0.995, 2, 16, 16, canary=True, explore_frac=0.03, explore_seed=41)
        tol = att.Tolerances(rank_depth=1, rank_min_mass=0.25)
        out = gpu_adaptive(gc, q, tol, sel)
        check_against_oracle(oc, q, tol, sel, out)
        explored = np.stack([ad.explored_blocks(oc.n_blocks, g, sel) for g in range(2)])
        assert explored.sum() > 0 and (out["promoted"][0] >= explored).all()
        assert not (out["flags"] & att.FLAG_PRECOND).any()
        assert (out["score_dev"] > 0).all() and (out["score_dev"] <= out["cert"]["delta_h"] * (1 + 1e-3)).all()
        say(f"  explored blocks per group {explored.sum(axis=1).tolist()}, largest |s_fp16 - s_int8| / Delta_h = "
            f"{float((out['score_dev'] / out['cert']['delta_h']).max()):.3f}")
        # another seed draws other blocks
        sel2 = ad.SelectorParams(0.995, 2, 16, 16, canary=True, explore_frac=0.03, explore_seed=42)
        out2 = gpu_adaptive(gc, q, tol, sel2)
        check_against_oracle(oc, q, tol, sel2, out2)
        assert (out2["promoted"] != out["promoted"]).any()
        # the firing path, forced from the host: a guard so negative that every deviation exceeds the
        # bound; every head reports PRECOND and the ladder recomputes the whole layer (Rung 4)
        tolf = att.Tolerances(eps_guard=-10.0)
        fired = gpu_adaptive(gc, q, tolf, sel, step=True)
        assert fired["rung"] == 4
        check_against_oracle(oc, q, tolf, sel, fired, served={(0, h): 4 for h in range(8)})


@pytest.mark.parametrize("hq,hkv", [(2, 2), (4, 2), (8, 2)])
def test_adaptive_gqa_widths_ragged_appends_and_reset(hq, hkv):
    say(f"adaptive: {hq} query / {hkv} KV heads, appended steps with ragged block counts, reset")
    g = hq // hkv
    sel = ad.SelectorParams(0.9, 1, 8, 16, v_limit=8, canary=True, explore_frac=0.02, explore_seed=3)
    tol = att.Tolerances(rank_depth=1, v_tol=0.2)
    k, v, q = make_case(20 + hq, 1, hq, hkv, 10)
    oc = oracle.OracleLayerCache(1, hkv)
    with GpuLayerCache(1, hq, hkv, 700) as gc:
        # fewer than 16 tokens: nothing is sealed, the exact trailing tokens are the whole answer
        oc.append(k, v)
        gc.append(k, v)
        out = gpu_adaptive(gc, q, tol, sel)
        ref = oc.certified_decode(q, tol)
        for h in range(hq):
            assert np.linalg.norm(out["O"][0, h] - ref[h]["O"]) <= 1e-3 * np.linalg.norm(ref[h]["O"]) + 1e-6
            assert out["cert"]["E_key"][0, h] == 0 and out["cert"]["E_val"][0, h] == 0
        # grow through ragged lengths (block counts 1, 2, 5, 6, 13, 41: partial quads, partial blocks)
        rng = np.random.Generator(np.random.Philox(900 + hq))
        for n_new in (7, 16, 50, 13, 120, 440):
            ks, vs = workloads.normal_f16(rng, (1, hkv, n_new, 128)), workloads.normal_f16(rng, (1, hkv, n_new, 128))
            oc.append(ks, vs)
            gc.append(ks, vs)
            qq = workloads.normal_f16(rng, (1, hq, 128))
            out = gpu_adaptive(gc, qq, tol, sel)
            check_against_oracle(oc, qq, tol, sel, out)
        # reset and start over with a shorter cache: nothing of the old run may show through
        gc.cqa.cqa_cache_reset(gc.h, 0)
        oc2 = oracle.OracleLayerCache(1, hkv)
        k2, v2, q2 = make_case(40 + hq, 1, hq, hkv, 100)
        oc2.append(k2, v2)
        gc.append(k2, v2)
        out = gpu_adaptive(gc, q2, tol, sel)
        check_against_oracle(oc2, q2, tol, sel, out)


def test_adaptive_error_paths():
    cqa = load_binding()
    k, v, q = make_case(4, 1, 4, 1, 64)
    with GpuLayerCache(1, 4, 1, 128, tier2=False) as gc:
        gc.append(k, v)
        with pytest.raises(cqa.CqaError) as e:
            cqa.cqa_adaptive_decode(gc.h, 0, gc.to_dev(q), cqa.Tolerances(), cqa.Selector(), gc.O, gc.cert, gc.flags)
        assert e.value.status == cqa.ERR_NO_TIER2
    with GpuLayerCache(1, 4, 1, 128) as gc:
        gc.append(k, v)
        for bad in (cqa.Selector(0.9, 4, 2, 2), cqa.Selector(0.9, 0, 600, 600), cqa.Selector(0.9, -1, 2, 2),
                    cqa.Selector(0.9, 0, 8, 4), cqa.Selector(0.9, 0, 8, 8, v_limit=513),
                    cqa.Selector(0.9, 0, 8, 8, v_limit=-1)):
            with pytest.raises(cqa.CqaError) as e:
                cqa.cqa_adaptive_decode(gc.h, 0, gc.to_dev(q), cqa.Tolerances(), bad, gc.O, gc.cert, gc.flags)
            assert e.value.status == cqa.ERR_INVALID_ARG


def test_adaptive_128k_sampled_heads():
    say("adaptive: N=131072, Student-t(3) keys; selector exact on every head, oracle attend pass on 3 heads")
    sh = workloads.SHAPES["t128k"]
    k, v = workloads.make_kv("t128k", seed=0)
    q = workloads.make_q("t128k", 3, seed=0)
    oc = oracle.OracleLayerCache(sh.batch, sh.n_kv_heads)
    oc.append(k, v)
    ks, vs = workloads.make_step_kv("t128k", 0, seed=0)
    oc.append(ks, vs)
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.context + 64) as gc:
        gc.append(k, v)
        gc.append(ks, vs)
        sel = ad.SelectorParams(0.995, 2, 128, 128)
        tol = att.Tolerances(rank_depth=1, rank_min_mass=0.25)
        out = gpu_adaptive(gc, q, tol, sel)
        # selector decisions on every head (cheap), attend pass on the heads of one KV group
        bt, hq = sh.batch, sh.n_q_heads
        nb = oc.n_blocks
        for h in range(hq):
            c0 = out["cert0"][0, h]
            s = ad.select_blocks(out["l8"][0, h].astype(np.float64), float(c0["lse"]), sel)
            kk = ad.rung1_expand(s, float(c0["delta_h"]), float(c0["v_max"]), tol, sel)
            assert int(out["k_star"][0, h]) == kk and out["selected"][0, h, :kk].tolist() == s["order"][:kk].tolist()
        check_against_oracle(oc, q, tol, sel, out, heads=[(0, 8), (0, 9), (0, 11)])
        say(f"  K* min/median/max {out['k_star'].min()}/{int(np.median(out['k_star']))}/{out['k_star'].max()}, "
            f"promoted per group {out['promoted'].sum(axis=2).ravel().tolist()} of {nb}")


def test_key_scratch_does_not_change_results_and_holds_recent_blocks():
    say("adaptive: FP16 scratch on the device (hits, misses, eviction) gives the same bits as reading the host")
    k, v, q = make_case(21, 2, 8, 2, 16 * 300 + 9, peaked=[(0, 1, 1500, 0.9), (1, 6, 40, 1.0)])
    rng = np.random.Generator(np.random.Philox(77))
    qs = [q] + [workloads.normal_f16(rng, q.shape) for _ in range(3)]
    sel = ad.SelectorParams(0.9, 4, 64, 64)
    tol = att.Tolerances(rank_depth=1)
    with GpuLayerCache(2, 8, 2, 16 * 300 + 64) as gc:
        cqa = gc.cqa
        gc.append(k, v)
        assert cqa.cqa_scratch_stats(gc.h) == (0, 0, 0)    # off until asked for
        # reference: scratch off, every promoted block read from the pinned originals
        ref = [gpu_adaptive(gc, x, tol, sel) for x in qs]
        assert cqa.cqa_scratch_stats(gc.h) == (0, 0, 0)
        promoted = [int(r["promoted"].sum()) for r in ref]

        def same(a, b, w):
            assert (a["O"] == b["O"]).all() and a["cert"].tobytes() == b["cert"].tobytes(), w
            assert (a["flags"] == b["flags"]).all() and (a["promoted"] == b["promoted"]).all(), w
            assert (a["lx"] == b["lx"]).all(), w

        # (i) room for everything (capacity 304 blocks -> at most 512 slots): first use misses,
        # the same query again hits every block
        cqa.cqa_set_scratch_slots(gc.h, 512)
        same(gpu_adaptive(gc, qs[0], tol, sel), ref[0], "cold")
        assert cqa.cqa_scratch_stats(gc.h) == (512, 0, promoted[0])
        same(gpu_adaptive(gc, qs[0], tol, sel), ref[0], "warm")
        assert cqa.cqa_scratch_stats(gc.h) == (512, promoted[0], promoted[0])
        for i in (1, 2, 3, 1):
            same(gpu_adaptive(gc, qs[i], tol, sel), ref[i], ("other queries", i))
        # (ii) fewer slots than one step promotes per group: the overflow is read from the host,
        # later steps evict the least recently used slots; results stay the same
        per_group = ref[0]["promoted"].sum(axis=2).max()
        small = max(2, int(per_group) // 2)
        cqa.cqa_set_scratch_slots(gc.h, small)
        _, h1, m1 = cqa.cqa_scratch_stats(gc.h)
        for rep in range(2):
            for i in (0, 1, 0, 2, 3):
                same(gpu_adaptive(gc, qs[i], tol, sel), ref[i], ("small scratch", rep, i))
        _, h2, m2 = cqa.cqa_scratch_stats(gc.h)
        assert h2 > h1 and m2 > m1
        say(f"  {small} slots per head: {h2 - h1} hits, {m2 - m1} misses over 10 steps")
        # (iii) a reset empties the layer's scratch: appending other keys must not find the old ones
        cqa.cqa_set_scratch_slots(gc.h, 512)
        gpu_adaptive(gc, qs[0], tol, sel)
        cqa.cqa_cache_reset(gc.h, 0)
        k2, v2, _ = make_case(22, 2, 8, 2, 16 * 300 + 9)
        gc.append(k2, v2)
        oc2 = oracle.OracleLayerCache(2, 2)
        oc2.append(k2, v2)
        out = gpu_adaptive(gc, qs[0], tol, sel)
        check_against_oracle(oc2, qs[0], tol, sel, out)
        out = gpu_adaptive(gc, qs[0], tol, sel)          # now from the scratch
        check_against_oracle(oc2, qs[0], tol, sel, out)
        with pytest.raises(cqa.CqaError):
            cqa.cqa_set_scratch_slots(gc.h, 513)


def test_scratch_holds_promoted_values_too():
    say("adaptive: the scratch's value halves (cold, warm, a slot that held only keys, eviction) give the same bits")
    k, v, q = make_case(23, 2, 8, 2, 16 * 300 + 9, peaked=[(0, 1, 1500, 0.9), (1, 6, 40, 1.0)])
    rng = np.random.Generator(np.random.Philox(78))
    qs = [q] + [workloads.normal_f16(rng, q.shape) for _ in range(2)]
    tol = att.Tolerances(rank_depth=1, v_tol=0.004)

    def same(a, b, w):
        assert (a["O"] == b["O"]).all() and a["cert"].tobytes() == b["cert"].tobytes(), w
        assert (a["flags"] == b["flags"]).all() and (a["promoted"] == b["promoted"]).all(), w
        assert (a["v_promoted"] == b["v_promoted"]).all() and (a["lx"] == b["lx"]).all(), w

    for per_head in (False, True):
        sel_v = ad.SelectorParams(0.5, 2, 6, 6, v_limit=24, per_head=per_head)
        with GpuLayerCache(2, 8, 2, 16 * 300 + 64) as gc:
            cqa = gc.cqa
            gc.append(k, v)
            ref = [gpu_adaptive(gc, x, tol, sel_v) for x in qs]
            ref_k = gpu_adaptive(gc, qs[0], tol, ad.SelectorParams(0.5, 2, 6, 6, per_head=per_head))
            listed = [int((r["promoted"] | r["v_promoted"]).sum()) for r in ref]
            assert ref[0]["v_promoted"].sum() > 0 and (ref[0]["v_promoted"] & ~ref[0]["promoted"]).sum() > 0
            # the value promotion is really on: the value term shrinks against keys-only promotion
            assert (ref[0]["cert"]["E_val"] < ref_k["cert"]["E_val"]).any()
            # cold, then warm
            cqa.cqa_set_scratch_slots(gc.h, 512)
            same(gpu_adaptive(gc, qs[0], tol, sel_v), ref[0], "cold")
            assert cqa.cqa_scratch_stats(gc.h) == (512, 0, listed[0])
            same(gpu_adaptive(gc, qs[0], tol, sel_v), ref[0], "warm")
            assert cqa.cqa_scratch_stats(gc.h) == (512, listed[0], listed[0])
            # slots that hold only the keys: a step that also needs the block's values fills the other half
            cqa.cqa_set_scratch_slots(gc.h, 512)
            same(gpu_adaptive(gc, qs[0], tol, ad.SelectorParams(0.5, 2, 6, 6, per_head=per_head)), ref_k, "keys only")
            _, h0, m0 = cqa.cqa_scratch_stats(gc.h)
            same(gpu_adaptive(gc, qs[0], tol, sel_v), ref[0], "values join")
            _, h1, m1 = cqa.cqa_scratch_stats(gc.h)
            assert m1 - m0 >= int(ref[0]["v_promoted"].sum()) and (h1 - h0) + (m1 - m0) == listed[0]
            same(gpu_adaptive(gc, qs[0], tol, sel_v), ref[0], "both halves held")
            _, h2, m2 = cqa.cqa_scratch_stats(gc.h)
            assert (h2 - h1, m2 - m1) == (listed[0], 0)
            # fewer slots than a step lists: overflow from the host, eviction in later steps
            cqa.cqa_set_scratch_slots(gc.h, 3)
            for rep in range(2):
                for i in (0, 1, 0, 2):
                    same(gpu_adaptive(gc, qs[i], tol, sel_v), ref[i], ("small scratch", per_head, rep, i))


def test_long_context_beyond_the_selector_lds_window():
    say("long context: 16 * 20500 + 11 tokens, one KV head (the selector re-reads rows that do not fit its "
        "LDS key buffer; indices beyond 2^18 tokens), one-pass path and adaptive path against the oracle")
    n = 16 * 20500 + 11
    k, v, q = make_case(33, 1, 4, 1, n, student=True, peaked=[(0, 2, n - 5000, 0.8)])
    oc = oracle.OracleLayerCache(1, 1)
    oc.append(k, v)
    with GpuLayerCache(1, 4, 1, n + 16) as gc:
        for pos in range(0, n, 100000):            # appended in pieces: ragged joins between them
            gc.append(k[:, :, pos:pos + 100000], v[:, :, pos:pos + 100000])
        assert gc.length() == n
        O, cert, flags, lm = gc.certified_decode(q, want_logmass=True)
        ref = oc.certified_decode(q, att.Tolerances())
        for h, r in enumerate(ref):
            assert_head_matches(r, O[0, h], cert[0, h], flags[0, h], ("long", h))
            assert np.abs(lm[0, h] - r["blk_logmass"]).max() <= 1e-4
        for sel in (ad.SelectorParams(0.995, 2, 128, 128), ad.SelectorParams(0.9999, 8, 512, 512)):
            tol = att.Tolerances(rank_depth=1, rank_min_mass=0.25, v_tol=0.05)
            out = gpu_adaptive(gc, q, tol, sel)
            check_against_oracle(oc, q, tol, sel, out)
            say(f"  K* {out['k_star'].ravel().tolist()}, promoted {int(out['promoted'].sum())} of {oc.n_blocks}")
        # the enqueue-only step with one head over its tolerance
        tot = np.sort((cert["E_key"].astype(np.float64) + cert["E_val"]).ravel())
        if tot[-1] - tot[-2] > 1e-3 * tot[-1]:
            gtol = gc.cqa.Tolerances(eps_total=float(0.5 * (tot[-1] + tot[-2])))
            gc.cqa.cqa_decode_step_enqueue(gc.h, 0, None, None, gc.to_dev(q), gtol, gc.O, gc.cert, gc.flags)
            O2, cert2, _ = gc.results()
            sv = cert2["served_rung"] == 3
            assert sv.sum() == 1 and (O2[~sv] == O[~sv]).all()
            h = int(np.argwhere(sv)[0][1])
            dense = oracle.softmax_attention(q[0, h], k[0, 0], v[0, 0])
            assert np.linalg.norm(O2[0, h] - dense) <= 1e-3 * np.linalg.norm(dense) + 1e-6


def test_long_context_diffuse_heads_rung1_to_the_limit():
    say("long context, diffuse heads (normal keys): K* at K_max, Rung 1 doubling to k_limit = 512 on rows the "
        "selector re-reads")
    n = 16 * 10600 + 3
    k, v, q = make_case(34, 1, 4, 1, n)
    oc = oracle.OracleLayerCache(1, 1)
    oc.append(k, v)
    with GpuLayerCache(1, 4, 1, n + 16) as gc:
        gc.append(k, v)
        sel = ad.SelectorParams(0.995, 2, 128, 512)
        tol = att.Tolerances(eps_key=1e-3, rank_depth=1)
        out = gpu_adaptive(gc, q, tol, sel)
        check_against_oracle(oc, q, tol, sel, out)
        assert (out["k_star"] == 512).all()
        say(f"  promoted {int(out['promoted'].sum())} of {oc.n_blocks}")


def test_adaptive_batched_serving_shape():
    say("adaptive: batch 64 x 4096 tokens (2048 selector workgroups, 512 KV groups), three sampled sequences "
        "against the oracle")
    sh = workloads.SHAPES["serve64"]
    k, v = workloads.make_kv("serve64", seed=0)
    q = workloads.make_q("serve64", 1, seed=0)
    rows = [0, 31, 63]
    oc = oracle.OracleLayerCache(len(rows), sh.n_kv_heads)
    oc.append(k[rows], v[rows])
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.context + 16) as gc:
        gc.append(k, v)
        sel = ad.SelectorParams(0.995, 2, 64, 64, v_limit=32)
        tol = att.Tolerances(rank_depth=1, rank_min_mass=0.25, v_tol=0.05)
        out = gpu_adaptive(gc, q, tol, sel)
        sub = {name: (val[rows] if isinstance(val, np.ndarray) else val) for name, val in out.items()}
        check_against_oracle(oc, q[rows], tol, sel, sub)
        say(f"  K* median {int(np.median(out['k_star']))} max {out['k_star'].max()}, "
            f"promoted per group max {out['promoted'].sum(axis=2).max()}")


def test_random_small_shapes_and_selectors():
    say("24 seeded random small shapes and selector settings (keys and values promoted, canary, exploration) "
        "against the oracle")
    rng = np.random.default_rng(77)
    for case in range(24):
        bt = int(rng.integers(1, 3))
        hkv = int(rng.integers(1, 3))
        group = int(rng.choice([1, 2, 4]))
        hq = hkv * group
        n = int(rng.choice([16, 17, 33, 160, 161, 500, 1023, 1024, 2000]))
        k, v, q = make_case(1000 + case, bt, hq, hkv, n, student=bool(rng.integers(0, 2)))
        oc = oracle.OracleLayerCache(bt, hkv)
        oc.append(k, v)
        k_min = int(rng.integers(0, 4))
        k_max = int(k_min + rng.integers(0, 40))
        sel = ad.SelectorParams(float(rng.choice([0.5, 0.9, 0.995, 1.0])), k_min, k_max,
                                int(k_max + rng.integers(0, 64)), v_limit=int(rng.choice([0, 0, 16, 64])),
                                v_greedy=bool(rng.integers(0, 2)), canary=bool(rng.integers(0, 2)),
                                explore_frac=float(rng.choice([0.0, 0.0, 0.03])), explore_seed=case)
        tol = att.Tolerances(eps_key=float(rng.choice([np.inf, 0.05, 0.5])), v_tol=float(rng.choice([np.inf, 0.05])),
                             eps_val=float(rng.choice([np.inf, 0.2])), rank_depth=int(rng.choice([0, 1, 2, 3, 8])),
                             rank_min_mass=float(rng.choice([0.0, 0.25])))
        with GpuLayerCache(bt, hq, hkv, n + 8) as gc:
            gc.append(k, v)
            out = gpu_adaptive(gc, q, tol, sel)
            try:
                check_against_oracle(oc, q, tol, sel, out)
            except AssertionError as e:
                raise AssertionError(("case", case, bt, hkv, group, n, sel, tol)) from e


def test_random_small_shapes_with_quantised_query_and_per_head_sets():
    say("20 more seeded random small shapes: quantised-query scoring and per-head promoted sets drawn at random too")
    rng = np.random.default_rng(78)
    for case in range(20):
        bt = int(rng.integers(1, 3))
        hkv = int(rng.integers(1, 3))
        group = int(rng.choice([1, 2, 4]))
        hq = hkv * group
        n = int(rng.choice([16, 31, 48, 161, 500, 1024, 1500]))
        k, v, q = make_case(2000 + case, bt, hq, hkv, n, student=bool(rng.integers(0, 2)))
        oc = oracle.OracleLayerCache(bt, hkv)
        oc.append(k, v)
        k_min = int(rng.integers(0, 4))
        k_max = int(k_min + rng.integers(0, 40))
        sel = ad.SelectorParams(float(rng.choice([0.5, 0.9, 0.995])), k_min, k_max,
                                int(k_max + rng.integers(0, 64)), v_limit=int(rng.choice([0, 16])),
                                canary=bool(rng.integers(0, 2)), explore_frac=float(rng.choice([0.0, 0.03])),
                                explore_seed=case, per_head=bool(rng.integers(0, 2)))
        tol = att.Tolerances(v_tol=float(rng.choice([np.inf, 0.05])), rank_depth=int(rng.choice([0, 1, 2])),
                             rank_min_mass=float(rng.choice([0.0, 0.25])), int8_query=bool(case % 4 != 3),
                             mass_exp=int(rng.choice([2, 3])))
        with GpuLayerCache(bt, hq, hkv, n + 8) as gc:
            gc.append(k, v)
            out = gpu_adaptive(gc, q, tol, sel)
            try:
                check_against_oracle(oc, q, tol, sel, out)
            except AssertionError as e:
                raise AssertionError(("case", case, bt, hkv, group, n, sel, tol)) from e


def test_ranking_check_at_depth_r():
    say("adaptive: ranking check at depths 1..8 on diffuse heads, flags and margins against the oracle")
    k, v, q = make_case(41, 2, 8, 2, 16 * 220 + 5)
    oc = oracle.OracleLayerCache(2, 2)
    oc.append(k, v)
    with GpuLayerCache(2, 8, 2, 16 * 220 + 16) as gc:
        gc.append(k, v)
        sel = ad.SelectorParams(0.5, 4, 24, 24)
        flagged = {}
        for depth in (1, 2, 3, 5, 8):
            tol = att.Tolerances(rank_depth=depth, rank_min_mass=0.0, eps_guard=0.0)
            out = gpu_adaptive(gc, q, tol, sel)
            check_against_oracle(oc, q, tol, sel, out)
            flagged[depth] = (out["flags"] & att.FLAG_RANK) != 0
        say("  heads with RANK by depth: " + ", ".join(f"{d}: {int(f.sum())}" for d, f in flagged.items()))
        # a group with fewer promoted blocks than the depth: the depth is their number
        sel2 = ad.SelectorParams(0.0, 2, 2, 2)
        tol = att.Tolerances(rank_depth=8, rank_min_mass=0.0)
        out = gpu_adaptive(gc, q, tol, sel2)
        check_against_oracle(oc, q, tol, sel2, out)
        with pytest.raises(gc.cqa.CqaError) as e:
            gpu_adaptive(gc, q, att.Tolerances(rank_depth=9), sel)
        assert e.value.status == gc.cqa.ERR_UNSUPPORTED


def test_ranking_depth_two_catches_a_swap_below_the_top_block():
    say("adaptive: a dominant block, then two nearly tied blocks that the INT8 scores order the other way round: "
        "certified at depth 1, RANK at depth 2 and deeper")
    # the tied pair of test_adaptive_ranking_check_and_ladder (with this seed the INT8 scores swap it) ...
    k, v, q = make_case(10, 1, 8, 2, 4096 + 3)
    p1, p2 = workloads.plant_near_tie(k, v, q, 0, 5, 8, seed=10, gap=12.0, nudge=0.002)
    # ... under a third key along the same direction whose logit lies 3 above the pair's
    qf = q[0, 5].astype(np.float64)
    base = k[0, 1, p1].astype(np.float64)
    l1 = float(qf @ base) / math.sqrt(128.0)
    p0 = 16 * 100 + 7
    assert p0 // 16 not in (p1 // 16, p2 // 16)
    k[0, 1, p0] = (base * (1.0 + 3.0 / l1)).astype(np.float16)
    oc = oracle.OracleLayerCache(1, 2)
    oc.append(k, v)
    with GpuLayerCache(1, 8, 2, 4200) as gc:
        gc.append(k, v)
        sel = ad.SelectorParams(0.995, 3, 32, 32)
        got = {}
        for depth in (1, 2, 3):
            tol = att.Tolerances(rank_depth=depth, rank_min_mass=0.25)
            out = gpu_adaptive(gc, q, tol, sel)
            check_against_oracle(oc, q, tol, sel, out)
            got[depth] = bool(out["flags"][0, 5] & att.FLAG_RANK)
            assert int(out["cert"]["top_block"][0, 5]) == p0 // 16
            assert out["promoted"][0, 1, [p0 // 16, p1 // 16, p2 // 16]].all()
        assert got == {1: False, 2: True, 3: True}


def test_adaptive_end_to_end_from_raw_inputs_where_margins_are_clear():
    """No GPU number enters the oracle here: oracle.adaptive.adaptive_decode runs on the raw FP16
    inputs (its own scoring pass, its own selection, its own attend pass) and the GPU's decisions
    and results are compared with it.  Every head is peaked on planted keys so that the selection
    is decided by wide margins (coverage far from tau_cov on both sides of K*, log-mass gaps at the
    selection boundary far above the 1e-4 accuracy of the log-masses); the test checks that the
    margins really are wide before it compares."""
    say("adaptive: end to end against the oracle on raw inputs (clear selection margins)")
    bt, hq, hkv, n = 2, 8, 2, 4000 + 9
    g = hq // hkv
    rng = np.random.Generator(np.random.Philox(77))
    k = workloads.normal_f16(rng, (bt, hkv, n, 128))
    v = workloads.normal_f16(rng, (bt, hkv, n, 128))
    q = np.zeros((bt, hq, 128), np.float16)
    for b in range(bt):
        for h in range(hq):
            kh = h // g
            p1 = 16 * (7 + 11 * h + 3 * b) + (h % 16)          # distinct blocks per head
            p2 = 16 * (100 + 13 * h + 5 * b) + ((3 * h) % 16)
            if h % 2:                                           # odd heads: a second key, slightly weaker
                k[b, kh, p2] = (k[b, kh, p1].astype(np.float32) * 0.97).astype(np.float16)
            q[b, h] = (k[b, kh, p1].astype(np.float32) * 1.3).astype(np.float16)
    oc = oracle.OracleLayerCache(bt, hkv)
    oc.append(k, v)
    sel = ad.SelectorParams(0.9, 1, 8, 8)
    tol = att.Tolerances(rank_depth=1)
    ref = ad.adaptive_decode(oc, q, tol, sel)
    # the margins that make the comparison meaningful
    for (b, h), r in ref.items():
        s = ad.select_blocks(r["scoring"]["blk_logmass"], r["scoring"]["lse"], sel)
        kk = r["k_star"]
        assert kk == (2 if h % 2 else 1), (b, h, kk)
        cov = s["rho_trail"] + np.concatenate([[0.0], np.cumsum(s["p_sorted"])])
        assert cov[kk] - sel.tau_cov > 1e-3 and (kk == sel.k_min or sel.tau_cov - cov[kk - 1] > 1e-3), (b, h)
        lsort = r["scoring"]["blk_logmass"][s["order"]]
        assert (lsort[:kk] - lsort[1:kk + 1]).min() > 0.05, (b, h)      # every rank up to the boundary is clear
    with GpuLayerCache(bt, hq, hkv, n + 64) as gc:
        gc.append(k, v)
        out = gpu_adaptive(gc, q, tol, sel)
        for (b, h), r in ref.items():
            w = ("raw adaptive", b, h)
            kk = r["k_star"]
            assert int(out["k_star"][b, h]) == kk, w
            assert out["selected"][b, h, :kk].tolist() == [int(x) for x in r["selected"]], w
            assert (out["promoted"][b, h // g] == r["promoted"]).all(), w
            assert not out["v_promoted"][b, h // g].any(), w
            ct = out["cert"][b, h]
            err = np.linalg.norm(out["O"][b, h] - r["O"])
            assert err <= 1e-3 * np.linalg.norm(r["O"]) + 2e-6 * r["v_max"], (w, "O", err)
            assert np.abs(out["O"][b, h] - r["O"]).max() <= 1e-3 * np.abs(r["O"]).max() + 2e-6 * r["v_max"], (w, "O element")
            for name in ("E_key", "E_val", "delta_h", "v_max", "alpha_tail_hat", "max_block_contrib"):
                x, y = float(ct[name]), r[name]
                assert abs(x - y) <= 1e-4 * abs(y) + 1e-9, (w, name, x, y)
            assert abs(float(ct["lse"]) - r["lse"]) <= 1e-4 * max(1.0, abs(r["lse"])), (w, "lse")
            assert np.abs(out["l8"][b, h] - r["scoring"]["blk_logmass"]).max() <= 1e-4, (w, "scoring log-masses")
            assert np.abs(out["lx"][b, h] - r["blk_logmass"]).max() <= 1e-4, (w, "attend log-masses")
            assert int(ct["top_block"]) == r["ranking"]["top_fp16"], (w, "top block")
            assert int(out["flags"][b, h]) == r["flags"], (w, "flags", int(out["flags"][b, h]), r["flags"])
            # the key term shrank with the tail
            assert float(ct["E_key"]) < 0.2 * float(out["cert0"]["E_key"][b, h]), w


def test_per_head_promoted_sets_against_the_union_variant():
    """The paper's default (every head promotes its own selection) next to the per-KV-group union:
    both against the oracle, keys and values, with exploration and the canary on; the head bits
    differ between the modes, the group-level masks do not."""
    say("adaptive: per-head promoted sets (the paper's default) and the per-group union")
    k, v, q = make_case(31, 2, 8, 2, 3000 + 7, peaked=[(0, 1, 333, 0.9), (0, 2, 1900, 1.1), (1, 4, 77, 0.8),
                                                       (1, 6, 1500, 1.2), (1, 7, 1501, 0.6)])
    oc = oracle.OracleLayerCache(2, 2)
    oc.append(k, v)
    with GpuLayerCache(2, 8, 2, 3100) as gc:
        gc.append(k, v)
        outs = {}
        for per_head in (True, False):
            for tau, kmin, kmax, vlim in ((0.9, 1, 8, 0), (0.995, 2, 16, 8)):
                sel = ad.SelectorParams(tau, kmin, kmax, kmax, v_limit=vlim, canary=True, explore_frac=0.02,
                                        explore_seed=5, per_head=per_head)
                tol = att.Tolerances(rank_depth=2, v_tol=0.01 if vlim else math.inf)
                out = gpu_adaptive(gc, q, tol, sel)
                check_against_oracle(oc, q, tol, sel, out)
                outs[(per_head, kmax)] = out
        for kmax in (8, 16):
            ph, un = outs[(True, kmax)], outs[(False, kmax)]
            assert (ph["promoted"] == un["promoted"]).all() and (ph["k_star"] == un["k_star"]).all()
            assert (ph["head_keys"] != un["head_keys"]).any()
            # a head's own set only loses blocks against the union: its achieved tail is no smaller
            assert (ph["cert"]["alpha_tail_hat"] >= un["cert"]["alpha_tail_hat"] * (1 - 1e-6)).all()
            say(f"  K_max {kmax}: (head, block) pairs with FP16 keys per-head "
                f"{int(sum(bin(int(x)).count('1') for x in ph['head_keys'].ravel()))} / union "
                f"{int(sum(bin(int(x)).count('1') for x in un['head_keys'].ravel()))}")
