"""GPU parity: the HIP path through the C ABI against the CPU oracle, same seeded inputs.

Bars: bit-exact codes, scales, offsets and (away from thresholds) flags;
||O_gpu - O_oracle|| <= 1e-3 ||O_oracle|| + 1e-6; certificate terms within 1e-4
relative; block log-masses within 1e-4 absolute; eta, nu within 1e-6 relative.
"""
import math

import numpy as np
import pytest

import oracle
import workloads
from oracle import quantizer as qz
from helpers import GpuLayerCache, assert_head_matches, load_binding, to_gpu_tol

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def check_blocks(gc, oc, blocks, heads=None, layer=0):
    """Exported Tier-1 blocks against the oracle's sealed blocks: exact codes and metadata."""
    heads = heads or [(b, h) for b in range(oc.bt) for h in range(oc.hkv)]
    for b, h in heads:
        for blk in blocks:
            kc, sg, z, vc, vs, vo, eta, nu = gc.export(b, h, blk, layer)
            w = (b, h, blk)
            assert (kc == oc.k_codes[b, h, blk]).all(), ("k codes", w)
            assert (sg.view(np.uint32) == oc.sigma[b, h, blk].view(np.uint32)).all(), ("sigma", w)
            assert (z.view(np.uint32) == oc.z[b, h, blk].view(np.uint32)).all(), ("z", w)
            assert (vc == oc.v_codes[b, h, blk]).all(), ("v codes", w)
            assert (vs.view(np.uint16) == oc.v_scale[b, h, blk].view(np.uint16)).all(), ("v scale", w)
            assert (vo.view(np.uint16) == oc.v_offset[b, h, blk].view(np.uint16)).all(), ("v offset", w)
            assert abs(float(eta) - float(oc.eta[b, h, blk])) <= 1e-6 * float(oc.eta[b, h, blk]) + 1e-12, ("eta", w)
            assert abs(float(nu) - float(oc.nu[b, h, blk])) <= 1e-6 * float(oc.nu[b, h, blk]), ("nu", w)


def compare_all(gc, ref, O, cert, flags, where, check_flags=True):
    hq = gc.hq
    for i, r in enumerate(ref):
        b, h = divmod(i, hq)
        assert_head_matches(r, O[b, h], cert[b, h], flags[b, h], (where, b, h), check_flags)


# ------------------------------------------------------------------ config 1: tiny

def test_tiny_quantize_and_decode():
    say("tiny: N=1024, GQA 4")
    sh = workloads.SHAPES["tiny"]
    k, v = workloads.make_kv("tiny", seed=0)
    q = workloads.make_q("tiny", seed=0)
    oc = oracle.OracleLayerCache(sh.batch, sh.n_kv_heads)
    oc.append(k, v)
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, 2048) as gc:
        gc.append(k, v)
        assert gc.length() == 1024
        check_blocks(gc, oc, range(64))
        O, cert, flags, lm = gc.certified_decode(q, want_logmass=True)
        ref = oc.certified_decode(q, oracle.Tolerances())
        compare_all(gc, ref, O, cert, flags, "tiny")
        for i, r in enumerate(ref):
            assert np.abs(lm[0, i] - r["blk_logmass"]).max() <= 1e-4, ("blk_logmass", i)
        # forced fallback goes through Tier-2 paging and returns the dense result
        rung, O2, cert2, flags2 = gc.decode_step(q, gc.cqa.Tolerances(force_flags=gc.cqa.FLAG_TOTAL))
        assert rung == 3
        ref2 = oc.decode_step(q, oracle.Tolerances(force_flags=oracle.FLAG_TOTAL))
        compare_all(gc, ref2, O2, cert2, flags2, "tiny forced")


@pytest.mark.parametrize("pieces", [[1] * 20, [15, 1, 1, 16, 17, 31, 32, 3], [16, 16], [5], [100, 7, 9]])
def test_ragged_appends_seal_the_same_blocks(pieces):
    say(f"ragged appends {pieces}")
    total = sum(pieces)
    rng = np.random.default_rng(total)
    bt, hkv, hq = 2, 2, 4
    k = rng.standard_normal((bt, hkv, total, 128)).astype(np.float16)
    v = rng.standard_normal((bt, hkv, total, 128)).astype(np.float16)
    q = rng.standard_normal((bt, hq, 128)).astype(np.float16)
    oc = oracle.OracleLayerCache(bt, hkv)
    with GpuLayerCache(bt, hq, hkv, 256) as gc:
        pos = 0
        for n in pieces:
            oc.append(k[:, :, pos:pos + n], v[:, :, pos:pos + n])
            gc.append(k[:, :, pos:pos + n], v[:, :, pos:pos + n])
            pos += n
            assert gc.length() == pos
            O, cert, flags = gc.certified_decode(q)
            ref = oc.certified_decode(q, oracle.Tolerances())
            compare_all(gc, ref, O, cert, flags, ("ragged", pos))
        check_blocks(gc, oc, range(total // 16))


@pytest.mark.parametrize("group", [1, 2, 4])
def test_gqa_group_sizes(group):
    say(f"GQA group {group}")
    rng = np.random.default_rng(group)
    bt, hkv, n = 1, 2, 16 * 37 + 9
    hq = hkv * group
    k = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    v = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    q = (rng.standard_normal((bt, hq, 128)) * 2).astype(np.float16)
    oc = oracle.OracleLayerCache(bt, hkv)
    oc.append(k, v)
    with GpuLayerCache(bt, hq, hkv, 1024) as gc:
        gc.append(k, v)
        O, cert, flags = gc.certified_decode(q)
        compare_all(gc, oc.certified_decode(q, oracle.Tolerances()), O, cert, flags, ("gqa", group))


def test_vector_alu_variant_and_standalone_reduction():
    say("vector-ALU split kernel + stand-alone reduction")
    rng = np.random.default_rng(17)
    bt, hkv, hq, n = 2, 2, 8, 16 * 150 + 7
    k = (rng.standard_normal((bt, hkv, n, 128)) * 1.5).astype(np.float16)
    v = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    q = rng.standard_normal((bt, hq, 128)).astype(np.float16)
    oc = oracle.OracleLayerCache(bt, hkv)
    oc.append(k, v)
    ref = oc.certified_decode(q, oracle.Tolerances(rank_depth=1))
    with GpuLayerCache(bt, hq, hkv, 4096) as gc:
        gc.append(k, v)
        for variant in (1, 0):
            gc.cqa.cqa_set_kernel_variant(gc.h, variant)
            O, cert, flags = gc.certified_decode(q, gc.cqa.Tolerances(rank_depth=1))
            compare_all(gc, ref, O, cert, flags, ("variant", variant))


def test_split_invariance():
    say("split invariance")
    rng = np.random.default_rng(3)
    bt, hkv, hq, n = 1, 2, 8, 16 * 200 + 3
    k = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    v = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    q = rng.standard_normal((bt, hq, 128)).astype(np.float16)
    with GpuLayerCache(bt, hq, hkv, 4096) as gc:
        gc.append(k, v)
        base = None
        for s in (1, 2, 7, 25, 64, 0):
            gc.cqa.cqa_set_splits(gc.h, s)
            O, cert, flags = gc.certified_decode(q)
            if base is None:
                base = (O.copy(), cert.copy())
                continue
            # value weights enter the matrix cores as two bf16 terms (16 significant bits), so O
            # moves by up to ~2^-16 relative when the split boundaries move; the certificate
            # scalars are accumulated in FP32 on the vector ALU
            assert np.abs(O - base[0]).max() <= 1e-4 * np.abs(base[0]).max()
            for name in ("E_key", "E_val", "delta_h", "v_max", "lse", "max_block_contrib"):
                assert np.allclose(cert[name], base[1][name], rtol=5e-6, atol=1e-9), (s, name)
            assert (cert["top_block"] == base[1]["top_block"]).all()


def test_exactly_representable_cache_has_zero_bounds():
    say("exactly representable cache")
    rng = np.random.default_rng(5)
    nb, d = 12, 128
    k = np.repeat(rng.standard_normal((1, 1, nb, 1, d)).astype(np.float16), 16, axis=3).reshape(1, 1, nb * 16, d)
    v = (rng.integers(0, 16, size=(1, 1, nb * 16, d)) * 0.25 - 2.0).astype(np.float16)
    v[..., 0::16] = -2.0
    v[..., 1::16] = 1.75
    q = rng.standard_normal((1, 4, d)).astype(np.float16)
    with GpuLayerCache(1, 4, 1, 256) as gc:
        gc.append(k, v)
        O, cert, flags = gc.certified_decode(q)
        assert (cert["E_key"] == 0).all() and (cert["E_val"] == 0).all() and (cert["delta_h"] == 0).all()
        for h in range(4):
            dense = oracle.softmax_attention(q[0, h], k[0, 0], v[0, 0])
            assert np.linalg.norm(O[0, h] - dense) <= 5e-5 * np.linalg.norm(dense) + 1e-7


# ------------------------------------------------------------------ errors and fallback

def test_error_paths():
    say("error paths")
    cqa = load_binding()
    import torch
    rng = np.random.default_rng(0)
    k = rng.standard_normal((1, 1, 40, 128)).astype(np.float16)
    v = rng.standard_normal((1, 1, 40, 128)).astype(np.float16)
    q = rng.standard_normal((1, 4, 128)).astype(np.float16)
    with GpuLayerCache(1, 4, 1, 48, tier2=False) as gc:
        with pytest.raises(cqa.CqaError) as e:            # empty cache
            gc.certified_decode(q)
        assert e.value.status == cqa.ERR_INVALID_ARG
        gc.append(k, v)
        with pytest.raises(cqa.CqaError) as e:            # capacity
            gc.append(k[:, :, :9], v[:, :, :9])
        assert e.value.status == cqa.ERR_CAPACITY
        assert gc.length() == 40
        O, cert, flags = gc.certified_decode(q)
        keep = O.copy()
        # Tier-2 absent: a required fallback is an error and O keeps the certified values
        with pytest.raises(cqa.CqaError) as e:
            gc.decode_step(q, cqa.Tolerances(force_flags=cqa.FLAG_RANK))
        assert e.value.status == cqa.ERR_NO_TIER2
        torch.cuda.synchronize()
        assert (gc.O.cpu().numpy() == keep.astype(np.float32)).all()
        with pytest.raises(cqa.CqaError) as e:
            cqa.cqa_certified_decode(gc.h, 3, gc.to_dev(q), cqa.Tolerances(), gc.O, gc.cert, gc.flags)
        assert e.value.status == cqa.ERR_INVALID_ARG
        # tolerance sets out of range; a ranking depth above 1 is refused, not served at depth 1
        for bad, status in ((cqa.Tolerances(mass_exp=-1), cqa.ERR_INVALID_ARG),
                            (cqa.Tolerances(key_bound_mode=3), cqa.ERR_INVALID_ARG),
                            (cqa.Tolerances(rank_depth=-1), cqa.ERR_INVALID_ARG),
                            (cqa.Tolerances(rank_depth=2), cqa.ERR_UNSUPPORTED)):
            with pytest.raises(cqa.CqaError) as e:
                cqa.cqa_certified_decode(gc.h, 0, gc.to_dev(q), bad, gc.O, gc.cert, gc.flags)
            assert e.value.status == status
    with pytest.raises(cqa.CqaError) as e:
        cqa.cqa_cache_create(1, 1, 24, 8, 1024)
    assert e.value.status == cqa.ERR_UNSUPPORTED


def test_fallback_equals_dense_kernel_bit_for_bit():
    say("fallback == dense kernel on resident copies")
    import torch
    rng = np.random.default_rng(8)
    bt, hkv, hq, n = 2, 2, 8, 16 * 90 + 11
    k = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    v = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    q = rng.standard_normal((bt, hq, 128)).astype(np.float16)
    oc = oracle.OracleLayerCache(bt, hkv)
    oc.append(k, v)
    with GpuLayerCache(bt, hq, hkv, 2048) as gc:
        cqa = gc.cqa
        gc.append(k, v)
        kd, vd, qd = gc.to_dev(k), gc.to_dev(v), gc.to_dev(q)
        ws = torch.zeros(cqa.cqa_dense_workspace_bytes(bt, hq, n), dtype=torch.uint8, device=gc.dev)
        Od = torch.zeros((bt, hq, 128), dtype=torch.float32, device=gc.dev)
        cqa.cqa_dense_attention(qd, kd, vd, bt, hq, hkv, n, Od, ws)
        torch.cuda.synchronize()
        dense = Od.cpu().numpy()
        for b in range(bt):
            for h in range(hq):
                ref = oracle.softmax_attention(q[b, h], k[b, h // 4], v[b, h // 4])
                assert np.linalg.norm(dense[b, h] - ref) <= 1e-3 * np.linalg.norm(ref) + 1e-6
        # Rung 4: every row equals the dense kernel's output exactly
        rung, O, cert, flags = gc.decode_step(q, cqa.Tolerances(force_flags=cqa.FLAG_PRECOND))
        assert rung == 4
        assert (O.astype(np.float32) == dense).all()
        assert (cert["served_rung"] == 4).all() and (cert["E_key"] == 0).all() and (cert["E_val"] == 0).all()
        assert (flags == (cqa.FLAG_PRECOND | (4 << cqa.RUNG_SHIFT))).all()
        # Rung 3 on a chosen subset: those rows are dense, the others keep the certified output
        Oq, certq, _ = gc.certified_decode(q)
        tot = np.sort((certq["E_key"].astype(np.float64) + certq["E_val"]).ravel())
        eps = 0.5 * (tot[-3] + tot[-4])
        tol = oracle.Tolerances(eps_total=eps)
        rung, O, cert, flags = gc.decode_step(q, to_gpu_tol(cqa, tol))
        assert rung == 3
        ref = oc.decode_step(q, tol)
        compare_all(gc, ref, O, cert, flags, "rung3 subset")
        served = cert["served_rung"] == 3
        assert served.sum() == 3
        assert (O.astype(np.float32)[served] == dense[served]).all()
        assert (O.astype(np.float32)[~served] == Oq.astype(np.float32)[~served]).all()
        # explicit head selection through cqa_dense_fallback
        sel = np.zeros((bt, hq), dtype=np.uint32)
        sel[1, 5] = 1
        gc.certified_decode(q)
        cqa.cqa_dense_fallback(gc.h, 0, qd, sel, 0, 3, gc.O, gc.cert, gc.flags)
        O, cert, flags = gc.results()
        assert (O.astype(np.float32)[1, 5] == dense[1, 5]).all()
        assert cert["served_rung"][1, 5] == 3 and cert["served_rung"].sum() == 3


# ------------------------------------------------------------------ config 2: 8K, 64 steps

def test_l8k_sixty_four_steps():
    say("l8k: N=8192 (+64 appended tokens), outlier key channels")
    sh = workloads.SHAPES["l8k"]
    k, v = workloads.make_kv("l8k", seed=0)
    oc = oracle.OracleLayerCache(sh.batch, sh.n_kv_heads)
    oc.append(k, v)
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, 8192 + 64) as gc:
        gc.append(k, v)
        check_blocks(gc, oc, list(range(0, 512, 23)) + [511])
        for step in range(sh.steps):
            ks, vs = workloads.make_step_kv("l8k", step, seed=0)
            q = workloads.make_q("l8k", step, seed=0)
            oc.append(ks, vs)
            gc.append(ks, vs)
            O, cert, flags = gc.certified_decode(q)
            if step % 8 in (0, 7) or step == sh.steps - 1:
                ref = oc.certified_decode(q, oracle.Tolerances())
                compare_all(gc, ref, O, cert, flags, ("l8k", step))
        assert gc.length() == 8192 + 64
        check_blocks(gc, oc, range(512, 516))


# ------------------------------------------------------------------ config 3: 32K, batch 4, mixed regimes

def test_mixed32k_five_percent_fallback():
    say("mixed32k: Bt=4, N=32768, peaked and diffuse heads, ~5% fallback")
    sh = workloads.SHAPES["mixed32k"]
    k, v = workloads.make_kv("mixed32k", seed=0)
    q, planted = workloads.make_peaked_q(k, sh.n_q_heads, gap=10.0, seed=0)
    oc = oracle.OracleLayerCache(sh.batch, sh.n_kv_heads)
    oc.append(k, v)
    ref0 = oc.certified_decode(q, oracle.Tolerances())
    tot = np.sort([r["E_key"] + r["E_val"] for r in ref0])[::-1]
    eps = 0.5 * (tot[5] + tot[6])          # exactly 6 of 128 heads (~5 %) exceed it
    assert (tot[5] - tot[6]) > 1e-3 * tot[5]
    tol = oracle.Tolerances(eps_total=eps)
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.context) as gc:
        gc.append(k, v)
        check_blocks(gc, oc, [0, 1, 1000, 2047], heads=[(0, 0), (3, 7)])
        O, cert, flags, lm = gc.certified_decode(q, want_logmass=True)
        compare_all(gc, ref0, O, cert, flags, "mixed32k certified")
        for i in (0, 1, 64, 127):
            assert np.abs(lm.reshape(-1, lm.shape[-1])[i] - ref0[i]["blk_logmass"]).max() <= 1e-4
        # peaked heads put (almost) all their mass on the planted block
        for b in range(sh.batch):
            for h in range(0, sh.n_q_heads, 2):
                assert cert["top_block"][b, h] == planted[b, h] // 16
        rung, O, cert, flags = gc.decode_step(q, to_gpu_tol(gc.cqa, tol))
        assert rung == 3
        ref = oc.decode_step(q, tol)
        assert sum(r["served_rung"] == 3 for r in ref) == 6
        compare_all(gc, ref, O, cert, flags, "mixed32k ladder")


# ------------------------------------------------------------------ config 4: 128K, heavy-tailed keys

def test_t128k_steps():
    say("t128k: N=131072, Student-t(3) keys, appended steps")
    sh = workloads.SHAPES["t128k"]
    k, v = workloads.make_kv("t128k", seed=0)
    oc = oracle.OracleLayerCache(sh.batch, sh.n_kv_heads)
    oc.append(k, v)
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.context + 64) as gc:
        gc.append(k, v)
        check_blocks(gc, oc, [0, 4095, 8191])
        check_blocks(gc, oc, range(100, 8192, 997), heads=[(0, 3)])
        for step in range(sh.steps):
            ks, vs = workloads.make_step_kv("t128k", step, seed=0)
            q = workloads.make_q("t128k", step, seed=0)
            oc.append(ks, vs)
            gc.append(ks, vs)
            O, cert, flags = gc.certified_decode(q)
            if step == 0:
                heads = [(0, h) for h in range(sh.n_q_heads)]      # every head once
            elif step in (7, 15):
                heads = [(0, h) for h in (1, 14, 31)]              # sampled heads later
            else:
                continue
            say(f"  step {step}: oracle on {len(heads)} heads")
            ref = oc.certified_decode(q, oracle.Tolerances(), heads=heads)
            for (b, h), r in zip(heads, ref):
                assert_head_matches(r, O[b, h], cert[b, h], flags[b, h], ("t128k", step, h))
        # Rung 3 at full size: eps_total is placed in the widest gap among the eight largest
        # totals, at least 2e-4 relative away from both neighbours, so the heads above it (one
        # to seven of them) fall back and no head sits near the threshold
        tot = (cert["E_key"].astype(np.float64) + cert["E_val"]).ravel()
        srt = np.sort(tot)[::-1]
        gaps = (srt[:7] - srt[1:8]) / srt[:7]
        j = int(np.argmax(gaps))
        assert gaps[j] > 4e-4, ("no usable gap among the largest totals", srt[:8])
        eps = 0.5 * (srt[j] + srt[j + 1])
        n_over = j + 1
        rung, O2, cert2, flags2 = gc.decode_step(q, gc.cqa.Tolerances(eps_total=eps))
        assert rung == 3 and (cert2["served_rung"] == 3).sum() == n_over
        assert ((cert2["served_rung"] == 3).ravel() == (tot > eps)).all()
        served = [tuple(x) for x in np.argwhere(cert2["served_rung"] == 3)]
        dense = {}
        for b, h in served:
            dense[(b, h)] = oracle.softmax_attention(q[b, h], oc.k16[b, h // 4], oc.v16[b, h // 4])
            assert np.linalg.norm(O2[b, h] - dense[(b, h)]) <= 1e-3 * np.linalg.norm(dense[(b, h)]) + 1e-6
            assert np.abs(O2[b, h] - dense[(b, h)]).max() <= 1e-3 * np.abs(dense[(b, h)]).max() + 1e-6
        # the same step enqueue-only (the launch configuration bench.py times): the ladder
        # kernel serves the heads from the pinned originals, everything else is untouched
        gc.cqa.cqa_decode_step_enqueue(gc.h, 0, None, None, gc.to_dev(q), gc.cqa.Tolerances(eps_total=eps),
                                       gc.O, gc.cert, gc.flags)
        O3, cert3, flags3 = gc.results()
        assert (flags3 == flags2).all() and (cert3["served_rung"] == cert2["served_rung"]).all()
        sv = cert3["served_rung"] == 3
        assert (O3[~sv] == O2[~sv]).all() and (O3[~sv] == O[~sv]).all()
        for b, h in served:
            assert np.linalg.norm(O3[b, h] - dense[(b, h)]) <= 1e-3 * np.linalg.norm(dense[(b, h)]) + 1e-6
            # the two dense paths split the 131K tokens differently (64 against 1024 partial sums
            # in FP32), so they agree to accumulation rounding, not bit for bit
            assert np.abs(O3[b, h] - O2[b, h]).max() <= 3e-5 * np.abs(O2[b, h]).max()
        # and with nothing flagged it is the certified pass, bit for bit
        gc.cqa.cqa_decode_step_enqueue(gc.h, 0, None, None, gc.to_dev(q), gc.cqa.Tolerances(), gc.O, gc.cert,
                                       gc.flags)
        O4, cert4, flags4 = gc.results()
        assert (O4 == O).all() and cert4.tobytes() == cert.tobytes() and (flags4 == flags).all()


def test_append_decode_step_equals_the_two_calls():
    say("one-call append + decode step against append followed by decode step, 40 steps across seals")
    cqa = load_binding()
    sh = workloads.SHAPES["l8k"]
    k, v = workloads.make_kv("l8k", seed=0, context=2048 + 5)
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, 2200) as a, \
            GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, 2200) as b:
        a.append(k, v)
        b.append(k, v)
        tol = cqa.Tolerances()
        for step in range(40):
            ks, vs = workloads.make_step_kv("l8k", step, seed=1)
            q = workloads.make_q("l8k", step, seed=1)
            kd, vd, qd = a.to_dev(ks), a.to_dev(vs), a.to_dev(q)
            a.cqa.cqa_cache_append(a.h, 0, kd, vd, 1)
            a.cqa.cqa_decode_step(a.h, 0, qd, tol, a.O, a.cert, a.flags, None)
            b.cqa.cqa_append_decode_step(b.h, 0, kd, vd, qd, tol, b.O, b.cert, b.flags)
            Oa, ca, fa = a.results()
            Ob, cb, fb = b.results()
            assert a.length() == b.length() == 2048 + 5 + step + 1
            assert (Oa == Ob).all() and (fa == fb).all(), ("step", step)
            assert ca.tobytes() == cb.tobytes(), ("certificate", step)
        # the caches hold the same blocks and the same originals: every block sealed on the way,
        # and a forced fallback (which reads the pinned originals incl. the tokens that rode along)
        for blk in (126, 127, 128, 129):
            xa, xb = a.export(0, 3, blk), b.export(0, 3, blk)
            for u, w in zip(xa, xb):
                assert np.array_equal(np.asarray(u), np.asarray(w)), ("block", blk)
        forced = cqa.Tolerances(force_flags=cqa.FLAG_TOTAL)
        qd = a.to_dev(workloads.make_q("l8k", 99, seed=1))
        a.cqa.cqa_decode_step(a.h, 0, qd, forced, a.O, a.cert, a.flags, None)
        b.cqa.cqa_decode_step(b.h, 0, qd, forced, b.O, b.cert, b.flags, None)
        assert (a.results()[0] == b.results()[0]).all()


def test_stream_hint_does_not_change_results():
    say("plain and non-temporal Tier-1 loads give the same bits")
    rng = np.random.default_rng(23)
    bt, hkv, hq, n = 2, 2, 8, 16 * 301 + 5
    k = (rng.standard_normal((bt, hkv, n, 128)) * 1.5).astype(np.float16)
    v = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    q = rng.standard_normal((bt, hq, 128)).astype(np.float16)
    with GpuLayerCache(bt, hq, hkv, 8192) as gc:
        gc.append(k, v)
        out = []
        for mode in (1, 2, 0):
            gc.cqa.cqa_set_stream_hint(gc.h, mode)
            O, cert, flags, lm = gc.certified_decode(q, want_logmass=True)
            out.append((O.copy(), cert.tobytes(), flags.copy(), lm.copy()))
        for o in out[1:]:
            assert (o[0] == out[0][0]).all() and o[1] == out[0][1]
            assert (o[2] == out[0][2]).all() and (o[3] == out[0][3]).all()
        with pytest.raises(gc.cqa.CqaError):
            gc.cqa.cqa_set_stream_hint(gc.h, 3)


@pytest.mark.parametrize("k_scale", [600.0, 650.0])
def test_large_delta_tail_form_matches_up_to_the_binary32_range(k_scale):
    """Keys so coarse that Delta_h is 35 .. 49: the tail form of the key term (key_bound_mode 1) is
    2 V_max (e^{2 Delta_h} - 1) ~ 1e30 .. 1e38 where it fits binary32 and +inf (with PRECOND) where
    it does not; the default mode takes the tanh form and stays finite."""
    say(f"large Delta, keys x{k_scale}")
    rng = np.random.default_rng(41)
    bt, hkv, hq, n = 1, 2, 8, 16 * 40 + 3
    k = (rng.standard_normal((bt, hkv, n, 128)) * k_scale).astype(np.float16)
    v = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    q = rng.standard_normal((bt, hq, 128)).astype(np.float16)
    oc = oracle.OracleLayerCache(bt, hkv)
    oc.append(k, v)
    with GpuLayerCache(bt, hq, hkv, 2048) as gc:
        gc.append(k, v)
        for mode in (1, 0):
            ref = oc.certified_decode(q, oracle.Tolerances(key_bound_mode=mode))
            O, cert, flags = gc.certified_decode(q, gc.cqa.Tolerances(key_bound_mode=mode))
            compare_all(gc, ref, O, cert, flags, ("large delta", k_scale, mode))
            if mode == 1:
                assert max(r["delta_h"] for r in ref) > 44.4 and min(r["delta_h"] for r in ref) < 44.0
                assert any(math.isinf(r["E_key"]) for r in ref) and any(math.isfinite(r["E_key"]) for r in ref)
                assert all(bool(r["flags"] & oracle.FLAG_PRECOND) == math.isinf(r["E_key"]) for r in ref)
            else:
                assert all(r["flags"] == 0 for r in ref)
