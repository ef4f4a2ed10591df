"""GPU parity of the INT8 x INT8 scoring mode (cqa_tolerances.int8_query: the scaled query quantised
to 8 bits per block and scored on the INT8 matrix cores) against the oracle's, through the C ABI.

The integer decisions (the 8-bit codes of the scaled query) are taken in binary32 on both sides, so
block log-masses agree to 1e-4 as in the default mode -- one differing code would move a block's
scores by ~1e-2.  Delta_h carries the explicit third error term and is held to 1e-4 relative like
every certificate scalar.
"""
import numpy as np
import pytest

import oracle
import workloads
from oracle import adaptive as ad
from helpers import GpuLayerCache, assert_head_matches, to_gpu_tol
from test_gpu_adaptive import check_against_oracle, gpu_adaptive, make_case

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def compare(gc, oc, q, tol, where, heads=None, lm=None):
    gtol = to_gpu_tol(gc.cqa, tol)
    O, cert, flags, glm = gc.certified_decode(q, gtol, want_logmass=True)
    bt, hq, _ = q.shape
    heads = heads or [(b, h) for b in range(bt) for h in range(hq)]
    ref = oc.certified_decode(q, tol, heads=heads)
    for (b, h), r in zip(heads, ref):
        assert_head_matches(r, O[b, h], cert[b, h], flags[b, h], (where, b, h))
        assert np.abs(glm[b, h] - r["blk_logmass"]).max() <= 1e-4, (where, "block log-masses", b, h)
    return O, cert, flags, ref


def test_tiny_and_group_sizes():
    say("int8 query: tiny (GQA 4) and GQA 1 / 2, ragged tails")
    for hq, hkv, n, seed in ((4, 1, 1024 + 5, 0), (2, 2, 16 * 37 + 9, 1), (4, 2, 16 * 130 + 15, 2)):
        rng = np.random.default_rng(seed)
        k = (rng.standard_normal((2, hkv, n, 128)) * (1.0 + seed)).astype(np.float16)
        v = rng.standard_normal((2, hkv, n, 128)).astype(np.float16)
        q = (rng.standard_normal((2, hq, 128)) * (1.0 + 0.5 * seed)).astype(np.float16)
        oc = oracle.OracleLayerCache(2, hkv)
        oc.append(k, v)
        with GpuLayerCache(2, hq, hkv, n + 32) as gc:
            gc.append(k, v)
            O8, c8, _, ref8 = compare(gc, oc, q, oracle.Tolerances(int8_query=True, rank_depth=1), ("int8", hq, hkv))
            O0, c0, _, ref0 = compare(gc, oc, q, oracle.Tolerances(rank_depth=1), ("exact", hq, hkv))
            # the mode is really on: the certificate widens, the output moves (a little)
            assert (c8["delta_h"] > c0["delta_h"]).all()
            assert (O8 != O0).any()
            for mass_exp, mode in ((3, 1), (2, 2)):
                compare(gc, oc, q, oracle.Tolerances(int8_query=True, mass_exp=mass_exp, key_bound_mode=mode),
                        ("int8", hq, hkv, mass_exp, mode))


def test_l8k_outlier_channels_with_steps():
    say("int8 query: l8k (outlier channels x20), 20 steps across a seal")
    sh = workloads.SHAPES["l8k"]
    k, v = workloads.make_kv("l8k", seed=0, context=8192 - 6)
    oc = oracle.OracleLayerCache(sh.batch, sh.n_kv_heads)
    oc.append(k, v)
    tol = oracle.Tolerances(int8_query=True)
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, 8192 + 64) as gc:
        gc.append(k, v)
        for step in range(20):
            ks, vs = workloads.make_step_kv("l8k", step, seed=0)
            q = workloads.make_q("l8k", step, seed=0)
            oc.append(ks, vs)
            gc.append(ks, vs)
            if step in (0, 5, 6, 19):
                heads = [(0, h) for h in range(sh.n_q_heads)] if step == 6 else [(0, 0), (0, 13), (0, 31)]
                compare(gc, oc, q, tol, ("l8k", step), heads=heads)


def test_t128k_sampled_heads_and_error_paths():
    say("int8 query: t128k (Student-t keys), sampled heads; unsupported combinations")
    sh = workloads.SHAPES["t128k"]
    k, v = workloads.make_kv("t128k", seed=0)
    q = workloads.make_q("t128k", 2, seed=0)
    oc = oracle.OracleLayerCache(sh.batch, sh.n_kv_heads)
    oc.append(k, v)
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.context + 64) as gc:
        gc.append(k, v)
        O1, c1, f1, _ = compare(gc, oc, q, oracle.Tolerances(int8_query=True), "t128k", heads=[(0, 2), (0, 17), (0, 28)])
        cqa = gc.cqa
        qd = gc.to_dev(q)
        # the load hint (plain / non-temporal Tier-1 loads) does not change a bit in this mode either
        for hint in (2, 1):
            cqa.cqa_set_stream_hint(gc.h, hint)
            O2, c2, f2 = gc.certified_decode(q, to_gpu_tol(cqa, oracle.Tolerances(int8_query=True)))
            assert np.array_equal(O1, O2) and c1.tobytes() == c2.tobytes() and (f1 == f2).all(), ("hint", hint)
        cqa.cqa_set_stream_hint(gc.h, 0)
        # the vector-ALU cross-check kernel does not have the mode
        cqa.cqa_set_kernel_variant(gc.h, 1)
        with pytest.raises(cqa.CqaError) as e:
            cqa.cqa_certified_decode(gc.h, 0, qd, cqa.Tolerances(int8_query=True), gc.O, gc.cert, gc.flags, None)
        assert e.value.status == cqa.ERR_UNSUPPORTED
        with pytest.raises(cqa.CqaError) as e:
            cqa.cqa_adaptive_decode(gc.h, 0, qd, cqa.Tolerances(int8_query=True), cqa.Selector(), gc.O, gc.cert,
                                    gc.flags)
        assert e.value.status == cqa.ERR_UNSUPPORTED
        cqa.cqa_set_kernel_variant(gc.h, 0)
        # the enqueue-only step takes it (split pass + reduction + device-resolved ladder)
        cqa.cqa_decode_step_enqueue(gc.h, 0, None, None, qd, cqa.Tolerances(int8_query=True), gc.O, gc.cert, gc.flags)
        O, cert, flags = gc.results()
        ref = oc.certified_decode(q, oracle.Tolerances(int8_query=True), heads=[(0, 9)])[0]
        assert_head_matches(ref, O[0, 9], cert[0, 9], flags[0, 9], ("t128k enqueue", 9))


def test_more_sequences_than_compute_units():
    """With more (batch, kv-head) sequences than compute units the split pass runs in workgroups of
    four waves, two per compute unit: both scoring modes, GQA 2, one split and a forced three."""
    say("280 sequences (batch 70 x 4 kv heads, GQA 2): four-wave workgroups, default and int8 query, 1 and 3 splits")
    bt, hq, hkv, n = 70, 8, 4, 16 * 23 + 7
    rng = np.random.default_rng(5)
    k = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    v = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    q = (rng.standard_normal((bt, hq, 128)) * 1.5).astype(np.float16)
    rows = [0, 33, 69]
    oc = oracle.OracleLayerCache(len(rows), hkv)
    oc.append(k[rows], v[rows])
    with GpuLayerCache(bt, hq, hkv, n + 16) as gc:
        gc.append(k, v)
        for splits in (0, 3):
            gc.cqa.cqa_set_splits(gc.h, splits)
            for tol in (oracle.Tolerances(), oracle.Tolerances(int8_query=True)):
                O, cert, flags, glm = gc.certified_decode(q, to_gpu_tol(gc.cqa, tol), want_logmass=True)
                ref = oc.certified_decode(q[rows], tol)
                for (i, h), r in zip([(i, h) for i in range(len(rows)) for h in range(hq)], ref):
                    b = rows[i]
                    assert_head_matches(r, O[b, h], cert[b, h], flags[b, h], (splits, tol.int8_query, b, h))
                    assert np.abs(glm[b, h] - r["blk_logmass"]).max() <= 1e-4
        gc.cqa.cqa_set_splits(gc.h, 0)


def test_adaptive_precision_on_top_of_the_quantised_query():
    """The adaptive calls in this mode: the pass over all blocks scores with the 8-bit scaled query,
    the promoted-block pass reproduces those scores for what stays in INT8 (per-group and per-head
    promoted sets, value promotion, exploration and the score-consistency check on)."""
    say("int8 query + adaptive precision: small planted case (all heads), both promoted-set modes; t128k sampled heads")
    k, v, q = make_case(41, 2, 8, 2, 3000 + 5, peaked=[(0, 1, 333, 0.9), (0, 2, 1900, 1.1), (1, 4, 77, 0.8), (1, 6, 1500, 1.2)])
    oc = oracle.OracleLayerCache(2, 2)
    oc.append(k, v)
    with GpuLayerCache(2, 8, 2, 3100) as gc:
        gc.append(k, v)
        plain = gpu_adaptive(gc, q, oracle.Tolerances(rank_depth=2), ad.SelectorParams(0.9, 1, 8, 16))
        for per_head in (False, True):
            for tau, kmin, kmax, vlim in ((0.9, 1, 8, 0), (0.995, 2, 16, 8)):
                sel = ad.SelectorParams(tau, kmin, kmax, 2 * kmax, v_limit=vlim, canary=True, explore_frac=0.02,
                                        explore_seed=7, per_head=per_head)
                tol = oracle.Tolerances(int8_query=True, rank_depth=2, v_tol=0.01 if vlim else np.inf)
                out = gpu_adaptive(gc, q, tol, sel)
                check_against_oracle(oc, q, tol, sel, out)
                assert (out["cert"]["delta_h"] > plain["cert"]["delta_h"]).all()    # the third term is in
        # the enqueue-only step (nothing over a threshold and no ranking check: the ladder serves no head)
        sel = ad.SelectorParams(0.9, 1, 8, 16)
        tol = oracle.Tolerances(int8_query=True, rank_depth=0)
        enq = gpu_adaptive(gc, q, tol, sel, step="enqueue")
        check_against_oracle(oc, q, tol, sel, enq)
        assert (enq["cert"]["served_rung"] == 0).all()
    sh = workloads.SHAPES["t128k"]
    k, v = workloads.make_kv("t128k", seed=0)
    q = workloads.make_q("t128k", 4, seed=0)
    oc = oracle.OracleLayerCache(sh.batch, sh.n_kv_heads)
    oc.append(k, v)
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.context + 64) as gc:
        gc.append(k, v)
        sel = ad.SelectorParams(0.995, 2, 128, 128)
        tol = oracle.Tolerances(int8_query=True, rank_depth=1, rank_min_mass=0.25)
        out = gpu_adaptive(gc, q, tol, sel)
        check_against_oracle(oc, q, tol, sel, out, heads=[(0, 4), (0, 5), (0, 7)])
