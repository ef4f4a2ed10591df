"""The entry point for callers that cannot allocate (cqa_certified_decode_noalloc) against the
ordinary cqa_certified_decode, through the C ABI: two calls in a row, the second on a smaller
input, each compared with the existing entry point's output on the same cache and query.

Both run the same kernels on the same inputs; only the home of the split partials differs (a fixed
array inside the library's device image instead of the cache's workspace), so beyond the parity
bars (O 1e-3 relative, certificate terms 1e-4 relative, flags equal) the results are expected to
be bit-identical, which is checked too.
"""
import numpy as np
import pytest

import workloads
from helpers import GpuLayerCache, load_binding

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def both_calls(gc, q16, tol):
    """(O, cert, flags) of the existing entry point, then of the no-allocation one."""
    t = gc.torch
    qd = gc.to_dev(q16)
    gc.cqa.cqa_certified_decode(gc.h, 0, qd, tol, gc.O, gc.cert, gc.flags, None)
    ref = gc.results()
    # poison the outputs so that a call that wrote nothing cannot pass
    gc.O.fill_(float("nan"))
    gc.cert.zero_()
    gc.flags.fill_(-1)
    t.cuda.synchronize()
    gc.cqa.cqa_certified_decode_noalloc(gc.h, 0, qd, tol, gc.O, gc.cert, gc.flags)
    got = gc.results()
    return ref, got


def assert_same(ref, got, where):
    O0, c0, f0 = ref
    O1, c1, f1 = got
    assert np.isfinite(O1).all(), where
    for b in range(O0.shape[0]):
        for h in range(O0.shape[1]):
            n0 = np.linalg.norm(O0[b, h])
            assert np.linalg.norm(O1[b, h] - O0[b, h]) <= 1e-3 * n0 + 1e-6, (where, "O", b, h)
            assert np.abs(O1[b, h] - O0[b, h]).max() <= 1e-3 * np.abs(O0[b, h]).max() + 1e-6, (where, "O elem", b, h)
            for name in ("E_key", "E_val", "delta_h", "v_max", "alpha_tail_hat", "max_block_contrib", "lse"):
                x0, x1 = float(c0[b, h][name]), float(c1[b, h][name])
                assert abs(x1 - x0) <= 1e-4 * abs(x0) + 1e-9, (where, name, b, h, x0, x1)
            assert int(c1[b, h]["top_block"]) == int(c0[b, h]["top_block"]), (where, "top_block", b, h)
    assert (f0 == f1).all(), (where, "flags")
    # same kernels, same inputs, no atomics in the arithmetic: identical bits
    assert np.array_equal(O0, O1), (where, "O bits")
    assert c0.tobytes() == c1.tobytes(), (where, "cert bits")


def test_noalloc_entry_point_matches_the_existing_one_twice_in_a_row():
    cqa = load_binding()
    # first call: the 8K single-layer shape with a ragged tail (512 sealed blocks + 5 trailing tokens)
    sh = workloads.SHAPES["l8k"]
    n1 = sh.context + 5
    say(f"no-alloc call 1: {sh.n_q_heads} q / {sh.n_kv_heads} kv heads, {n1} tokens")
    k1, v1 = workloads.make_kv("l8k", seed=0, context=n1)
    q1 = workloads.make_q("l8k", step=3, seed=0)
    # second call: a smaller input (one KV head, 1000 tokens: 62 blocks + 8 trailing tokens)
    st = workloads.SHAPES["tiny"]
    n2 = 1000
    k2, v2 = workloads.make_kv("tiny", seed=1, context=n2)
    q2 = workloads.make_q("tiny", step=1, seed=1)
    tol = cqa.Tolerances(rank_depth=1, eps_total=1.0)   # some flags set, so the flag words are not all zero
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, n1 + 64) as g1, \
            GpuLayerCache(st.batch, st.n_q_heads, st.n_kv_heads, 2048) as g2:
        g1.append(k1, v1)
        g2.append(k2, v2)
        ref1, got1 = both_calls(g1, q1, tol)
        say(f"no-alloc call 2: {st.n_q_heads} q / {st.n_kv_heads} kv heads, {n2} tokens")
        ref2, got2 = both_calls(g2, q2, tol)
        assert_same(ref1, got1, "call 1 (8K)")
        assert_same(ref2, got2, "call 2 (1000 tokens)")
        # and the larger one once more after the smaller: the array keeps old contents, none is read
        ref3, got3 = both_calls(g1, q1, tol)
        assert_same(ref3, got3, "call 3 (8K again)")
        assert np.array_equal(ref1[0], ref3[0])


def test_noalloc_entry_point_rejects_what_does_not_fit_its_scratch():
    cqa = load_binding()
    bt, hq, hkv, n = 4, 32, 8, 32800     # 513 quads of blocks per head: room for 64 workgroups of 8 waves
    say(f"no-alloc limit: batch {bt}, {hq} q heads, 64 forced splits")
    rng = np.random.default_rng(5)
    k = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    v = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    q = rng.standard_normal((bt, hq, 128)).astype(np.float16)
    with GpuLayerCache(bt, hq, hkv, n + 64) as gc:
        gc.append(k, v)
        ref, got = both_calls(gc, q, cqa.Tolerances())
        assert_same(ref, got, "default splits")
        gc.cqa.cqa_set_splits(gc.h, 64)
        assert gc.cqa.cqa_decode_splits(gc.h, 0) == 64
        assert bt * hq * 64 * 576 > cqa.STATIC_SCRATCH_BYTES
        gc.O.fill_(7.0)
        gc.torch.cuda.synchronize()
        with pytest.raises(cqa.CqaError) as e:
            gc.cqa.cqa_certified_decode_noalloc(gc.h, 0, gc.to_dev(q), cqa.Tolerances(), gc.O, gc.cert, gc.flags)
        assert e.value.status == cqa.ERR_SCRATCH
        gc.torch.cuda.synchronize()
        assert (gc.O.cpu().numpy() == 7.0).all()      # nothing was launched
        gc.cqa.cqa_set_splits(gc.h, 0)
        ref, got = both_calls(gc, q, cqa.Tolerances())
        assert_same(ref, got, "after the refused call")
