"""GPU parity of the enqueue-only decode step: the fallback ladder resolved by a device kernel.

Same bars as the host-resolved step: heads that are not served are bit-identical to the certified
pass, served heads equal the dense FP16 result (1e-3 against the oracle, ~1e-6 against the
host-resolved ladder, whose dense pass splits the sequence differently), flags and rungs exact.
"""
import numpy as np
import pytest

import oracle
import workloads
from helpers import GpuLayerCache, assert_head_matches, load_binding, to_gpu_tol

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def compare_all(gc, ref, O, cert, flags, where):
    for i, r in enumerate(ref):
        b, h = divmod(i, gc.hq)
        assert_head_matches(r, O[b, h], cert[b, h], flags[b, h], (where, b, h))


def enqueue(gc, q, tol, k=None, v=None):
    qd = gc.to_dev(q)
    kd = None if k is None else gc.to_dev(k)
    vd = None if v is None else gc.to_dev(v)
    gc.cqa.cqa_decode_step_enqueue(gc.h, 0, kd, vd, qd, tol, gc.O, gc.cert, gc.flags)
    return gc.results()


def make(seed, bt, hkv, hq, n):
    rng = np.random.default_rng(seed)
    k = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    v = rng.standard_normal((bt, hkv, n, 128)).astype(np.float16)
    q = rng.standard_normal((bt, hq, 128)).astype(np.float16)
    return k, v, q


@pytest.mark.parametrize("group", [1, 2, 4])
def test_every_rung_against_oracle_and_host_ladder(group):
    say(f"device-resolved ladder, GQA group {group}: no flags, Rung 3 subset, Rung 4 by PRECOND and by group count")
    bt, hkv, n = 2, 2, 16 * 90 + 11
    hq = hkv * group
    k, v, q = make(8 + group, bt, hkv, hq, n)
    oc = oracle.OracleLayerCache(bt, hkv)
    oc.append(k, v)
    with GpuLayerCache(bt, hq, hkv, 2048) as gc:
        cqa = gc.cqa
        gc.append(k, v)
        assert cqa.cqa_ladder_counts(gc.h) == (0, 0)
        # nothing flagged: exactly the certified pass
        Oq, certq, flagsq = gc.certified_decode(q)
        O, cert, flags = enqueue(gc, q, cqa.Tolerances())
        assert (O == Oq).all() and cert.tobytes() == certq.tobytes() and (flags == flagsq).all()
        assert cqa.cqa_ladder_counts(gc.h) == (0, 0)
        # Rung 3 for the heads whose total bound exceeds eps_total (about a third of them)
        tot = np.sort((certq["E_key"].astype(np.float64) + certq["E_val"]).ravel())
        cut = len(tot) - max(1, len(tot) // 3)
        eps = 0.5 * (tot[cut] + tot[cut - 1])
        tol = oracle.Tolerances(eps_total=eps)
        ref = oc.decode_step(q, tol)
        n_served = sum(r["served_rung"] == 3 for r in ref)
        assert 0 < n_served < bt * hq
        O, cert, flags = enqueue(gc, q, to_gpu_tol(cqa, tol))
        compare_all(gc, ref, O, cert, flags, "rung 3")
        served = cert["served_rung"] == 3
        assert served.sum() == n_served
        assert (O[~served] == Oq[~served]).all()
        rung, Oh, certh, flagsh = gc.decode_step(q, to_gpu_tol(cqa, tol))
        assert rung == 3 and (flagsh == flags).all() and (certh["served_rung"] == cert["served_rung"]).all()
        assert np.abs(Oh - O).max() <= 2e-6 * np.abs(Oh).max()
        assert cqa.cqa_ladder_counts(gc.h) == (1, 0)
        # Rung 4: a PRECOND flag anywhere serves every head
        tol4 = oracle.Tolerances(force_flags=oracle.FLAG_PRECOND)
        O, cert, flags = enqueue(gc, q, to_gpu_tol(cqa, tol4))
        compare_all(gc, oc.decode_step(q, tol4), O, cert, flags, "rung 4 precond")
        assert (cert["served_rung"] == 4).all() and (cert["E_key"] == 0).all() and (cert["E_val"] == 0).all()
        assert (flags == (cqa.FLAG_PRECOND | (4 << cqa.RUNG_SHIFT))).all()
        # Rung 4 by the number of flagged KV groups
        groups_flagged = len({(i // hq, (i % hq) // group) for i, r in enumerate(ref) if r["served_rung"] == 3})
        tolg = oracle.Tolerances(eps_total=eps, rung4_min_groups=groups_flagged)
        O, cert, flags = enqueue(gc, q, to_gpu_tol(cqa, tolg))
        compare_all(gc, oc.decode_step(q, tolg), O, cert, flags, "rung 4 by groups")
        assert (cert["served_rung"] == 4).all()
        tolg = oracle.Tolerances(eps_total=eps, rung4_min_groups=groups_flagged + 1)
        O, cert, flags = enqueue(gc, q, to_gpu_tol(cqa, tolg))
        assert (cert["served_rung"] == np.where(served, 3, 0)).all()
        assert cqa.cqa_ladder_counts(gc.h) == (2, 2)
        # the arrival counters are back at zero: the same step again gives the same bits
        O2, cert2, flags2 = enqueue(gc, q, to_gpu_tol(cqa, tolg))
        assert (O2 == O).all() and cert2.tobytes() == cert.tobytes() and (flags2 == flags).all()


def test_steps_with_appends_match_the_two_calls():
    say("enqueue-only steps with a token appended each, across seals, one head falling back per step")
    cqa = load_binding()
    sh = workloads.SHAPES["l8k"]
    k, v = workloads.make_kv("l8k", seed=0, context=2048 + 5)
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, 2200) as a, \
            GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, 2200) as b:
        a.append(k, v)
        b.append(k, v)
        served_steps = 0
        for step in range(36):
            ks, vs = workloads.make_step_kv("l8k", step, seed=1)
            q = workloads.make_q("l8k", step, seed=1)
            kd, vd, qd = a.to_dev(ks), a.to_dev(vs), a.to_dev(q)
            # tolerance between the two largest totals of this step: exactly one head is flagged
            a.cqa.cqa_cache_append(a.h, 0, kd, vd, 1)
            _, certq, _ = a.certified_decode(q)
            tot = np.sort((certq["E_key"].astype(np.float64) + certq["E_val"]).ravel())
            flagged = step % 3 != 0 and (tot[-1] - tot[-2]) > 1e-3 * tot[-1]
            tol = cqa.Tolerances(eps_total=0.5 * (tot[-1] + tot[-2])) if flagged else cqa.Tolerances()
            rung = a.cqa.cqa_decode_step(a.h, 0, qd, tol, a.O, a.cert, a.flags, None)
            b.cqa.cqa_decode_step_enqueue(b.h, 0, kd, vd, qd, tol, b.O, b.cert, b.flags)
            Oa, ca, fa = a.results()
            Ob, cb, fb = b.results()
            assert a.length() == b.length() == 2048 + 5 + step + 1
            assert rung == (3 if flagged else 0)
            assert (fa == fb).all() and (ca["served_rung"] == cb["served_rung"]).all(), ("step", step)
            sv = ca["served_rung"] == 3
            assert sv.sum() == (1 if flagged else 0)
            served_steps += int(flagged)
            assert (Oa[~sv] == Ob[~sv]).all(), ("step", step)
            if flagged:
                assert np.abs(Oa[sv] - Ob[sv]).max() <= 2e-6 * np.abs(Oa[sv]).max(), ("step", step)
        assert b.cqa.cqa_ladder_counts(b.h) == (served_steps, 0)


def test_error_paths():
    say("enqueue-only step: error paths")
    cqa = load_binding()
    k, v, q = make(3, 1, 2, 8, 40)
    with GpuLayerCache(1, 8, 2, 41, tier2=False) as gc:
        gc.append(k, v)
        with pytest.raises(cqa.CqaError) as e:
            enqueue(gc, q, cqa.Tolerances())
        assert e.value.status == cqa.ERR_NO_TIER2
    with GpuLayerCache(1, 8, 2, 41) as gc:
        with pytest.raises(cqa.CqaError) as e:      # empty cache, nothing appended
            enqueue(gc, q, cqa.Tolerances())
        assert e.value.status == cqa.ERR_INVALID_ARG
        gc.append(k, v)
        with pytest.raises(cqa.CqaError) as e:      # only one of k, v
            gc.cqa.cqa_decode_step_enqueue(gc.h, 0, gc.to_dev(k[:, :, :1]), None, gc.to_dev(q),
                                           cqa.Tolerances(), gc.O, gc.cert, gc.flags)
        assert e.value.status == cqa.ERR_INVALID_ARG
        enqueue(gc, q, cqa.Tolerances(), k[:, :, :1], v[:, :, :1])
        assert gc.length() == 41
        with pytest.raises(cqa.CqaError) as e:      # full
            enqueue(gc, q, cqa.Tolerances(), k[:, :, :1], v[:, :, :1])
        assert e.value.status == cqa.ERR_CAPACITY
        assert gc.length() == 41


def test_serve64_batched_shape():
    say("serve64: batch 64 x 4096 tokens (one split per KV group), sampled sequences against the oracle, "
        "ladder over 2048 heads")
    cqa = load_binding()
    sh = workloads.SHAPES["serve64"]
    k, v = workloads.make_kv("serve64", seed=0)
    q = workloads.make_q("serve64", 0, seed=0)
    rows = [0, 17, 63]
    oc = oracle.OracleLayerCache(len(rows), sh.n_kv_heads)
    oc.append(k[rows], v[rows])
    ref = oc.certified_decode(q[rows], oracle.Tolerances())
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.context + 16) as gc:
        gc.append(k, v)
        assert cqa.cqa_decode_splits(gc.h, 0) == 1
        Oq, certq, flagsq = gc.certified_decode(q)
        for i, r in enumerate(ref):
            b, h = rows[i // sh.n_q_heads], i % sh.n_q_heads
            assert_head_matches(r, Oq[b, h], certq[b, h], flagsq[b, h], ("serve64", b, h))
        # a tolerance that flags the seven heads with the largest totals; the device-resolved ladder
        # serves exactly those, everything else stays bit-identical to the certified pass
        tot = (certq["E_key"].astype(np.float64) + certq["E_val"]).ravel()
        order = np.argsort(tot)
        assert tot[order[-7]] - tot[order[-8]] > 1e-4 * tot[order[-7]]
        eps = 0.5 * (tot[order[-7]] + tot[order[-8]])
        O, cert, flags = enqueue(gc, q, cqa.Tolerances(eps_total=float(eps)))
        sv = cert["served_rung"] == 3
        assert sorted(np.flatnonzero(sv.ravel())) == sorted(order[-7:])
        assert (O[~sv] == Oq[~sv]).all() and (flags[~sv] == flagsq[~sv]).all()
        assert (flags[sv] == (cqa.FLAG_TOTAL | (3 << cqa.RUNG_SHIFT))).all()
        g = sh.n_q_heads // sh.n_kv_heads
        for b, h in np.argwhere(sv):
            dense = oracle.softmax_attention(q[b, h], k[b, h // g], v[b, h // g])
            assert np.linalg.norm(O[b, h] - dense) <= 1e-3 * np.linalg.norm(dense) + 1e-6, (b, h)
            assert cert["E_key"][b, h] == 0 and cert["E_val"][b, h] == 0
        assert cqa.cqa_ladder_counts(gc.h) == (1, 0)


def test_caller_provided_tier2():
    say("originals in pinned host arrays the caller provides: filled in place, used by every fallback path")
    import torch
    cqa = load_binding()
    bt, hkv, hq, n, cap = 2, 2, 8, 16 * 40 + 7, 1024
    k, v, q = make(31, bt, hkv, hq, n)
    elems = bt * hkv * cap * 128
    t2k = torch.zeros(elems, dtype=torch.float16, pin_memory=True)
    t2v = torch.zeros(elems, dtype=torch.float16, pin_memory=True)
    with pytest.raises(cqa.CqaError) as e:          # too small
        cqa.cqa_cache_create_caller_tier2(1, bt, hq, hkv, cap, t2k, t2v, elems * 2 - 2)
    assert e.value.status == cqa.ERR_INVALID_ARG
    plain = np.zeros(elems, dtype=np.float16)       # ordinary pageable memory is refused
    with pytest.raises(cqa.CqaError) as e:
        cqa.cqa_cache_create_caller_tier2(1, bt, hq, hkv, cap, plain.ctypes.data, t2v, elems * 2)
    assert e.value.status == cqa.ERR_INVALID_ARG
    h = cqa.cqa_cache_create_caller_tier2(1, bt, hq, hkv, cap, t2k, t2v, elems * 2)
    dev = torch.device("cuda:0")
    try:
        O = torch.zeros((bt, hq, 128), dtype=torch.float32, device=dev)
        cert = torch.zeros((bt * hq, cqa.CERT_BYTES), dtype=torch.uint8, device=dev)
        flags = torch.zeros((bt * hq,), dtype=torch.int32, device=dev)
        kd, vd, qd = (torch.from_numpy(x).to(dev) for x in (k, v, q))
        cqa.cqa_cache_append(h, 0, kd[:, :, :600].contiguous(), vd[:, :, :600].contiguous(), 600)   # copy engines
        for t in range(600, n):                                                                  # kernel stores
            cqa.cqa_decode_step_enqueue(h, 0, kd[:, :, t:t + 1].contiguous(), vd[:, :, t:t + 1].contiguous(), qd,
                                        cqa.Tolerances(), O, cert, flags)
        torch.cuda.synchronize()
        got_k = t2k.numpy().reshape(bt, hkv, cap, 128)[:, :, :n]
        got_v = t2v.numpy().reshape(bt, hkv, cap, 128)[:, :, :n]
        assert (got_k.view(np.uint16) == k.view(np.uint16)).all()
        assert (got_v.view(np.uint16) == v.view(np.uint16)).all()
        assert not t2k.numpy().reshape(bt, hkv, cap, 128)[:, :, n:].any()
        forced = cqa.Tolerances(force_flags=cqa.FLAG_TOTAL)
        outs = []
        cqa.cqa_decode_step_enqueue(h, 0, None, None, qd, forced, O, cert, flags)      # ladder kernel
        torch.cuda.synchronize()
        outs.append(O.cpu().numpy().astype(np.float64))
        rung = cqa.cqa_decode_step(h, 0, qd, forced, O, cert, flags, None)             # host ladder, copy + kernel
        torch.cuda.synchronize()
        assert rung == 3
        outs.append(O.cpu().numpy().astype(np.float64))
        for o in outs:
            for b in range(bt):
                for hh in range(hq):
                    dense = oracle.softmax_attention(q[b, hh], k[b, hh // 4], v[b, hh // 4])
                    assert np.linalg.norm(o[b, hh] - dense) <= 1e-3 * np.linalg.norm(dense) + 1e-6
    finally:
        cqa.cqa_cache_destroy(h)
    # the arrays are the caller's: still there, still holding the originals
    assert (t2k.numpy().reshape(bt, hkv, cap, 128)[:, :, :n].view(np.uint16) == k.view(np.uint16)).all()


def test_random_small_shapes_against_oracle():
    say("40 seeded random small shapes (batch, GQA width, lengths incl. < 16, = 16 k, ragged), random tolerance: "
        "enqueue-only step with append against the oracle's append + decode_step")
    cqa = load_binding()
    rng = np.random.default_rng(2024)
    lengths = [1, 2, 15, 16, 17, 31, 32, 33, 47, 48, 64, 100, 255, 256, 257, 1000]
    for case in range(40):
        bt = int(rng.integers(1, 4))
        hkv = int(rng.integers(1, 4))
        group = int(rng.choice([1, 2, 4]))
        hq = hkv * group
        n = int(lengths[case % len(lengths)] if case < 2 * len(lengths) else rng.integers(1, 700))
        k = (rng.standard_normal((bt, hkv, n + 1, 128)) * rng.choice([0.5, 1.0, 3.0])).astype(np.float16)
        v = rng.standard_normal((bt, hkv, n + 1, 128)).astype(np.float16)
        q = rng.standard_normal((bt, hq, 128)).astype(np.float16)
        oc = oracle.OracleLayerCache(bt, hkv)
        oc.append(k[:, :, :n], v[:, :, :n])
        oc.append(k[:, :, n:], v[:, :, n:])
        ref0 = oc.certified_decode(q, oracle.Tolerances())
        tot = np.sort([r["E_key"] + r["E_val"] for r in ref0])
        # a tolerance in the widest gap between the heads' totals (none: everything passes)
        tol = oracle.Tolerances()
        if len(tot) > 1:
            gaps = np.diff(tot)
            j = int(np.argmax(gaps))
            if gaps[j] > 1e-3 * tot[j + 1]:
                tol = oracle.Tolerances(eps_total=float(0.5 * (tot[j] + tot[j + 1])),
                                        rung4_min_groups=int(rng.choice([0, 0, 2])))
        if case % 5 == 0:      # every head served, whatever its bound (also at lengths of a few tokens)
            tol = oracle.Tolerances(force_flags=oracle.FLAG_TOTAL if case % 10 else oracle.FLAG_PRECOND)
        ref = oc.decode_step(q, tol)
        with GpuLayerCache(bt, hq, hkv, n + 8) as gc:
            gc.append(k[:, :, :n], v[:, :, :n])
            O, cert, flags = enqueue(gc, q, to_gpu_tol(cqa, tol), k[:, :, n:], v[:, :, n:])
            assert gc.length() == n + 1
            compare_all(gc, ref, O, cert, flags, ("case", case, bt, hkv, group, n))
