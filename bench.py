#!/usr/bin/env python3
"""Benchmark of the certified-decode hot path on one MI355X.

A step = one pass of the whole hot path over the 128K single-layer workload:
append one (k, v) token per KV head (trailing FP16 block, Tier-2 copy, block seal
when 16 tokens have arrived), the split-K certified decode over the packed
cache, the cross-split reduction with the certificate, and the fallback ladder resolved
by a device kernel (tolerances +inf in the headline run, so no head falls back).

Prints ONE JSON line.  `value` is whole-step throughput (steps/s for the one
layer) with all inputs resident in HBM; `roofline` prices the dominant kernel
(the split-K decode pass) against HBM bandwidth using its algorithmic bytes and
the MEDIAN of its duration over a fixed 210 dispatches of the same step loop (the
first 10 dropped), each carrying a HIP event pair on its launch stream; that pass
runs after the pass that yields `value` (event-carrying dispatches slow the
step).  `roofline.no_reuse` is the same kernel alternating over four resident
copies of the layer (1.2 GB between two visits of a record), so that nothing it
reads can still sit in the 256 MB memory-side cache.  `cpu_baseline` is the CPU
oracle timed on the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

import workloads

PEAK_HBM_GBS = 8000.0
# the arithmetic the path computes in: scores and weighted values are matrix-core contractions whose
# FP32 operands are split into two FP16 (scores) / two BF16 (values) terms, accumulated in FP32;
# softmax state and the certificate are FP32
DTYPE = "f16x2/bf16x2 mfma operands, f32 accumulate"
ROOF_DISPATCHES = 210          # event-carrying dispatches of the roofline leg ...
ROOF_DROP = 10                 # ... of which the first ones are dropped
NO_REUSE_LAYERS = 4            # resident copies of the layer the no-reuse leg alternates over
BYTES_PER_TOKEN = 288.5        # Tier-1 bytes per token per KV head (codes + metadata + eta, nu)
WORKLOAD = "t128k"


def read_traffic_note():
    """HBM bytes per launch of the split kernel from the committed rocprofv3 counter summary."""
    path = os.path.join(ROOT, "profiles", "certified_split_t128k_pmc.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1].strip())
    except OSError:
        pass
    return None


def cpu_baseline(k, v, steps_budget_s=12.0):
    """Times the oracle (as it stands) on full steps of the same workload, before the GPU is touched."""
    import oracle

    sh = workloads.SHAPES[WORKLOAD]
    oc = oracle.OracleLayerCache(sh.batch, sh.n_kv_heads)
    oc.append(k, v)                                   # prefix build: set-up, not timed
    tol = oracle.Tolerances()
    n = 0
    t0 = time.perf_counter()
    c0 = os.times()
    while True:
        ks, vs = workloads.make_step_kv(WORKLOAD, 1000 + n, seed=0)
        q = workloads.make_q(WORKLOAD, 1000 + n, seed=0)
        oc.append(ks, vs)
        oc.decode_step(q, tol)
        n += 1
        if time.perf_counter() - t0 > steps_budget_s or n >= 8:
            break
    wall = time.perf_counter() - t0
    c1 = os.times()
    cpu = (c1.user + c1.system) - (c0.user + c0.system)
    return {"value": n / wall, "unit": "steps/s", "cores": max(1, int(round(cpu / wall))),
            "kind": "oracle",
            "sample": f"{n} full steps (append 1 token + certified decode of all 32 heads, 128K context) "
                      f"of the same workload; numpy float64, host has {len(os.sched_getaffinity(0))} cores"}


def bench_small(args, name) -> int:
    """tiny / l8k / mixed32k: kernel-only and end-to-end step rates plus the oracle's rate, one JSON line.
    mixed32k also times the step with its calibrated tolerance (6 of 128 heads served by Rung 3)."""
    import oracle

    sh = workloads.SHAPES[name]
    k, v = workloads.make_kv(name, seed=0)
    if name == "mixed32k":
        q_fixed, _ = workloads.make_peaked_q(k, sh.n_q_heads)
    else:
        q_fixed = None
    # oracle first (before the GPU is touched): prefix build untimed, then whole steps
    oc = oracle.OracleLayerCache(sh.batch, sh.n_kv_heads)
    oc.append(k, v)
    n_or = 0
    t0 = time.perf_counter()
    c0 = os.times()
    while n_or < 8 and time.perf_counter() - t0 < 10.0:
        ks1, vs1 = workloads.make_step_kv(name, 1000 + n_or)
        qo = q_fixed if q_fixed is not None else workloads.make_q(name, 1000 + n_or)
        oc.append(ks1, vs1)
        oc.decode_step(qo, oracle.Tolerances())
        n_or += 1
    wall = time.perf_counter() - t0
    c1 = os.times()
    cores = max(1, int(round(((c1.user + c1.system) - (c0.user + c0.system)) / wall)))
    del oc

    import torch
    from paper_2605_20868_amd import binding as cqa

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, W = args.steps, args.warmup
    h = cqa.cqa_cache_create(1, sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.context + K + W + 64)
    try:
        cqa.cqa_cache_append(h, 0, torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev), sh.context)
        torch.cuda.synchronize()
        rng = np.random.Generator(np.random.Philox(7))
        n_in = K + W
        ks = torch.from_numpy(workloads.normal_f16(rng, (n_in, sh.batch, sh.n_kv_heads, 1, 128))).to(dev)
        vs = torch.from_numpy(workloads.normal_f16(rng, (n_in, sh.batch, sh.n_kv_heads, 1, 128))).to(dev)
        if q_fixed is not None:
            qs = torch.from_numpy(np.broadcast_to(q_fixed, (n_in,) + q_fixed.shape).copy()).to(dev)
        else:
            qs = torch.from_numpy(workloads.normal_f16(rng, (n_in, sh.batch, sh.n_q_heads, 128))).to(dev)
        O = torch.empty((sh.batch, sh.n_q_heads, 128), dtype=torch.float32, device=dev)
        cert = torch.zeros((sh.batch * sh.n_q_heads, cqa.CERT_BYTES), dtype=torch.uint8, device=dev)
        flags = torch.zeros((sh.batch * sh.n_q_heads,), dtype=torch.int32, device=dev)
        tol = cqa.Tolerances()
        stream = torch.cuda.current_stream().cuda_stream
        kp, vp, qp = ks.data_ptr(), vs.data_ptr(), qs.data_ptr()
        kv_stride, q_stride = ks[0].numel() * 2, qs[0].numel() * 2
        Op, certp, flagsp = O.data_ptr(), cert.data_ptr(), flags.data_ptr()

        def step(i, t):
            cqa.cqa_decode_step_enqueue(h, 0, kp + i * kv_stride, vp + i * kv_stride,
                                        qp + i * q_stride, t, Op, certp, flagsp, stream)

        for i in range(W):
            step(i, tol)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(W, W + K):
            step(i, tol)
        torch.cuda.synchronize()
        e2e_ms = (time.perf_counter() - t0) * 1e3 / K
        cqa.cqa_profile_begin(h, 50)
        ko_ms = cqa.cqa_time_certified_decode(h, 0, qp, tol, Op, certp, flagsp, None, 50, stream)
        mean_ms, min_ms, _ = cqa.cqa_profile_end(h)
        fb = None
        if name == "mixed32k":
            cqa.cqa_certified_decode(h, 0, qp, tol, Op, certp, flagsp, None, stream)
            torch.cuda.synchronize()
            ct = cert.cpu().numpy().view(np.dtype(cqa.CERT_FIELDS)).ravel()
            tot = np.sort(ct["E_key"].astype(np.float64) + ct["E_val"])[::-1]
            tight = cqa.Tolerances(eps_total=float(0.5 * (tot[5] + tot[6])))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(5):
                rung = cqa.cqa_decode_step(h, 0, qp, tight, Op, certp, flagsp, None, stream)
            torch.cuda.synchronize()
            served = int((cert.cpu().numpy().view(np.dtype(cqa.CERT_FIELDS)).ravel()["served_rung"] == 3).sum())
            fb = {"ms_per_step": (time.perf_counter() - t0) * 1e3 / 5, "heads_served_by_rung3": served,
                  "rung": rung}
        n_tokens = cqa.cqa_cache_length(h, 0)
        splits = cqa.cqa_decode_splits(h, 0)
    finally:
        cqa.cqa_cache_destroy(h)
    alg_bytes = sh.batch * sh.n_kv_heads * (n_tokens // 16) * 16 * BYTES_PER_TOKEN
    achieved = alg_bytes / (mean_ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": f"certified decode attention steps/s per layer, workload {name}",
        "value": 1e3 / e2e_ms, "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": e2e_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": f"{name}: 1 layer, batch {sh.batch}, {sh.n_q_heads} q / {sh.n_kv_heads} kv heads, "
                               f"context {sh.context}+steps, tolerances +inf", "splits": splits},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBS, "traffic": None,
                     "kernel": "certified_split_mfma_kernel", "kernel_mean_ms": mean_ms, "kernel_min_ms": min_ms,
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "note": "effective rate; workloads that fit the caches are not an HBM-roofline claim"},
        "kernel_only": {"ms_per_step": ko_ms, "steps_per_s": 1e3 / ko_ms},
        "fallback_step": fb,
        "cpu_baseline": {"value": n_or / wall, "unit": "steps/s", "cores": cores, "kind": "oracle",
                         "sample": f"{n_or} full steps of the same workload"},
    }))
    return 0


def bench_stack(args) -> int:
    """The 32-layer stack (batch 2, 128K per sequence): all layers resident, one pass = every layer's
    append + decode step.  Not the headline line; prints its own JSON line."""
    import torch
    from paper_2605_20868_amd import binding as cqa

    sh = workloads.SHAPES["stack"]
    ctx = args.context or sh.context
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, W = min(args.steps, 20), min(args.warmup, 3)
    L = sh.n_layers
    h = cqa.cqa_cache_create(L, sh.batch, sh.n_q_heads, sh.n_kv_heads, ctx + K + W + 16)
    try:
        for layer in range(L):
            kd, vd = workloads.torch_device_kv("stack", layer, dev, context=ctx)
            cqa.cqa_cache_append(h, layer, kd, vd, ctx)
            torch.cuda.synchronize()
            del kd, vd
        rng = np.random.Generator(np.random.Philox(11))
        n_in = K + W
        ks = torch.from_numpy(workloads.student_t3_f16(rng, (n_in, L, sh.batch, sh.n_kv_heads, 1, 128))).to(dev)
        vs = torch.from_numpy(workloads.normal_f16(rng, (n_in, L, sh.batch, sh.n_kv_heads, 1, 128))).to(dev)
        qs = torch.from_numpy(workloads.normal_f16(rng, (n_in, L, sh.batch, sh.n_q_heads, 128))).to(dev)
        O = torch.empty((sh.batch, sh.n_q_heads, 128), dtype=torch.float32, device=dev)
        cert = torch.zeros((sh.batch * sh.n_q_heads, cqa.CERT_BYTES), dtype=torch.uint8, device=dev)
        flags = torch.zeros((sh.batch * sh.n_q_heads,), dtype=torch.int32, device=dev)
        tol = cqa.Tolerances()
        stream = torch.cuda.current_stream().cuda_stream
        kp, vp, qp = ks.data_ptr(), vs.data_ptr(), qs.data_ptr()
        kv_stride, q_stride = ks[0, 0].numel() * 2, qs[0, 0].numel() * 2
        Op, certp, flagsp = O.data_ptr(), cert.data_ptr(), flags.data_ptr()

        def step(i):
            for layer in range(L):
                j = i * L + layer
                cqa.cqa_decode_step_enqueue(h, layer, kp + j * kv_stride, vp + j * kv_stride,
                                            qp + j * q_stride, tol, Op, certp, flagsp, stream)

        for i in range(W):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(W, W + K):
            step(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        cqa.cqa_profile_begin(h, K * L)
        for i in range(W, W + K):
            for layer in range(L):
                cqa.cqa_decode_step_enqueue(h, layer, None, None, qp + (i * L + layer) * q_stride, tol, Op,
                                            certp, flagsp, stream)
        torch.cuda.synchronize()
        mean_ms, min_ms, n_timed = cqa.cqa_profile_end(h)
        splits = cqa.cqa_decode_splits(h, 0)
        # streaming-read ceiling: the load-only kernel, one launch per layer in turn (fresh memory
        # every launch, as in the step loop)
        torch.cuda.synchronize()
        ts0 = time.perf_counter()
        sr_total, sr_bytes = 0.0, 0
        for rep in range(2):
            for layer in range(L):
                ms1, sr_bytes = cqa.cqa_time_stream_read(h, layer, 1, stream)
                sr_total += ms1
        sr_ms = sr_total / (2 * L)
    finally:
        cqa.cqa_cache_destroy(h)
    nb_mid = (ctx + W + K // 2) // 16
    alg_bytes = sh.batch * sh.n_kv_heads * nb_mid * 16 * BYTES_PER_TOKEN
    achieved = alg_bytes / (mean_ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "certified decode attention layer-steps/s, 32-layer stack at 128K ctx, batch 2",
        "value": K * L / (t1 - t0), "unit": "layer-steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": (t1 - t0) * 1e3 / K, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": f"stack: {L} layers, batch {sh.batch}, {sh.n_q_heads} q / {sh.n_kv_heads} kv heads, "
                               f"context {ctx}+steps, K ~ Student-t(3), V ~ N(0,1), tolerances +inf",
                   "step": "for each of the 32 layers: append 1 token + decode step with the ladder resolved on the device (cqa_decode_step_enqueue)", "splits": splits},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBS, "traffic": None,
                     "kernel": "certified_split_mfma_kernel<4>", "kernel_mean_ms": mean_ms,
                     "kernel_min_ms": min_ms, "algorithmic_bytes_per_launch": alg_bytes,
                     "stream_ceiling": {"GBps": sr_bytes / (sr_ms * 1e-3) / 1e9, "ms": sr_ms,
                                        "frac_of_ceiling": (alg_bytes / (mean_ms * 1e-3)) / (sr_bytes / (sr_ms * 1e-3)),
                                        "what": "load-only kernel with the split kernel's launch shape and load "
                                                "instructions, one launch per layer in turn"}},
        "cpu_baseline": None,
    }))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--context", type=int, default=None, help="override the context length (debug)")
    ap.add_argument("--workload", default=WORKLOAD, choices=[WORKLOAD, "stack", "tiny", "l8k", "mixed32k", "serve64"],
                    help="t128k (default, the headline line); stack: 32 layers x batch 2 x 128K, a step = append + "
                         "decode step on every layer (layer-steps/s); tiny / l8k / mixed32k: the small parity "
                         "workloads, reported for the results table only")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives or sharding are part of it); "
              "run with --gpus 1", file=sys.stderr)
        return 2
    if int(os.environ.get("RANK", "0")) != 0:
        return 0

    if args.workload == "stack":
        return bench_stack(args)
    if args.workload != WORKLOAD:
        return bench_small(args, args.workload)
    sh = workloads.SHAPES[WORKLOAD]
    ctx = args.context or sh.context
    k, v = workloads.make_kv(WORKLOAD, seed=0, context=ctx)

    base = None
    if not args.no_cpu_baseline:
        base = cpu_baseline(k, v)

    import torch
    from paper_2605_20868_amd import binding as cqa     # raises if libcqa.so is missing

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, W = args.steps, args.warmup
    cap = ctx + K + W + 64
    h = cqa.cqa_cache_create(1, sh.batch, sh.n_q_heads, sh.n_kv_heads, cap)
    try:
        kd = torch.from_numpy(k).to(dev)
        vd = torch.from_numpy(v).to(dev)
        # bulk append (prefill-sized): quantize + pack + annotate all blocks, Tier-2 copy to pinned RAM
        torch.cuda.synchronize()
        tb0 = time.perf_counter()
        cqa.cqa_cache_append(h, 0, kd, vd, ctx)
        torch.cuda.synchronize()
        bulk_s = time.perf_counter() - tb0
        del kd, vd
        rng = np.random.Generator(np.random.Philox(7))
        n_in = K + W
        ks = torch.from_numpy(workloads.student_t3_f16(rng, (n_in, sh.batch, sh.n_kv_heads, 1, 128))).to(dev)
        vs = torch.from_numpy(workloads.normal_f16(rng, (n_in, sh.batch, sh.n_kv_heads, 1, 128))).to(dev)
        qs = torch.from_numpy(workloads.normal_f16(rng, (n_in, sh.batch, sh.n_q_heads, 128))).to(dev)
        O = torch.empty((sh.batch, sh.n_q_heads, 128), dtype=torch.float32, device=dev)
        cert = torch.zeros((sh.batch * sh.n_q_heads, cqa.CERT_BYTES), dtype=torch.uint8, device=dev)
        flags = torch.zeros((sh.batch * sh.n_q_heads,), dtype=torch.int32, device=dev)
        tol = cqa.Tolerances()                          # headline: every threshold at +inf
        stream = torch.cuda.current_stream().cuda_stream

        # the binding takes raw device addresses: per-step slices are computed as integers here
        kp, vp, qp = ks.data_ptr(), vs.data_ptr(), qs.data_ptr()
        kv_stride, q_stride = ks[0].numel() * 2, qs[0].numel() * 2
        Op, certp, flagsp = O.data_ptr(), cert.data_ptr(), flags.data_ptr()

        # One step = append the new token + split pass + reduction + fallback ladder, all enqueued on
        # the stream: the ladder is resolved by a device kernel, so the host never waits inside the
        # loop (the timed region ends with a synchronisation).
        def step(i):
            cqa.cqa_decode_step_enqueue(h, 0, kp + i * kv_stride, vp + i * kv_stride,
                                        qp + i * q_stride, tol, Op, certp, flagsp, stream)

        if args.copy_probe:
            src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
            dst = torch.empty_like(src)
            dst.copy_(src)
            torch.cuda.synchronize()
            del src, dst
        # Spin-up before the W warm-up steps: a GPU that has idled through the set-up above needs a few
        # milliseconds of work before its clocks settle (measured: the first ~150 steps of a fresh
        # loop run ~8 % slower than the next 150).  Untimed decode steps without an append.
        for i in range(300):
            cqa.cqa_decode_step_enqueue(h, 0, None, None, qp + (i % n_in) * q_stride, tol, Op, certp, flagsp, stream)
        torch.cuda.synchronize()
        for i in range(W):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(W, W + K):
            step(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()

        # Duration of the dominant kernel: a second pass over the same step loop (a fixed number
        # of steps whatever --steps says), with a HIP event pair attached to every dispatch of the
        # split kernel on its launch stream.  (Kept out of the pass that yields `value`:
        # event-carrying dispatches slow the step.)  The first dispatches are dropped and the
        # median is what the roofline uses: a few slow dispatches drag a mean.
        cqa.cqa_profile_begin(h, ROOF_DISPATCHES)
        for i in range(ROOF_DISPATCHES):
            cqa.cqa_decode_step_enqueue(h, 0, None, None, qp + ((W + i) % n_in) * q_stride, tol, Op, certp,
                                        flagsp, stream)
        torch.cuda.synchronize()
        _, _, n_timed = cqa.cqa_profile_end(h)
        assert n_timed == ROOF_DISPATCHES
        kdur = np.sort(cqa.cqa_profile_durations(h)[ROOF_DROP:].astype(np.float64))
        median_ms, mean_ms, min_ms = float(np.median(kdur)), float(kdur.mean()), float(kdur[0])
        p90_ms = float(kdur[int(0.9 * (len(kdur) - 1))])
        ladder_counts = cqa.cqa_ladder_counts(h)

        # the optional INT8 x INT8 scoring mode (quantised scaled query on the INT8 matrix cores):
        # the same event-timed loop, reported next to the default kernel's figure
        tol8 = cqa.Tolerances(int8_query=True)
        cqa.cqa_profile_begin(h, 110)
        for i in range(110):
            cqa.cqa_decode_step_enqueue(h, 0, None, None, qp + ((W + i) % n_in) * q_stride, tol8, Op, certp,
                                        flagsp, stream)
        torch.cuda.synchronize()
        cqa.cqa_profile_end(h)
        q8_median_ms = float(np.median(cqa.cqa_profile_durations(h)[ROOF_DROP:]))

        # the same steps with the ladder resolved on the host (flag words read back through mapped
        # pinned memory after every step, fallback by copy + dense kernel): reported apart from `value`
        torch.cuda.synchronize()
        th0 = time.perf_counter()
        for i in range(W, W + K):
            cqa.cqa_decode_step(h, 0, qp + i * q_stride, tol, Op, certp, flagsp, None, stream)
        torch.cuda.synchronize()
        host_ms = (time.perf_counter() - th0) * 1e3 / K

        # Rung 3 through the device-resolved ladder: a tolerance between the two largest totals of
        # this query flags exactly one head; its KV group's originals are read from pinned host RAM
        # by the ladder kernel itself
        cqa.cqa_certified_decode(h, 0, qp, tol, Op, certp, flagsp, None, stream)
        torch.cuda.synchronize()
        cv = cert.cpu().numpy().view(np.dtype(cqa.CERT_FIELDS)).ravel()
        tot = np.sort(cv["E_key"].astype(np.float64) + cv["E_val"])
        tight = cqa.Tolerances(eps_total=float(0.5 * (tot[-1] + tot[-2])))
        n_fbd = 5
        cqa.cqa_decode_step_enqueue(h, 0, None, None, qp, tight, Op, certp, flagsp, stream)
        torch.cuda.synchronize()
        served_heads = int((cert.cpu().numpy().view(np.dtype(cqa.CERT_FIELDS)).ravel()["served_rung"] == 3).sum())
        td0 = time.perf_counter()
        for i in range(n_fbd):
            cqa.cqa_decode_step_enqueue(h, 0, None, None, qp, tight, Op, certp, flagsp, stream)
        torch.cuda.synchronize()
        fbd_ms = (time.perf_counter() - td0) * 1e3 / n_fbd

        # the ladder's cost, reported apart from `value`: the same decode with ONE of the 32 heads
        # served by Rung 3 (its KV group's FP16 originals paged in from pinned host RAM, dense
        # recompute, row overwritten)
        sel = np.zeros(sh.batch * sh.n_q_heads, np.uint32)
        sel[5] = 1
        n_fb = 5
        torch.cuda.synchronize()
        tf0 = time.perf_counter()
        for i in range(n_fb):
            cqa.cqa_certified_decode(h, 0, qp + i * q_stride, tol, Op, certp, flagsp, None, stream)
            cqa.cqa_dense_fallback(h, 0, qp + i * q_stride, sel, 0, 3, Op, certp, flagsp, stream)
        torch.cuda.synchronize()
        fb_ms = (time.perf_counter() - tf0) * 1e3 / n_fb

        # adaptive key precision, reported apart from `value`: scoring pass, selection (tau_cov 0.995,
        # K in [2, 128]), FP16-key gather from pinned host RAM, attend pass, ranking check, ladder
        sel = cqa.Selector(0.995, 2, 128, 128)
        atol = cqa.Tolerances(rank_depth=1, rank_min_mass=0.25)
        n_ad = 20
        for i in range(3):
            cqa.cqa_adaptive_step_enqueue(h, 0, qp + i * q_stride, atol, sel, Op, certp, flagsp, stream)
        torch.cuda.synchronize()
        lc0 = cqa.cqa_ladder_counts(h)
        ta0 = time.perf_counter()
        for i in range(n_ad):
            cqa.cqa_adaptive_step_enqueue(h, 0, qp + (W + i) * q_stride, atol, sel, Op, certp, flagsp, stream)
        torch.cuda.synchronize()
        ad_ms = (time.perf_counter() - ta0) * 1e3 / n_ad
        lc1 = cqa.cqa_ladder_counts(h)
        kst, _, prom, *_ = cqa.cqa_adaptive_state(h, 0, sh.batch, sh.n_q_heads, sh.n_kv_heads)
        prom = prom & 1
        # the same with value promotion (second rung) on: blocks whose estimated contribution exceeds
        # the paper's v_tol = 0.05 are attended from their FP16 values
        vsel = cqa.Selector(0.995, 2, 128, 128, v_limit=128)
        vtol = cqa.Tolerances(rank_depth=1, rank_min_mass=0.25, v_tol=0.05)
        for i in range(3):
            cqa.cqa_adaptive_step_enqueue(h, 0, qp + i * q_stride, vtol, vsel, Op, certp, flagsp, stream)
        torch.cuda.synchronize()
        tv0 = time.perf_counter()
        for i in range(n_ad):
            cqa.cqa_adaptive_step_enqueue(h, 0, qp + (W + i) * q_stride, vtol, vsel, Op, certp, flagsp, stream)
        torch.cuda.synchronize()
        adv_ms = (time.perf_counter() - tv0) * 1e3 / n_ad
        vstate = cqa.cqa_adaptive_state(h, 0, sh.batch, sh.n_q_heads, sh.n_kv_heads)
        # the optional FP16 scratch (off above): switched on, the 20 queries once with an empty
        # scratch (every promoted block is read from pinned host RAM and kept) and once more (every
        # promoted block is now held on the device)
        def timed_adaptive(first, tl, sl):
            torch.cuda.synchronize()
            tt = time.perf_counter()
            for i in range(n_ad):
                cqa.cqa_adaptive_step_enqueue(h, 0, qp + (first + i) * q_stride, tl, sl, Op, certp, flagsp, stream)
            torch.cuda.synchronize()
            return (time.perf_counter() - tt) * 1e3 / n_ad
        # the paper's default promoted sets (every head its own selection) against the per-group union
        # used above: same first pass and selection; the promoted-block pass gates each head on its own bits
        sel_ph = cqa.Selector(0.995, 2, 128, 128, per_head=True)
        timed_adaptive(0, atol, sel_ph)
        ad_ph_ms = timed_adaptive(W, atol, sel_ph)
        ph_state = cqa.cqa_adaptive_state(h, 0, sh.batch, sh.n_q_heads, sh.n_kv_heads)[2]
        ph_pairs = int(sum(bin(int(x)).count("1") for x in ((ph_state >> 4) & 15).ravel()))
        ph_blocks = int((ph_state & 1).sum())
        cqa.cqa_set_scratch_slots(h, 1024)
        ad_cold_ms = timed_adaptive(W, atol, sel)
        ad_warm_ms = timed_adaptive(W, atol, sel)
        sc_slots, sc_hits, sc_misses = cqa.cqa_scratch_stats(h)
        cqa.cqa_set_scratch_slots(h, 0)
        ad_info = {"ms_per_step": ad_ms, "ms_per_step_with_value_promotion": adv_ms,
                   "per_head_sets": {"ms_per_step": ad_ph_ms, "key_promoted_blocks_last_step": ph_blocks,
                                     "head_block_pairs_with_fp16_keys_last_step": ph_pairs,
                                     "what": "sel.per_head = 1 (the paper's default: each head's promoted set is its own "
                                             "selection); the FP16 keys of a block are read once per KV group when any head "
                                             "asks for them, so the bytes over the host link equal the union variant's "
                                             "(blocks x 4 KB); a union would give every listed block to all 4 heads"},
                   "key_scratch": {"ms_per_step_filling": ad_cold_ms, "ms_per_step_all_hits": ad_warm_ms,
                                   "slots_per_kv_head": sc_slots, "hits": sc_hits, "misses": sc_misses},
                   "value_blocks_per_head_median": float(np.median(vstate[5])), "steps_with_fallback": int(sum(lc1) - sum(lc0)),
                   "k_star_median": float(np.median(kst)), "k_star_max": int(kst.max()),
                   "promoted_blocks_per_group_max": int(prom.sum(axis=2).max()),
                   "what": f"cqa_adaptive_step_enqueue, wall time, mean of {n_ad} (tau_cov 0.995, K in [2, 128], ranking "
                           "check on, rank_min_mass 0.25; steps that fall back include the dense recompute); "
                           "promoted keys are read from pinned host RAM by the kernel; key_scratch: the same "
                           "20 queries with the optional device-resident FP16 scratch switched on, "
                           "first filling it, then hitting it"}

        # the streaming-read ceiling for this access pattern: the same records, launch shape and load
        # instructions, no arithmetic
        sr_ms, sr_bytes = cqa.cqa_time_stream_read(h, 0, 50, stream)
        # kernel-only rate: split pass + reduction back to back, no host synchronisation in between
        ko_ms = cqa.cqa_time_certified_decode(h, 0, qs[0], tol, O, cert, flags, None, 50, stream)
        splits = cqa.cqa_decode_splits(h, 0)
        n_tokens = cqa.cqa_cache_length(h, 0)
    finally:
        cqa.cqa_cache_destroy(h)

    # The same kernel with no reuse between launches: NO_REUSE_LAYERS resident copies of the layer,
    # visited in turn, so a record is read again only after (copies - 1) x 303 MB of other records
    # have gone through the memory system (the library picks the non-temporal load hint from the
    # footprint, as it does for a model's real layer stack).  Split pass + reduction only: this
    # cache keeps no FP16 originals.
    h2 = cqa.cqa_cache_create(NO_REUSE_LAYERS, sh.batch, sh.n_q_heads, sh.n_kv_heads, ctx + 64, cqa.TIER2_NONE)
    try:
        kd = torch.from_numpy(k).to(dev)
        vd = torch.from_numpy(v).to(dev)
        for layer in range(NO_REUSE_LAYERS):
            cqa.cqa_cache_append(h2, layer, kd, vd, ctx)
        torch.cuda.synchronize()
        del kd, vd
        for i in range(2 * NO_REUSE_LAYERS):
            cqa.cqa_certified_decode(h2, i % NO_REUSE_LAYERS, qp, tol, Op, certp, flagsp, None, stream)
        torch.cuda.synchronize()
        cqa.cqa_profile_begin(h2, ROOF_DISPATCHES)
        for i in range(ROOF_DISPATCHES):
            cqa.cqa_certified_decode(h2, i % NO_REUSE_LAYERS, qp + (i % n_in) * q_stride, tol, Op, certp,
                                     flagsp, None, stream)
        torch.cuda.synchronize()
        cqa.cqa_profile_end(h2)
        ndur = np.sort(cqa.cqa_profile_durations(h2)[ROOF_DROP:].astype(np.float64))
        nr_median, nr_mean, nr_min = float(np.median(ndur)), float(ndur.mean()), float(ndur[0])
        nr_sr = [cqa.cqa_time_stream_read(h2, i % NO_REUSE_LAYERS, 1, stream) for i in range(6 * NO_REUSE_LAYERS)]
        nr_sr_ms = float(np.median([x[0] for x in nr_sr[NO_REUSE_LAYERS:]]))
        nr_sr_bytes = nr_sr[0][1]
    finally:
        cqa.cqa_cache_destroy(h2)
    nr_bytes = sh.batch * sh.n_kv_heads * (ctx // 16) * 16 * BYTES_PER_TOKEN

    ms_per_step = (t1 - t0) * 1e3 / K
    nb_mid = (ctx + W + K // 2) // 16
    alg_bytes = sh.batch * sh.n_kv_heads * nb_mid * 16 * BYTES_PER_TOKEN
    achieved = alg_bytes / (median_ms * 1e-3) / 1e9
    out = {
        "metric": "certified decode attention steps/s per layer at 128K ctx; HBM GB/s vs peak",
        "value": K / (t1 - t0),
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": DTYPE,
        "data": "synthetic",
        "config": {
            "workload": f"t128k: 1 layer, batch {sh.batch}, {sh.n_q_heads} q / {sh.n_kv_heads} kv heads, "
                        f"d 128, context {ctx}+steps, K ~ Student-t(3), V ~ N(0,1), INT8 K / INT4 V "
                        f"(B=16, g=16), tolerances +inf, Tier-2 FP16 originals in pinned host RAM",
            "step": "append 1 token + certified decode + reduce + fallback ladder resolved on the device "
                    "(cqa_decode_step_enqueue; no host wait inside the loop)",
            "splits": splits,
            "final_tokens": n_tokens,
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": PEAK_HBM_GBS,
            "unit": "GB/s",
            "frac": achieved / PEAK_HBM_GBS,
            "traffic": read_traffic_note(),
            "traffic_source": "profiles/certified_split_t128k_pmc.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                              "command, committed; not measured in this run)",
            "kernel": "certified_split_mfma_kernel<4>",
            "kernel_median_ms": median_ms,
            "kernel_mean_ms": mean_ms,
            "kernel_min_ms": min_ms,
            "kernel_p90_ms": p90_ms,
            "kernel_timing": f"HIP event pair on each of {ROOF_DISPATCHES} dispatches of the step loop (a pass of its "
                             f"own after the timed one), first {ROOF_DROP} dropped; achieved and frac use the median",
            "algorithmic_bytes_per_launch": alg_bytes,
            "no_reuse": {
                "achieved": nr_bytes / (nr_median * 1e-3) / 1e9, "frac": nr_bytes / (nr_median * 1e-3) / 1e9 / PEAK_HBM_GBS,
                "kernel_median_ms": nr_median, "kernel_mean_ms": nr_mean, "kernel_min_ms": nr_min,
                "algorithmic_bytes_per_launch": nr_bytes,
                "stream_ceiling_GBps": nr_sr_bytes / (nr_sr_ms * 1e-3) / 1e9,
                "what": f"the same kernel alternating over {NO_REUSE_LAYERS} resident copies of the layer "
                        f"({NO_REUSE_LAYERS - 1} x 303 MB of other records between two visits of a record; "
                        f"non-temporal loads chosen by the library), {ROOF_DISPATCHES} event-timed dispatches, "
                        f"first {ROOF_DROP} dropped, median; stream_ceiling: the load-only kernel in the same rotation",
            },
            "stream_ceiling": {
                "GBps": sr_bytes / (sr_ms * 1e-3) / 1e9, "ms": sr_ms, "bytes": sr_bytes,
                "frac_of_ceiling": (alg_bytes / (median_ms * 1e-3)) / (sr_bytes / (sr_ms * 1e-3)),
                "what": "a load-only kernel over the same Tier-1 records with the split kernel's launch shape "
                        "and load instructions, 50 back-to-back launches: what the memory system delivers "
                        "for this access pattern (one 303 MB layer read repeatedly: part of it is served "
                        "by the memory-side cache)",
            },
        },
        "step_level": {
            "achieved": alg_bytes / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s",
            "frac": alg_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "what": "the same algorithmic bytes over the whole step's time (ms_per_step): the split pass plus "
                    "the reduction, the ladder kernel, the append and their dispatch gaps",
        },
        "kernel_only": {
            "ms_per_step": ko_ms,
            "steps_per_s": 1e3 / ko_ms,
            "what": "split pass + reduction, 50 back-to-back launches between two HIP events",
        },
        "int8_query_scoring": {
            "kernel_median_ms": q8_median_ms,
            "what": "split kernel with cqa_tolerances.int8_query = 1 (scaled query quantised to 8 bits per block, "
                    "mfma_i32_16x16x64_i8 scoring, explicit third error term in Delta_h), event-timed over 100 "
                    "dispatches of the step loop, median; compare roofline.kernel_median_ms",
        },
        "adaptive_step": ad_info,
        "host_ladder_step": {
            "ms_per_step": host_ms,
            "what": f"cqa_decode_step (no append): flag words read back by the host after every step, mean of {K}",
        },
        "ladder": {
            "rung3_steps": ladder_counts[0], "rung4_steps": ladder_counts[1],
            "what": "steps of the timed and the profiled pass that the device-resolved ladder served by a rung",
        },
        "fallback_step_device": {
            "ms_per_step": fbd_ms, "heads_served": served_heads,
            "what": "cqa_decode_step_enqueue with one head over its tolerance: Rung 3 by the ladder kernel, which "
                    f"reads the KV group's originals from pinned host RAM itself, wall time, mean of {n_fbd}",
        },
        "fallback_step": {
            "ms_per_step": fb_ms,
            "what": "certified decode + Rung 3 for 1 of 32 heads (one KV group paged from pinned host RAM: "
                    f"{2 * n_tokens * 128 * 2 / 1e6:.1f} MB host-to-device), wall time, mean of {n_fb}",
        },
        "bulk_append": {
            "GBps_in": 2 * k.nbytes / bulk_s / 1e9,
            "ms": bulk_s * 1e3,
            "what": f"one append of {ctx} tokens x {sh.n_kv_heads} KV heads (FP16 K and V in, Tier-1 records out, "
                    "FP16 originals copied to pinned host RAM), wall time incl. the device-to-host copy",
        },
        "cpu_baseline": base,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
