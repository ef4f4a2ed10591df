"""The no-allocation decode under HIP graph capture: the call is recorded into a graph (it launches
kernels and does nothing else: no allocation, no memory-set node, no host wait) and replayed several
times with eager work and synchronisations between the replays; every replay must reproduce the
eager result bit for bit, also after the query buffer has been refilled in place.
"""
import numpy as np
import pytest

import workloads
from helpers import GpuLayerCache

pytestmark = pytest.mark.gpu


def test_noalloc_decode_replays_from_a_graph():
    print("graph capture of cqa_certified_decode_noalloc: l8k shape, 4 replays, 3 queries", flush=True)
    sh = workloads.SHAPES["l8k"]
    n = 8192 - 11
    k, v = workloads.make_kv("l8k", seed=0, context=n)
    qs = [workloads.make_q("l8k", i, seed=0) for i in range(3)]
    with GpuLayerCache(sh.batch, sh.n_q_heads, sh.n_kv_heads, 8192 + 64) as gc:
        t, cqa = gc.torch, gc.cqa
        gc.append(k, v)
        tol = cqa.Tolerances()
        qd = gc.to_dev(qs[0]).clone()                 # the buffer the graph reads
        eager = []
        for q in qs:
            qd.copy_(gc.to_dev(q))
            cqa.cqa_certified_decode_noalloc(gc.h, 0, qd, tol, gc.O, gc.cert, gc.flags)
            eager.append(gc.results())
        s = t.cuda.Stream()
        g = t.cuda.CUDAGraph()
        qd.copy_(gc.to_dev(qs[0]))
        t.cuda.synchronize()
        with t.cuda.graph(g, stream=s):
            cqa.cqa_certified_decode_noalloc(gc.h, 0, qd, tol, gc.O, gc.cert, gc.flags, s.cuda_stream)
        for rep, qi in enumerate((0, 1, 2, 1)):
            qd.copy_(gc.to_dev(qs[qi]))
            gc.O.fill_(float("nan"))                  # eager work between the replays
            gc.cert.zero_()
            gc.flags.fill_(-1)
            t.cuda.synchronize()
            g.replay()
            t.cuda.synchronize()
            O, cert, flags = gc.results()
            O0, c0, f0 = eager[qi]
            assert np.array_equal(O, O0), ("replay", rep, "O")
            assert cert.tobytes() == c0.tobytes(), ("replay", rep, "cert")
            assert (flags == f0).all(), ("replay", rep, "flags")
            # an eager call of the ordinary entry point in between (it shares nothing with the graph's scratch)
            cqa.cqa_certified_decode(gc.h, 0, qd, tol, gc.O, gc.cert, gc.flags, None)
            assert np.array_equal(gc.results()[0], O0)
