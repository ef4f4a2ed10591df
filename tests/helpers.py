"""Shared plumbing for the GPU parity tests: device buffers via torch, calls via the C ABI."""
import math
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def load_binding():
    """Loads the built library; builds it first only if nothing has been built."""
    from paper_2605_20868_amd import build as b
    if not os.path.exists(b.OUT):
        b.build(verbose=False)
    from paper_2605_20868_amd import binding
    return binding


class GpuLayerCache:
    """One-layer cache on cuda:0 driven through the C ABI."""

    def __init__(self, batch, n_q_heads, n_kv_heads, max_tokens, tier2=True, n_layers=1):
        import torch
        self.torch = torch
        self.cqa = load_binding()
        self.dev = torch.device("cuda:0")
        self.bt, self.hq, self.hkv = batch, n_q_heads, n_kv_heads
        self.h = self.cqa.cqa_cache_create(
            n_layers, batch, n_q_heads, n_kv_heads, max_tokens,
            self.cqa.TIER2_PINNED if tier2 else self.cqa.TIER2_NONE)
        n = batch * n_q_heads
        self.O = torch.zeros((batch, n_q_heads, 128), dtype=torch.float32, device=self.dev)
        self.cert = torch.zeros((n, self.cqa.CERT_BYTES), dtype=torch.uint8, device=self.dev)
        self.flags = torch.zeros((n,), dtype=torch.int32, device=self.dev)

    def close(self):
        if self.h is not None:
            self.cqa.cqa_cache_destroy(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def length(self, layer=0):
        return self.cqa.cqa_cache_length(self.h, layer)

    def append(self, k16, v16, layer=0):
        t = self.torch
        kd = k16 if isinstance(k16, t.Tensor) else t.from_numpy(np.ascontiguousarray(k16)).to(self.dev)
        vd = v16 if isinstance(v16, t.Tensor) else t.from_numpy(np.ascontiguousarray(v16)).to(self.dev)
        self.cqa.cqa_cache_append(self.h, layer, kd, vd, kd.shape[2])
        t.cuda.synchronize()

    def to_dev(self, q16):
        return self.torch.from_numpy(np.ascontiguousarray(q16)).to(self.dev)

    def results(self):
        self.torch.cuda.synchronize()
        O = self.O.cpu().numpy().astype(np.float64)
        cert = self.cert.cpu().numpy().view(np.dtype(self.cqa.CERT_FIELDS)).reshape(self.bt, self.hq)
        flags = self.flags.cpu().numpy().view(np.uint32).reshape(self.bt, self.hq)
        return O, cert, flags

    def certified_decode(self, q16, tol=None, layer=0, want_logmass=False):
        qd = self.to_dev(q16)
        lm = None
        if want_logmass:
            nb = self.length(layer) // 16
            lm = self.torch.zeros((self.bt, self.hq, max(nb, 1)), dtype=self.torch.float32,
                                  device=self.dev)
        self.cqa.cqa_certified_decode(self.h, layer, qd, tol or self.cqa.Tolerances(), self.O,
                                      self.cert, self.flags, lm)
        O, cert, flags = self.results()
        if want_logmass:
            return O, cert, flags, lm.cpu().numpy()
        return O, cert, flags

    def decode_step(self, q16, tol=None, layer=0):
        qd = self.to_dev(q16)
        rung = self.cqa.cqa_decode_step(self.h, layer, qd, tol or self.cqa.Tolerances(), self.O,
                                        self.cert, self.flags, None)
        O, cert, flags = self.results()
        return rung, O, cert, flags

    def export(self, b, kvh, block, layer=0):
        return self.cqa.cqa_cache_export_block(self.h, layer, b, kvh, block)


def to_gpu_tol(cqa, tol):
    """oracle.Tolerances -> binding.Tolerances (same fields)."""
    return cqa.Tolerances(tol.eps_total, tol.eps_key, tol.eps_val, tol.v_tol, tol.rank_min_mass,
                          tol.eps_guard, tol.rank_depth, tol.mass_exp, tol.key_bound_mode,
                          tol.rung4_min_groups, tol.force_flags, tol.int8_query)


CERT_REL = 1e-4      # bounds: |gpu - oracle| <= 1e-4 |oracle| + 1e-9
O_REL = 1e-3         # outputs: ||gpu - oracle|| <= 1e-3 ||oracle|| + 1e-6, and element-wise
                     # |gpu_c - oracle_c| <= 1e-3 max_c |oracle_c| + 1e-6 (a few wrong channels
                     # cannot hide in the norm of a head with a large output)


def assert_head_matches(ref, O_row, cert_row, flags_word, where, check_flags=True):
    err = np.linalg.norm(O_row - ref["O"])
    assert err <= O_REL * np.linalg.norm(ref["O"]) + 1e-6, (where, "O", err, np.linalg.norm(ref["O"]))
    worst = np.abs(O_row - ref["O"]).max()
    assert worst <= O_REL * np.abs(ref["O"]).max() + 1e-6, (where, "O element", worst, np.abs(ref["O"]).max())
    served = ref.get("served_rung", 0)
    for name in ("E_key", "E_val"):
        a, b = float(cert_row[name]), ref[name]
        if math.isinf(b):
            assert a == b, (where, name, a, b)      # a bound beyond binary32 is +inf on both sides
            continue
        assert abs(a - b) <= CERT_REL * abs(b) + 1e-9, (where, name, a, b)
    if served == 0:
        for name in ("delta_h", "v_max", "alpha_tail_hat", "max_block_contrib"):
            a, b = float(cert_row[name]), ref[name]
            assert abs(a - b) <= CERT_REL * abs(b) + 1e-9, (where, name, a, b)
        assert abs(float(cert_row["lse"]) - ref["lse"]) <= 1e-4 * max(1.0, abs(ref["lse"])), (where, "lse")
        if math.isfinite(ref["rank_margin"]):
            # a difference of two FP32 log-masses: 2e-4 absolute at ordinary logit sizes, relative to
            # the log-masses' own magnitude when the logits are in the thousands
            assert abs(float(cert_row["rank_margin"]) - ref["rank_margin"]) <= 2e-4 * max(1.0, abs(ref["lse"])), \
                (where, "margin", float(cert_row["rank_margin"]), ref["rank_margin"])
            if ref["rank_margin"] > 1e-3:
                assert int(cert_row["top_block"]) == ref["top_block"], (where, "top_block")
        else:
            assert math.isinf(float(cert_row["rank_margin"]))
    assert int(cert_row["served_rung"]) == served, (where, "served_rung")
    if check_flags:
        assert int(flags_word) == ref["flags"], (where, "flags", int(flags_word), ref["flags"])
