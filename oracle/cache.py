"""CPU oracle, part 3: the tiered cache and the fallback ladder (test infrastructure only).

Follows the paper's cache description: tokens are appended to a trailing FP16
partial block; when B=16 tokens have arrived the block is sealed (quantized
atomically from those B tokens alone) and is immutable afterwards; the FP16
originals of every token are retained (Tier 2) and are what the dense fallback
recomputes from.

Ladder reading (the paper's Rung 3 is per head, Rung 4 per layer and all heads;
the adaptive selector's Rungs 1-2 are outside the hot path, so every request for
more precision is served by the first rung that exists here, which is sound
because the ladder only ever increases precision):

* a head whose flag word has any of KEY/VAL/RANK/TOTAL/PRECOND set needs the
  dense recompute;
* Rung 4 (all heads of the layer) if any head has PRECOND, or if
  rung4_min_groups > 0 and at least that many (batch, kv-head) groups hold a
  flagged head; otherwise Rung 3 for exactly the flagged heads;
* a served head returns O_dense = softmax(q K^T / sqrt d) V on the FP16
  originals, its certificate terms become (0, 0), and the rung served is written
  to the certificate and to bits 8-10 of the flag word.
"""
from __future__ import annotations

import numpy as np

from . import attention as att
from . import quantizer as qz


class OracleLayerCache:
    """One layer's cache for Bt sequences and Hkv KV heads (all the same length)."""

    def __init__(self, batch: int, n_kv_heads: int, head_dim: int = 128, tier2: bool = True):
        self.bt, self.hkv, self.d = batch, n_kv_heads, head_dim
        self.tier2 = tier2
        self.k16 = np.zeros((batch, n_kv_heads, 0, head_dim), dtype=np.float16)
        self.v16 = np.zeros((batch, n_kv_heads, 0, head_dim), dtype=np.float16)
        shp = (batch, n_kv_heads, 0)
        self.k_codes = np.zeros(shp + (qz.B, head_dim), dtype=np.int8)
        self.sigma = np.zeros(shp + (head_dim,), dtype=np.float32)
        self.z = np.zeros(shp + (head_dim,), dtype=np.float32)
        self.v_codes = np.zeros(shp + (qz.B, head_dim), dtype=np.uint8)
        self.v_scale = np.zeros(shp + (qz.B, head_dim // qz.G), dtype=np.float16)
        self.v_offset = np.zeros(shp + (qz.B, head_dim // qz.G), dtype=np.float16)
        self.eta = np.zeros(shp, dtype=np.float32)
        self.nu = np.zeros(shp, dtype=np.float32)

    @property
    def length(self) -> int:
        return self.k16.shape[2]

    @property
    def n_blocks(self) -> int:
        return self.k_codes.shape[2]

    def append(self, k16: np.ndarray, v16: np.ndarray) -> None:
        """k16, v16 float16 [Bt, Hkv, n_new, d]; seals every block that completes."""
        assert k16.dtype == np.float16 and v16.dtype == np.float16
        self.k16 = np.concatenate([self.k16, k16], axis=2)
        self.v16 = np.concatenate([self.v16, v16], axis=2)
        nb_new = self.length // qz.B
        nb_old = self.n_blocks
        if nb_new == nb_old:
            return
        lo, hi = nb_old * qz.B, nb_new * qz.B
        kb = self.k16[:, :, lo:hi].reshape(self.bt, self.hkv, nb_new - nb_old, qz.B, self.d)
        vb = self.v16[:, :, lo:hi].reshape(self.bt, self.hkv, nb_new - nb_old, qz.B, self.d)
        codes, sigma, z = qz.quantize_key_blocks(kb)
        vc, vs, vo = qz.quantize_values(vb)
        v_hat = qz.dequantize_values(vc, vs, vo)
        eta, nu = qz.block_annotations(vb, v_hat)
        self.k_codes = np.concatenate([self.k_codes, codes], axis=2)
        self.sigma = np.concatenate([self.sigma, sigma], axis=2)
        self.z = np.concatenate([self.z, z], axis=2)
        self.v_codes = np.concatenate([self.v_codes, vc], axis=2)
        self.v_scale = np.concatenate([self.v_scale, vs], axis=2)
        self.v_offset = np.concatenate([self.v_offset, vo], axis=2)
        self.eta = np.concatenate([self.eta, eta], axis=2)
        self.nu = np.concatenate([self.nu, nu], axis=2)

    def certified_decode(self, q16: np.ndarray, tol: att.Tolerances, heads=None) -> list:
        """q16 float16 [Bt, Hq, d].  Returns a list of per-(b, h) result dicts (row-major).

        `heads` optionally restricts the work to an iterable of (b, h) pairs.
        """
        bt, hq, d = q16.shape
        g = hq // self.hkv
        nb = self.n_blocks
        todo = [(b, h) for b in range(bt) for h in range(hq)] if heads is None else list(heads)
        out = {}
        cache_kv = {}
        for b, h in todo:
            kh = h // g
            if (b, kh) not in cache_kv:
                k_hat = qz.dequantize_keys(self.k_codes[b, kh], self.sigma[b, kh], self.z[b, kh])
                v_hat = qz.dequantize_values(self.v_codes[b, kh], self.v_scale[b, kh],
                                             self.v_offset[b, kh])
                cache_kv = {(b, kh): (k_hat.reshape(nb * qz.B, d), v_hat.reshape(nb * qz.B, d))}
            k_hat, v_hat = cache_kv[(b, kh)]
            out[(b, h)] = att.certified_head(
                q16[b, h], k_hat, v_hat, self.sigma[b, kh], self.eta[b, kh], self.nu[b, kh],
                self.k16[b, kh, nb * qz.B:], self.v16[b, kh, nb * qz.B:], tol,
                k_codes=self.k_codes[b, kh], z=self.z[b, kh])
        return [out[key] for key in todo]

    def dense_head(self, q16: np.ndarray, b: int, h: int, n_q_heads: int) -> np.ndarray:
        if not self.tier2:
            raise RuntimeError("Tier-2 originals unavailable: cannot fall back")
        g = n_q_heads // self.hkv
        return att.softmax_attention(q16[b, h], self.k16[b, h // g], self.v16[b, h // g])

    def decode_step(self, q16: np.ndarray, tol: att.Tolerances) -> list:
        """Certified decode followed by the ladder.  Results carry 'served_rung'."""
        bt, hq, _ = q16.shape
        g = hq // self.hkv
        res = self.certified_decode(q16, tol)
        need = [(r["flags"] & att.FLAG_ANY) != 0 for r in res]
        rung = ladder_decision([r["flags"] for r in res], bt, hq, g, tol.rung4_min_groups)
        for i, r in enumerate(res):
            b, h = divmod(i, hq)
            r["served_rung"] = 0
            if rung == 4 or (rung == 3 and need[i]):
                r["O"] = self.dense_head(q16, b, h, hq)
                r["E_key"] = 0.0
                r["E_val"] = 0.0
                r["served_rung"] = rung
                r["flags"] |= rung << att.RUNG_SHIFT
        return res


def ladder_decision(flags, batch: int, n_q_heads: int, group: int, rung4_min_groups: int) -> int:
    """0 = nothing to do, 3 = per-head recompute of flagged heads, 4 = whole layer."""
    need = [(f & att.FLAG_ANY) != 0 for f in flags]
    if not any(need):
        return 0
    if any(f & att.FLAG_PRECOND for f in flags):
        return 4
    groups = {(i // n_q_heads, (i % n_q_heads) // group) for i, n in enumerate(need) if n}
    if rung4_min_groups > 0 and len(groups) >= rung4_min_groups:
        return 4
    return 3
