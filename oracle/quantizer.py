"""CPU oracle, part 1: the cache-write quantizers (test infrastructure only).

This file is the slow, plain reference the HIP kernels are checked against.
It is NOT part of the product path: only tests, the smoke check and the
bench's cpu_baseline leg may import it.  It shares no code with the HIP path.

What it follows (paper sections, in the paper's notation):

* Keys -- "Per-channel INT8 keys" (Quantization Schemes): for one sealed block
  of B=16 tokens and each channel c, with channel minimum l_c and maximum u_c,
      sigma_c = (u_c - l_c) / 255,    z_c = l_c + 128 sigma_c,
      code    = clamp(round((k - z_c) / sigma_c), -128, 127),
      k_hat   = code * sigma_c + z_c.
  sigma_c and z_c are FP32 per block and per channel.
* Values -- "Per-group INT4 values": every token's d channels are cut into
  groups of g=16; each group gets an FP16 scale and an offset and 4-bit codes,
  two codes per byte.
* Annotations -- "Value error annotation": eta_b = max_t ||v_hat_t - v_t||_2
  and nu_b = max_t ||v_t||_2 over the block's tokens, one float each.

Readings where the paper leaves the arithmetic open (the HIP path follows the
same readings so that codes and scales can be compared bit for bit):

* All quantizer arithmetic is IEEE binary32, one rounding per operation, in
  exactly the order written above (subtract, true divide; multiply, add;
  subtract, true divide, round-half-even, clamp).  numpy's float32 ufuncs do
  exactly this (no fused multiply-add).
* "round" is round-half-to-even.
* z_c = l_c + 128 sigma_c (the paper's other form u_c - 127 sigma_c differs in
  floating point).
* Constant channel (u_c == l_c): sigma_c = 0, z_c = l_c, code = 0, k_hat = l_c.
* INT4 codes are unsigned 0..15; offset = group minimum (already FP16, exact);
  scale = fp16_round((hi - lo) / 15); codes use the rounded scale so that
  v_hat = code * scale + offset is self-consistent.  Scale 0 (constant group, or
  a range so small that it rounds to FP16 zero): code = 0, v_hat = offset.
* Canonical packing: byte j holds channel 2j in its low nibble, 2j+1 in its high.
* eta_b and nu_b are evaluated in float64 from the real-number reconstruction
  and then rounded once to float32.
"""
from __future__ import annotations

import numpy as np

B = 16  # tokens per block
G = 16  # value channels per group


def quantize_key_blocks(k16: np.ndarray):
    """k16: float16 [..., B, d] (one or many sealed blocks).

    Returns (codes int8 [..., B, d], sigma float32 [..., d], z float32 [..., d]).
    """
    assert k16.dtype == np.float16 and k16.shape[-2] == B
    k = k16.astype(np.float32)
    lo = k.min(axis=-2)
    hi = k.max(axis=-2)
    sigma = (hi - lo) / np.float32(255.0)
    z = lo + np.float32(128.0) * sigma
    safe = np.where(sigma == 0, np.float32(1.0), sigma)
    t = (k - z[..., None, :]) / safe[..., None, :]
    codes = np.clip(np.rint(t), -128.0, 127.0)
    codes = np.where(sigma[..., None, :] == 0, np.float32(0.0), codes).astype(np.int8)
    assert sigma.dtype == np.float32 and z.dtype == np.float32
    return codes, sigma, z


def dequantize_keys(codes: np.ndarray, sigma: np.ndarray, z: np.ndarray) -> np.ndarray:
    """k_hat = code * sigma + z as real numbers (float64)."""
    return codes.astype(np.float64) * sigma.astype(np.float64)[..., None, :] \
        + z.astype(np.float64)[..., None, :]


def quantize_values(v16: np.ndarray):
    """v16: float16 [..., d].

    Returns (codes uint8 [..., d] in 0..15, scale float16 [..., d/G],
    offset float16 [..., d/G]).
    """
    assert v16.dtype == np.float16 and v16.shape[-1] % G == 0
    d = v16.shape[-1]
    v = v16.astype(np.float32).reshape(v16.shape[:-1] + (d // G, G))
    lo = v.min(axis=-1)
    hi = v.max(axis=-1)
    scale_h = ((hi - lo) / np.float32(15.0)).astype(np.float16)
    s = scale_h.astype(np.float32)
    safe = np.where(s == 0, np.float32(1.0), s)
    t = (v - lo[..., None]) / safe[..., None]
    codes = np.clip(np.rint(t), 0.0, 15.0)
    codes = np.where(s[..., None] == 0, np.float32(0.0), codes).astype(np.uint8)
    offset_h = lo.astype(np.float16)  # exact: lo is one of the FP16 inputs
    return codes.reshape(v16.shape), scale_h, offset_h


def dequantize_values(codes: np.ndarray, scale_h: np.ndarray, offset_h: np.ndarray) -> np.ndarray:
    """v_hat = code * scale + offset as real numbers (float64)."""
    d = codes.shape[-1]
    c = codes.astype(np.float64).reshape(codes.shape[:-1] + (d // G, G))
    vh = c * scale_h.astype(np.float64)[..., None] + offset_h.astype(np.float64)[..., None]
    return vh.reshape(codes.shape)


def pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """Canonical packing: byte j = codes[2j] | codes[2j+1] << 4."""
    assert codes.dtype == np.uint8
    lo = codes[..., 0::2]
    hi = codes[..., 1::2]
    return (lo | (hi << 4)).astype(np.uint8)


def unpack_nibbles(packed: np.ndarray) -> np.ndarray:
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = packed & 0x0F
    out[..., 1::2] = packed >> 4
    return out


def block_annotations(v16: np.ndarray, v_hat: np.ndarray):
    """v16 float16 [..., NB, B, d], v_hat float64 same shape.

    Returns (eta float32 [..., NB], nu float32 [..., NB]).
    """
    v = v16.astype(np.float64)
    err = np.sqrt(((v_hat - v) ** 2).sum(axis=-1))
    nrm = np.sqrt((v ** 2).sum(axis=-1))
    return err.max(axis=-1).astype(np.float32), nrm.max(axis=-1).astype(np.float32)


# Storage arithmetic of the Tier-1 layout (bytes per token per KV head),
# following the paper's storage table: codes + metadata, d=128, B=16, g=16.
def tier1_bytes_per_token(d: int = 128, block: int = B, group: int = G) -> dict:
    return {
        "k_codes": float(d),
        "k_meta": 2.0 * d * 4.0 / block,
        "v_codes": d / 2.0,
        "v_meta": 2.0 * (d / group) * 2.0,
        "eta": 4.0 / block,
        "nu": 4.0 / block,
    }
