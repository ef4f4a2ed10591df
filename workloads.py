"""Seeded synthetic inputs for the certified-decode hot path.

This module only draws random numbers and shapes them into LLaMA-3.1-8B-like
KV caches (32 query heads, 8 KV heads, head_dim 128).  It holds none of the
method's arithmetic: no quantizer, no softmax, no bound.  Both the CPU oracle's
tests and the HIP path's tests/bench take their FP16 bit patterns from here so
the two sides see identical inputs.

The five named workloads stand in for the model caches the paper measures on
(its text corpora and weights are not available offline); only their shapes and
value statistics are imitated:

  tiny      Bt=1 Hkv=1 Hq=4  N=1024    K,V,q ~ N(0,1)
  l8k       Bt=1 Hkv=8 Hq=32 N=8192    K ~ N(0,1) with 4 outlier channels x20
  mixed32k  Bt=4 Hkv=8 Hq=32 N=32768   half the heads peaked (logit gap 10)
  t128k     Bt=1 Hkv=8 Hq=32 N=131072  K ~ Student-t(3), V ~ N(0,1)
  stack     32 layers of t128k-like data at Bt=2 (generated on the device)

All arrays are numpy float16, laid out [Bt, H, T, d].
"""
from __future__ import annotations

import dataclasses
import zlib

import numpy as np

HEAD_DIM = 128
BLOCK = 16


@dataclasses.dataclass(frozen=True)
class Shape:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    context: int
    steps: int
    n_layers: int = 1
    head_dim: int = HEAD_DIM

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


SHAPES = {
    "tiny": Shape("tiny", 1, 4, 1, 1024, 1),
    "l8k": Shape("l8k", 1, 32, 8, 8192, 64),
    "mixed32k": Shape("mixed32k", 4, 32, 8, 32768, 1),
    "t128k": Shape("t128k", 1, 32, 8, 131072, 16),
    "stack": Shape("stack", 2, 32, 8, 131072, 8, n_layers=32),
    # batched serving: many short sequences, one split per KV group
    "serve64": Shape("serve64", 64, 32, 8, 4096, 1),
}


def _rng(seed: int, *key) -> np.random.Generator:
    """Independent sub-stream per (seed, key...) so tensors can be drawn in any order."""
    words = [seed & 0xFFFFFFFF]
    for k in key:
        if isinstance(k, str):
            words.append(zlib.crc32(k.encode()))
        else:
            words.append(int(k) & 0xFFFFFFFF)
    return np.random.Generator(np.random.Philox(np.random.SeedSequence(words)))


def normal_f16(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.standard_normal(shape, dtype=np.float32).astype(np.float16)


def student_t3_f16(rng: np.random.Generator, shape) -> np.ndarray:
    """t(3) = z0 / sqrt((z1^2+z2^2+z3^2)/3), drawn in float32, cast to float16."""
    z0 = rng.standard_normal(shape, dtype=np.float32)
    acc = np.zeros(shape, dtype=np.float32)
    for _ in range(3):
        z = rng.standard_normal(shape, dtype=np.float32)
        acc += z * z
    np.sqrt(acc / np.float32(3.0), out=acc)
    return (z0 / acc).astype(np.float16)


def outlier_channels(seed: int, n_kv_heads: int, head_dim: int = HEAD_DIM, count: int = 4):
    """The `count` channel indices per KV head that carry the x20 outliers."""
    out = []
    for h in range(n_kv_heads):
        r = _rng(seed, "outlier", h)
        out.append(np.sort(r.choice(head_dim, size=count, replace=False)))
    return np.stack(out)


def make_kv(name: str, seed: int = 0, layer: int = 0, context: int | None = None,
            batch: int | None = None, n_kv_heads: int | None = None):
    """FP16 K and V of shape [Bt, Hkv, N, d] for a named workload."""
    sh = SHAPES[name]
    n = sh.context if context is None else context
    bt = sh.batch if batch is None else batch
    hkv = sh.n_kv_heads if n_kv_heads is None else n_kv_heads
    shape = (bt, hkv, n, sh.head_dim)
    rk = _rng(seed, name, layer, "K")
    rv = _rng(seed, name, layer, "V")
    if name in ("t128k", "stack", "serve64"):
        k = student_t3_f16(rk, shape)
    else:
        k = normal_f16(rk, shape)
    if name == "l8k":
        ch = outlier_channels(seed, hkv, sh.head_dim)
        k32 = k.astype(np.float32)
        for h in range(hkv):
            k32[:, h, :, ch[h]] *= np.float32(20.0)
        k = k32.astype(np.float16)
    v = normal_f16(rv, shape)
    return k, v


def make_step_kv(name: str, step: int, seed: int = 0, layer: int = 0,
                 batch: int | None = None, n_kv_heads: int | None = None):
    """One appended (k, v) token per (batch, kv-head): shape [Bt, Hkv, 1, d]."""
    sh = SHAPES[name]
    bt = sh.batch if batch is None else batch
    hkv = sh.n_kv_heads if n_kv_heads is None else n_kv_heads
    shape = (bt, hkv, 1, sh.head_dim)
    rk = _rng(seed, name, layer, "Kstep", step)
    rv = _rng(seed, name, layer, "Vstep", step)
    if name in ("t128k", "stack", "serve64"):
        k = student_t3_f16(rk, shape)
    else:
        k = normal_f16(rk, shape)
    if name == "l8k":
        ch = outlier_channels(seed, hkv, sh.head_dim)
        k32 = k.astype(np.float32)
        for h in range(hkv):
            k32[:, h, :, ch[h]] *= np.float32(20.0)
        k = k32.astype(np.float16)
    v = normal_f16(rv, shape)
    return k, v


def make_q(name: str, step: int = 0, seed: int = 0, layer: int = 0,
           batch: int | None = None, n_q_heads: int | None = None) -> np.ndarray:
    """FP16 queries [Bt, Hq, d] ~ N(0,1)."""
    sh = SHAPES[name]
    bt = sh.batch if batch is None else batch
    hq = sh.n_q_heads if n_q_heads is None else n_q_heads
    return normal_f16(_rng(seed, name, layer, "q", step), (bt, hq, sh.head_dim))


def make_peaked_q(k: np.ndarray, n_q_heads: int, gap: float = 10.0, seed: int = 0,
                  name: str = "mixed32k"):
    """Queries for the mixed-regime workload.

    Even query heads are aligned with one planted key of their KV head so that
    this key's logit exceeds every other logit by `gap` (on the FP16 keys, before
    the query is rounded to FP16); odd heads are diffuse N(0,1) draws.
    Returns (q [Bt,Hq,d] float16, planted positions [Bt,Hq] with -1 for diffuse).
    """
    bt, hkv, n, d = k.shape
    g = n_q_heads // hkv
    q = normal_f16(_rng(seed, name, "q_diffuse"), (bt, n_q_heads, d))
    planted = -np.ones((bt, n_q_heads), dtype=np.int64)
    rp = _rng(seed, name, "planted")
    inv = 1.0 / np.sqrt(float(d))
    for b in range(bt):
        for h in range(0, n_q_heads, 2):
            kh = k[b, h // g].astype(np.float64)
            p = int(rp.integers(0, n))
            dots = (kh @ kh[p]) * inv
            a = dots[p]
            dots[p] = -np.inf
            c = gap / (a - dots.max())
            q[b, h] = (c * kh[p]).astype(np.float16)
            planted[b, h] = p
    return q, planted


def plant_near_tie(k: np.ndarray, v: np.ndarray, q: np.ndarray, b: int, hq: int,
                   n_q_heads: int, seed: int = 0, gap: float = 10.0, nudge: float = 0.01,
                   longest_key: bool = False):
    """Adversarial head: two keys in different blocks whose logits nearly tie.

    Position p2 receives a copy of key p1 with one channel nudged so the two
    FP16 logits differ by about `nudge`, both exceeding every other logit by
    about `gap`; the value at p2 is the negation of the value at p1.  Edits k, v
    and q in place and returns (p1, p2).

    p1 is a seeded position in the first half of the context, or, with
    `longest_key`, the longest key of the first half: on heavy-tailed keys a
    typical key is out-scored along its own direction by some far longer key,
    and only the longest one can be given a positive logit gap by scaling.
    """
    bt, hkv, n, d = k.shape
    g = n_q_heads // hkv
    kh = hq // g
    r = _rng(seed, "near_tie", b, hq)
    p1 = int(r.integers(0, n // 2))
    if longest_key:
        kk = k[b, kh, : n // 2].astype(np.float32)
        p1 = int(np.argmax(np.einsum("td,td->t", kk, kk)))
    p2 = int(n // 2 + r.integers(0, n // 2))
    p2 = min(p2, n - 1)
    if p1 // BLOCK == p2 // BLOCK:
        p2 = (p2 + BLOCK) % n
    inv = 1.0 / np.sqrt(float(d))
    base = k[b, kh, p1].astype(np.float64)
    dots = (k[b, kh].astype(np.float64) @ base) * inv
    a = dots[p1]
    dots[p1] = -np.inf
    dots[p2] = -np.inf
    assert a > dots.max(), "the planted key does not lead along its own direction"
    c = gap / (a - dots.max())
    q[b, hq] = (c * base).astype(np.float16)
    qf = q[b, hq].astype(np.float64)
    ch = int(np.argmax(np.abs(qf)))
    twin = base.copy()
    twin[ch] -= nudge / (qf[ch] * inv)
    k[b, kh, p2] = twin.astype(np.float16)
    v[b, kh, p2] = -v[b, kh, p1]
    return p1, p2


def torch_device_kv(name: str, layer: int, device, seed: int = 0, batch: int | None = None,
                    context: int | None = None):
    """Device-side generator for the 32-layer stack: same distributions, torch RNG.

    Returns torch float16 tensors (k, v) of shape [Bt, Hkv, N, d] on `device`.
    Used where 8 host cores cannot draw tens of GB of samples in reasonable time;
    the oracle then receives these exact bits copied back to the host.
    """
    import torch

    sh = SHAPES[name]
    bt = sh.batch if batch is None else batch
    n = sh.context if context is None else context
    gen = torch.Generator(device=device)
    gen.manual_seed((seed * 1000003 + layer * 7919 + zlib.crc32(name.encode())) & 0x7FFFFFFF)
    shape = (bt, sh.n_kv_heads, n, sh.head_dim)
    z0 = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    acc = torch.zeros(shape, device=device, dtype=torch.float32)
    for _ in range(3):
        z = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
        acc.addcmul_(z, z)
    k = (z0 / torch.sqrt(acc / 3.0)).to(torch.float16)
    del z0, acc, z
    v = torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(torch.float16)
    return k, v
