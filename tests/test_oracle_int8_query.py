"""Pins of the oracle's INT8 x INT8 scoring mode (quantised scaled query, the paper's optional
tensor-core scoring in "Per-Channel Key Scoring") and of the explicit third error term that this
build adds to the block score bound.  None of these re-evaluates the oracle's own formula: they
check it against brute force over tokens, closed special cases, the quantiser's own guarantees
and the end-to-end bound.
"""
import math
import struct

import numpy as np
import pytest
import scipy.special

from oracle import quantizer as qz
from oracle.attention import Tolerances, certified_head, quantize_scaled_query


def f32(x):
    """Rounds a Python float to binary32 through struct (independent of numpy's casts)."""
    return struct.unpack("f", struct.pack("f", x))[0]


def build(seed, n, trail=0, q_scale=1.0, k_scale=1.0, outlier=False):
    rng = np.random.default_rng(seed)
    d = 128
    k16 = (rng.standard_normal((n + trail, d)) * k_scale).astype(np.float16)
    if outlier:
        k16[:, 5] *= np.float16(20.0)
        k16[:, 77] *= np.float16(20.0)
    v16 = rng.standard_normal((n + trail, d)).astype(np.float16)
    q16 = (rng.standard_normal(d) * q_scale).astype(np.float16)
    nb = n // 16
    codes, sigma, z = qz.quantize_key_blocks(k16[:n].reshape(nb, 16, d))
    k_hat = qz.dequantize_keys(codes, sigma, z).reshape(n, d)
    vc, vs, vo = qz.quantize_values(v16[:n])
    v_hat = qz.dequantize_values(vc, vs, vo)
    eta, nu = qz.block_annotations(v16[:n].reshape(nb, 16, d), v_hat.reshape(nb, 16, d))
    return dict(q16=q16, k16=k16, v16=v16, codes=codes, sigma=sigma, z=z, k_hat=k_hat, v_hat=v_hat,
                eta=eta, nu=nu, n=n)


def run(c, tol):
    n = c["n"]
    return certified_head(c["q16"], c["k_hat"], c["v_hat"], c["sigma"], c["eta"], c["nu"], c["k16"][n:],
                          c["v16"][n:], tol, k_codes=c["codes"], z=c["z"])


@pytest.mark.parametrize("seed", range(6))
def test_query_quantiser_guarantees_and_scalar_recomputation(seed):
    c = build(seed, 64, q_scale=1.0 + seed, outlier=seed % 2 == 1)
    t, s_q = quantize_scaled_query(c["q16"], c["sigma"])
    assert t.dtype == np.int8 and np.abs(t.astype(int)).max() <= 127
    qt = c["q16"].astype(np.float64)[None, :] * c["sigma"].astype(np.float64)
    for b in range(t.shape[0]):
        # the largest element of the block maps to +-127, everything lies within half a step
        cmax = int(np.argmax(np.abs(qt[b])))
        assert abs(int(t[b, cmax])) == 127
        step = float(s_q[b])
        assert np.abs(qt[b] - step * t[b]).max() <= 0.5 * step * (1 + 1e-5) + 1e-12
        # scalar binary32 recomputation of three channels, rounding through struct
        amax = max(abs(f32(float(c["q16"][ch]) * float(c["sigma"][b, ch]))) for ch in range(128))
        assert f32(amax / 127.0) == float(s_q[b])
        inv = f32(127.0 / amax)
        for ch in (0, cmax, 127):
            prod = f32(float(c["q16"][ch]) * float(c["sigma"][b, ch])) * inv     # exact in binary64
            lo = math.floor(prod)
            want = lo if prod - lo < 0.5 else lo + 1
            if prod - lo == 0.5:
                want = lo if lo % 2 == 0 else lo + 1
            assert int(t[b, ch]) == want


def test_query_already_on_the_grid_changes_nothing():
    """q~ = (integers in [-127, 127]) x a power of two, with +-127 present: the quantiser is exact,
    the third term vanishes and the scores are those of the unquantised query."""
    rng = np.random.default_rng(11)
    d, n = 128, 48
    c = build(3, n)
    sig = np.full((n // 16, d), 0.25, dtype=np.float32)
    ints = rng.integers(-127, 128, d)
    ints[7], ints[90] = 127, -127
    q16 = (ints * 0.5).astype(np.float16)                    # exact in FP16
    c = dict(c, q16=q16, sigma=sig)
    c["k_hat"] = qz.dequantize_keys(c["codes"], sig, c["z"]).reshape(n, d)
    t, s_q = quantize_scaled_query(q16, sig)
    assert (t == ints[None, :]).all() and (s_q == np.float32(0.125)).all()
    r8 = run(c, Tolerances(int8_query=True))
    r0 = run(c, Tolerances())
    assert (r8["delta_q"] == 0).all() and r8["delta_h"] == r0["delta_h"]
    assert np.allclose(r8["scores_sealed"], r0["scores_sealed"], rtol=1e-13, atol=1e-13)
    assert np.allclose(r8["O"], r0["O"], rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("seed,q_scale,k_scale,outlier", [(0, 1.0, 1.0, False), (1, 3.0, 1.0, True),
                                                          (2, 0.3, 4.0, False), (3, 6.0, 2.0, True),
                                                          (4, 1.0, 1.0, True)])
def test_scores_by_brute_force_and_the_third_error_term(seed, q_scale, k_scale, outlier):
    c = build(seed, 80, trail=5, q_scale=q_scale, k_scale=k_scale, outlier=outlier)
    r8 = run(c, Tolerances(int8_query=True))
    r0 = run(c, Tolerances())
    t, s_q = quantize_scaled_query(c["q16"], c["sigma"])
    q = c["q16"].astype(np.float64)
    d = 128
    # brute force, token by token, channel by channel
    for tok in (0, 17, 33, 79):
        b = tok // 16
        acc = 0
        for ch in range(d):
            acc += int(t[b, ch]) * int(c["codes"][b, tok % 16, ch])
        cz = sum(float(q[ch]) * float(c["z"][b, ch]) for ch in range(d))
        assert abs(r8["scores_sealed"][tok] - (float(s_q[b]) * acc + cz) / math.sqrt(d)) < 1e-10
    # the third term bounds the distance to the scores of the unquantised scaled query, block by
    # block, and is itself at most 64 sqrt(d) s_q
    diff = np.abs(r8["scores_sealed"] - r0["scores_sealed"]).reshape(-1, 16).max(axis=1)
    assert (diff <= r8["delta_q"] * (1 + 1e-9) + 1e-12).all()
    assert (diff > 0).any()
    assert (r8["delta_q"] <= 64 * math.sqrt(d) * s_q.astype(np.float64) * (1 + 1e-6)).all()
    # and against the TRUE scores (FP16 keys): Delta_b + Delta^q_b
    s_true = c["k16"][:80].astype(np.float64) @ q / math.sqrt(d)
    delta_b = (np.abs(q)[None] * c["sigma"].astype(np.float64)).sum(1) / (2 * math.sqrt(d))
    err = np.abs(r8["scores_sealed"] - s_true).reshape(-1, 16).max(axis=1)
    assert (err <= (delta_b + r8["delta_q"]) * (1 + 2.0 ** -6) + 1e-12).all()
    assert abs(r8["delta_h"] - (delta_b + r8["delta_q"]).max()) < 1e-12
    assert r8["delta_h"] > r0["delta_h"]


@pytest.mark.parametrize("seed,n,trail,q_scale,k_scale", [(0, 64, 0, 1.0, 1.0), (1, 48, 7, 3.0, 1.0),
                                                          (2, 32, 1, 1.0, 6.0), (3, 256, 3, 0.5, 1.0),
                                                          (4, 16, 15, 5.0, 3.0)])
def test_total_bound_holds_with_the_quantised_query(seed, n, trail, q_scale, k_scale):
    c = build(seed + 40, n, trail=trail, q_scale=q_scale, k_scale=k_scale, outlier=seed % 2 == 0)
    q = c["q16"].astype(np.float64)
    K = c["k16"].astype(np.float64)
    V = c["v16"].astype(np.float64)
    a = scipy.special.softmax(K @ q / math.sqrt(128))
    o_ref = a @ V
    for mass_exp in (2, 3):
        for mode in (0, 1):
            r = run(c, Tolerances(int8_query=True, mass_exp=mass_exp, key_bound_mode=mode))
            assert np.linalg.norm(r["O"] - o_ref) <= r["E_key"] + r["E_val"]
            tv = 0.5 * np.abs(a - r["weights"]).sum()
            assert 2 * r["v_max"] * tv <= r["E_key"] * (1 + 1e-9) + 1e-15
            assert tv <= math.tanh(r["delta_h"]) + 1e-15
    # softmax consistency of the quantised-query scores
    r = run(c, Tolerances(int8_query=True))
    s_all = np.concatenate([r["scores_sealed"], K[n:] @ q / math.sqrt(128)])
    assert np.allclose(r["weights"], scipy.special.softmax(s_all), rtol=1e-12, atol=1e-16)
    assert abs(r["lse"] - scipy.special.logsumexp(s_all)) < 1e-10


# ---------------------------------------------------------------- the adaptive path in this mode

def _small_cache(seed, n_tokens=300, scale=1.0, outlier=False):
    import oracle
    rng = np.random.Generator(np.random.Philox(seed))
    k = (rng.standard_normal((1, 1, n_tokens, 128)) * scale).astype(np.float32)
    if outlier:
        k[..., 5] *= 20.0
    v = rng.standard_normal((1, 1, n_tokens, 128)).astype(np.float32)
    q = (rng.standard_normal((1, 4, 128)) * 1.5).astype(np.float16)
    oc = oracle.OracleLayerCache(1, 1)
    oc.append(k.astype(np.float16), v.astype(np.float16))
    return oc, q


@pytest.mark.parametrize("seed,scale,outlier", [(0, 1.0, False), (1, 2.5, True), (2, 0.6, False), (3, 4.0, True)])
def test_adaptive_path_with_the_quantised_query(seed, scale, outlier):
    """Adaptive precision on top of quantised-query scoring.  Special cases that reduce to known
    results (nothing promoted = the one-pass result of the mode; everything promoted = textbook
    attention on the FP16 keys), token-level brute force of the mixed scores, the tail theorem
    with the widened Delta_h and the end-to-end bound against dense attention on the originals."""
    from oracle import adaptive as ad
    oc, q = _small_cache(100 + seed, n_tokens=16 * 18 + 11, scale=scale, outlier=outlier)
    nb = oc.n_blocks
    K = oc.k16[0, 0].astype(np.float64)
    V = oc.v16[0, 0].astype(np.float64)
    tol8 = Tolerances(int8_query=True, key_bound_mode=1, rank_depth=1)
    one_pass = oc.certified_decode(q, Tolerances(int8_query=True, key_bound_mode=1))
    # (i) nothing promoted: the one-pass result of the mode, bit for bit in the oracle's arithmetic
    none = ad.adaptive_decode(oc, q, tol8, ad.SelectorParams(tau_cov=0.0, k_min=0, k_max=0, k_limit=0))
    for h in range(4):
        r = none[(0, h)]
        assert not r["promoted"].any()
        assert np.allclose(r["O"], one_pass[h]["O"], rtol=1e-13, atol=1e-15)
        assert abs(r["E_key"] - one_pass[h]["E_key"]) <= 1e-12 * max(1.0, one_pass[h]["E_key"])
        assert r["delta_h"] == one_pass[h]["delta_h"] and r["delta_h"] > oc.certified_decode(q, Tolerances())[h]["delta_h"]
    # (ii) everything promoted: exact keys everywhere, the quantised query no longer matters
    every = ad.adaptive_decode(oc, q, tol8, ad.SelectorParams(tau_cov=2.0, k_min=nb, k_max=nb, k_limit=nb))
    v_hat = qz.dequantize_values(oc.v_codes[0, 0], oc.v_scale[0, 0], oc.v_offset[0, 0]).reshape(nb * 16, 128)
    v_mixed = np.concatenate([v_hat, V[nb * 16:]])
    for h in range(4):
        r = every[(0, h)]
        a = scipy.special.softmax(K @ q[0, h].astype(np.float64) / math.sqrt(128))
        assert r["promoted"].all() and r["E_key"] == 0.0 and r["alpha_tail_hat"] == 0.0
        assert np.allclose(r["O"], a @ v_mixed, rtol=1e-12, atol=1e-14)
    # (iii) partial promotion
    for tau, kmax in ((0.5, 3), (0.9, 7)):
        part = ad.adaptive_decode(oc, q, tol8, ad.SelectorParams(tau_cov=tau, k_min=1, k_max=kmax, k_limit=kmax))
        for h in range(4):
            r = part[(0, h)]
            qf = q[0, h].astype(np.float64)
            sc = r["scoring"]
            prom = r["promoted"]
            assert prom.any() and not prom.all()
            # the selection was made on the quantised-query log-masses
            assert np.array_equal(sc["blk_logmass"], one_pass[h]["blk_logmass"])
            # token-level brute force: promoted tokens from the FP16 keys and the exact query, the
            # rest from integer products of the query codes and the key codes
            t, s_q = quantize_scaled_query(q[0, h], oc.sigma[0, 0])
            s = np.empty(nb * 16)
            for tok in range(nb * 16):
                b = tok // 16
                if prom[b]:
                    s[tok] = sum(float(qf[c]) * float(K[tok, c]) for c in range(128)) / math.sqrt(128)
                else:
                    acc = sum(int(t[b, c]) * int(oc.k_codes[0, 0][b, tok % 16, c]) for c in range(0, 128))
                    cz = float(oc.z[0, 0][b].astype(np.float64) @ qf)
                    s[tok] = (float(s_q[b]) * acc + cz) / math.sqrt(128)
            s_all = np.concatenate([s, K[nb * 16:] @ qf / math.sqrt(128)])
            w = scipy.special.softmax(s_all)
            assert np.allclose(r["weights"], w, rtol=1e-10, atol=1e-16)
            assert np.allclose(r["O"], w @ v_mixed, rtol=1e-10, atol=1e-13)
            # tail theorem with the widened Delta_h: the true mass of the unpromoted blocks
            a_true = scipy.special.softmax(K @ qf / math.sqrt(128))
            tail_tok = np.concatenate([np.repeat(~prom, 16), np.zeros(oc.length - nb * 16, bool)])
            assert a_true[tail_tok].sum() <= math.exp(2 * r["delta_h"]) * r["alpha_tail_hat"] * (1 + 1e-9) + 1e-15
            # key-side distortion and the total bound, against dense attention on the originals
            assert 2 * r["v_max"] * 0.5 * np.abs(a_true - r["weights"]).sum() <= r["E_key"] * (1 + 1e-9) + 1e-15
            assert np.linalg.norm(r["O"] - a_true @ V) <= r["E_key"] + r["E_val"]
            # the score-consistency figure: FP16 against quantised-query scores on promoted tokens
            dev = np.abs(s - sc["scores_sealed"])[np.repeat(prom, 16)].max()
            assert abs(r["score_dev"] - dev) < 1e-12 and r["score_dev"] <= r["delta_h"] * (1 + 2.0 ** -6) + 1e-12
