"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of
the oracle's own code.  None of these need a GPU."""
import math
import os

import numpy as np
import pytest
import scipy.special

import oracle
from oracle import quantizer as qz
from oracle.attention import Tolerances, certified_head, key_term, softmax_attention

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_worked_numbers.txt")


def golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, val, dec = line.split()
            out[name] = (float(val), int(dec))
    return out


def rnd(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float16)


# --------------------------------------------------------------------------- quantizers

def test_key_quantizer_integer_grid_is_exact():
    # a channel that holds integers spanning exactly [-128, 127] has sigma=1, z=0, code=k
    k = np.zeros((16, 4), dtype=np.float16)
    k[:, 0] = [-128, 127, 0, 1, -1, 5, 77, -90, 100, -100, 64, -64, 3, 2, 126, -127]
    k[:, 1] = 2.5                                   # constant channel
    k[:, 2] = np.linspace(-1, 1, 16)
    k[:, 3] = [0, 255] + [17] * 14                  # min 0, max 255 -> sigma 1, z 128
    codes, sigma, z = qz.quantize_key_blocks(k)
    assert sigma[0] == 1.0 and z[0] == 0.0
    assert (codes[:, 0] == k[:, 0].astype(np.int64)).all()
    assert sigma[1] == 0.0 and z[1] == 2.5 and (codes[:, 1] == 0).all()
    assert sigma[3] == 1.0 and z[3] == 128.0
    assert codes[0, 3] == -128 and codes[1, 3] == 127 and codes[2, 3] == 17 - 128
    k_hat = qz.dequantize_keys(codes, sigma, z)
    assert (k_hat[:, [0, 1, 3]] == k[:, [0, 1, 3]].astype(np.float64)).all()


@pytest.mark.parametrize("seed,scale", [(0, 1.0), (1, 20.0), (2, 1e-3), (3, 300.0)])
def test_key_quantizer_bound_and_no_clipping(seed, scale):
    k = rnd((50, 16, 128), seed, scale)
    codes, sigma, z = qz.quantize_key_blocks(k)
    k_hat = qz.dequantize_keys(codes, sigma, z)
    err = np.abs(k_hat - k.astype(np.float64))
    half = sigma.astype(np.float64)[:, None, :] / 2
    # reconstruction bound |k - k_hat| <= sigma/2, up to the float32 rounding of z and the quotient
    assert (err <= half * (1 + 2.0 ** -6) + 1e-12).all()
    assert np.median(err / np.maximum(half, 1e-30)) < 0.6
    # the fitted extremes map to the ends of the code range (no clipping of fitted data)
    k32 = k.astype(np.float32)
    amin = k32.argmin(axis=1)
    amax = k32.argmax(axis=1)
    cmin = np.take_along_axis(codes, amin[:, None, :], axis=1)[:, 0]
    cmax = np.take_along_axis(codes, amax[:, None, :], axis=1)[:, 0]
    assert (cmin <= -127).all() and (cmax >= 126).all()
    assert codes.min() >= -128 and codes.max() <= 127


def test_key_quantizer_independent_scalar_recompute():
    # python-float recomputation with struct-packed float32 rounding after every operation
    import struct

    def f32(x):
        return struct.unpack("f", struct.pack("f", x))[0]

    k = rnd((16, 3), 7)
    codes, sigma, z = qz.quantize_key_blocks(k)
    for c in range(3):
        col = [float(x) for x in k[:, c]]
        lo, hi = min(col), max(col)
        s = f32(f32(hi - lo) / 255.0)
        zz = f32(lo + f32(128.0 * s))
        assert s == float(sigma[c]) and zz == float(z[c])
        for t in range(16):
            quo = f32(f32(col[t] - zz) / s)
            r = round(quo)                          # python round() is half-to-even
            assert max(-128, min(127, r)) == int(codes[t, c])


def test_value_quantizer_grid_aligned_is_exact():
    # a group holding offset + {0..15} * 2^e has scale 2^e and zero reconstruction error
    v = np.zeros((16, 128), dtype=np.float16)
    for t in range(16):
        for g in range(8):
            e = 2.0 ** (g - 5)
            vals = (np.arange(16) * e + (t - 8) * e * 4).astype(np.float16)
            v[t, g * 16:(g + 1) * 16] = np.roll(vals, t + g)
    codes, scale, off = qz.quantize_values(v)
    for g in range(8):
        assert (scale[:, g].astype(np.float64) == 2.0 ** (g - 5)).all()
    v_hat = qz.dequantize_values(codes, scale, off)
    assert (v_hat == v.astype(np.float64)).all()
    eta, nu = qz.block_annotations(v[None], v_hat[None])
    assert eta[0] == 0.0
    assert nu[0] == np.float32(np.sqrt((v.astype(np.float64) ** 2).sum(-1)).max())
    assert set(np.unique(codes)) == set(range(16))


def test_value_quantizer_error_bound_and_typical_size():
    v = rnd((4096, 128), 11)
    codes, scale, off = qz.quantize_values(v)
    assert codes.max() == 15 and codes.min() == 0
    v_hat = qz.dequantize_values(codes, scale, off)
    err = np.abs(v_hat - v.astype(np.float64)).reshape(4096, 8, 16)
    s = scale.astype(np.float64)[..., None]
    # half a step, plus the drift of the FP16-rounded scale over 15 steps
    assert (err <= s / 2 * (1 + 2 ** -8) + 15 * s * 2.0 ** -11).all()
    rel = np.sqrt(((v_hat - v.astype(np.float64)) ** 2).sum()) / np.sqrt((v.astype(np.float64) ** 2).sum())
    # 4-bit, g=16 on Gaussian values: a few percent relative error (the paper quotes ~5 %)
    assert 0.04 < rel < 0.09
    # uniform-noise model: per-element rms error ~ step / sqrt(12)
    rms = np.sqrt((err ** 2).mean())
    assert abs(rms / (scale.astype(np.float64).mean() / math.sqrt(12)) - 1) < 0.1


def test_value_quantizer_degenerate_groups():
    v = np.zeros((2, 32), dtype=np.float16)
    v[0, :16] = 3.0                                   # constant group
    v[0, 16:] = np.float16(6e-8) * (np.arange(16) % 2)  # range far below an FP16 step of 15ths
    v[1] = np.linspace(-2, 2, 32)
    codes, scale, off = qz.quantize_values(v)
    assert scale[0, 0] == 0 and (codes[0, :16] == 0).all() and off[0, 0] == 3.0
    assert scale[0, 1] == 0 and (codes[0, 16:] == 0).all()
    v_hat = qz.dequantize_values(codes, scale, off)
    assert (v_hat[0, :16] == 3.0).all()


def test_nibble_packing_roundtrip_and_order():
    codes = np.arange(32, dtype=np.uint8).reshape(2, 16) % 16
    packed = qz.pack_nibbles(codes)
    assert packed.shape == (2, 8)
    assert packed[0, 0] == (0 | (1 << 4)) and packed[0, 7] == (14 | (15 << 4))
    assert (qz.unpack_nibbles(packed) == codes).all()


def test_storage_arithmetic_matches_paper_table():
    g = golden()
    b = qz.tier1_bytes_per_token()
    assert b["k_codes"] == g["k_codes_bytes"][0]
    assert b["k_meta"] == g["k_meta_bytes"][0]
    assert b["v_codes"] == g["v_codes_bytes"][0]
    assert b["v_meta"] == g["v_meta_bytes"][0]
    total = b["k_codes"] + b["k_meta"] + b["v_codes"] + b["v_meta"]
    assert total == g["tier1_bytes_total"][0]
    assert b["eta"] < 1 and b["nu"] < 1
    assert round(total / g["fp16_bytes_total"][0], 2) == g["tier1_fraction_of_fp16"][0]
    assert (b["k_codes"] + b["k_meta"]) / 256 == g["key_side_fraction"][0]
    assert (b["v_codes"] + b["v_meta"]) / 256 == g["value_side_fraction"][0]
    staging = 2 * 131072 * 128 * 8 * 2 / 2 ** 30
    assert round(staging, 1) == g["rung4_staging_gb"][0]


# --------------------------------------------------------------------------- worked numbers

def test_worked_numbers_from_the_paper():
    g = golden()
    d = 0.18
    assert round(math.exp(2 * d), 2) == g["exp_2delta_at_0.18"][0]
    assert round(math.exp(3 * d), 2) == g["exp_3delta_at_0.18"][0]
    assert round(math.expm1(2 * d), 2) == g["expm1_2delta_at_0.18"][0]
    tight = key_term(d, 0.005, 1.0, mass_exp=2, mode=1)
    impl = key_term(d, 0.005, 1.0, mass_exp=3, mode=1)
    assert round(tight, 3) == g["ekey_over_vmax_tight"][0]
    assert round(impl, 3) == g["ekey_over_vmax_impl"][0]
    assert abs(tight - 0.006211) < 5e-7 and abs(impl - 0.007436) < 5e-7
    assert abs(impl / tight - math.exp(d)) < 1e-12
    # mode 2 is the full-sequence lemma, mode 0 the smaller of the two
    assert key_term(d, 1.0, 3.0, 2, 2) == 2 * 3.0 * math.tanh(d)
    assert key_term(d, 0.005, 1.0, 2, 0) == tight
    assert key_term(d, 1.0, 1.0, 2, 0) == 2 * math.tanh(d)
    # overflow-safe for saturated Delta
    assert key_term(500.0, 1.0, 2.0, 2, 0) == 4.0
    assert key_term(0.0, 1.0, 2.0, 2, 0) == 0.0
    # the tail form with a large Delta: exact below the binary32 range of the certificate
    # (2 V_max (e^{2 Delta} - 1) once the mass factor has saturated at 1), +inf beyond it
    assert key_term(42.0, 0.5, 3.0, 2, 1) == pytest.approx(6.0 * math.expm1(84.0), rel=1e-12)
    assert key_term(42.0, 1e-40, 3.0, 2, 1) == pytest.approx(6.0 * math.exp(84.0) * 1e-40 * math.expm1(84.0), rel=1e-12)
    assert key_term(50.0, 0.5, 3.0, 2, 1) == math.inf
    assert key_term(400.0, 0.5, 3.0, 2, 1) == math.inf
    assert key_term(400.0, 0.5, 3.0, 2, 0) == 6.0        # the default mode still takes the tanh form


# --------------------------------------------------------------------------- attention + certificate

def build_case(seed, n, d=128, q_scale=1.0, k_scale=1.0, trail=0, adversarial=False):
    rng = np.random.default_rng(seed)
    k16 = (rng.standard_normal((n + trail, d)) * k_scale).astype(np.float16)
    v16 = rng.standard_normal((n + trail, d)).astype(np.float16)
    nb = n // 16
    codes, sigma, z = qz.quantize_key_blocks(k16[:n].reshape(nb, 16, d))
    k_hat = qz.dequantize_keys(codes, sigma, z).reshape(n, d)
    vc, vs, vo = qz.quantize_values(v16[:n])
    v_hat = qz.dequantize_values(vc, vs, vo)
    eta, nu = qz.block_annotations(v16[:n].reshape(nb, 16, d), v_hat.reshape(nb, 16, d))
    if adversarial:
        # query aligned with the sign pattern of the first block's rounding errors, scaled up
        e = (k_hat[:16] - k16[:16].astype(np.float64))[3]
        q16 = (np.sign(e) * q_scale).astype(np.float16)
    else:
        q16 = (rng.standard_normal(d) * q_scale).astype(np.float16)
    return dict(q16=q16, k16=k16, v16=v16, k_hat=k_hat, v_hat=v_hat, sigma=sigma, eta=eta, nu=nu,
                n=n, trail=trail)


def run_case(c, tol=None):
    n = c["n"]
    return certified_head(c["q16"], c["k_hat"], c["v_hat"], c["sigma"], c["eta"], c["nu"],
                          c["k16"][n:], c["v16"][n:], tol or Tolerances())


def test_key_term_beyond_binary32_raises_precond():
    """A head whose tail-form key term leaves the binary32 range reports +inf and PRECOND."""
    c = build_case(3, 64, k_scale=900.0)
    res = run_case(c, Tolerances(key_bound_mode=1))
    assert res["delta_h"] > 45.0
    assert res["E_key"] == math.inf and res["flags"] & 8
    res0 = run_case(c, Tolerances(key_bound_mode=0))
    assert math.isfinite(res0["E_key"]) and not res0["flags"] & 8


@pytest.mark.parametrize("seed,n,trail,q_scale,k_scale,adv", [
    (0, 64, 0, 1.0, 1.0, False), (1, 64, 5, 1.0, 1.0, False), (2, 48, 15, 3.0, 1.0, False),
    (3, 32, 1, 1.0, 8.0, False), (4, 64, 0, 4.0, 1.0, True), (5, 16, 7, 2.0, 3.0, True),
    (6, 256, 3, 0.3, 1.0, False), (7, 64, 0, 6.0, 4.0, True),
])
def test_total_bound_and_every_link_of_the_chain(seed, n, trail, q_scale, k_scale, adv):
    c = build_case(seed, n, q_scale=q_scale, k_scale=k_scale, trail=trail, adversarial=adv)
    r = run_case(c)
    q = c["q16"].astype(np.float64)
    K = c["k16"].astype(np.float64)
    V = c["v16"].astype(np.float64)
    d = q.shape[0]
    # independent recomputation with library softmax (not the oracle's own formula)
    s_ref = K @ q / math.sqrt(d)
    a = scipy.special.softmax(s_ref)
    o_ref = a @ V
    k_mix = np.concatenate([c["k_hat"], K[n:]])
    v_mix = np.concatenate([c["v_hat"], V[n:]])
    s_q = k_mix @ q / math.sqrt(d)
    a_q = scipy.special.softmax(s_q)
    # naive special case: all certification off == textbook attention on (K_hat, V_hat)
    assert np.allclose(r["O"], a_q @ v_mix, rtol=1e-12, atol=1e-14)
    assert abs(r["weights"].sum() - 1) < 1e-12
    assert abs(r["lse"] - scipy.special.logsumexp(s_q)) < 1e-10
    # contract: measured error within the two-term bound
    err = np.linalg.norm(r["O"] - o_ref)
    assert err <= r["E_key"] + r["E_val"]
    # value chain: ||sum a'(V_hat - V)|| <= sum_b rho_b eta_b <= max_b eta_b
    e_val_meas = np.linalg.norm(a_q @ (v_mix - V))
    assert e_val_meas <= r["E_val"] * (1 + 1e-6) + 1e-12
    assert r["E_val"] <= float(c["eta"].max()) * (1 + 1e-12)
    assert r["max_block_contrib"] <= r["E_val"] + 1e-15
    # key chain: ||sum (a'-a) V|| <= 2 V_max TV <= E_key, and TV <= tanh(Delta_h)
    tv = 0.5 * np.abs(a - a_q).sum()
    e_key_meas = np.linalg.norm((a_q - a) @ V)
    v_max = np.linalg.norm(V, axis=1).max()
    assert abs(r["v_max"] - np.float32(v_max)) <= 1e-6 * v_max
    assert e_key_meas <= 2 * r["v_max"] * tv * (1 + 1e-6) + 1e-12
    assert 2 * r["v_max"] * tv <= r["E_key"] * (1 + 1e-9) + 1e-15
    assert tv <= math.tanh(r["delta_h"]) + 1e-15
    # score perturbation within Delta_b (tight L1 form) <= Cauchy-Schwarz form
    sig = c["sigma"].astype(np.float64)
    delta_b = (np.abs(q)[None] * sig).sum(1) / (2 * math.sqrt(d))
    cs = np.linalg.norm(q) * np.linalg.norm(sig, axis=1) / (2 * math.sqrt(d))
    assert (delta_b <= cs + 1e-15).all()
    assert abs(r["delta_h"] - delta_b.max()) < 1e-12
    ds = np.abs(s_q - s_ref)[:n].reshape(-1, 16).max(1)
    assert (ds <= delta_b * (1 + 2.0 ** -6) + 1e-12).all()
    assert (np.abs(s_q - s_ref)[n:] == 0).all()
    # probability-ratio lemma and the normalised tail implication for random token subsets
    ratio = a_q / a
    dh = r["delta_h"] * (1 + 2.0 ** -6)
    assert ratio.max() <= math.exp(2 * dh) and ratio.min() >= math.exp(-2 * dh)
    rng = np.random.default_rng(seed + 100)
    for _ in range(8):
        sub = rng.random(a.shape[0]) < 0.3
        assert a[sub].sum() <= math.exp(2 * dh) * a_q[sub].sum() + 1e-15
    # block masses: sum_b rho_b + trailing mass = 1 and l_b is the block log-sum-exp
    rho = np.exp(r["blk_logmass"] - r["lse"])
    assert abs(rho.sum() + a_q[n:].sum() - 1) < 1e-12
    assert abs(r["alpha_tail_hat"] - rho.sum()) < 1e-12
    lb = scipy.special.logsumexp(s_q[:n].reshape(-1, 16), axis=1)
    assert np.allclose(r["blk_logmass"], lb, atol=1e-10)
    top = int(np.argmax(lb))
    assert r["top_block"] == top
    if n >= 32:
        assert abs(r["rank_margin"] - (lb[top] - np.delete(lb, top).max())) < 1e-10


def test_uniform_scale_special_case():
    # sigma_c = delta for every channel: the Cauchy-Schwarz form reduces to ||q|| delta / 2
    d = 128
    q = rnd((d,), 3).astype(np.float64)
    delta = 0.03
    sig = np.full(d, delta)
    cs = np.linalg.norm(q) * np.linalg.norm(sig) / (2 * math.sqrt(d))
    assert abs(cs - np.linalg.norm(q) * delta / 2) < 1e-15


def test_exactly_representable_cache_gives_zero_bounds_and_exact_output():
    # channel-constant key blocks (sigma = 0) and grid-aligned values (eta = 0)
    d, nb = 128, 6
    rng = np.random.default_rng(5)
    k16 = np.repeat(rng.standard_normal((nb, 1, d)).astype(np.float16), 16, axis=1).reshape(nb * 16, d)
    base = (rng.integers(0, 16, size=(nb * 16, d)) * 0.25 - 2.0).astype(np.float16)
    base[:, 0::16] = -2.0
    base[:, 1::16] = 1.75                    # every group spans the full 0..15 grid
    v16 = base
    codes, sigma, z = qz.quantize_key_blocks(k16.reshape(nb, 16, d))
    assert (sigma == 0).all()
    k_hat = qz.dequantize_keys(codes, sigma, z).reshape(-1, d)
    vc, vs, vo = qz.quantize_values(v16)
    v_hat = qz.dequantize_values(vc, vs, vo)
    eta, nu = qz.block_annotations(v16.reshape(nb, 16, d), v_hat.reshape(nb, 16, d))
    assert (eta == 0).all()
    q16 = rnd((d,), 9)
    r = certified_head(q16, k_hat, v_hat, sigma, eta, nu, k16[:0], v16[:0], Tolerances())
    assert r["E_key"] == 0.0 and r["E_val"] == 0.0 and r["delta_h"] == 0.0
    assert (k_hat == k16.astype(np.float64)).all() and (v_hat == v16.astype(np.float64)).all()
    o_ref = softmax_attention(q16, k16, v16)
    assert np.allclose(r["O"], o_ref, rtol=1e-14, atol=1e-15)   # same inputs; rounding order only


def test_tv_lemmas_on_random_perturbations():
    rng = np.random.default_rng(0)
    for trial in range(200):
        n = int(rng.integers(2, 40))
        delta = float(rng.uniform(0.01, 2.0))
        s = rng.standard_normal(n) * rng.uniform(0.1, 5)
        pert = rng.uniform(-delta, delta, n)
        if trial % 3 == 0:
            pert = np.where(rng.random(n) < 0.5, delta, -delta)
        a = scipy.special.softmax(s)
        # full-sequence lemma
        tv = 0.5 * np.abs(a - scipy.special.softmax(s + pert)).sum()
        assert tv <= math.tanh(delta) + 1e-15
        # tail-restricted lemma: an exact set F and a perturbed tail T of true mass alpha_T
        tail = rng.random(n) < 0.5
        a2 = scipy.special.softmax(s + np.where(tail, pert, 0.0))
        tv2 = 0.5 * np.abs(a - a2).sum()
        alpha_true = a[tail].sum()
        assert tv2 <= alpha_true * math.expm1(2 * delta) + 1e-15
        # the oracle's key term covers it when fed the INT8-estimated tail mass
        alpha_hat = a2[tail].sum()
        assert 2 * tv2 <= key_term(delta, alpha_hat, 1.0, 2, 1) + 1e-15
        assert 2 * tv2 <= key_term(delta, alpha_hat, 1.0, 2, 0) + 1e-15
        assert key_term(delta, alpha_hat, 1.0, 2, 1) <= key_term(delta, alpha_hat, 1.0, 3, 1)


def test_flags_and_thresholds():
    c = build_case(21, 64, trail=3)
    base = run_case(c)
    assert base["flags"] == 0
    mid = lambda x: (x * 0.5, x * 2.0)
    lo, hi = mid(base["E_key"])
    assert run_case(c, Tolerances(eps_key=lo))["flags"] == oracle.FLAG_KEY
    assert run_case(c, Tolerances(eps_key=hi))["flags"] == 0
    lo, hi = mid(base["E_val"])
    assert run_case(c, Tolerances(eps_val=lo))["flags"] == oracle.FLAG_VAL
    assert run_case(c, Tolerances(eps_val=hi))["flags"] == 0
    lo, hi = mid(base["max_block_contrib"])
    assert run_case(c, Tolerances(v_tol=lo))["flags"] == oracle.FLAG_VAL
    assert run_case(c, Tolerances(v_tol=hi))["flags"] == 0
    lo, hi = mid(base["E_key"] + base["E_val"])
    assert run_case(c, Tolerances(eps_total=lo))["flags"] == oracle.FLAG_TOTAL
    assert run_case(c, Tolerances(eps_total=hi))["flags"] == 0
    assert run_case(c, Tolerances(force_flags=oracle.FLAG_RANK))["flags"] == oracle.FLAG_RANK
    # diffuse head: top-2 block log-masses are closer than 2 Delta_h -> RANK fires when unconditional
    assert base["rank_margin"] < 2 * base["delta_h"]
    assert run_case(c, Tolerances(rank_depth=1))["flags"] == oracle.FLAG_RANK
    assert run_case(c, Tolerances(rank_depth=1, rank_min_mass=0.9))["flags"] == 0
    assert run_case(c, Tolerances(rank_depth=0))["flags"] == 0


def test_rank_check_passes_for_a_clearly_peaked_head():
    c = build_case(22, 64)
    k = c["k16"].astype(np.float64)
    c["q16"] = (k[37] * 1.5).astype(np.float16)
    r = run_case(c, Tolerances(rank_depth=1))
    assert r["top_block"] == 37 // 16
    assert r["rank_margin"] > 2 * r["delta_h"] + 1e-6
    assert r["flags"] == 0


# --------------------------------------------------------------------------- cache + ladder

def test_cache_sealing_is_block_local_and_immutable():
    rng = np.random.default_rng(1)
    bt, hkv, d = 2, 2, 128
    k = rng.standard_normal((bt, hkv, 53, d)).astype(np.float16)
    v = rng.standard_normal((bt, hkv, 53, d)).astype(np.float16)
    one = oracle.OracleLayerCache(bt, hkv)
    one.append(k, v)
    inc = oracle.OracleLayerCache(bt, hkv)
    for lo, hi in [(0, 1), (1, 16), (16, 17), (17, 40), (40, 53)]:
        inc.append(k[:, :, lo:hi], v[:, :, lo:hi])
    assert one.n_blocks == inc.n_blocks == 3 and one.length == 53
    for name in ("k_codes", "sigma", "z", "v_codes", "v_scale", "v_offset", "eta", "nu"):
        assert (getattr(one, name) == getattr(inc, name)).all(), name
    # block 1's metadata depends on its own 16 tokens only
    codes, sigma, z = qz.quantize_key_blocks(k[0, 1, 16:32])
    assert (one.sigma[0, 1, 1] == sigma).all() and (one.k_codes[0, 1, 1] == codes).all()


def test_ladder_forced_fallback_returns_dense_exactly():
    rng = np.random.default_rng(2)
    bt, hkv, hq, d = 1, 2, 8, 128
    k = rng.standard_normal((bt, hkv, 70, d)).astype(np.float16)
    v = rng.standard_normal((bt, hkv, 70, d)).astype(np.float16)
    q = rng.standard_normal((bt, hq, d)).astype(np.float16)
    c = oracle.OracleLayerCache(bt, hkv)
    c.append(k, v)
    plain = c.decode_step(q, Tolerances())
    assert all(r["served_rung"] == 0 and r["flags"] == 0 for r in plain)
    forced = c.decode_step(q, Tolerances(force_flags=oracle.FLAG_TOTAL))
    for i, r in enumerate(forced):
        dense = scipy.special.softmax(k[0, i // 4].astype(np.float64) @ q[0, i].astype(np.float64)
                                      / math.sqrt(d)) @ v[0, i // 4].astype(np.float64)
        assert np.allclose(r["O"], dense, rtol=1e-12, atol=1e-14)
        assert r["E_key"] == 0.0 and r["E_val"] == 0.0 and r["served_rung"] == 3
        assert r["flags"] == oracle.FLAG_TOTAL | (3 << oracle.RUNG_SHIFT)
    # only the flagged heads are recomputed by Rung 3
    tot = sorted(r["E_key"] + r["E_val"] for r in plain)
    eps = 0.5 * (tot[-2] + tot[-1])
    some = c.decode_step(q, Tolerances(eps_total=eps))
    assert sum(r["served_rung"] == 3 for r in some) == 1
    for r0, r1 in zip(plain, some):
        if r1["served_rung"] == 0:
            assert (r0["O"] == r1["O"]).all() and r1["E_key"] == r0["E_key"]
    # Rung 4 when enough groups are flagged, or on a precondition flag
    all4 = c.decode_step(q, Tolerances(eps_total=eps, rung4_min_groups=1))
    assert all(r["served_rung"] == 4 for r in all4)
    pre = c.decode_step(q, Tolerances(force_flags=oracle.FLAG_PRECOND))
    assert all(r["served_rung"] == 4 for r in pre)
    no_t2 = oracle.OracleLayerCache(bt, hkv, tier2=False)
    no_t2.append(k, v)
    with pytest.raises(RuntimeError):
        no_t2.decode_step(q, Tolerances(force_flags=oracle.FLAG_TOTAL))


def test_ladder_decision_table():
    f = [0] * 8
    assert oracle.ladder_decision(f, 1, 8, 4, 0) == 0
    f[5] = oracle.FLAG_VAL
    assert oracle.ladder_decision(f, 1, 8, 4, 0) == 3
    assert oracle.ladder_decision(f, 1, 8, 4, 2) == 3
    f[1] = oracle.FLAG_KEY
    assert oracle.ladder_decision(f, 1, 8, 4, 2) == 4
    f[1] = 0
    f[6] = oracle.FLAG_KEY          # same KV group as head 5
    assert oracle.ladder_decision(f, 1, 8, 4, 2) == 3
    f[6] = oracle.FLAG_PRECOND
    assert oracle.ladder_decision(f, 1, 8, 4, 0) == 4
