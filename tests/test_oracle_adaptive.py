"""Pins for the adaptive-precision part of the oracle: each test checks it against something
other than itself (brute force, the paper's theorem and worked numbers, textbook special cases)."""
import math

import numpy as np
import pytest

import oracle
import workloads
from oracle import adaptive as ad
from oracle import attention as att
from oracle import quantizer as qz


def small_cache(seed, n_tokens=300, scale=1.0, outlier=False):
    """One KV head with 4 query heads, a few hundred tokens (18 sealed blocks + 12 trailing)."""
    rng = np.random.Generator(np.random.Philox(seed))
    k = (rng.standard_normal((1, 1, n_tokens, 128)) * scale).astype(np.float32)
    if outlier:
        k[..., 5] *= 20.0
    v = rng.standard_normal((1, 1, n_tokens, 128)).astype(np.float32)
    q = (rng.standard_normal((1, 4, 128)) * 1.5).astype(np.float16)
    oc = oracle.OracleLayerCache(1, 1)
    oc.append(k.astype(np.float16), v.astype(np.float16))
    return oc, q


# ---------------------------------------------------------------- selector (steps 1-4)

def brute_force_k(masses, rho_trail, tau):
    """Smallest number of blocks whose masses, taken largest first, cover tau with the trailing mass."""
    best = sorted(masses, reverse=True)
    c = rho_trail
    for k in range(len(best) + 1):
        if c >= tau:
            return k
        if k < len(best):
            c += best[k]
    return len(best)


@pytest.mark.parametrize("seed", range(6))
def test_selector_is_the_minimal_cover(seed):
    rng = np.random.Generator(np.random.Philox(100 + seed))
    nb = 40
    logits = rng.standard_normal(nb) * 3.0
    rho_trail = 0.07
    masses = np.exp(logits) / np.exp(logits).sum() * (1.0 - rho_trail)
    lse = 1.234
    logmass = np.log(masses) + lse
    for tau in (0.5, 0.9, 0.995):
        sel = ad.select_blocks(logmass, lse, ad.SelectorParams(tau_cov=tau, k_min=0, k_max=nb))
        assert sel["k_star"] == brute_force_k(list(masses), rho_trail, tau)
        k = sel["k_star"]
        # the chosen blocks are the k heaviest, the tail mass is what the others hold
        chosen = set(sel["order"][:k].tolist())
        assert chosen == set(np.argsort(-masses, kind="stable")[:k].tolist())
        others = [masses[i] for i in range(nb) if i not in chosen]
        assert ad.tail_mass(sel, k) == pytest.approx(sum(others), rel=1e-12, abs=1e-15)
        assert abs(sel["rho_trail"] - rho_trail) < 1e-12
        if k < nb:
            assert ad.tail_mass(sel, k) <= 1.0 - tau + 1e-12       # target met when not clamped


def test_selector_clamps_and_ties():
    logmass = np.array([0.0, 2.0, 2.0, -1.0, 2.0, 0.5])
    lse = math.log(np.exp(logmass).sum())
    sel = ad.select_blocks(logmass, lse, ad.SelectorParams(tau_cov=0.0, k_min=2, k_max=4))
    assert sel["k_star"] == 2                                     # K_min
    assert sel["order"].tolist() == [1, 2, 4, 5, 0, 3]            # equal masses: lower index first
    sel = ad.select_blocks(logmass, lse, ad.SelectorParams(tau_cov=1.1, k_min=2, k_max=4))
    assert sel["k_star"] == 4                                     # K_max
    sel = ad.select_blocks(logmass, lse, ad.SelectorParams(tau_cov=1.1, k_min=2, k_max=100))
    assert sel["k_star"] == 6                                     # never more than the blocks there are


def test_rung1_doubles_until_the_key_term_fits():
    nb = 64
    logmass = -0.05 * np.arange(nb)
    lse = math.log(np.exp(logmass).sum())
    par = ad.SelectorParams(tau_cov=0.2, k_min=1, k_max=4, k_limit=64)
    sel = ad.select_blocks(logmass, lse, par)
    k0 = sel["k_star"]
    delta, vmax = 0.18, 10.0
    loose = att.Tolerances(eps_key=math.inf, key_bound_mode=1)
    assert ad.rung1_expand(sel, delta, vmax, loose, par) == k0
    target = att.key_term(delta, ad.tail_mass(sel, 4 * k0), vmax, 2, 1)
    tol = att.Tolerances(eps_key=target * 1.0001, key_bound_mode=1)
    assert ad.rung1_expand(sel, delta, vmax, tol, par) == 4 * k0  # two doublings, not three
    never = att.Tolerances(eps_key=0.0, key_bound_mode=1)
    assert ad.rung1_expand(sel, delta, vmax, never, par) == 64    # stops at the cap


def test_worked_operating_point():
    """tau_cov = 0.995, Delta = 0.18: tail mass 0.005 gives 0.006211 V_max (0.007436 with e^{3 Delta}),
    the numbers of the paper's tail-restricted key bound."""
    masses = np.array([0.9, 0.095, 0.003, 0.002])
    logmass = np.log(masses)
    sel = ad.select_blocks(logmass, 0.0, ad.SelectorParams(tau_cov=0.995, k_min=0, k_max=4))
    assert sel["k_star"] == 2
    alpha = ad.tail_mass(sel, 2)
    assert alpha == pytest.approx(0.005, rel=1e-12)
    assert att.key_term(0.18, alpha, 1.0, 2, 1) == pytest.approx(0.006211, abs=5e-7)
    assert att.key_term(0.18, alpha, 1.0, 3, 1) == pytest.approx(0.007436, abs=5e-7)


# ---------------------------------------------------------------- attend pass with gated key precision

@pytest.mark.parametrize("seed", range(4))
def test_special_cases_reduce_to_known_attention(seed):
    oc, q = small_cache(seed)
    nb = oc.n_blocks
    k_hat = qz.dequantize_keys(oc.k_codes[0, 0], oc.sigma[0, 0], oc.z[0, 0]).reshape(nb * 16, 128)
    v_hat = qz.dequantize_values(oc.v_codes[0, 0], oc.v_scale[0, 0], oc.v_offset[0, 0]).reshape(nb * 16, 128)
    k_tr, v_tr = oc.k16[0, 0, nb * 16:], oc.v16[0, 0, nb * 16:]
    tol = att.Tolerances()
    one_pass = att.certified_head(q[0, 1], k_hat, v_hat, oc.sigma[0, 0], oc.eta[0, 0], oc.nu[0, 0],
                                  k_tr, v_tr, tol)
    args = (q[0, 1], k_hat, oc.k16[0, 0, :nb * 16], v_hat, oc.eta[0, 0], oc.nu[0, 0], k_tr, v_tr)
    tail = (one_pass["blk_logmass"], one_pass["lse"], one_pass["delta_h"], tol)
    # nothing promoted: the one-pass result
    none = ad.mixed_head(*args, np.zeros(nb, bool), *tail)
    assert np.allclose(none["O"], one_pass["O"], rtol=0, atol=1e-14)
    for f in ("E_key", "E_val", "alpha_tail_hat", "lse", "max_block_contrib"):
        assert none[f] == pytest.approx(one_pass[f], rel=1e-12)
    # everything promoted: textbook attention over the FP16 keys and the INT4-reconstructed values
    full = ad.mixed_head(*args, np.ones(nb, bool), *tail)
    ref = att.softmax_attention(q[0, 1], oc.k16[0, 0].astype(np.float64),
                                np.concatenate([v_hat, v_tr.astype(np.float64)]))
    assert np.allclose(full["O"], ref, rtol=0, atol=1e-13)
    assert full["alpha_tail_hat"] == 0.0 and full["E_key"] == 0.0


@pytest.mark.parametrize("seed,scale,outlier", [(0, 1.0, False), (1, 1.0, True), (2, 3.0, False),
                                                (3, 0.3, True), (4, 2.0, True)])
def test_tail_theorem_and_bounds_hold(seed, scale, outlier):
    """The true (FP16-key) mass of the unpromoted blocks is at most e^{2 Delta_h} alpha_hat_T, the key
    term bounds the output change caused by the INT8 keys that remain, and key + value terms bound
    the distance to the FP16 reference."""
    oc, q = small_cache(10 + seed, scale=scale, outlier=outlier)
    nb = oc.n_blocks
    v_hat = qz.dequantize_values(oc.v_codes[0, 0], oc.v_scale[0, 0], oc.v_offset[0, 0]).reshape(nb * 16, 128)
    v_mixed_all = np.concatenate([v_hat, oc.v16[0, 0, nb * 16:].astype(np.float64)])
    for tau, kmax in ((0.5, 3), (0.9, 8), (0.995, nb)):
        par = ad.SelectorParams(tau_cov=tau, k_min=1, k_max=kmax, k_limit=kmax)
        res = ad.adaptive_decode(oc, q, att.Tolerances(key_bound_mode=1), par)
        for h in range(4):
            r = res[(0, h)]
            qf = q[0, h].astype(np.float64)
            s_true = oc.k16[0, 0].astype(np.float64) @ qf / math.sqrt(128.0)
            a_true = np.exp(s_true - s_true.max())
            a_true /= a_true.sum()
            tail_tok = np.concatenate([np.repeat(~r["promoted"], 16), np.zeros(oc.length - nb * 16, bool)])
            true_tail = a_true[tail_tok].sum()
            assert true_tail <= min(1.0, math.exp(2 * r["delta_h"]) * r["alpha_tail_hat"]) * (1 + 1e-9)
            # the head's own selection is inside the union, the union holds at most 4 K_max blocks
            assert r["promoted"][r["selected"]].all() and r["promoted"].sum() <= 4 * kmax
            o_exact_keys = a_true @ v_mixed_all
            assert np.linalg.norm(r["O"] - o_exact_keys) <= r["E_key"] * (1 + 1e-9) + 1e-12
            o_ref = att.softmax_attention(q[0, h], oc.k16[0, 0], oc.v16[0, 0])
            assert np.linalg.norm(r["O"] - o_ref) <= (r["E_key"] + r["E_val"]) * (1 + 1e-9) + 1e-12
            # promotion can only lower the estimated tail
            assert r["alpha_tail_hat"] <= r["scoring"]["alpha_tail_hat"] + 1e-15


def test_promotion_shrinks_the_key_term_by_orders_of_magnitude():
    """A peaked head: a handful of promoted blocks hold almost all the mass, so the key term with the
    achieved tail is far below the one-pass key term (the reason for the second pass)."""
    oc, q = small_cache(77, n_tokens=1024 + 5)
    q = q.copy()
    q[0, 2] = (oc.k16[0, 0, 321].astype(np.float32) * 0.9).astype(np.float16)   # aligned with one key
    res = ad.adaptive_decode(oc, q, att.Tolerances(key_bound_mode=1),
                             ad.SelectorParams(tau_cov=0.995, k_min=2, k_max=16, k_limit=16))
    r = res[(0, 2)]
    assert r["promoted"][321 // 16]
    assert r["E_key"] < 0.05 * r["scoring"]["E_key"]


# ---------------------------------------------------------------- ranking consistency

def test_ranking_check_hand_cases():
    l8 = np.array([5.0, 4.0, 1.0, 0.5, 0.2])
    prom = np.array([True, True, False, False, False])
    ok = ad.ranking_check(l8, np.array([5.1, 3.9, 0, 0, 0]), prom, 0.2, 1e-6)
    assert not ok["disagree"] and not ok["boundary"] and ok["top_fp16"] == 0
    swap = ad.ranking_check(l8, np.array([4.4, 4.6, 0, 0, 0]), prom, 0.2, 1e-6)
    assert swap["disagree"] and swap["top_fp16"] == 1 and swap["top_int8"] == 0
    # a tail block whose upper-bounded log-mass reaches the best promoted FP16 log-mass
    near = ad.ranking_check(np.array([5.0, 4.0, 4.95, 0.5, 0.2]), np.array([5.1, 3.9, 0, 0, 0]), prom, 0.2, 1e-6)
    assert near["boundary"] and not near["disagree"]
    # exactly at the boundary counts as not certified once the guard is added, strictly below passes
    edge = ad.ranking_check(np.array([5.0, 4.0, 4.75, 0.5, 0.25]), np.array([5.0, 3.5, 0, 0, 0]), prom, 0.25, 0.0)
    assert not edge["boundary"]                                  # 4.75 + 0.25 = 5.0 is not > 5.0
    over = ad.ranking_check(np.array([5.0, 4.0, 4.75, 0.5, 0.25]), np.array([5.0, 3.5, 0, 0, 0]), prom, 0.25, 2.0 ** -20)
    assert over["boundary"]
    empty = ad.ranking_check(l8, l8, np.zeros(5, bool), 0.2, 1e-6)
    assert not empty["disagree"] and not empty["boundary"]


def test_boundary_check_is_sound():
    """When no flag is raised, the block with the largest true (FP16-key) log-mass is the promoted
    block the check names: an unpromoted block cannot outrank it."""
    hits = 0
    for seed in range(12):
        oc, q = small_cache(200 + seed, outlier=bool(seed & 1))
        nb = oc.n_blocks
        res = ad.adaptive_decode(oc, q, att.Tolerances(rank_depth=1),
                                 ad.SelectorParams(tau_cov=0.9, k_min=1, k_max=6, k_limit=6))
        for h in range(4):
            r = res[(0, h)]
            if r["flags"] & att.FLAG_RANK:
                continue
            hits += 1
            s_true = (oc.k16[0, 0, :nb * 16].astype(np.float64) @ q[0, h].astype(np.float64)) / math.sqrt(128.0)
            sb = s_true.reshape(nb, 16)
            l_true = sb.max(axis=1) + np.log(np.exp(sb - sb.max(axis=1, keepdims=True)).sum(axis=1))
            assert int(np.argmax(l_true)) == r["ranking"]["top_fp16"]
    assert hits > 0


# ---------------------------------------------------------------- value promotion (second rung)

def test_value_selection_policies():
    """Threshold policy = every block whose estimated contribution exceeds v_tol; greedy policy = the
    smallest prefix (largest contributions first) that brings the estimated value term under the
    budget: checked against brute force over all prefixes."""
    rng = np.random.Generator(np.random.Philox(300))
    nb = 30
    logits = rng.standard_normal(nb) * 2.0
    p = np.exp(logits) / np.exp(logits).sum() * 0.9
    lse = 0.7
    l = np.log(p) + lse
    eta = rng.uniform(0.1, 1.0, nb).astype(np.float32)
    c = p * eta.astype(np.float64)
    order = sorted(range(nb), key=lambda i: (-c[i], i))
    for v_tol in (0.01, 0.03, math.inf):
        got = ad.select_value_blocks(l, lse, eta, att.Tolerances(v_tol=v_tol),
                                     ad.SelectorParams(v_limit=nb))
        want = [i for i in order if c[i] > v_tol]
        assert got.tolist() == want
    for budget in (0.05, 0.2, c.sum() * 1.01):
        got = ad.select_value_blocks(l, lse, eta, att.Tolerances(eps_val=budget),
                                     ad.SelectorParams(v_limit=nb, v_greedy=True))
        k = next(k for k in range(nb + 1) if sum(c[i] for i in order[k:]) <= budget)
        assert got.tolist() == order[:k]
        assert c.sum() - c[got].sum() <= budget + 1e-15
    capped = ad.select_value_blocks(l, lse, eta, att.Tolerances(eps_val=0.0),
                                    ad.SelectorParams(v_limit=5, v_greedy=True))
    assert capped.tolist() == order[:5]
    assert ad.select_value_blocks(l, lse, eta, att.Tolerances(v_tol=0.0), ad.SelectorParams()).size == 0


@pytest.mark.parametrize("seed", range(3))
def test_value_promotion_special_cases_and_bound(seed):
    oc, q = small_cache(400 + seed)
    nb = oc.n_blocks
    k_hat = qz.dequantize_keys(oc.k_codes[0, 0], oc.sigma[0, 0], oc.z[0, 0]).reshape(nb * 16, 128)
    v_hat = qz.dequantize_values(oc.v_codes[0, 0], oc.v_scale[0, 0], oc.v_offset[0, 0]).reshape(nb * 16, 128)
    k_tr, v_tr = oc.k16[0, 0, nb * 16:], oc.v16[0, 0, nb * 16:]
    tol = att.Tolerances()
    sc = att.certified_head(q[0, 0], k_hat, v_hat, oc.sigma[0, 0], oc.eta[0, 0], oc.nu[0, 0], k_tr, v_tr, tol)
    args = (q[0, 0], k_hat, oc.k16[0, 0, :nb * 16], v_hat, oc.eta[0, 0], oc.nu[0, 0], k_tr, v_tr)
    tail = (sc["blk_logmass"], sc["lse"], sc["delta_h"], tol)
    v16 = oc.v16[0, 0, :nb * 16]
    # every value promoted, no key promoted: attention over the INT8-reconstructed keys and the FP16
    # values; the value term vanishes
    allv = ad.mixed_head(*args, np.zeros(nb, bool), *tail, v_promoted=np.ones(nb, bool), v16_sealed=v16)
    ref = att.softmax_attention(q[0, 0], np.concatenate([k_hat, k_tr.astype(np.float64)]), oc.v16[0, 0])
    assert np.allclose(allv["O"], ref, rtol=0, atol=1e-13)
    assert allv["E_val"] == 0.0 and allv["max_block_contrib"] == 0.0
    # keys and values all promoted: the dense FP16 reference itself
    both = ad.mixed_head(*args, np.ones(nb, bool), *tail, v_promoted=np.ones(nb, bool), v16_sealed=v16)
    dense = att.softmax_attention(q[0, 0], oc.k16[0, 0], oc.v16[0, 0])
    assert np.allclose(both["O"], dense, rtol=0, atol=1e-13) and both["E_key"] == 0.0 and both["E_val"] == 0.0
    # a partial promotion: E_val drops by exactly the promoted blocks' share, and still bounds the
    # value-side error against the same attention weights applied to the FP16 values
    vp = np.zeros(nb, bool)
    vp[np.argsort(-sc["blk_logmass"])[:4]] = True
    part = ad.mixed_head(*args, np.zeros(nb, bool), *tail, v_promoted=vp, v16_sealed=v16)
    rho = np.exp(part["blk_logmass"] - part["lse"])
    assert part["E_val"] == pytest.approx(float((rho * oc.eta[0, 0])[~vp].sum()), rel=1e-12)
    assert part["E_val"] < sc["E_val"]
    o_fp16v = part["weights"] @ oc.v16[0, 0].astype(np.float64)
    assert np.linalg.norm(part["O"] - o_fp16v) <= part["E_val"] * (1 + 1e-9) + 1e-12


def test_greedy_budget_is_met_in_the_attend_pass_when_nothing_is_capped():
    """With FP16 keys nowhere (masses unchanged between the passes) the achieved value term equals
    the estimate the greedy rule stopped on, so it is under the budget."""
    oc, q = small_cache(500, n_tokens=1024 + 3)
    tol = att.Tolerances(eps_val=0.3)
    par = ad.SelectorParams(tau_cov=0.0, k_min=0, k_max=0, k_limit=0, v_limit=512, v_greedy=True)
    res = ad.adaptive_decode(oc, q, tol, par)
    for h in range(4):
        r = res[(0, h)]
        assert not r["promoted"].any()
        assert r["E_val"] <= 0.3 * (1 + 1e-9)
        assert not (r["flags"] & att.FLAG_VAL)
        assert r["E_val"] < r["scoring"]["E_val"]


# ---------------------------------------------------------------- monitors

def scalar_mix(block, group, seed):
    """The exploration hash written out for one block with Python integers."""
    x = (block * 0x9E3779B1) & 0xFFFFFFFF
    x ^= (group * 0x85EBCA77) & 0xFFFFFFFF
    x ^= (seed * 0xC2B2AE3D) & 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x7FEB352D) & 0xFFFFFFFF
    x ^= x >> 15
    x = (x * 0x846CA68B) & 0xFFFFFFFF
    x ^= x >> 16
    return x


def test_exploration_draw():
    par = ad.SelectorParams(explore_frac=0.05, explore_seed=12345)
    nb = 20000
    m = ad.explored_blocks(nb, 3, par)
    for blk in (0, 1, 77, 4096, 19999):
        assert bool(m[blk]) == (scalar_mix(blk, 3, 12345) < int(0.05 * 2 ** 32))
    assert abs(m.mean() - 0.05) < 0.005                      # the budget is met on average
    assert (m != ad.explored_blocks(nb, 4, par)).any()       # another group, another draw
    assert (m != ad.explored_blocks(nb, 3, ad.SelectorParams(explore_frac=0.05, explore_seed=12346))).any()
    assert not ad.explored_blocks(nb, 3, ad.SelectorParams()).any()
    assert ad.explored_blocks(nb, 3, ad.SelectorParams(explore_frac=1.0)).mean() > 0.9999


def test_canary_passes_on_sound_metadata_and_fires_on_corruption():
    """|s_fp16 - s_int8| <= Delta_b <= Delta_h on every token (the per-token bound behind the key term),
    so the check is silent on a sound cache; a scale that no longer describes the block's data (the
    failure the monitor exists for) breaks the bound and raises PRECOND."""
    oc, q = small_cache(600, n_tokens=1024 + 2, outlier=True)
    par = ad.SelectorParams(0.9, 1, 8, 8, canary=True, explore_frac=0.05, explore_seed=7)
    res = ad.adaptive_decode(oc, q, att.Tolerances(), par)
    for h in range(4):
        r = res[(0, h)]
        assert r["score_dev"] <= r["delta_h"] * (1 + 1e-4) and not (r["flags"] & att.FLAG_PRECOND)
        assert r["promoted"].sum() > r["selected"].size       # exploration added blocks
    # corrupt sigma of one explored block: its INT8 reconstruction no longer matches the data
    victim = int(np.nonzero(ad.explored_blocks(oc.n_blocks, 0, par))[0][0])
    oc.sigma[0, 0, victim] *= 3.0
    res = ad.adaptive_decode(oc, q, att.Tolerances(), par)
    fired = [bool(res[(0, h)]["flags"] & att.FLAG_PRECOND) for h in range(4)]
    assert any(fired)
    quiet = ad.adaptive_decode(oc, q, att.Tolerances(), ad.SelectorParams(0.9, 1, 8, 8, explore_frac=0.05, explore_seed=7))
    assert not any(quiet[(0, h)]["flags"] & att.FLAG_PRECOND for h in range(4))   # check switched off


def test_ranking_check_at_depth_r():
    """Depth r of the paper's ranking-consistency check: hand cases, then an independent
    formulation (sorted() on tuples) on random inputs, and depth 1 as the special case."""
    l8 = np.array([5.0, 4.0, 3.0, 2.0, 1.0, 0.5])
    prom = np.array([True, True, True, True, False, False])
    # the top block agrees, the second and third are swapped by the FP16 scores
    lx = np.array([5.2, 3.1, 3.9, 2.0, 0, 0])
    d1 = ad.ranking_check(l8, lx, prom, 0.1, 1e-6, depth=1)
    d2 = ad.ranking_check(l8, lx, prom, 0.1, 1e-6, depth=2)
    d3 = ad.ranking_check(l8, lx, prom, 0.1, 1e-6, depth=3)
    assert not d1["disagree"] and d1["rank_fp16"] == [0]
    assert d2["disagree"] and d2["rank_fp16"] == [0, 2] and d2["rank_int8"] == [0, 1]
    assert d3["disagree"] and d3["rank_fp16"] == [0, 2, 1] and d3["rank_int8"] == [0, 1, 2]
    # the boundary moves with the depth: the tail's best (1.0 + 0.1) is below the 3rd FP16 log-mass
    # (3.1) but above a 4th one lowered to 1.05
    lx4 = np.array([5.2, 4.1, 3.1, 1.05, 0, 0])
    assert not ad.ranking_check(l8, lx4, prom, 0.1, 1e-6, depth=3)["boundary"]
    b4 = ad.ranking_check(l8, lx4, prom, 0.1, 1e-6, depth=4)
    assert b4["boundary"] and not b4["disagree"] and b4["kth_fp16"] == 1.05
    # more depth than promoted blocks: the depth is the size of the promoted set
    assert ad.ranking_check(l8, lx4, prom, 0.1, 1e-6, depth=9)["rank_fp16"] == [0, 1, 2, 3]
    # ties go to the lower block index under both rankings
    t = ad.ranking_check(np.array([2.0, 2.0, 2.0, 0.0]), np.array([1.0, 1.0, 1.0, 0.0]),
                         np.array([True, True, True, False]), 0.1, 0.0, depth=2)
    assert t["rank_fp16"] == [0, 1] and t["rank_int8"] == [0, 1] and not t["disagree"]
    rng = np.random.default_rng(5)
    for trial in range(300):
        nb = int(rng.integers(2, 40))
        l8r = np.round(rng.normal(0, 2, nb), 1)              # rounded: ties occur
        lxr = np.round(l8r + rng.normal(0, 0.15, nb), 1)
        pr = rng.random(nb) < 0.4
        r = int(rng.integers(1, 6))
        delta, guard = 0.2, 1e-6
        got = ad.ranking_check(l8r, lxr, pr, delta, guard, depth=r)
        F = [b for b in range(nb) if pr[b]]
        if not F:
            assert not got["disagree"] and not got["boundary"]
            continue
        rr = min(r, len(F))
        by_x = sorted(F, key=lambda b: (-lxr[b], b))[:rr]
        by_8 = sorted(F, key=lambda b: (-l8r[b], b))[:rr]
        assert got["rank_fp16"] == by_x and got["rank_int8"] == by_8
        assert got["disagree"] == (by_x != by_8)
        tail = [l8r[b] for b in range(nb) if not pr[b]]
        assert got["boundary"] == (bool(tail) and max(tail) + delta + guard > lxr[by_x[-1]])
        one = ad.ranking_check(l8r, lxr, pr, delta, guard)
        assert one["rank_fp16"] == by_x[:1] and one["top_fp16"] == by_x[0]


# ---------------------------------------------------------------- per-head promoted sets

@pytest.mark.parametrize("seed,scale,outlier", [(0, 1.0, False), (1, 2.0, True), (2, 0.5, False)])
def test_per_head_promoted_sets(seed, scale, outlier):
    """The paper's default: every head promotes its own selection.  The head's F is exactly its
    K* best blocks (plus explored ones), lies inside the group's union, its tail is the union
    variant's tail plus the masses of the union's blocks it did not pick, and every bound that
    holds for the union holds for it (tail theorem, key term, total)."""
    oc, q = small_cache(60 + seed, n_tokens=400, scale=scale, outlier=outlier)
    nb = oc.n_blocks
    v_hat = qz.dequantize_values(oc.v_codes[0, 0], oc.v_scale[0, 0], oc.v_offset[0, 0]).reshape(nb * 16, 128)
    v_mixed_all = np.concatenate([v_hat, oc.v16[0, 0, nb * 16:].astype(np.float64)])
    tol = att.Tolerances(key_bound_mode=1, rank_depth=1, v_tol=0.02)
    for tau, kmax in ((0.6, 3), (0.9, 6)):
        ph = ad.SelectorParams(tau_cov=tau, k_min=1, k_max=kmax, k_limit=kmax, v_limit=4, per_head=True,
                               explore_frac=0.1, explore_seed=3)
        un = ad.SelectorParams(tau_cov=tau, k_min=1, k_max=kmax, k_limit=kmax, v_limit=4, explore_frac=0.1,
                               explore_seed=3)
        rp = ad.adaptive_decode(oc, q, tol, ph)
        ru = ad.adaptive_decode(oc, q, tol, un)
        explored = ad.explored_blocks(nb, 0, ph)
        differs = False
        for h in range(4):
            p, u = rp[(0, h)], ru[(0, h)]
            own = np.zeros(nb, bool)
            own[p["selected"]] = True
            assert (p["promoted"] == (own | explored)).all()
            assert (u["promoted"] >= p["promoted"]).all() and (p["group_promoted"] == u["promoted"]).all()
            vown = np.zeros(nb, bool)
            vown[p["v_selected"]] = True
            assert (p["v_promoted"] == vown).all() and (u["v_promoted"] >= vown).all()
            differs = differs or (u["promoted"] != p["promoted"]).any()
            # tail: the union's tail plus the estimated masses of the union's blocks this head left in INT8
            extra = np.exp(p["scoring"]["blk_logmass"][u["promoted"] & ~p["promoted"]] - p["scoring"]["lse"]).sum()
            assert abs(p["alpha_tail_hat"] - (u["alpha_tail_hat"] + extra)) < 1e-12
            # the theorems, with the head's own F
            qf = q[0, h].astype(np.float64)
            s_true = oc.k16[0, 0].astype(np.float64) @ qf / math.sqrt(128.0)
            a_true = np.exp(s_true - s_true.max())
            a_true /= a_true.sum()
            tail_tok = np.concatenate([np.repeat(~p["promoted"], 16), np.zeros(oc.length - nb * 16, bool)])
            assert a_true[tail_tok].sum() <= min(1.0, math.exp(2 * p["delta_h"]) * p["alpha_tail_hat"]) * (1 + 1e-9)
            v_mix = v_mixed_all.copy()
            vp_tok = np.repeat(p["v_promoted"], 16)
            v_mix[:nb * 16][vp_tok] = oc.v16[0, 0, :nb * 16].astype(np.float64)[vp_tok]
            assert np.linalg.norm(p["O"] - a_true @ v_mix) <= p["E_key"] * (1 + 1e-9) + 1e-12
            o_ref = att.softmax_attention(q[0, h], oc.k16[0, 0], oc.v16[0, 0])
            assert np.linalg.norm(p["O"] - o_ref) <= (p["E_key"] + p["E_val"]) * (1 + 1e-9) + 1e-12
            # ranking check runs over the head's own F
            assert p["ranking"]["top_fp16"] == -1 or p["promoted"][p["ranking"]["top_fp16"]]
        assert differs      # the two modes are not the same thing on this data
