"""CPU oracle, part 4: adaptive key precision (test infrastructure only).

Follows the paper's "Adaptive Precision Selection" steps, the first rung of its
"Fallback Ladder", the tail-restricted key bound with the achieved INT8-estimated
tail mass (total error bound), the "INT8 Mass Estimation" theorem's normalised
tail implication, and the "Ranking-Consistency Check" with its boundary
verification.  All real-number arithmetic is float64.

Readings where the paper is silent or offers a choice (the HIP path follows the same):

* Mass fractions are taken over EVERYTHING the head attends to, i.e. the sealed
  blocks and the trailing FP16 tokens.  The trailing tokens are exact, so their
  mass counts as covered: C_k = rho_trail + sum of the k largest block masses,
  and the estimated tail mass is alpha_hat_T = 1 - C_K = sum over unpromoted
  blocks of p_b^int8.  With nothing promoted this is the alpha_hat of the one-pass
  certificate.
* Blocks are ranked by INT8 log-mass, ties by lower block index.
* K* = min{k : C_k >= tau_cov}, then clamped to [K_min, K_max] and to the number
  of sealed blocks.
* Rung 1: while the key term computed from the achieved alpha_hat_T exceeds
  eps_key and K can still grow, K doubles (capped at k_limit >= K_max, the
  scratch capacity, and at the number of blocks).
* Key precision is chosen per KV group by default: the promoted set of a group is
  the union of its query heads' selections (the paper's per-KV-group selection
  variant).  A head's tail is then the complement of the union, which only shrinks
  alpha_hat_T; the bound stays valid.  With SelectorParams.per_head the promoted set
  F of a head is its OWN selection (the paper's default: steps 1-6 of "Adaptive
  Precision Selection" and the ranking check run per head over the head's F); the
  blocks the exploration budget draws are promoted for every head of the group in
  either mode.  Value promotion follows the same switch.
* Delta in the bound is Delta_h of the scoring pass (maximum over all sealed
  blocks): the global-max-shift factor of the mass theorem ranges over all blocks.
* Value promotion (the ladder's second rung) is decided from the scoring pass too: a block's
  estimated contribution is c_b = p_b^int8 * eta_b.  Default policy: promote every block with
  c_b > v_tol.  Hard-budget variant (v_greedy): additionally promote blocks in descending c_b
  (ties: lower index) until the estimated value term left, sum of the unpromoted c_b, is at
  most eps_val.  Both are prefixes of the same ordering, so the head's selection is the longer
  of the two, capped at v_limit.  Like keys, values are promoted per KV group (union of the
  group's heads' selections).  A promoted block is attended with its FP16 values and enters
  E_val and max_b rho_b eta_b with eta_b = 0; E_val is the achieved one (attend-pass masses).
  Using the estimated masses for the greedy stop is this build's reading: the paper states the
  stop on the achieved term, which is only known after the pass.
* Monitors (the paper's "Instability Detection").  Score-consistency check (canary): on every
  key-promoted block the FP16 score of each token is compared with its INT8 score; a head with
  |s_fp16 - s_int8| > Delta_h + eps_guard anywhere gets PRECOND (the quantization error left the
  declared bound: metadata corruption or a hardware fault), which the ladder serves by Rung 4.
  Exploration budget: a fraction of the blocks, drawn per (seed, KV group, block) by a counter-
  based hash so both sides draw the same ones, is key-promoted on top of the selection, which
  puts blocks the selector would never pick under the same check.  The hash is the 32-bit
  multiply-xorshift mixer with constants 0x7FEB352D / 0x846CA68B applied to
  block * 0x9E3779B1 ^ group * 0x85EBCA77 ^ seed * 0xC2B2AE3D; a block is explored when the
  result is below explore_frac * 2^32.
* Quantised-query scoring (Tolerances.int8_query, the paper's optional INT8 x INT8 scoring of
  "Per-Channel Key Scoring"): the scoring pass scores every sealed block with the 8-bit scaled
  query; selection, Rung 1 and the ranking check read its log-masses, its Delta_h (which
  contains the explicit third term) is the Delta of the bound, blocks left in INT8 keep its
  scores in the attend pass, promoted blocks are scored exactly from FP16 keys and the exact
  query.  The score-consistency check compares a promoted token's FP16 score with the
  quantised-query score.
* Ranking check at depth r (Tolerances.rank_depth, the paper's configurable depth;
  default 1) over the head's promoted set F (the group's union, or the head's own
  selection with per_head): (i) the r blocks with the largest FP16 log-masses in F
  must be, in the same order, the r blocks with the largest INT8 log-masses in F
  (ties by lower index; fewer than r promoted blocks: r = their number);
  (ii) boundary: no unpromoted block may have l_b^int8 + Delta_h (+ eps_guard) >
  the r-th largest FP16 log-mass in F.  Either failure sets RANK.  The optional rank_min_mass gate of the one-pass path
  applies here too (0 = the paper's unconditional check).
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

from . import attention as att


@dataclasses.dataclass
class SelectorParams:
    tau_cov: float = 0.995
    k_min: int = 2
    k_max: int = 128
    k_limit: int = 128          # cap for Rung-1 doubling (>= k_max)
    v_limit: int = 0            # blocks one head may promote to FP16 values (0 = off)
    v_greedy: bool = False      # hard-budget variant: also promote until the estimate fits eps_val
    canary: bool = False        # score-consistency check on key-promoted blocks
    explore_frac: float = 0.0   # exploration budget: fraction of blocks key-promoted at random
    explore_seed: int = 0       # counter of the draw (e.g. the decode step)
    per_head: bool = False      # promoted sets per query head (the paper's default) instead of per KV group


def rank_blocks(logmass: np.ndarray) -> np.ndarray:
    """Block indices by descending INT8 log-mass; equal masses keep the lower index first."""
    return np.argsort(-np.asarray(logmass, dtype=np.float64), kind="stable")


def select_blocks(logmass: np.ndarray, lse: float, par: SelectorParams) -> dict:
    """Steps 1-4 of the adaptive selection for one head.

    logmass [NB]: INT8 block log-masses of the scoring pass; lse: log of the total
    estimated mass (sealed + trailing tokens).  Returns the ranking, K* before any
    Rung-1 growth, and the estimated tail mass left after promoting the K* best.
    """
    l = np.asarray(logmass, dtype=np.float64)
    nb = l.shape[0]
    order = rank_blocks(l)
    p = np.exp(l[order] - lse)                 # estimated normalised block masses, descending
    total_blocks = float(p.sum())
    rho_trail = 1.0 - total_blocks             # exact FP16 tokens: always covered
    covered = rho_trail + np.concatenate([[0.0], np.cumsum(p)])   # C_0 .. C_NB
    hit = np.nonzero(covered >= par.tau_cov)[0]
    k = int(hit[0]) if hit.size else nb
    k = max(par.k_min, min(k, par.k_max))
    k = min(k, nb)
    return dict(order=order, k_star=k, p_sorted=p, rho_trail=rho_trail)


def tail_mass(sel: dict, k: int) -> float:
    """alpha_hat_T after promoting the k best-ranked blocks: sum of the other blocks' masses."""
    return float(sel["p_sorted"][k:].sum())


def rung1_expand(sel: dict, delta_h: float, v_max: float, tol: att.Tolerances,
                 par: SelectorParams) -> int:
    """Rung 1: double K while the key term of the achieved tail exceeds eps_key."""
    nb = sel["order"].shape[0]
    cap = min(max(par.k_limit, par.k_max), nb)
    k = sel["k_star"]
    while k < cap and att.key_term(delta_h, tail_mass(sel, k), v_max, tol.mass_exp,
                                   tol.key_bound_mode) > tol.eps_key:
        k = min(max(2 * k, 1), cap)
    return k


def value_contributions(logmass: np.ndarray, lse: float, eta: np.ndarray) -> np.ndarray:
    """Estimated contribution of each block to the value term: c_b = p_b^int8 * eta_b."""
    return np.exp(np.asarray(logmass, dtype=np.float64) - lse) * np.asarray(eta, dtype=np.float64)


def select_value_blocks_from(contrib: np.ndarray, tol: att.Tolerances, par: SelectorParams) -> np.ndarray:
    """The head's blocks to promote to FP16 values, in descending estimated contribution."""
    c = np.asarray(contrib, dtype=np.float64)
    nb = c.shape[0]
    if par.v_limit <= 0 or nb == 0:
        return np.zeros(0, dtype=np.int64)
    order = np.argsort(-c, kind="stable")
    cs = c[order]
    k = int((cs > tol.v_tol).sum())                                 # local policy: a prefix
    if par.v_greedy:
        left = cs.sum() - np.concatenate([[0.0], np.cumsum(cs)])    # estimate left after k blocks
        hit = np.nonzero(left <= tol.eps_val)[0]
        k = max(k, int(hit[0]) if hit.size else nb)
    k = min(k, par.v_limit, nb)
    return order[:k]


def select_value_blocks(logmass: np.ndarray, lse: float, eta: np.ndarray, tol: att.Tolerances,
                        par: SelectorParams) -> np.ndarray:
    return select_value_blocks_from(value_contributions(logmass, lse, eta), tol, par)


def explored_blocks(nb: int, group: int, par: SelectorParams) -> np.ndarray:
    """Boolean mask [NB] of the blocks the exploration budget key-promotes for KV group `group`
    (= batch * n_kv_heads + kv_head)."""
    if par.explore_frac <= 0.0 or nb == 0:
        return np.zeros(nb, dtype=bool)
    m = np.uint64(0xFFFFFFFF)
    x = (np.arange(nb, dtype=np.uint64) * np.uint64(0x9E3779B1)) & m
    x ^= np.uint64((group * 0x85EBCA77) & 0xFFFFFFFF)
    x ^= np.uint64(((par.explore_seed & 0xFFFFFFFF) * 0xC2B2AE3D) & 0xFFFFFFFF)
    x ^= x >> np.uint64(16)
    x = (x * np.uint64(0x7FEB352D)) & m
    x ^= x >> np.uint64(15)
    x = (x * np.uint64(0x846CA68B)) & m
    x ^= x >> np.uint64(16)
    threshold = min(int(par.explore_frac * 4294967296.0), 0xFFFFFFFF)
    return x < np.uint64(threshold)


def group_union(selections, nb: int) -> np.ndarray:
    """Boolean mask [NB]: union of the heads' promoted sets (each an index array)."""
    mask = np.zeros(nb, dtype=bool)
    for idx in selections:
        mask[np.asarray(idx, dtype=np.int64)] = True
    return mask


def ranking_check(l_int8: np.ndarray, l_fp16: np.ndarray, promoted: np.ndarray, delta_h: float,
                  eps_guard: float, depth: int = 1) -> dict:
    """Ranking consistency at depth r plus boundary verification for one head (the paper's
    "Ranking-Consistency Check": the two top-r rankings over the promoted set must agree, and no
    tail block may have an upper-bounded log-mass above the r-th highest FP16 log-mass).

    l_fp16 holds FP16 log-masses on promoted blocks (its values elsewhere are ignored).
    Order: larger log-mass first, equal log-masses by lower block index.  With fewer than r
    promoted blocks the depth is the number of promoted blocks.  Returns the two rankings
    (block indices, best first), their heads top_fp16 / top_int8, and the two verdicts.
    """
    promoted = np.asarray(promoted, dtype=bool)
    if not promoted.any():
        return dict(disagree=False, boundary=False, top_fp16=-1, top_int8=-1, rank_fp16=[], rank_int8=[],
                    kth_fp16=-math.inf)
    idx = np.nonzero(promoted)[0]
    r = max(1, min(int(depth), len(idx)))
    # stable sort on the negated log-masses: ties keep ascending block order
    rank_fp16 = [int(b) for b in idx[np.argsort(-l_fp16[idx], kind="stable")][:r]]
    rank_int8 = [int(b) for b in idx[np.argsort(-l_int8[idx], kind="stable")][:r]]
    kth = float(l_fp16[rank_fp16[-1]])
    tail = ~promoted
    boundary = bool(tail.any() and float(l_int8[tail].max()) + delta_h + eps_guard > kth)
    return dict(disagree=rank_fp16 != rank_int8, boundary=boundary, top_fp16=rank_fp16[0],
                top_int8=rank_int8[0], rank_fp16=rank_fp16, rank_int8=rank_int8, kth_fp16=kth)


def mixed_head(q16: np.ndarray, k_hat: np.ndarray, k16_sealed: np.ndarray, v_hat: np.ndarray,
               eta: np.ndarray, nu: np.ndarray, k_trail16: np.ndarray, v_trail16: np.ndarray,
               promoted: np.ndarray, l_int8: np.ndarray, lse_int8: float, delta_h: float,
               tol: att.Tolerances, v_promoted: np.ndarray | None = None,
               v16_sealed: np.ndarray | None = None, canary: bool = False,
               s_scored: np.ndarray | None = None) -> dict:
    """The attend pass with mask-gated key precision, one head, one step.

    k_hat float64 [NB*B, d] INT8 reconstructions; k16_sealed float16 [NB*B, d] the FP16
    originals of the same tokens; promoted bool [NB]; l_int8, lse_int8, delta_h: the scoring
    pass's block log-masses, total log-mass and Delta_h for this head.
    Values are INT4 reconstructions, except in the blocks of v_promoted (bool [NB], optional),
    which use the FP16 originals v16_sealed [NB*B, d] and count with eta_b = 0.
    s_scored float64 [NB*B] (optional): the scoring pass's own scores of the sealed tokens,
    given when that pass scored with a quantised scaled query (Tolerances.int8_query): the
    blocks left in INT8 then keep exactly those scores (scoring and attending are one pass
    over them), the promoted blocks are scored exactly from their FP16 keys as always, and
    delta_h already carries the third error term of the quantised query, so the tail theorem
    and the key bound hold with it unchanged.
    """
    q = q16.astype(np.float64)
    d = q.shape[0]
    nb = promoted.shape[0]
    blk = k_hat.shape[0] // nb if nb else 16
    inv = 1.0 / math.sqrt(d)
    tok_prom = np.repeat(np.asarray(promoted, dtype=bool), blk)
    k_mix = np.where(tok_prom[:, None], k16_sealed.astype(np.float64), k_hat)
    s_seal = (k_mix @ q) * inv if nb else np.zeros(0)
    if s_scored is not None and nb:
        s_seal = np.where(tok_prom, s_seal, np.asarray(s_scored, dtype=np.float64))
    r = k_trail16.shape[0]
    kt = k_trail16.astype(np.float64)
    vt = v_trail16.astype(np.float64)
    s_trail = (kt @ q) * inv if r else np.zeros(0)
    s_all = np.concatenate([s_seal, s_trail])
    m = s_all.max()
    e = np.exp(s_all - m)
    z_sum = e.sum()
    a = e / z_sum
    lse = m + math.log(z_sum)
    eta_eff = eta.astype(np.float64)
    v_seal = v_hat
    if v_promoted is not None and np.asarray(v_promoted, dtype=bool).any():
        vp = np.asarray(v_promoted, dtype=bool)
        v_seal = np.where(np.repeat(vp, blk)[:, None], v16_sealed.astype(np.float64), v_hat)
        eta_eff = np.where(vp, 0.0, eta_eff)
    v_all = np.concatenate([v_seal, vt]) if r else v_seal
    o = a @ v_all

    sb = s_seal.reshape(nb, blk)
    m_b = sb.max(axis=1)
    l_b = m_b + np.log(np.exp(sb - m_b[:, None]).sum(axis=1))
    rho = np.exp(l_b - lse)
    contrib = rho * eta_eff
    e_val = float(contrib.sum())
    max_contrib = float(contrib.max())
    v_max = float(nu.max())
    if r:
        v_max = max(v_max, float(np.sqrt((vt ** 2).sum(axis=1)).max()))
    alpha_hat = float(np.exp(np.asarray(l_int8, dtype=np.float64)[~promoted] - lse_int8).sum())
    e_key = att.key_term(delta_h, alpha_hat, v_max, tol.mass_exp, tol.key_bound_mode)

    rk = ranking_check(np.asarray(l_int8, dtype=np.float64), l_b, promoted, delta_h, tol.eps_guard,
                       max(1, tol.rank_depth))
    # score-consistency check: FP16 against INT8 scores on the key-promoted tokens
    score_dev = 0.0
    if nb and tok_prom.any():
        s_int8 = (k_hat[tok_prom] @ q) * inv if s_scored is None else np.asarray(s_scored, dtype=np.float64)[tok_prom]
        score_dev = float(np.abs(s_seal[tok_prom] - s_int8).max())
    flags = 0
    if canary and score_dev > delta_h + tol.eps_guard:
        flags |= att.FLAG_PRECOND
    if e_key > tol.eps_key:
        flags |= att.FLAG_KEY
    if e_val > tol.eps_val or max_contrib > tol.v_tol:
        flags |= att.FLAG_VAL
    if tol.rank_depth >= 1 and promoted.any():
        rho_top = float(rho[rk["top_fp16"]])
        if rho_top >= tol.rank_min_mass and (rk["disagree"] or rk["boundary"]):
            flags |= att.FLAG_RANK
    if not all(math.isfinite(x) for x in (e_key, e_val, delta_h, v_max, lse)) \
            or not np.isfinite(o).all():
        flags |= att.FLAG_PRECOND
    if e_key + e_val > tol.eps_total:
        flags |= att.FLAG_TOTAL
    flags |= tol.force_flags
    return dict(O=o, E_key=e_key, E_val=e_val, delta_h=delta_h, v_max=v_max,
                alpha_tail_hat=alpha_hat, lse=lse, max_block_contrib=max_contrib,
                flags=flags, blk_logmass=l_b, weights=a, ranking=rk, score_dev=score_dev)


def adaptive_decode(cache, q16: np.ndarray, tol: att.Tolerances, par: SelectorParams,
                    groups=None) -> dict:
    """Scoring pass, selection (+ Rung 1), per-group union, attend pass with gated key precision.

    cache: an OracleLayerCache.  q16 float16 [Bt, Hq, d].  `groups` optionally restricts the
    work to an iterable of (b, kv_head) pairs.  Returns {(b, h): result dict}; each result is
    mixed_head's, plus 'k_star' (the head's own K after Rung 1), 'selected' (its own block
    indices, best first), 'promoted' (the group's union mask) and 'scoring' (the one-pass result).
    The scoring pass runs with every threshold disabled: its flags are not part of the result.
    """
    from . import quantizer as qz

    bt, hq, d = q16.shape
    g = hq // cache.hkv
    nb = cache.n_blocks
    todo = [(b, kh) for b in range(bt) for kh in range(cache.hkv)] if groups is None else list(groups)
    out = {}
    for b, kh in todo:
        k_hat = qz.dequantize_keys(cache.k_codes[b, kh], cache.sigma[b, kh],
                                   cache.z[b, kh]).reshape(nb * qz.B, d)
        v_hat = qz.dequantize_values(cache.v_codes[b, kh], cache.v_scale[b, kh],
                                     cache.v_offset[b, kh]).reshape(nb * qz.B, d)
        k_tr, v_tr = cache.k16[b, kh, nb * qz.B:], cache.v16[b, kh, nb * qz.B:]
        scoring, picks, ks, vpicks = [], [], [], []
        for i in range(g):
            h = kh * g + i
            sc = att.certified_head(q16[b, h], k_hat, v_hat, cache.sigma[b, kh], cache.eta[b, kh],
                                    cache.nu[b, kh], k_tr, v_tr, att.Tolerances(int8_query=tol.int8_query),
                                    k_codes=cache.k_codes[b, kh], z=cache.z[b, kh])
            sel = select_blocks(sc["blk_logmass"], sc["lse"], par)
            k = rung1_expand(sel, sc["delta_h"], sc["v_max"], tol, par)
            scoring.append(sc)
            picks.append(sel["order"][:k])
            ks.append(k)
            vpicks.append(select_value_blocks(sc["blk_logmass"], sc["lse"], cache.eta[b, kh], tol, par))
        explored = explored_blocks(nb, b * cache.hkv + kh, par)
        union = group_union(picks, nb) | explored
        vunion = group_union(vpicks, nb)
        for i in range(g):
            h = kh * g + i
            sc = scoring[i]
            # the head's promoted sets: its own selection, or the group's union
            f_keys = (group_union([picks[i]], nb) | explored) if par.per_head else union
            f_vals = group_union([vpicks[i]], nb) if par.per_head else vunion
            res = mixed_head(q16[b, h], k_hat, cache.k16[b, kh, :nb * qz.B], v_hat, cache.eta[b, kh],
                             cache.nu[b, kh], k_tr, v_tr, f_keys, sc["blk_logmass"], sc["lse"],
                             sc["delta_h"], tol, v_promoted=f_vals,
                             v16_sealed=cache.v16[b, kh, :nb * qz.B], canary=par.canary,
                             s_scored=sc["scores_sealed"] if tol.int8_query else None)
            res.update(k_star=ks[i], selected=picks[i], promoted=f_keys, scoring=sc,
                       v_selected=vpicks[i], v_promoted=f_vals, group_promoted=union,
                       group_v_promoted=vunion)
            out[(b, h)] = res
    return out
