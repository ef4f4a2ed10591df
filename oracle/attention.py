"""CPU oracle, part 2: certified decode attention and its certificate.

Test infrastructure only (see quantizer.py's header); float64 throughout; no
blocking, fusion or reordering beyond what the paper's definitions state.

For ONE query head at ONE decode step (paper notation):

* quantized-key logits  s'_t = q . k_hat_t / sqrt(d)  for tokens of sealed
  blocks and  s'_t = q . k_t / sqrt(d)  for the trailing FP16 tokens (Algorithm 1
  scoring line; the trailing block stays FP16 until B tokens arrive);
* a' = softmax(s'),  O_quant = sum_t a'_t v_hat_t  (v_hat = v on trailing tokens);
* block statistics of Algorithm 1, Phase 1:  m_b = max_t s',  S_b = sum_t
  exp(s' - m_b),  l_b = m_b + log S_b,  and block masses rho_b = exp(l_b - LSE);
* score-error bound (Theorem 2 discussion, the tighter runtime form):
  Delta_b = (1 / (2 sqrt d)) sum_c |q_c| sigma_c^(b),  Delta_h = max_b Delta_b
  over sealed blocks only;
* key term: E_key <= 2 V_max TV(a, a') with TV <= tanh(Delta) (full-sequence
  lemma) and TV <= alpha_T (e^{2 Delta} - 1) (tail-restricted lemma), the true
  tail mass bounded through the mass-estimation theorem by
  alpha_T <= min{1, e^{c Delta} alpha_hat_T}, c = 2 (theorems) or 3 (the
  paper's implementation);
* value term (blockwise corollary): E_val = sum_b rho_b eta_b;
* the total  ||O_quant - O_ref|| <= E_key + E_val  (total error bound).

Readings where the paper is silent (the HIP path follows the same ones):

* No block is promoted to FP16 keys here (the adaptive selector is outside the
  hot path), so the INT8 tail is "all sealed blocks":
  alpha_hat_T = sum_b rho_b = 1 - (mass of the trailing FP16 tokens).
* key_bound_mode 0: E_key = 2 V_max min(tanh Delta_h, T_tail); mode 1: T_tail
  only (the literal total-bound formula with the min{1,.} cap on the mass);
  mode 2: tanh only.  T_tail = min{1, e^{c Delta_h} alpha_hat_T} (e^{2 Delta_h} - 1).
* V_max ranges over every attended token: max over sealed blocks of nu_b and
  over trailing tokens of ||v_t||.
* Ranking check without FP16 scores (interval form of the boundary test): each
  block's FP16 log-mass lies within +-Delta_h of its INT8 log-mass, so the top-1
  block is certified iff  l_(1) - l_(2) > 2 Delta_h + eps_guard.  The check is
  skipped for heads whose top block holds less than rank_min_mass.  Ties in
  l_b go to the lower block index.
* The certificate is reported in binary32 (the paper's policy table keeps the
  certificate's accumulators in FP32): a key term whose value exceeds the
  binary32 range (2 Delta_h beyond ~88.7 in the tail form) is +inf, which is a
  non-finite certificate quantity and raises PRECOND.
* INT8 x INT8 scoring (Tolerances.int8_query; the paper's "Per-Channel Key
  Scoring" offers it as the tensor-core alternative to FP16 scoring and names the
  quantisation of the scaled query as a third error source).  Per sealed block the
  scaled query q~_c = q_c sigma_c is quantised symmetrically to 8 bits with one
  scale per block, s_q = max_c |q~_c| / 127, T_c = round(q~_c / s_q) in
  [-127, 127]; the block's logits are (s_q sum_c T_c code_c + q . z) / sqrt(d).
  The paper budgets "one more Delta" for this (its e^{3 Delta} substitution) without
  bounding it; here the third source gets an explicit term: every code has
  magnitude <= 128, so the scores move by at most
      Delta^q_b = (128 / sqrt d) sum_c |q~_c - s_q T_c|
  (<= 64 sqrt(d) s_q), and the block's score-error bound becomes
  Delta_b + Delta^q_b; Delta_h, E_key and the ranking test use that sum, so every
  theorem applies unchanged.  The integer decisions T_c are taken in binary32, as
  the kernel takes them: q~ = fl(q sigma), inv = fl(127 / max|q~|),
  T = round-half-even(q~ inv) on the exact product, s_q = fl(max|q~| / 127).
* Flag word: bit0 KEY (E_key > eps_key), bit1 VAL (E_val > eps_val or
  max_b rho_b eta_b > v_tol), bit2 RANK, bit3 PRECOND (a non-finite certificate
  quantity), bit4 TOTAL (E_key + E_val > eps_total); force_flags is OR-ed in.
  All comparisons are strict.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

FLAG_KEY = 1
FLAG_VAL = 2
FLAG_RANK = 4
FLAG_PRECOND = 8
FLAG_TOTAL = 16
FLAG_ANY = FLAG_KEY | FLAG_VAL | FLAG_RANK | FLAG_PRECOND | FLAG_TOTAL
RUNG_SHIFT = 8
FLT_MAX = float(np.finfo(np.float32).max)   # certificates are reported in binary32


@dataclasses.dataclass
class Tolerances:
    eps_total: float = math.inf
    eps_key: float = math.inf
    eps_val: float = math.inf
    v_tol: float = math.inf
    rank_min_mass: float = 0.0
    eps_guard: float = 1e-6
    rank_depth: int = 0
    mass_exp: int = 2
    key_bound_mode: int = 0
    rung4_min_groups: int = 0
    force_flags: int = 0
    int8_query: bool = False      # INT8 x INT8 scoring of a quantised scaled query


def softmax_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """Textbook single-query attention, softmax(q K^T / sqrt d) V, in float64."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    s = (k @ q) / math.sqrt(q.shape[-1])
    a = np.exp(s - s.max())
    a /= a.sum()
    return a @ v


def key_term(delta_h: float, alpha_hat: float, v_max: float, mass_exp: int = 2,
             mode: int = 0) -> float:
    """E_key from Delta_h, the INT8-estimated tail mass and V_max (see header)."""
    if alpha_hat <= 0.0 or delta_h == 0.0:
        t_tail = 0.0
    else:
        # beyond the binary64 range the factors are +inf; the cap keeps math.exp from raising
        grow = math.exp(mass_exp * delta_h) if mass_exp * delta_h < 700.0 else math.inf
        widen = math.expm1(2.0 * delta_h) if 2.0 * delta_h < 700.0 else math.inf
        t_tail = min(1.0, grow * alpha_hat) * widen
    t_full = math.tanh(delta_h)
    if mode == 0:
        tv = min(t_full, t_tail)
    elif mode == 1:
        tv = t_tail
    else:
        tv = t_full
    e_key = 2.0 * v_max * tv
    return e_key if abs(e_key) <= FLT_MAX else math.copysign(math.inf, e_key)


def quantize_scaled_query(q16: np.ndarray, sigma: np.ndarray):
    """INT8 quantisation of the scaled query, one scale per sealed block (see header).

    q16 float16 [d]; sigma float32 [NB, d].  Returns (T int8 [NB, d], s_q float32 [NB]).
    The decisions are binary32's: the product q sigma and the two quotients are rounded to
    binary32; T rounds the exact product q~ inv (which binary64 holds exactly) half to even.
    """
    q32 = q16.astype(np.float32)
    qt = (q32[None, :] * sigma.astype(np.float32)).astype(np.float32)       # one rounding per element
    amax = np.abs(qt).max(axis=1).astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        inv = np.where(amax > 0, np.float32(127.0) / amax, np.float32(0.0)).astype(np.float32)
        s_q = (amax / np.float32(127.0)).astype(np.float32)
    t = np.rint(qt.astype(np.float64) * inv.astype(np.float64)[:, None])
    assert np.abs(t).max(initial=0.0) <= 127
    return t.astype(np.int8), s_q


def certified_head(q16: np.ndarray, k_hat: np.ndarray, v_hat: np.ndarray, sigma: np.ndarray,
                   eta: np.ndarray, nu: np.ndarray, k_trail16: np.ndarray,
                   v_trail16: np.ndarray, tol: Tolerances, k_codes: np.ndarray = None,
                   z: np.ndarray = None) -> dict:
    """One head, one step.

    q16 float16 [d]; k_hat, v_hat float64 [NB*B, d] (reconstructions of the sealed
    tokens); sigma float32 [NB, d]; eta, nu float32 [NB]; k_trail16, v_trail16
    float16 [r, d] (r may be 0).  tol.int8_query also needs the stored key codes
    k_codes int8 [NB, B, d] and zero points z float32 [NB, d].
    """
    q = q16.astype(np.float64)
    d = q.shape[0]
    nb = sigma.shape[0]
    blk = k_hat.shape[0] // nb if nb else 16
    r = k_trail16.shape[0]
    inv = 1.0 / math.sqrt(d)

    s_seal = (k_hat @ q) * inv if nb else np.zeros(0)
    delta_q = np.zeros(nb)
    if tol.int8_query and nb:
        t_q, s_q = quantize_scaled_query(q16, sigma)
        codes = k_codes.astype(np.float64)                                   # [NB, B, d]
        dots = np.einsum("btc,bc->bt", codes, t_q.astype(np.float64))       # exact integers
        c_b = z.astype(np.float64) @ q                                       # q . z per block
        s_seal = ((s_q.astype(np.float64)[:, None] * dots + c_b[:, None]) * inv).reshape(-1)
        resid = np.abs(q[None, :] * sigma.astype(np.float64) - s_q.astype(np.float64)[:, None] * t_q)
        delta_q = resid.sum(axis=1) * (128.0 * inv)
    kt = k_trail16.astype(np.float64)
    vt = v_trail16.astype(np.float64)
    s_trail = (kt @ q) * inv if r else np.zeros(0)
    s_all = np.concatenate([s_seal, s_trail])
    m = s_all.max()
    e = np.exp(s_all - m)
    z_sum = e.sum()
    a = e / z_sum
    lse = m + math.log(z_sum)
    v_all = np.concatenate([v_hat, vt]) if r else v_hat
    o = a @ v_all

    if nb:
        sb = s_seal.reshape(nb, blk)
        m_b = sb.max(axis=1)
        s_b = np.exp(sb - m_b[:, None]).sum(axis=1)
        l_b = m_b + np.log(s_b)
        rho = np.exp(l_b - lse)
        delta_b = (np.abs(q)[None, :] * sigma.astype(np.float64)).sum(axis=1) * (0.5 * inv) + delta_q
        delta_h = float(delta_b.max())
        contrib = rho * eta.astype(np.float64)
        e_val = float(contrib.sum())
        max_contrib = float(contrib.max())
        alpha_hat = float(rho.sum())
        top = int(np.argmax(l_b))
        if nb >= 2:
            rest = l_b.copy()
            rest[top] = -np.inf
            margin = float(l_b[top] - rest.max())
        else:
            margin = math.inf
        rho_top = float(rho[top])
        v_max = float(nu.max())
    else:
        l_b = np.zeros(0)
        delta_h = 0.0
        e_val = 0.0
        max_contrib = 0.0
        alpha_hat = 0.0
        top = -1
        margin = math.inf
        rho_top = 0.0
        v_max = 0.0
    if r:
        v_max = max(v_max, float(np.sqrt((vt ** 2).sum(axis=1)).max()))

    e_key = key_term(delta_h, alpha_hat, v_max, tol.mass_exp, tol.key_bound_mode)

    flags = 0
    if e_key > tol.eps_key:
        flags |= FLAG_KEY
    if e_val > tol.eps_val or max_contrib > tol.v_tol:
        flags |= FLAG_VAL
    if tol.rank_depth >= 1 and nb >= 2 and rho_top >= tol.rank_min_mass \
            and margin <= 2.0 * delta_h + tol.eps_guard:
        flags |= FLAG_RANK
    if not all(math.isfinite(x) for x in (e_key, e_val, delta_h, v_max, lse)) \
            or not np.isfinite(o).all():
        flags |= FLAG_PRECOND
    if e_key + e_val > tol.eps_total:
        flags |= FLAG_TOTAL
    flags |= tol.force_flags

    return dict(O=o, E_key=e_key, E_val=e_val, delta_h=delta_h, v_max=v_max,
                alpha_tail_hat=alpha_hat, lse=lse, max_block_contrib=max_contrib,
                rank_margin=margin, top_block=top, flags=flags, blk_logmass=l_b,
                weights=a, delta_q=delta_q, scores_sealed=s_seal)
