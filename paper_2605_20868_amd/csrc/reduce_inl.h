// Cross-split reduction of one (batch, query head), executed by ONE wave of 64 lanes.
//
// Merges the per-split partial states (m, l, o[128], value-term sums, maxima, two largest block
// log-masses) with the usual log-sum-exp factors, attends the trailing FP16 tokens exactly
// (their keys and values are not quantized: eta = 0, no contribution to Delta_h), and
// evaluates the certificate of the paper's total error bound:
//   E_val = sum_b rho_b eta_b,   E_key = 2 V_max min(tanh Delta_h, min{1, e^{c Delta_h} alpha_hat}(e^{2 Delta_h} - 1))
// (key_bound_mode 1 / 2 select the second / first factor alone), the interval form of the
// ranking test  l_(1) - l_(2) <= 2 Delta_h + eps_guard,  and the flag word.
// Used by the reduction kernels of the one-pass and of the adaptive decode.
#pragma once

#include "cqa_internal.h"

namespace cqa {

struct ReduceArgs {
  const float* partials;  // [Bt][Hq][nsplit][PART_FLOATS]
  const __half* q;        // [Bt][Hq][128]
  const __half* trail_k;  // layer base [Bt*Hkv][16][128]
  const __half* trail_v;
  float* O;
  cqa_head_cert* cert;
  uint32_t* flags;
  uint32_t* flags_mirror;  // optional second copy of the flag words (mapped pinned host memory)
  uint32_t mirror_tag;     // OR-ed into each mirrored word (bits 16-31): the host polls for it
  cqa_tolerances tol;
  int nsplit, nb, r, n_q, n_kv;
  int pstride;           // partial sets per (batch, q-head) row of `partials`; 0 = nsplit
};

// LDS operations of one wave execute in order; this only stops the compiler from moving LDS
// accesses across a point where the lanes of a wave exchange data through LDS.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// merges top-2 state (t1, i1, t2) with (u1, j1, u2); ties go to the lower block index
__device__ __forceinline__ void top2_merge(float& t1, int& i1, float& t2, float u1, int j1,
                                           float u2) {
  const bool keep = (t1 > u1) || (t1 == u1 && (unsigned)i1 <= (unsigned)j1);
  if (keep) {
    t2 = fmaxf(t2, u1);
  } else {
    t2 = fmaxf(u2, t1);
    t1 = u1;
    i1 = j1;
  }
}
// DPP move inside a row of 16 lanes (no LDS round trip)
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
  return __uint_as_float(
      (uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(x), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_movi(int x) {
  return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, true);
}
// all-reduce over the 16 lanes of a row: quad xor 1, quad xor 2, half-row mirror, row mirror
__device__ __forceinline__ float row_max(float x) {
  x = fmaxf(x, dpp_mov<0xB1>(x));
  x = fmaxf(x, dpp_mov<0x4E>(x));
  x = fmaxf(x, dpp_mov<0x141>(x));
  x = fmaxf(x, dpp_mov<0x140>(x));
  return x;
}
__device__ __forceinline__ float row_sum(float x) {
  x += dpp_mov<0xB1>(x);
  x += dpp_mov<0x4E>(x);
  x += dpp_mov<0x141>(x);
  x += dpp_mov<0x140>(x);
  return x;
}
// all-reduce over the 64 lanes of the wave: the row step on DPP, two cross-row exchanges
__device__ __forceinline__ float wave_sum(float v) {
  v = row_sum(v);
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
  v = row_max(v);
  v = fmaxf(v, __shfl_xor(v, 16));
  v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}
template <int CTRL>
__device__ __forceinline__ void top2_step_dpp(float& t1, int& i1, float& t2) {
  const float u1 = dpp_mov<CTRL>(t1), u2 = dpp_mov<CTRL>(t2);
  const int j1 = dpp_movi<CTRL>(i1);
  top2_merge(t1, i1, t2, u1, j1, u2);
}
__device__ __forceinline__ void wave_top2(float& t1, int& i1, float& t2) {
  top2_step_dpp<0xB1>(t1, i1, t2);
  top2_step_dpp<0x4E>(t1, i1, t2);
  top2_step_dpp<0x141>(t1, i1, t2);
  top2_step_dpp<0x140>(t1, i1, t2);
#pragma unroll
  for (int m = 16; m < 64; m <<= 1) {
    const float u1 = __shfl_xor(t1, m), u2 = __shfl_xor(t2, m);
    const int j1 = __shfl_xor(i1, m);
    top2_merge(t1, i1, t2, u1, j1, u2);
  }
}

// What the adaptive decode (gated key precision) substitutes in the certificate (the paper's total
// error bound with the achieved tail mass, and its ranking-consistency check): the estimated mass
// of the blocks left in INT8 and Delta_h come from the first (all-INT8) pass, the ranking verdict from a scan
// over the block log-masses of both passes.
struct AdaptiveIn {
  float alpha;       // sum over unpromoted blocks of the first pass's normalised masses
  float delta;       // Delta_h of the first pass
  float top_fp16;    // largest FP16 log-mass among promoted blocks (-inf if none)
  float kth_fp16;    // the r-th largest (r = ranking depth; = top_fp16 at depth 1)
  float tail_ub;     // largest unpromoted INT8 log-mass + Delta_h (-inf if none)
  int top_block;     // the promoted block with the largest FP16 log-mass (-1 if none)
  int rank_fail;     // the two rankings disagree on the top block, or the boundary test failed
  int precond;       // the score-consistency check found a score outside its declared bound
  // The partial sets outside [pos_set0, pos_set1) -- the one pass over all sealed blocks and the
  // negated sets that take the listed blocks back out of it -- contribute their output
  // accumulators only.  A difference of two nearly equal sums would leave the certificate's
  // scalars with the rounding of the large terms, so the mass, the value term and the largest
  // rho_b eta_b of the blocks that are NOT listed come from the scan over the block log-masses
  // instead, relative to the first pass's lse8:  L8u = sum exp(l_b - lse8),
  // EV8u = sum exp(l_b - lse8) eta_b,  maxc8 = max exp(l_b - lse8) eta_b.
  int pos_set0, pos_set1;
  float L8u, EV8u, maxc8, lse8;
};

// wsm: wave-private LDS scratch of at least 64 floats.  All 64 lanes of the wave must call.
// This code runs on the critical tail of the launch: it is written for few dependent memory
// round trips (all loads of a chunk of 64 splits are issued before anything is consumed) and
// short cross-lane chains, not for few instructions.
__device__ __forceinline__ void reduce_head_wave(const ReduceArgs& a, int b, int hq, float* wsm,
                                                 const AdaptiveIn* ad = nullptr) {
  const int l = threadIdx.x & 63;
  const int kvh = hq / (a.n_q / a.n_kv);
  const float inv_sqrt_d = 0.08838834764831845f;
  const float* part = a.partials + ((int64_t)b * a.n_q + hq) * (a.pstride > 0 ? a.pstride : a.nsplit) * PART_FLOATS;

  // trailing FP16 tokens (at most 15): request them first, they are used last.
  //   scores / norms: lane (t = l >> 2, cpart = l & 3) covers channels 32 cpart .. 32 cpart + 31 of
  //   token t; values for the output: lane l covers channels 2l, 2l+1 of every token.
  const __half* tk = a.trail_k + ((int64_t)b * a.n_kv + kvh) * BLK * D;
  const __half* tv = a.trail_v + ((int64_t)b * a.n_kv + kvh) * BLK * D;
  const int tt = min(l >> 2, max(a.r - 1, 0)), cpart = l & 3;
  uint4 kq[4], vq[4], qq[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    kq[i] = reinterpret_cast<const uint4*>(tk + tt * D + cpart * 32)[i];
    vq[i] = reinterpret_cast<const uint4*>(tv + tt * D + cpart * 32)[i];
    qq[i] = reinterpret_cast<const uint4*>(a.q + ((int64_t)b * a.n_q + hq) * D + cpart * 32)[i];
  }
  __half2 vt[BLK - 1];
#pragma unroll
  for (int t = 0; t < BLK - 1; ++t)
    vt[t] = reinterpret_cast<const __half2*>(tv + min(t, max(a.r - 1, 0)) * D)[l];

  float M = -INFINITY, L = 0.0f, EV = 0.0f, EVM = 0.0f, DM = 0.0f, VM = 0.0f;
  float T1 = -INFINITY, T2 = -INFINITY;
  int I1 = -1;
  float2 o2 = make_float2(0.0f, 0.0f);
  for (int s0 = 0; s0 < a.nsplit; s0 += 64) {
    // scalars of split s0 + l (one split per lane) and, for my two channels, the partial
    // outputs of all 64 splits of the chunk
    const int s = s0 + l;
    const bool on = s < a.nsplit;
    const float* ps = part + (int64_t)(on ? s : a.nsplit - 1) * PART_FLOATS;
    float sc[9];
#pragma unroll
    for (int i = 0; i < 9; ++i) sc[i] = ps[i];
    float2 x[64];
#pragma unroll
    for (int i = 0; i < 64; ++i)
      x[i] = *reinterpret_cast<const float2*>(part + (int64_t)min(s0 + i, a.nsplit - 1) * PART_FLOATS + P_O + 2 * l);

    const float m = on ? sc[P_M] : -INFINITY;
    const float Mn = fmaxf(M, wave_max(m));
    const float fo = __expf(M - Mn);        // rescales what earlier chunks accumulated
    const float f = on ? __expf(m - Mn) : 0.0f;
    wsm[l] = f;
    const float fc = (ad == nullptr || (s >= ad->pos_set0 && s < ad->pos_set1)) ? f : 0.0f;
    L = L * fo + wave_sum(fc * sc[P_L]);
    EV = EV * fo + wave_sum(fc * sc[P_EV]);
    EVM = fmaxf(EVM * fo, wave_max(fc * sc[P_EVMAX]));
    DM = fmaxf(DM, wave_max(on ? sc[P_DMAX] : 0.0f));
    VM = fmaxf(VM, wave_max(on ? sc[P_VMAX] : 0.0f));
    float u1 = on ? sc[P_T1] : -INFINITY, u2 = on ? sc[P_T2] : -INFINITY;
    int j1 = on ? __float_as_int(sc[P_I1]) : -1;
    wave_top2(u1, j1, u2);
    top2_merge(T1, I1, T2, u1, j1, u2);
    M = Mn;
    wave_sync();
    o2.x *= fo;
    o2.y *= fo;
#pragma unroll
    for (int i = 0; i < 64; ++i) {
      const float fi = wsm[i];            // zero for splits past the end
      o2.x = fmaf(fi, x[i].x, o2.x);
      o2.y = fmaf(fi, x[i].y, o2.y);
    }
    wave_sync();
  }
  if (ad != nullptr) {
    // the blocks no second pass touched: their mass and value term from the scan
    const float g8 = __expf(ad->lse8 - M);
    L += g8 * ad->L8u;
    EV += g8 * ad->EV8u;
    EVM = fmaxf(EVM, g8 * ad->maxc8);
  }
  float L_sealed = L;

  // ---- trailing FP16 tokens: exact keys and values, eta = 0
  if (a.r > 0) {
    float dot = 0.0f, n2 = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const __half2* kh = reinterpret_cast<const __half2*>(&kq[i]);
      const __half2* vh = reinterpret_cast<const __half2*>(&vq[i]);
      const __half2* qh = reinterpret_cast<const __half2*>(&qq[i]);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        dot = fmaf(__low2float(qh[e]), __low2float(kh[e]), dot);
        dot = fmaf(__high2float(qh[e]), __high2float(kh[e]), dot);
        n2 = fmaf(__low2float(vh[e]), __low2float(vh[e]), n2);
        n2 = fmaf(__high2float(vh[e]), __high2float(vh[e]), n2);
      }
    }
    dot += dpp_mov<0xB1>(dot);      // the four parts of a token are one quad of lanes
    dot += dpp_mov<0x4E>(dot);
    n2 += dpp_mov<0xB1>(n2);
    n2 += dpp_mov<0x4E>(n2);
    const bool live = (l >> 2) < a.r;
    const float st = live ? dot * inv_sqrt_d : -INFINITY;
    const float M2 = fmaxf(M, wave_max(st));
    VM = fmaxf(VM, wave_max(live ? sqrtf(n2) : 0.0f));
    const float fs = __expf(M - M2);
    const float pt = live ? __expf(st - M2) : 0.0f;
    L *= fs;
    o2.x *= fs;
    o2.y *= fs;
    EV *= fs;
    EVM *= fs;
    L_sealed = L;
    L += wave_sum(pt) * 0.25f;      // every token is held by four lanes
    if (cpart == 0) wsm[l >> 2] = pt;
    wave_sync();
#pragma unroll
    for (int t = 0; t < BLK - 1; ++t) {
      const float p = wsm[t];       // zero for t >= r
      o2.x = fmaf(p, __low2float(vt[t]), o2.x);
      o2.y = fmaf(p, __high2float(vt[t]), o2.y);
    }
    M = M2;
  }

  const float out0 = o2.x / L, out1 = o2.y / L;
  reinterpret_cast<float2*>(a.O + ((int64_t)b * a.n_q + hq) * D)[l] = make_float2(out0, out1);
  const bool bad = __any(!isfinite(out0) || !isfinite(out1));

  if (l == 0) {
    // certificate scalars in FP32 (a handful of operations; their rounding is ~1e-7 relative)
    const float e_val = EV / L;
    const float lse = M + logf(L);
    const float maxc = EVM / L;
    const float alpha_hat = ad != nullptr ? ad->alpha : L_sealed / L;
    const float delta = ad != nullptr ? ad->delta : DM;
    const float vmax = VM;
    // No cap on the exponents: beyond the binary32 range the factors are +inf, the tail form of
    // the key term with them, and a non-finite key term raises PRECOND below (in the default
    // mode the tanh form, at most 1, still wins the min).
    float t_tail = 0.0f;
    if (alpha_hat > 0.0f && delta != 0.0f) {
      const float grow = expf((float)a.tol.mass_exp * delta);
      const float widen = expm1f(2.0f * delta);
      t_tail = fminf(1.0f, grow * alpha_hat) * widen;
    }
    const float t_full = tanhf(delta);
    const float tv = a.tol.key_bound_mode == 0 ? fminf(t_full, t_tail)
                                               : (a.tol.key_bound_mode == 1 ? t_tail : t_full);
    const float e_key = 2.0f * vmax * tv;
    float margin = a.nb >= 2 ? T1 - T2 : INFINITY;
    float rho_top = a.nb >= 1 ? expf(T1 - lse) : 0.0f;
    bool rank_flag = a.tol.rank_depth >= 1 && a.nb >= 2 && rho_top >= a.tol.rank_min_mass &&
                     margin <= 2.0f * delta + a.tol.eps_guard;
    if (ad != nullptr) {
      const bool any = ad->top_block >= 0;
      margin = any ? ad->kth_fp16 - ad->tail_ub : INFINITY;
      rho_top = any ? expf(ad->top_fp16 - lse) : 0.0f;
      rank_flag = a.tol.rank_depth >= 1 && any && rho_top >= a.tol.rank_min_mass && ad->rank_fail != 0;
      I1 = ad->top_block;
    }

    uint32_t fl = 0;
    if (e_key > a.tol.eps_key) fl |= CQA_FLAG_KEY;
    if (e_val > a.tol.eps_val || maxc > a.tol.v_tol) fl |= CQA_FLAG_VAL;
    if (rank_flag) fl |= CQA_FLAG_RANK;
    if (ad != nullptr && ad->precond != 0) fl |= CQA_FLAG_PRECOND;
    if (bad || !isfinite(e_key) || !isfinite(e_val) || !isfinite(delta) || !isfinite(vmax) ||
        !isfinite(lse))
      fl |= CQA_FLAG_PRECOND;
    if (e_key + e_val > a.tol.eps_total) fl |= CQA_FLAG_TOTAL;
    fl |= a.tol.force_flags;

    cqa_head_cert ct;
    ct.E_key = e_key;
    ct.E_val = e_val;
    ct.delta_h = delta;
    ct.v_max = VM;
    ct.alpha_tail_hat = alpha_hat;
    ct.lse = lse;
    ct.max_block_contrib = maxc;
    ct.rank_margin = margin;
    ct.top_block = I1;
    ct.served_rung = 0;
    a.cert[(int64_t)b * a.n_q + hq] = ct;
    a.flags[(int64_t)b * a.n_q + hq] = fl;
    // last store of this head: a host thread polling the mirror may take the tagged word as
    // "this head's row, certificate and flags have been issued" (device consumers rely on
    // stream order, not on this word)
    if (a.flags_mirror != nullptr)
      __hip_atomic_store(a.flags_mirror + (int64_t)b * a.n_q + hq, fl | a.mirror_tag,
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

}  // namespace cqa
