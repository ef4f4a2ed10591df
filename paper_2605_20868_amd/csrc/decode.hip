// Certified decode: split-K pass over Tier-1 and the cross-split reduction.
//
// What is computed (the paper's Algorithm 1 with no promoted blocks, its
// scaled-query scoring identity, and its two-term bound):
//   per sealed block b:  q~ = q (.) sigma^(b),  c_b = q . z^(b),
//                        s_t = (q~ . code_t + c_b) / sqrt(d),
//                        m_b = max_t s_t,  S_b = sum_t exp(s_t - m_b),  l_b = m_b + log S_b,
//                        Delta_b = (1 / (2 sqrt d)) sum_c |q_c| sigma_c^(b);
//   FP32 online softmax (m, l, o) with v_hat = code * scale + offset;
//   alongside it  sum_b rho_b eta_b  (value term),  max_b rho_b eta_b,
//   Delta_h = max_b Delta_b,  V_max = max_b nu_b,  and the two largest l_b;
//   the reduction merges the splits, attends the trailing FP16 tokens exactly and
//   evaluates  E_key = 2 V_max min(tanh Delta_h, min{1, e^{c Delta_h} alpha_hat}(e^{2 Delta_h} - 1)),
//   E_val = sum_b rho_b eta_b  and the flag word.
#include "cqa_internal.h"

namespace cqa {

__device__ __forceinline__ void wave_sync() {
  // LDS operations of one wave execute in order; this only stops the compiler from
  // moving LDS accesses across the point where lanes exchange data.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}


// merges top-2 state (t1, i1, t2) with (u1, j1, u2); ties go to the lower block index
__device__ __forceinline__ void top2_merge(float& t1, int& i1, float& t2, float u1, int j1, float u2) {
  const bool keep = (t1 > u1) || (t1 == u1 && (unsigned)i1 <= (unsigned)j1);
  if (keep) {
    t2 = fmaxf(t2, u1);
  } else {
    t2 = fmaxf(u2, t1);
    t1 = u1;
    i1 = j1;
  }
}

template <int G>
__global__ __launch_bounds__(256) void certified_split_kernel(DecodeArgs a) {
  const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int tok = l & 15, kg = l >> 4;              // roles in the score phase
  const int vn = l & 15, vgh = (l >> 4) & 1, vo = l >> 5;  // roles in the value phase
  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int64_t base_blk = ((int64_t)b * a.n_kv + kvh) * a.nb_cap;
  // blocks are dealt evenly over the splits (every split gets at least one: nsplit <= nb)
  const int b0 = (int)(((int64_t)split * a.nb) / a.nsplit);
  const int b1 = (int)(((int64_t)(split + 1) * a.nb) / a.nsplit);
  const float inv_sqrt_d = 0.08838834764831845f;  // 1 / sqrt(128)

  __shared__ __align__(16) float qs[4][G][D];     // scaled query of the block in flight, per wave
  __shared__ __align__(16) float ps[4][BLK][G];   // its probabilities
  __shared__ float ms[4][G][12];                  // per-wave scalars for the merge

  float qv[G][2];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const __half2 t = reinterpret_cast<const __half2*>(
        a.q + ((int64_t)b * a.n_q + kvh * G + h) * D)[l];
    qv[h][0] = __low2float(t);
    qv[h][1] = __high2float(t);
  }

  float m_run[G], l_run[G], ev[G], evmax[G], dmax[G], t1[G], t2[G];
  int i1[G];
  float acc[4][G];
  float vmax = 0.0f;
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m_run[h] = -INFINITY;
    l_run[h] = 0.0f;
    ev[h] = 0.0f;
    evmax[h] = 0.0f;
    dmax[h] = 0.0f;
    t1[h] = -INFINITY;
    t2[h] = -INFINITY;
    i1[h] = -1;
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) acc[gq][h] = 0.0f;
  }

  for (int blk = b0 + w; blk < b1; blk += 4) {
    const int64_t gb = base_blk + blk;
    // ---- scaled query, per-block constant, per-block score-error bound
    const float* kmb = a.km + gb * (KM_BYTES / 4);
    const float2 sg = reinterpret_cast<const float2*>(kmb)[l];
    const float2 zz = reinterpret_cast<const float2*>(kmb + D)[l];
    const float2 an = *reinterpret_cast<const float2*>(a.an + gb * 2);
    float csum[G], dsum[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float q0 = qv[h][0] * sg.x, q1 = qv[h][1] * sg.y;
      reinterpret_cast<float2*>(&qs[w][h][0])[l] = make_float2(q0, q1);
      // stored bytes are code + 128: fold the -128 * sum(q~) into the block constant
      csum[h] = qv[h][0] * zz.x + qv[h][1] * zz.y - 128.0f * (q0 + q1);
      dsum[h] = fabsf(qv[h][0]) * sg.x + fabsf(qv[h][1]) * sg.y;
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
#pragma unroll
      for (int h = 0; h < G; ++h) {
        csum[h] += __shfl_xor(csum[h], m);
        dsum[h] += __shfl_xor(dsum[h], m);
      }
    }
    wave_sync();

    // ---- scores: lane (tok, kg) covers channels cq*64 + kg*16 + 0..15, cq = 0, 1
    const uint8_t* kcb = a.kc + gb * KC_BYTES;
    float dot[G];
#pragma unroll
    for (int h = 0; h < G; ++h) dot[h] = 0.0f;
#pragma unroll
    for (int cq = 0; cq < 2; ++cq) {
      const uint4 x = reinterpret_cast<const uint4*>(kcb + cq * 1024)[l];
      const uint32_t wd[4] = {x.x, x.y, x.z, x.w};
      const int c0 = cq * 64 + kg * 16;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const float kf = (float)((wd[j >> 2] >> (8 * (j & 3))) & 0xffu);
#pragma unroll
        for (int h = 0; h < G; ++h) dot[h] = fmaf(qs[w][h][c0 + j], kf, dot[h]);
      }
    }
    float p[G], alpha[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      dot[h] += __shfl_xor(dot[h], 16);
      dot[h] += __shfl_xor(dot[h], 32);
      const float s = (dot[h] + csum[h]) * inv_sqrt_d;
      float mb = s;
#pragma unroll
      for (int m = 1; m < 16; m <<= 1) mb = fmaxf(mb, __shfl_xor(mb, m));
      const float pt = __expf(s - mb);
      float sb = pt;
#pragma unroll
      for (int m = 1; m < 16; m <<= 1) sb += __shfl_xor(sb, m);
      const float lb = mb + __logf(sb);
      const float m_new = fmaxf(m_run[h], mb);
      alpha[h] = __expf(m_run[h] - m_new);
      const float f = __expf(mb - m_new);
      p[h] = pt * f;
      const float sf = sb * f;
      const float ce = sf * an.x;
      l_run[h] = l_run[h] * alpha[h] + sf;
      ev[h] = ev[h] * alpha[h] + ce;
      evmax[h] = fmaxf(evmax[h] * alpha[h], ce);
      dmax[h] = fmaxf(dmax[h], dsum[h] * (0.5f * inv_sqrt_d));
      m_run[h] = m_new;
      if (lb > t1[h]) {
        t2[h] = t1[h];
        t1[h] = lb;
        i1[h] = blk;
      } else if (lb > t2[h]) {
        t2[h] = lb;
      }
      if (a.blk_logmass != nullptr && l == 0)
        a.blk_logmass[((int64_t)b * a.n_q + kvh * G + h) * a.nb + blk] = lb;
      if (kg == 0) ps[w][tok][h] = p[h];
    }
    vmax = fmaxf(vmax, an.y);
    wave_sync();

    // ---- values: lane (vo, vgh, vn) covers tokens vo*8..+7 of channels (vgh*4+gq)*16 + vn
    const uint4 vx = reinterpret_cast<const uint4*>(a.vc + gb * VC_BYTES)[l];
    const uint32_t vw[4] = {vx.x, vx.y, vx.z, vx.w};
    const __half* vmb = a.vm + gb * (VM_BYTES / 2);
    float pi[8][G];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int h = 0; h < G; ++h) pi[i][h] = ps[w][vo * 8 + i][h];
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const int g = vgh * 4 + gq;
      const uint4 sraw = *reinterpret_cast<const uint4*>(vmb + vo * 64 + g * 8);
      const uint4 oraw = *reinterpret_cast<const uint4*>(vmb + BLK * NG + vo * 64 + g * 8);
      const __half2* sh = reinterpret_cast<const __half2*>(&sraw);
      const __half2* oh = reinterpret_cast<const __half2*>(&oraw);
#pragma unroll
      for (int h = 0; h < G; ++h) acc[gq][h] *= alpha[h];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float sc = (i & 1) ? __high2float(sh[i >> 1]) : __low2float(sh[i >> 1]);
        const float of = (i & 1) ? __high2float(oh[i >> 1]) : __low2float(oh[i >> 1]);
        const float vh = fmaf((float)((vw[gq] >> (4 * i)) & 15u), sc, of);
#pragma unroll
        for (int h = 0; h < G; ++h) acc[gq][h] = fmaf(pi[i][h], vh, acc[gq][h]);
      }
    }
    wave_sync();
  }

  // ---- merge the four waves of the workgroup, then write one partial per q-head
  float* mo = &qs[0][0][0];  // reuse: [4][G][D]
  __syncthreads();
#pragma unroll
  for (int gq = 0; gq < 4; ++gq)
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float v = acc[gq][h] + __shfl_xor(acc[gq][h], 32);
      if (vo == 0) mo[(w * G + h) * D + (vgh * 4 + gq) * 16 + vn] = v;
    }
  if (l == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      ms[w][h][0] = m_run[h];
      ms[w][h][1] = l_run[h];
      ms[w][h][2] = ev[h];
      ms[w][h][3] = evmax[h];
      ms[w][h][4] = dmax[h];
      ms[w][h][5] = vmax;
      ms[w][h][6] = t1[h];
      ms[w][h][7] = t2[h];
      ms[w][h][8] = __int_as_float(i1[h]);
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * D; idx += 256) {
    const int h = idx / D, c = idx % D;
    float M = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) M = fmaxf(M, ms[ww][h][0]);
    float o = 0.0f;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) o += __expf(ms[ww][h][0] - M) * mo[(ww * G + h) * D + c];
    a.partials[(((int64_t)b * a.n_q + kvh * G + h) * a.nsplit + split) * PART_FLOATS + P_O + c] = o;
  }
  if (threadIdx.x < G) {
    const int h = threadIdx.x;
    float M = -INFINITY;
    for (int ww = 0; ww < 4; ++ww) M = fmaxf(M, ms[ww][h][0]);
    float L = 0.0f, EV = 0.0f, EVM = 0.0f, DM = 0.0f, VM = 0.0f, T1 = -INFINITY, T2 = -INFINITY;
    int I1 = -1;
    for (int ww = 0; ww < 4; ++ww) {
      const float f = __expf(ms[ww][h][0] - M);
      L += f * ms[ww][h][1];
      EV += f * ms[ww][h][2];
      EVM = fmaxf(EVM, f * ms[ww][h][3]);
      DM = fmaxf(DM, ms[ww][h][4]);
      VM = fmaxf(VM, ms[ww][h][5]);
      top2_merge(T1, I1, T2, ms[ww][h][6], __float_as_int(ms[ww][h][8]), ms[ww][h][7]);
    }
    float* pp = a.partials + (((int64_t)b * a.n_q + kvh * G + h) * a.nsplit + split) * PART_FLOATS;
    pp[P_M] = M;
    pp[P_L] = L;
    pp[P_EV] = EV;
    pp[P_EVMAX] = EVM;
    pp[P_DMAX] = DM;
    pp[P_VMAX] = VM;
    pp[P_T1] = T1;
    pp[P_T2] = T2;
    pp[P_I1] = __int_as_float(I1);
  }
}

struct ReduceArgs {
  const float* partials;
  const __half* q;
  const __half* trail_k;  // layer base [Bt*Hkv][16][128]
  const __half* trail_v;
  float* O;
  cqa_head_cert* cert;
  uint32_t* flags;
  cqa_tolerances tol;
  int nsplit, nb, r, n_q, n_kv;
};

constexpr int RED_THREADS = 256;

// block-wide sum / max over 256 threads; every thread gets the result
__device__ __forceinline__ float block_sum(float v, float* scratch4) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch4[threadIdx.x >> 6] = v;
  __syncthreads();
  return (scratch4[0] + scratch4[1]) + (scratch4[2] + scratch4[3]);
}
__device__ __forceinline__ float block_max(float v, float* scratch4) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) v = fmaxf(v, __shfl_xor(v, m));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch4[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(scratch4[0], scratch4[1]), fmaxf(scratch4[2], scratch4[3]));
}

__global__ __launch_bounds__(RED_THREADS) void certified_reduce_kernel(ReduceArgs a) {
  const int t = threadIdx.x, w = t >> 6, l = t & 63;
  const int c = t & (D - 1);            // channel owned by threads 0..127 in the epilogue
  const bool own = t < D;
  const int hq = blockIdx.x, b = blockIdx.y;
  const int group = a.n_q / a.n_kv;
  const int kvh = hq / group;
  const float inv_sqrt_d = 0.08838834764831845f;
  __shared__ float scratch4[4];
  __shared__ float wsm[MAX_SPLITS];     // per-split max, then per-split weight e^{m_s - M}
  __shared__ float t2s[4][3];
  __shared__ __align__(8) float osum[4][D];

  const float* part = a.partials + ((int64_t)b * a.n_q + hq) * a.nsplit * PART_FLOATS;
  // ---- per-split scalars, spread over the threads
  float m_loc = -INFINITY;
  for (int s = t; s < a.nsplit; s += RED_THREADS) {
    const float m = part[s * PART_FLOATS + P_M];
    wsm[s] = m;
    m_loc = fmaxf(m_loc, m);
  }
  float M = block_max(m_loc, scratch4);
  float L = 0.0f, EV = 0.0f, EVM = 0.0f, DM = 0.0f, VM = 0.0f;
  float T1 = -INFINITY, T2 = -INFINITY;
  int I1 = -1;
  for (int s = t; s < a.nsplit; s += RED_THREADS) {
    const float* ps = part + s * PART_FLOATS;
    const float f = __expf(wsm[s] - M);
    wsm[s] = f;
    L += f * ps[P_L];
    EV += f * ps[P_EV];
    EVM = fmaxf(EVM, f * ps[P_EVMAX]);
    DM = fmaxf(DM, ps[P_DMAX]);
    VM = fmaxf(VM, ps[P_VMAX]);
    top2_merge(T1, I1, T2, ps[P_T1], __float_as_int(ps[P_I1]), ps[P_T2]);
  }
  L = block_sum(L, scratch4);
  EV = block_sum(EV, scratch4);
  EVM = block_max(EVM, scratch4);
  DM = block_max(DM, scratch4);
  VM = block_max(VM, scratch4);
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    const float u1 = __shfl_xor(T1, m), u2 = __shfl_xor(T2, m);
    const int j1 = __shfl_xor(I1, m);
    top2_merge(T1, I1, T2, u1, j1, u2);
  }
  if (l == 0) {
    t2s[w][0] = T1;
    t2s[w][1] = T2;
    t2s[w][2] = __int_as_float(I1);
  }
  __syncthreads();   // also publishes wsm
  T1 = t2s[0][0];
  T2 = t2s[0][1];
  I1 = __float_as_int(t2s[0][2]);
#pragma unroll
  for (int ww = 1; ww < 4; ++ww)
    top2_merge(T1, I1, T2, t2s[ww][0], __float_as_int(t2s[ww][2]), t2s[ww][1]);

  // ---- weighted sum of the partial outputs: wave w takes splits w, w+4, ...; lane l channels 2l, 2l+1
  float2 o2 = make_float2(0.0f, 0.0f);
#pragma unroll 4
  for (int s = w; s < a.nsplit; s += 4) {
    const float f = wsm[s];
    const float2 x = reinterpret_cast<const float2*>(part + s * PART_FLOATS + P_O)[l];
    o2.x = fmaf(f, x.x, o2.x);
    o2.y = fmaf(f, x.y, o2.y);
  }
  reinterpret_cast<float2*>(&osum[w][0])[l] = o2;
  __syncthreads();
  float o = (osum[0][c] + osum[1][c]) + (osum[2][c] + osum[3][c]);
  float L_sealed = L;

  // ---- trailing FP16 tokens: exact keys and values, eta = 0
  if (a.r > 0) {
    const float qc = own ? __half2float(a.q[((int64_t)b * a.n_q + hq) * D + c]) : 0.0f;
    const __half* tk = a.trail_k + ((int64_t)b * a.n_kv + kvh) * BLK * D;
    const __half* tv = a.trail_v + ((int64_t)b * a.n_kv + kvh) * BLK * D;
    float st[BLK - 1];
    float vt[BLK - 1];
    float mt = -INFINITY;
    for (int tt = 0; tt < a.r; ++tt) {
      vt[tt] = own ? __half2float(tv[tt * D + c]) : 0.0f;
      st[tt] = block_sum(qc * __half2float(tk[tt * D + c]), scratch4) * inv_sqrt_d;
      mt = fmaxf(mt, st[tt]);
      const float n2 = block_sum(vt[tt] * vt[tt], scratch4);
      VM = fmaxf(VM, sqrtf(n2));
    }
    const float M2 = fmaxf(M, mt);
    const float fs = __expf(M - M2);
    L *= fs;
    o *= fs;
    EV *= fs;
    EVM *= fs;
    L_sealed = L;
    for (int tt = 0; tt < a.r; ++tt) {
      const float pt = __expf(st[tt] - M2);
      L += pt;
      o = fmaf(pt, vt[tt], o);
    }
    M = M2;
  }

  const float out = o / L;
  if (own) a.O[((int64_t)b * a.n_q + hq) * D + c] = out;
  const int bad = __syncthreads_or(!isfinite(out));

  if (t == 0) {
    const double Ld = (double)L;
    const double e_val = (double)EV / Ld;
    const double maxc = (double)EVM / Ld;
    const double lse = (double)M + log(Ld);
    const double alpha_hat = (double)L_sealed / Ld;
    const double delta = (double)DM;
    const double vmax = (double)VM;
    double t_tail = 0.0;
    if (alpha_hat > 0.0 && delta != 0.0) {
      const double grow = exp(fmin((double)a.tol.mass_exp * delta, 700.0));
      const double widen = expm1(fmin(2.0 * delta, 700.0));
      t_tail = fmin(1.0, grow * alpha_hat) * widen;
    }
    const double t_full = tanh(delta);
    double tv = a.tol.key_bound_mode == 0 ? fmin(t_full, t_tail)
                                          : (a.tol.key_bound_mode == 1 ? t_tail : t_full);
    const double e_key = 2.0 * vmax * tv;
    const double margin = a.nb >= 2 ? (double)T1 - (double)T2 : (double)INFINITY;
    const double rho_top = a.nb >= 1 ? exp((double)T1 - lse) : 0.0;

    uint32_t fl = 0;
    if (e_key > (double)a.tol.eps_key) fl |= CQA_FLAG_KEY;
    if (e_val > (double)a.tol.eps_val || maxc > (double)a.tol.v_tol) fl |= CQA_FLAG_VAL;
    if (a.tol.rank_depth >= 1 && a.nb >= 2 && rho_top >= (double)a.tol.rank_min_mass &&
        margin <= 2.0 * delta + (double)a.tol.eps_guard)
      fl |= CQA_FLAG_RANK;
    if (bad || !isfinite(e_key) || !isfinite(e_val) || !isfinite(delta) || !isfinite(vmax) ||
        !isfinite(lse))
      fl |= CQA_FLAG_PRECOND;
    if (e_key + e_val > (double)a.tol.eps_total) fl |= CQA_FLAG_TOTAL;
    fl |= a.tol.force_flags;

    cqa_head_cert ct;
    ct.E_key = (float)e_key;
    ct.E_val = (float)e_val;
    ct.delta_h = DM;
    ct.v_max = VM;
    ct.alpha_tail_hat = (float)alpha_hat;
    ct.lse = (float)lse;
    ct.max_block_contrib = (float)maxc;
    ct.rank_margin = (float)margin;
    ct.top_block = I1;
    ct.served_rung = 0;
    a.cert[(int64_t)b * a.n_q + hq] = ct;
    a.flags[(int64_t)b * a.n_q + hq] = fl;
  }
}

// Workgroups ("splits") per (batch, kv-head) and, for the vector-ALU kernel, blocks per split.
// The launch is sized to ONE resident generation: two workgroups of four waves per compute unit
// (the matrix-core kernel runs at two waves per SIMD), so no workgroup waits for a slot and the
// per-wave start-up latency is paid once.  The matrix-core kernel deals the head's quads of
// blocks evenly over all 4 * nsplit waves; short sequences get fewer workgroups so that every
// wave still has at least one quad.
void split_geometry(const Cache* c, int64_t n_blocks, int* nsplit, int* bps) {
  *nsplit = 0;
  *bps = 0;
  if (n_blocks <= 0) return;
  const int64_t heads = (int64_t)c->desc.batch * c->desc.n_kv_heads;
  int64_t want = c->forced_splits > 0 ? c->forced_splits : (2 * (int64_t)c->n_cu + heads - 1) / heads;
  if (want < 1) want = 1;
  if (want > c->max_splits) want = c->max_splits;
  if (want > MAX_SPLITS) want = MAX_SPLITS;
  const int64_t quads = (n_blocks + 3) / 4;
  const int64_t cap = (quads + 3) / 4;   // at least one quad per wave
  if (want > cap) want = cap;
  *nsplit = (int)want;
  *bps = (int)((n_blocks + want - 1) / want);
}

int pick_splits(const Cache* c, int64_t n_blocks) {
  int nsplit = 0, bps = 0;
  split_geometry(c, n_blocks, &nsplit, &bps);
  return nsplit;
}

int32_t launch_certified(Cache* c, int layer, const __half* q, const cqa_tolerances& tol, float* O,
                         cqa_head_cert* cert, uint32_t* flags, float* blk_logmass, hipStream_t st) {
  const int bt = c->desc.batch, hq = c->desc.n_q_heads, hkv = c->desc.n_kv_heads;
  const int64_t len = c->length[layer];
  const int64_t nb = len / BLK;
  const int r = (int)(len % BLK);
  int nsplit = 0, bps = 0;
  split_geometry(c, nb, &nsplit, &bps);
  const int64_t layer_head0 = head_index(c, layer, 0, 0);
  if (nb > 0) {
    DecodeArgs a;
    a.kc = c->kc + layer_head0 * c->nb_cap * KC_BYTES;
    a.km = c->km + layer_head0 * c->nb_cap * (KM_BYTES / 4);
    a.vc = c->vc + layer_head0 * c->nb_cap * VC_BYTES;
    a.vm = c->vm + layer_head0 * c->nb_cap * (VM_BYTES / 2);
    a.an = c->an + layer_head0 * c->nb_cap * 2;
    a.sigmax = c->sigmax + layer_head0;
    a.q = q;
    a.partials = c->partials;
    a.blk_logmass = blk_logmass;
    a.nb_cap = c->nb_cap;
    a.nb = (int)nb;
    a.nsplit = nsplit;
    a.bps = bps;
    a.n_q = hq;
    a.n_kv = hkv;
    a.debug = c->debug;
    const dim3 grid(nsplit, hkv, bt);
    const bool prof = c->prof_ev != nullptr && c->prof_n < c->prof_cap;
    if (prof) CQA_HIP(hipEventRecord(c->prof_ev[2 * c->prof_n], st));
    if (c->variant == 0) {
      const int32_t rc = launch_split_mfma(a, hq / hkv, grid, st);
      if (rc != CQA_OK) return rc;
    } else {
      switch (hq / hkv) {
        case 1: hipLaunchKernelGGL(certified_split_kernel<1>, grid, dim3(256), 0, st, a); break;
        case 2: hipLaunchKernelGGL(certified_split_kernel<2>, grid, dim3(256), 0, st, a); break;
        case 4: hipLaunchKernelGGL(certified_split_kernel<4>, grid, dim3(256), 0, st, a); break;
        default: return CQA_ERR_UNSUPPORTED;
      }
    }
    CQA_HIP(hipGetLastError());
    if (prof) {
      CQA_HIP(hipEventRecord(c->prof_ev[2 * c->prof_n + 1], st));
      ++c->prof_n;
    }
  }
  ReduceArgs ra;
  ra.partials = c->partials;
  ra.q = q;
  ra.trail_k = c->trail_k + layer_head0 * BLK * D;
  ra.trail_v = c->trail_v + layer_head0 * BLK * D;
  ra.O = O;
  ra.cert = cert;
  ra.flags = flags;
  ra.tol = tol;
  ra.nsplit = nsplit;
  ra.nb = (int)nb;
  ra.r = r;
  ra.n_q = hq;
  ra.n_kv = hkv;
  hipLaunchKernelGGL(certified_reduce_kernel, dim3(hq, bt), dim3(RED_THREADS), 0, st, ra);
  CQA_HIP(hipGetLastError());
  return CQA_OK;
}

}  // namespace cqa
