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
#include <mutex>

#include "cqa_internal.h"
#include "reduce_inl.h"

namespace cqa {

// PROM = false: the vector-ALU split pass over a contiguous range of sealed blocks (INT8 keys).
// PROM = true : the promoted-block pass of the adaptive decode (gated precision): the workgroups
//               of a KV group walk the group's list of promoted blocks.  A key-promoted block is
//               scored from its FP16 keys (sigma = 1, z = 0, no score error), a value-promoted
//               block is attended from its FP16 values and counts with eta_b = 0; both kinds of
//               originals are read by the device straight from the pinned Tier-2 arrays over the
//               host link.  Writes partial sets split0 + blockIdx.x.
template <int G, bool PROM>
__global__ __launch_bounds__(256) void certified_split_kernel(DecodeArgs a) {
  const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int tok = l & 15, kg = l >> 4;              // roles in the score phase
  const int vn = l & 15, vgh = (l >> 4) & 1, vo = l >> 5;  // roles in the value phase
  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int64_t head_rec = ((int64_t)b * a.n_kv + kvh) * a.nq_cap;
  // blocks are dealt evenly over the splits (every split gets at least one: nsplit <= nb)
  const int64_t grp = (int64_t)b * a.n_kv + kvh;
  // PROM: positions split * 4 + w, + 4 * gridDim.x, ... of the group's list; else a block range
  // PROM: the second half of the workgroups (neg) walks the same list with INT8 keys and INT4
  // values whatever the flags say and writes its partial set negated: it takes back what the one
  // pass over all sealed blocks added for the listed blocks, the first half adds them again with
  // the originals the flags ask for.
  const bool neg = PROM && split >= (int)gridDim.x / 2;
  const int psplit = PROM ? (neg ? split - (int)gridDim.x / 2 : split) : split;
  const int b0 = PROM ? psplit * 4 : (int)(((int64_t)split * a.nb) / a.nsplit);
  const int b1 = PROM ? min(a.ucount[grp], MAX_UNION) : (int)(((int64_t)(split + 1) * a.nb) / a.nsplit);
  const int bstep = PROM ? 2 * (int)gridDim.x : 4;   // PROM: 4 waves x gridDim.x / 2 workgroups
  const int out_split = PROM ? a.split0 + split : split;
  const float inv_sqrt_d = 0.08838834764831845f;  // 1 / sqrt(128)

  __shared__ __align__(16) float qs[4][G][D];     // scaled query of the block in flight, per wave
  __shared__ __align__(16) float ps[4][BLK][G];   // its probabilities
  __shared__ float ms[4][G][12];                  // per-wave scalars for the merge
  // FP16 values of a value-promoted block, one buffer per wave (rows padded against bank conflicts)
  __shared__ __align__(16) __half vst[PROM ? 4 : 1][PROM ? BLK : 1][PROM ? D + 8 : 8];

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
  float dev[G];               // canary: largest |s_fp16 - s_int8| seen on key-promoted tokens
#pragma unroll
  for (int h = 0; h < G; ++h) dev[h] = 0.0f;
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

  // the list entry of the next iteration is requested one iteration ahead
  int blk_next = (PROM && b0 + w < b1) ? a.ulist[grp * MAX_UNION + b0 + w] : b0 + w;
  for (int pos = b0 + w; pos < b1; pos += bstep) {
    // every index is bounded on the way in: a list entry outside [0, nb) is skipped
    const int blk = blk_next;
    blk_next = (PROM && pos + bstep < b1) ? a.ulist[grp * MAX_UNION + pos + bstep] : pos + bstep;
    if (PROM && (blk < 0 || blk >= a.nb)) continue;
    // Every load of the block is requested here, before anything is consumed: the block sits at
    // an address nothing else in this launch touches, so each dependent load costs a full
    // memory (and page-walk) latency.  First everything whose address follows from blk alone
    // (flags, INT8 codes, key and value metadata, INT4 codes), then the originals the flags ask
    // for.
    const int pf = PROM ? a.slot[grp * (a.nq_cap * 4) + blk] : 0;   // bit 0: FP16 keys, bit 1: FP16 values
    const float* kmb = reinterpret_cast<const float*>(a.t1 + t1_offset(head_rec, blk, Q_KM, KM_BYTES));
    const float2 sg8 = reinterpret_cast<const float2*>(kmb)[l];
    const float2 zz8 = reinterpret_cast<const float2*>(kmb + D)[l];
    float2 an = *reinterpret_cast<const float2*>(a.t1 + t1_offset(head_rec, blk, Q_AN, AN_BYTES));
    const uint8_t* kcb = a.t1 + t1_offset(head_rec, blk, Q_KC, KC_BYTES);
    uint4 kc8[2];
#pragma unroll
    for (int cq = 0; cq < 2; ++cq) kc8[cq] = reinterpret_cast<const uint4*>(kcb + cq * 1024)[l];
    const uint4 vx = reinterpret_cast<const uint4*>(a.t1 + t1_offset(head_rec, blk, Q_VC, VC_BYTES))[l];
    const __half* vmb = reinterpret_cast<const __half*>(a.t1 + t1_offset(head_rec, blk, Q_VM, VM_BYTES));
    uint4 sraw4[4], oraw4[4];
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const int g = vgh * 4 + gq;
      sraw4[gq] = *reinterpret_cast<const uint4*>(vmb + vo * 64 + g * 8);
      oraw4[gq] = *reinterpret_cast<const uint4*>(vmb + BLK * NG + vo * 64 + g * 8);
    }
    // which heads of the group score this block with FP16 keys / attend its FP16 values (the
    // per-head bits of the flag word; with per-group promotion they are all alike)
    const int hkb = (PROM && !neg) ? (pf >> SLOT_HK_SHIFT) & ((1 << G) - 1) : 0;
    const int hvb = (PROM && !neg) ? (pf >> SLOT_HV_SHIFT) & ((1 << G) - 1) : 0;
    const bool kfp = hkb != 0, vfp = hvb != 0;
    const bool kall = hkb == (1 << G) - 1;
    // FP16 keys of the block, [token][128 channels]: from its slot of the device-resident
    // scratch if it is held there, else from the host-resident originals -- and then, if the
    // block has just been given a slot, stored into it on the way
    uint4 k16[2][2];
    const int sc0 = (pf >> SLOT_SC_SHIFT) & 0xFFFF;   // bits 8-23: scratch slot + 1
    const int sc = (PROM && a.sc_k != nullptr && sc0 <= a.sc_cap) ? sc0 : 0;   // bounded whatever the word holds
    if (kfp) {
      const bool fill = sc > 0 && (pf & SLOT_FILL);
      __half* sck = sc > 0 ? a.sc_k + (((grp * a.sc_cap + (sc - 1)) * BLK) + tok) * D : nullptr;
      const __half* kf16 = (sc > 0 && !fill) ? sck
                                             : a.t2_k + ((grp * a.max_tokens + (int64_t)blk * BLK) + tok) * D;
#pragma unroll
      for (int cq = 0; cq < 2; ++cq) {
        const int c0 = cq * 64 + kg * 16;
        k16[cq][0] = *reinterpret_cast<const uint4*>(kf16 + c0);
        k16[cq][1] = *reinterpret_cast<const uint4*>(kf16 + c0 + 8);
      }
      if (fill) {
#pragma unroll
        for (int cq = 0; cq < 2; ++cq) {
          const int c0 = cq * 64 + kg * 16;
          *reinterpret_cast<uint4*>(sck + c0) = k16[cq][0];
          *reinterpret_cast<uint4*>(sck + c0 + 8) = k16[cq][1];
        }
      }
    }
    if (vfp) {
      // its FP16 values, row-major [token][128], coalesced into this wave's LDS buffer: from the
      // value half of the block's scratch slot, or from the host-resident originals (and then
      // into the slot, if the block has just been given one)
      const bool vfill = sc > 0 && (pf & SLOT_VFILL);
      const int64_t in_blk = (int64_t)(l >> 2) * D + (l & 3) * 32;
      __half* scv = sc > 0 ? a.sc_v + (grp * a.sc_cap + (sc - 1)) * (int64_t)(BLK * D) + in_blk : nullptr;
      const __half* v16 = (sc > 0 && !vfill) ? scv
                                             : a.t2_v + (grp * a.max_tokens + (int64_t)blk * BLK) * D + in_blk;
      uint4 v16r[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) v16r[j] = *reinterpret_cast<const uint4*>(v16 + j * 8);
      if (vfill) {
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<uint4*>(scv + j * 8) = v16r[j];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        *reinterpret_cast<uint4*>(&vst[w][l >> 2][(l & 3) * 32 + j * 8]) = v16r[j];
    }
    // ---- scores.  Lane (tok, kg) covers channels cq*64 + kg*16 + 0..15, cq = 0, 1.  First from
    //      the FP16 keys (sigma = 1, z = 0: the query itself in the LDS buffer) when some head asks
    //      for them, then from the INT8 codes (scaled query q~ = q sigma, block constant
    //      c_b = q.z, bound Delta_b) when some head keeps them -- or when the score-consistency
    //      check compares the two.
    float s16[G], s8[G], dsum[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      s16[h] = 0.0f;
      s8[h] = 0.0f;
      dsum[h] = 0.0f;
    }
    if (kfp) {
#pragma unroll
      for (int h = 0; h < G; ++h)
        reinterpret_cast<float2*>(&qs[w][h][0])[l] = make_float2(qv[h][0], qv[h][1]);
      wave_sync();
      float dot[G];
#pragma unroll
      for (int h = 0; h < G; ++h) dot[h] = 0.0f;
#pragma unroll
      for (int cq = 0; cq < 2; ++cq) {
        const int c0 = cq * 64 + kg * 16;
        const __half2* h0 = reinterpret_cast<const __half2*>(&k16[cq][0]);
        const __half2* h1 = reinterpret_cast<const __half2*>(&k16[cq][1]);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const __half2 pr = (j < 8) ? h0[j >> 1] : h1[(j - 8) >> 1];
          const float kf = (j & 1) ? __high2float(pr) : __low2float(pr);
#pragma unroll
          for (int h = 0; h < G; ++h) dot[h] = fmaf(qs[w][h][c0 + j], kf, dot[h]);
        }
      }
#pragma unroll
      for (int h = 0; h < G; ++h) {
        dot[h] += __shfl_xor(dot[h], 16);
        dot[h] += __shfl_xor(dot[h], 32);
        s16[h] = dot[h] * inv_sqrt_d;
      }
      wave_sync();   // the LDS buffer is rewritten below
    }
    const bool canary = PROM && kfp && a.score_dev != nullptr;
    if (!kfp || !kall || canary) {
      // a.int8_query: the scaled query is quantised to 8 bits per (head, block) exactly as the pass
      // over all blocks does it (binary32 decisions: s_q = max|q~| / 127, T = round-half-even of
      // q~ * fl(127 / max)), the codes T take the scaled query's place in the dot product, which is
      // then exact integer arithmetic, and the residual sum |q~ - s_q T| widens the block's bound
      float csum[G], tsum[G], rsum[G], sqv[G];
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float q0 = qv[h][0] * sg8.x, q1 = qv[h][1] * sg8.y;
        dsum[h] = fabsf(qv[h][0]) * sg8.x + fabsf(qv[h][1]) * sg8.y;
        tsum[h] = 0.0f;
        rsum[h] = 0.0f;
        sqv[h] = 1.0f;
        if (a.int8_query) {
          float amax = fmaxf(fabsf(q0), fabsf(q1));
#pragma unroll
          for (int m = 1; m < 64; m <<= 1) amax = fmaxf(amax, __shfl_xor(amax, m));
          const float inv = amax > 0.0f ? 127.0f / amax : 0.0f;
          const float sq = amax / 127.0f;
          const float MAGIC = 12582912.0f;   // 1.5 * 2^23: fl(x + MAGIC) - MAGIC = round-half-even(x)
          const float t0 = fmaf(q0, inv, MAGIC) - MAGIC, t1 = fmaf(q1, inv, MAGIC) - MAGIC;
          rsum[h] = fabsf(fmaf(-sq, t0, q0)) + fabsf(fmaf(-sq, t1, q1));
          q0 = t0;
          q1 = t1;
          tsum[h] = t0 + t1;                 // small integers: every partial sum below is exact
          sqv[h] = sq;
          csum[h] = qv[h][0] * zz8.x + qv[h][1] * zz8.y;
        } else {
          // stored bytes are code + 128: fold the -128 * sum(q~) into the block constant
          csum[h] = qv[h][0] * zz8.x + qv[h][1] * zz8.y - 128.0f * (q0 + q1);
        }
        reinterpret_cast<float2*>(&qs[w][h][0])[l] = make_float2(q0, q1);
      }
#pragma unroll
      for (int m = 1; m < 64; m <<= 1) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
          csum[h] += __shfl_xor(csum[h], m);
          dsum[h] += __shfl_xor(dsum[h], m);
          if (a.int8_query) {
            tsum[h] += __shfl_xor(tsum[h], m);
            rsum[h] += __shfl_xor(rsum[h], m);
          }
        }
      }
      if (a.int8_query) {
#pragma unroll
        for (int h = 0; h < G; ++h) dsum[h] = fmaf(256.0f, rsum[h], dsum[h]);   // (Delta_b + Delta^q_b) * 2 sqrt d
      }
      wave_sync();
      float dot[G];
#pragma unroll
      for (int h = 0; h < G; ++h) dot[h] = 0.0f;
#pragma unroll
      for (int cq = 0; cq < 2; ++cq) {
        const uint32_t wd[4] = {kc8[cq].x, kc8[cq].y, kc8[cq].z, kc8[cq].w};
        const int c0 = cq * 64 + kg * 16;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const float kf = (float)((wd[j >> 2] >> (8 * (j & 3))) & 0xffu);
#pragma unroll
          for (int h = 0; h < G; ++h) dot[h] = fmaf(qs[w][h][c0 + j], kf, dot[h]);
        }
      }
#pragma unroll
      for (int h = 0; h < G; ++h) {
        dot[h] += __shfl_xor(dot[h], 16);
        dot[h] += __shfl_xor(dot[h], 32);
        // quantised query: s_q * (sum T byte - 128 sum T) + q.z, the bracket in exact integers
        s8[h] = fmaf(sqv[h], dot[h] - 128.0f * tsum[h], csum[h]) * inv_sqrt_d;
      }
    }
    if (canary) {
      // score-consistency check: FP16 against INT8 scores, token by token, for the heads that
      // score this block from its FP16 keys
#pragma unroll
      for (int h = 0; h < G; ++h)
        if ((hkb >> h) & 1) dev[h] = fmaxf(dev[h], fabsf(s16[h] - s8[h]));
    }
    float p[G], alpha[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const bool use16 = ((hkb >> h) & 1) != 0;
      const float s = use16 ? s16[h] : s8[h];
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
      const float ce = ((hvb >> h) & 1) ? 0.0f : sf * an.x;   // exact values add nothing to the value term
      l_run[h] = l_run[h] * alpha[h] + sf;
      ev[h] = ev[h] * alpha[h] + ce;
      evmax[h] = fmaxf(evmax[h] * alpha[h], ce);
      dmax[h] = fmaxf(dmax[h], use16 ? 0.0f : dsum[h] * (0.5f * inv_sqrt_d));
      m_run[h] = m_new;
      if (lb > t1[h]) {
        t2[h] = t1[h];
        t1[h] = lb;
        i1[h] = blk;
      } else if (lb > t2[h]) {
        t2[h] = lb;
      }
      if (a.blk_logmass != nullptr && l == 0 && !neg)
        a.blk_logmass[((int64_t)b * a.n_q + kvh * G + h) * a.nb + blk] = lb;
      if (kg == 0) ps[w][tok][h] = p[h];
    }
    vmax = fmaxf(vmax, an.y);
    wave_sync();

    // ---- values: lane (vo, vgh, vn) covers tokens vo*8..+7 of channels (vgh*4+gq)*16 + vn
    const uint32_t vw[4] = {vx.x, vx.y, vx.z, vx.w};
    float pi[8][G];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int h = 0; h < G; ++h) pi[i][h] = ps[w][vo * 8 + i][h];
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const int g = vgh * 4 + gq;
      const __half2* sh = reinterpret_cast<const __half2*>(&sraw4[gq]);
      const __half2* oh = reinterpret_cast<const __half2*>(&oraw4[gq]);
#pragma unroll
      for (int h = 0; h < G; ++h) acc[gq][h] *= alpha[h];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float sc = (i & 1) ? __high2float(sh[i >> 1]) : __low2float(sh[i >> 1]);
        const float of = (i & 1) ? __high2float(oh[i >> 1]) : __low2float(oh[i >> 1]);
        const float v4 = fmaf((float)((vw[gq] >> (4 * i)) & 15u), sc, of);
        const float v16 = vfp ? __half2float(vst[w][vo * 8 + i][g * 16 + vn]) : v4;
#pragma unroll
        for (int h = 0; h < G; ++h) acc[gq][h] = fmaf(pi[i][h], ((hvb >> h) & 1) ? v16 : v4, acc[gq][h]);
      }
    }
    wave_sync();
  }

  if (PROM && a.score_dev != nullptr) {
    // deviations are non-negative floats: their bit patterns order like integers
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float d = dev[h];
#pragma unroll
      for (int m = 1; m < 64; m <<= 1) d = fmaxf(d, __shfl_xor(d, m));
      if (l == 0 && d > 0.0f)
        atomicMax(reinterpret_cast<int*>(a.score_dev + (int64_t)b * a.n_q + kvh * G + h), __float_as_int(d));
    }
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
    const float Mr = (M == -INFINITY) ? 0.0f : M;   // a workgroup without blocks writes zeros
    float o = 0.0f;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) o += __expf(ms[ww][h][0] - Mr) * mo[(ww * G + h) * D + c];
    a.partials[(((int64_t)b * a.n_q + kvh * G + h) * a.pstride + out_split) * PART_FLOATS + P_O + c] =
        neg ? -o : o;
  }
  if (threadIdx.x < G) {
    const int h = threadIdx.x;
    float M = -INFINITY;
    for (int ww = 0; ww < 4; ++ww) M = fmaxf(M, ms[ww][h][0]);
    const float Mr = (M == -INFINITY) ? 0.0f : M;
    float L = 0.0f, EV = 0.0f, EVM = 0.0f, DM = 0.0f, VM = 0.0f, T1 = -INFINITY, T2 = -INFINITY;
    int I1 = -1;
    for (int ww = 0; ww < 4; ++ww) {
      const float f = __expf(ms[ww][h][0] - Mr);
      L += f * ms[ww][h][1];
      EV += f * ms[ww][h][2];
      EVM = fmaxf(EVM, f * ms[ww][h][3]);
      DM = fmaxf(DM, ms[ww][h][4]);
      VM = fmaxf(VM, ms[ww][h][5]);
      top2_merge(T1, I1, T2, ms[ww][h][6], __float_as_int(ms[ww][h][8]), ms[ww][h][7]);
    }
    float* pp = a.partials + (((int64_t)b * a.n_q + kvh * G + h) * a.pstride + out_split) * PART_FLOATS;
    pp[P_M] = M;
    pp[P_L] = neg ? -L : L;
    pp[P_EV] = neg ? -EV : EV;
    pp[P_EVMAX] = neg ? 0.0f : EVM;
    pp[P_DMAX] = DM;
    pp[P_VMAX] = VM;
    pp[P_T1] = T1;
    pp[P_T2] = T2;
    pp[P_I1] = __int_as_float(I1);
  }
}

// Stand-alone cross-split reduction: one wave per (batch, query head); any number of waves per
// workgroup.
__global__ __launch_bounds__(256) void certified_reduce_kernel(ReduceArgs a) {
  __shared__ float wsm[4][64];
  const int w = threadIdx.x >> 6;
  const int hq = blockIdx.x * (int)(blockDim.x >> 6) + w, b = blockIdx.y;
  if (hq < a.n_q) reduce_head_wave(a, b, hq, wsm[w]);
}

// Waves per workgroup of the matrix-core split pass.  Eight -- one workgroup per compute unit, two
// waves per SIMD -- as long as there are no more (batch, kv-head) sequences than compute units: all
// of a launch's waves are then dispatched in one sweep (with two workgroups of four waves per
// compute unit the second one started ~2 us after the first and finished as much later), and a head
// has half as many partial sets to merge.  With more sequences than compute units every sequence is
// one workgroup anyway, and workgroups of four waves, two per compute unit, keep the launch at one
// resident generation for up to twice as many of them.
int waves_per_workgroup(const Cache* c) {
  return (int64_t)c->desc.batch * c->desc.n_kv_heads > c->n_cu ? 4 : 8;
}

// Workgroups ("splits") per (batch, kv-head) and, for the vector-ALU kernel, blocks per split.
// The launch is sized to ONE resident generation (the matrix-core kernel runs at two waves per
// SIMD), so no workgroup waits for a slot and the per-wave start-up latency is paid once.  The
// matrix-core kernel deals the head's quads of blocks evenly over all wpb * nsplit waves; short
// sequences get fewer workgroups so that every workgroup still has a quad.
void split_geometry(const Cache* c, int64_t n_blocks, int* nsplit, int* bps) {
  *nsplit = 0;
  *bps = 0;
  if (n_blocks <= 0) return;
  const int64_t heads = (int64_t)c->desc.batch * c->desc.n_kv_heads;
  const int wpb = waves_per_workgroup(c);
  int64_t want = c->forced_splits > 0 ? c->forced_splits
                                      : ((8 / wpb) * (int64_t)c->n_cu + heads - 1) / heads;
  if (want < 1) want = 1;
  if (want > c->max_splits) want = c->max_splits;
  if (want > MAX_SPLITS) want = MAX_SPLITS;
  const int64_t quads = (n_blocks + 3) / 4;
  const int64_t cap = (quads + wpb - 1) / wpb;   // at least one quad per workgroup's wave
  if (want > cap) want = cap;
  *nsplit = (int)want;
  *bps = (int)((n_blocks + want - 1) / want);
}

// Whether the matrix-core pass reads Tier-1 with the non-temporal hint.  One decode step of a
// model walks every layer, so the bytes read between two visits of the same record are one
// pass's bytes times the layer count.  Up to about the size of the memory-side cache (256 MB)
// plain loads gain from what is left there from the previous step (measured: 51.8 against
// 52.5 us at 303 MB); beyond it the hinted loads stream faster (98 against 109 us at 606 MB).
int stream_nt(const Cache* c, int64_t n_blocks) {
  if (c->stream_hint == 1) return 0;
  if (c->stream_hint == 2) return 1;
  const int64_t pass = (int64_t)c->desc.batch * c->desc.n_kv_heads * ((n_blocks + 3) / 4) * QUAD_BYTES;
  return pass * c->desc.n_layers > ((int64_t)384 << 20) ? 1 : 0;
}

int pick_splits(const Cache* c, int64_t n_blocks) {
  int nsplit = 0, bps = 0;
  split_geometry(c, n_blocks, &nsplit, &bps);
  return nsplit;
}

// Promoted-block pass of the adaptive decode (see certified_split_kernel).
int32_t launch_promoted_pass(const DecodeArgs& a, int group, dim3 grid, hipStream_t st) {
  if (a.ulist == nullptr || a.ucount == nullptr || a.slot == nullptr || a.t2_k == nullptr ||
      a.t2_v == nullptr)
    return CQA_ERR_INVALID_ARG;
  switch (group) {
    case 1: hipLaunchKernelGGL((certified_split_kernel<1, true>), grid, dim3(256), 0, st, a); break;
    case 2: hipLaunchKernelGGL((certified_split_kernel<2, true>), grid, dim3(256), 0, st, a); break;
    case 4: hipLaunchKernelGGL((certified_split_kernel<4, true>), grid, dim3(256), 0, st, a); break;
    default: return CQA_ERR_UNSUPPORTED;
  }
  CQA_HIP(hipGetLastError());
  return CQA_OK;
}

// Split partials of callers that must not allocate: one array per GPU, placed by the loader when
// the code object is loaded on that GPU and held until the process ends.  In host code the name
// `scratch` is only a handle for hipGetSymbolAddress; kernels receive the resolved address.
constexpr int64_t STATIC_SCRATCH_BYTES = CQA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES];   // per device: address of its copy of `scratch` (null = not resolved yet)
static std::mutex g_scratch_mutex;

// Address of the current device's copy of the static scratch; resolved once per device, with that
// device current (cqa_cache_create does it for the device it creates the cache on).
int32_t static_scratch(int device, void** out) {
  if (device < 0 || device >= MAX_DEVICES) return CQA_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[device] == nullptr) {
    int cur = -1;
    CQA_HIP(hipGetDevice(&cur));
    if (cur != device) return CQA_ERR_INVALID_ARG;
    void* p = nullptr;
    CQA_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return CQA_ERR_HIP;
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return CQA_OK;
}

int32_t launch_certified(Cache* c, int layer, const __half* q, const cqa_tolerances& tol, float* O,
                         cqa_head_cert* cert, uint32_t* flags, uint32_t* flags_mirror,
                         uint32_t mirror_tag, float* blk_logmass, hipStream_t st,
                         const __half* k_new, const __half* v_new, int pstride, float* eta_out,
                         float* partials) {
  const int bt = c->desc.batch, hq = c->desc.n_q_heads, hkv = c->desc.n_kv_heads;
  if (partials == nullptr) partials = c->partials;
  const int64_t len = c->length[layer];
  const int64_t nb = len / BLK;
  const int r = (int)(len % BLK);
  int nsplit = 0, bps = 0;
  split_geometry(c, nb, &nsplit, &bps);
  const int64_t layer_head0 = head_index(c, layer, 0, 0);
  ReduceArgs ra{};
  ra.partials = partials;
  ra.q = q;
  ra.trail_k = c->trail_k + layer_head0 * BLK * D;
  ra.trail_v = c->trail_v + layer_head0 * BLK * D;
  ra.O = O;
  ra.cert = cert;
  ra.flags = flags;
  ra.flags_mirror = flags_mirror;
  ra.mirror_tag = mirror_tag;
  ra.tol = tol;
  ra.nsplit = nsplit;
  ra.pstride = pstride;
  ra.nb = (int)nb;
  ra.r = r;
  ra.n_q = hq;
  ra.n_kv = hkv;
  if (nb > 0) {
    DecodeArgs a{};   // every field starts null / zero
    a.t1 = c->t1 + layer_head0 * c->nq_cap * QUAD_BYTES;
    a.sigmax = c->sigmax + layer_head0;
    a.q = q;
    a.partials = partials;
    a.blk_logmass = blk_logmass;
    a.nq_cap = c->nq_cap;
    a.nb = (int)nb;
    a.nsplit = nsplit;
    a.pstride = pstride > 0 ? pstride : nsplit;
    a.slot = nullptr;
    a.ulist = nullptr;
    a.ucount = nullptr;
    a.t2_k = nullptr;
    a.t2_v = nullptr;
    a.eta_out = nullptr;
    a.score_dev = nullptr;
    a.max_tokens = 0;
    a.split0 = 0;
    a.eta_out = blk_logmass != nullptr ? eta_out : nullptr;
    if (k_new != nullptr) {
      // the caller has already counted the new token in length[layer]: it is token len - 1
      if (c->variant != 0 || r == 0) return CQA_ERR_INVALID_ARG;   // needs this kernel and an open block
      a.ap_k_new = k_new;
      a.ap_v_new = v_new;
      a.ap_trail_k = c->trail_k + layer_head0 * BLK * D;
      a.ap_trail_v = c->trail_v + layer_head0 * BLK * D;
      const bool t2 = c->desc.tier2_mode == CQA_TIER2_PINNED;
      a.ap_t2_k = t2 ? c->t2_k + layer_head0 * c->desc.max_tokens * D : nullptr;
      a.ap_t2_v = t2 ? c->t2_v + layer_head0 * c->desc.max_tokens * D : nullptr;
      a.ap_slot = r - 1;
      a.ap_pos = len - 1;
      a.ap_max_tokens = c->desc.max_tokens;
    }
    a.bps = bps;
    a.n_q = hq;
    a.n_kv = hkv;
    a.stream_nt = stream_nt(c, nb);
    a.int8_query = tol.int8_query;
    a.wpb = waves_per_workgroup(c);
    // the quantised-query scoring exists in the matrix-core pass (and in the promoted-block pass of
    // the adaptive calls), not in the vector-ALU cross-check kernel
    if (tol.int8_query != 0 && c->variant != 0) return CQA_ERR_UNSUPPORTED;
    const dim3 grid(nsplit, hkv, bt);
    const bool prof = c->prof_ev != nullptr && c->prof_n < c->prof_cap;
    hipEvent_t ev0 = prof ? c->prof_ev[2 * c->prof_n] : nullptr;
    hipEvent_t ev1 = prof ? c->prof_ev[2 * c->prof_n + 1] : nullptr;
    if (prof && c->variant != 0) CQA_HIP(hipEventRecord(ev0, st));
    if (c->variant == 0 || a.eta_out != nullptr) {   // eta_b comes from this kernel only
      // one-dimensional grid: the kernel decodes (head, partial set) from the linear index
      const int32_t rc = launch_split_mfma(a, hq / hkv, dim3((unsigned)nsplit * hkv * bt), ev0, ev1, st);
      if (rc != CQA_OK) return rc;
    } else {
      switch (hq / hkv) {
        case 1: hipLaunchKernelGGL((certified_split_kernel<1, false>), grid, dim3(256), 0, st, a); break;
        case 2: hipLaunchKernelGGL((certified_split_kernel<2, false>), grid, dim3(256), 0, st, a); break;
        case 4: hipLaunchKernelGGL((certified_split_kernel<4, false>), grid, dim3(256), 0, st, a); break;
        default: return CQA_ERR_UNSUPPORTED;
      }
    }
    CQA_HIP(hipGetLastError());
    if (prof) {
      if (c->variant != 0) CQA_HIP(hipEventRecord(ev1, st));
      ++c->prof_n;
    }
  }
  // one wave per workgroup: each head's wave gets a compute unit's load path to itself
  // (measured 2 us faster at 32 heads than four heads per workgroup)
  hipLaunchKernelGGL(certified_reduce_kernel, dim3(hq, bt), dim3(64), 0, st, ra);
  CQA_HIP(hipGetLastError());
  return CQA_OK;
}

}  // namespace cqa
