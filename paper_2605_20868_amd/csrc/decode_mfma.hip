// Certified decode, split-K pass on the matrix cores (gfx950 MFMA, 64-wide waves).
//
// Same mathematics as the paper's Algorithm 1 with no promoted blocks and its
// scaled-query identity  q . k_hat = sum_c (q_c sigma_c) code_c + sum_c q_c z_c;
// the two contractions run as bf16 MFMAs with FP32 accumulation:
//
//  scores   S[token][(h, j)] = sum_c code[token][c] * q~[(h, j)][c]
//           One wave takes four consecutive blocks (a "quad") per iteration.
//           A = the 16 tokens of block i as exact bf16 integers (u = code + 128);
//           B = 16 columns = 4 query heads x the 4 blocks of the quad, each column
//           holding that block's scaled query q~ = q (.) sigma as THREE bf16 terms
//           (hi + mid + lo = 24 significant bits, i.e. FP32-exact); only the
//           columns of block i are kept from A_i's product.  Forming B once per
//           quad keeps every lane busy: lane (n, kg) owns column n, channels of kg.
//  values   O[(h, g')][c] = sum_t w[t][(h, g')] * (16 + code[t][c]),
//           w = p_t * scale_{t,g} as TWO bf16 terms, K = 32 tokens (two blocks),
//           one 16-channel value group per tile; the bias 16 (which makes the
//           4-bit code an exact bf16 by bit insertion) and the group offsets are
//           folded into  sum_t p_t (offset_{t,g} - 16 scale_{t,g}),  accumulated on the VALU.
//
// Lane roles (l = lane, n = l & 15, kg = l >> 4, h = n >> 2, j = g' = n & 3):
//   score phase : column n = (head h, block j of the quad); kg = 8-channel slice
//   value phase : row    n = (head h, group g' of the tile set); kg = 8-token slice
//   accumulators: C[row = 4 kg + v][col = n]  ->  head kg, vgpr v = g', channel n
#include "cqa_internal.h"

namespace cqa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

union BF8 {
  bf16x8 v;
  uint32_t u[4];
};

__device__ __forceinline__ void wave_sync_m() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// two FP32 values -> their upper 16 bits packed (x0 in the low half): bf16 by truncation
__device__ __forceinline__ uint32_t pack_hi16(float x1, float x0) {
  return __builtin_amdgcn_perm(__float_as_uint(x1), __float_as_uint(x0), 0x07060302u);
}
// two FP32 values -> bf16 by round-to-nearest-even (v_cvt_pk_bf16_f32), x0 in the low half
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_rne(float x1, float x0) {
  const f32x2_t x = {x0, x1};
  union {
    bf16x2_t v;
    uint32_t u;
  } r;
  r.v = __builtin_convertvector(x, bf16x2_t);
  return r.u;
}
__device__ __forceinline__ float trunc_bf16(float x) {
  return __uint_as_float(__float_as_uint(x) & 0xffff0000u);
}

__device__ __forceinline__ void top2_merge_m(float& t1, int& i1, float& t2, float u1, int j1,
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

template <int G>
__global__ __launch_bounds__(256) void certified_split_mfma_kernel(DecodeArgs a) {
  const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int n = l & 15, kg = l >> 4;
  const int h = n >> 2, j = n & 3;
  const bool hvalid = h < G;
  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int64_t base_blk = ((int64_t)b * a.n_kv + kvh) * a.nb_cap;
  const int b0 = split * a.bps;
  const int b1 = min(b0 + a.bps, a.nb);
  const float inv_sqrt_d = 0.08838834764831845f;

  __shared__ __align__(16) float pbuf[4][4][4][BLK];  // [wave][head][block of quad][token]
  __shared__ __align__(16) float mo[4][G][D];
  __shared__ float ms[4][G][12];

  // query of my head, my 32 channels: channel(u, e) = (u>>1)*64 + kg*16 + (u&1)*8 + e
  float qreg[32];
  {
    const __half* qh = a.q + ((int64_t)b * a.n_q + kvh * G + (hvalid ? h : 0)) * D;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint4 x = *reinterpret_cast<const uint4*>(qh + (u >> 1) * 64 + kg * 16 + (u & 1) * 8);
      const __half2* hh = reinterpret_cast<const __half2*>(&x);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        qreg[u * 8 + 2 * e] = hvalid ? __low2float(hh[e]) : 0.0f;
        qreg[u * 8 + 2 * e + 1] = hvalid ? __high2float(hh[e]) : 0.0f;
      }
    }
  }

  float m_run = -INFINITY, l_run = 0.0f, ev = 0.0f, evmax = 0.0f, dmax = 0.0f, vmax = 0.0f;
  float t1 = -INFINITY, t2 = -INFINITY;
  int i1 = -1;
  float offacc[2] = {0.0f, 0.0f};
  f32x4 acc[8];
#pragma unroll
  for (int g = 0; g < 8; ++g) acc[g] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

  for (int qb = b0 + 4 * w; qb < b1; qb += 16) {
    const int myblk = qb + j;
    const bool bvalid = myblk < b1;
    const int64_t gbj = base_blk + min(myblk, a.nb - 1);

    // ---- loads of the quad
    uint4 kraw[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint8_t* kcb = a.kc + (base_blk + min(qb + i, a.nb - 1)) * KC_BYTES;
#pragma unroll
      for (int cq = 0; cq < 2; ++cq) kraw[i][cq] = reinterpret_cast<const uint4*>(kcb + cq * 1024)[l];
    }
    const float* kmb = a.km + gbj * (KM_BYTES / 4);
    const float2 an = *reinterpret_cast<const float2*>(a.an + gbj * 2);
    uint4 vraw[2][2], sraw[2][2], oraw[2][2];
#pragma unroll
    for (int P = 0; P < 2; ++P) {
      const int64_t gbp = base_blk + min(qb + 2 * P + (kg >> 1), a.nb - 1);
      const uint8_t* vcb = a.vc + gbp * VC_BYTES + (kg & 1) * 512 + n * 16;
      const __half* vmb = a.vm + gbp * (VM_BYTES / 2) + (kg & 1) * 64;
#pragma unroll
      for (int gs = 0; gs < 2; ++gs) {
        vraw[P][gs] = *reinterpret_cast<const uint4*>(vcb + gs * 256);
        sraw[P][gs] = *reinterpret_cast<const uint4*>(vmb + (4 * gs + j) * 8);
        oraw[P][gs] = *reinterpret_cast<const uint4*>(vmb + BLK * NG + (4 * gs + j) * 8);
      }
    }

    // ---- scores: B (scaled query, 3 bf16 terms) per channel slice u, A per block
    f32x4 C[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) C[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    float csum = 0.0f, qsum = 0.0f, dsum = 0.0f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c0 = (u >> 1) * 64 + kg * 16 + (u & 1) * 8;
      const float4 s0 = *reinterpret_cast<const float4*>(kmb + c0);
      const float4 s1 = *reinterpret_cast<const float4*>(kmb + c0 + 4);
      const float4 z0 = *reinterpret_cast<const float4*>(kmb + D + c0);
      const float4 z1 = *reinterpret_cast<const float4*>(kmb + D + c0 + 4);
      const float sg[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
      const float zz[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
      float qt[8], r1[8], r2[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float qv = qreg[u * 8 + e];
        qt[e] = qv * sg[e];
        csum = fmaf(qv, zz[e], csum);
        qsum += qt[e];
        dsum = fmaf(fabsf(qv), sg[e], dsum);
        r1[e] = qt[e] - trunc_bf16(qt[e]);
        r2[e] = r1[e] - trunc_bf16(r1[e]);
      }
      BF8 bh, bm, bl;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        bh.u[p] = pack_hi16(qt[2 * p + 1], qt[2 * p]);
        bm.u[p] = pack_hi16(r1[2 * p + 1], r1[2 * p]);
        bl.u[p] = pack_rne(r2[2 * p + 1], r2[2 * p]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint4 kx = kraw[i][u >> 1];
        const uint32_t d0 = (u & 1) ? kx.z : kx.x, d1 = (u & 1) ? kx.w : kx.y;
        float kf[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          kf[e] = (float)((d0 >> (8 * e)) & 0xffu);
          kf[4 + e] = (float)((d1 >> (8 * e)) & 0xffu);
        }
        BF8 av;
#pragma unroll
        for (int p = 0; p < 4; ++p) av.u[p] = pack_hi16(kf[2 * p + 1], kf[2 * p]);
        C[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av.v, bh.v, C[i], 0, 0, 0);
        C[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av.v, bm.v, C[i], 0, 0, 0);
        C[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av.v, bl.v, C[i], 0, 0, 0);
      }
    }
    // per-block constant c_b = q.z - 128 sum(q~) (stored bytes are code + 128) and Delta_b
    float cb = fmaf(-128.0f, qsum, csum);
    cb += __shfl_xor(cb, 16);
    cb += __shfl_xor(cb, 32);
    dsum += __shfl_xor(dsum, 16);
    dsum += __shfl_xor(dsum, 32);

    // my column's block is j: tokens 4 kg .. 4 kg + 3 of it
    float s[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float raw = j == 0 ? C[0][v] : (j == 1 ? C[1][v] : (j == 2 ? C[2][v] : C[3][v]));
      s[v] = (raw + cb) * inv_sqrt_d;
    }

    // ---- block statistics and online softmax (state replicated over the lanes of a head)
    float mb = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
    mb = fmaxf(mb, __shfl_xor(mb, 16));
    mb = fmaxf(mb, __shfl_xor(mb, 32));
    float pt[4];
    float sb = 0.0f;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      pt[v] = bvalid ? __expf(s[v] - mb) : 0.0f;
      sb += pt[v];
    }
    sb += __shfl_xor(sb, 16);
    sb += __shfl_xor(sb, 32);
    const float lb = bvalid ? mb + __logf(sb) : -INFINITY;
    float mq = bvalid ? mb : -INFINITY;
    mq = fmaxf(mq, __shfl_xor(mq, 1));
    mq = fmaxf(mq, __shfl_xor(mq, 2));
    const float m_new = fmaxf(m_run, mq);
    const float alpha = __expf(m_run - m_new);
    const float f = bvalid ? __expf(mb - m_new) : 0.0f;
    const float sf = sb * f;
    const float ce = sf * an.x;
    float sq = sf, ceq = ce, cem = ce;
    sq += __shfl_xor(sq, 1);
    ceq += __shfl_xor(ceq, 1);
    cem = fmaxf(cem, __shfl_xor(cem, 1));
    sq += __shfl_xor(sq, 2);
    ceq += __shfl_xor(ceq, 2);
    cem = fmaxf(cem, __shfl_xor(cem, 2));
    l_run = fmaf(l_run, alpha, sq);
    ev = fmaf(ev, alpha, ceq);
    evmax = fmaxf(evmax * alpha, cem);
    m_run = m_new;
    if (bvalid) {
      dmax = fmaxf(dmax, dsum * (0.5f * inv_sqrt_d));
      vmax = fmaxf(vmax, an.y);
      if (lb > t1) {
        t2 = t1;
        t1 = lb;
        i1 = myblk;
      } else if (lb > t2) {
        t2 = lb;
      }
      if (a.blk_logmass != nullptr && kg == 0 && hvalid)
        a.blk_logmass[((int64_t)b * a.n_q + kvh * G + h) * a.nb + myblk] = lb;
    }
    *reinterpret_cast<float4*>(&pbuf[w][h][j][kg * 4]) =
        make_float4(pt[0] * f, pt[1] * f, pt[2] * f, pt[3] * f);
    wave_sync_m();

    // ---- rescale the output accumulators (head of an accumulator lane is kg)
    const float alpha_acc = __shfl(alpha, kg * 4);
    if (__any(alpha_acc != 1.0f)) {
#pragma unroll
      for (int g = 0; g < 8; ++g)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[g][v] *= alpha_acc;
    }
    offacc[0] *= alpha;
    offacc[1] *= alpha;

    // ---- values: two pairs of blocks, K = 32 tokens each
#pragma unroll
    for (int P = 0; P < 2; ++P) {
      const float4 pa = *reinterpret_cast<const float4*>(&pbuf[w][h][2 * P + (kg >> 1)][(kg & 1) * 8]);
      const float4 pb = *reinterpret_cast<const float4*>(&pbuf[w][h][2 * P + (kg >> 1)][(kg & 1) * 8 + 4]);
      const float p8[8] = {pa.x, pa.y, pa.z, pa.w, pb.x, pb.y, pb.z, pb.w};
#pragma unroll
      for (int gs = 0; gs < 2; ++gs) {
        const __half2* sh = reinterpret_cast<const __half2*>(&sraw[P][gs]);
        const __half2* oh = reinterpret_cast<const __half2*>(&oraw[P][gs]);
        float wv[8], wr[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float sc0 = __low2float(sh[e]), sc1 = __high2float(sh[e]);
          const float of0 = __low2float(oh[e]), of1 = __high2float(oh[e]);
          wv[2 * e] = p8[2 * e] * sc0;
          wv[2 * e + 1] = p8[2 * e + 1] * sc1;
          offacc[gs] = fmaf(p8[2 * e], fmaf(-16.0f, sc0, of0), offacc[gs]);
          offacc[gs] = fmaf(p8[2 * e + 1], fmaf(-16.0f, sc1, of1), offacc[gs]);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) wr[e] = wv[e] - trunc_bf16(wv[e]);
        // slot pairing: slots (2p, 2p+1) hold tokens (p, p+4) of the octet, matching the nibble pairs
        BF8 ah, al;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          ah.u[p] = pack_hi16(wv[p + 4], wv[p]);
          al.u[p] = pack_rne(wr[p + 4], wr[p]);
        }
        const uint32_t xs[4] = {vraw[P][gs].x, vraw[P][gs].y, vraw[P][gs].z, vraw[P][gs].w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint32_t x = xs[t];
          BF8 bv;   // bf16(16 + code): exponent bits 0x4180, code in mantissa bits 6..3
          bv.u[0] = ((x << 3) & 0x00780078u) | 0x41804180u;
          bv.u[1] = ((x >> 1) & 0x00780078u) | 0x41804180u;
          bv.u[2] = ((x >> 5) & 0x00780078u) | 0x41804180u;
          bv.u[3] = ((x >> 9) & 0x00780078u) | 0x41804180u;
          acc[4 * gs + t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah.v, bv.v, acc[4 * gs + t], 0, 0, 0);
          acc[4 * gs + t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al.v, bv.v, acc[4 * gs + t], 0, 0, 0);
        }
      }
    }
    wave_sync_m();
  }

  // ---- per-wave epilogue: fold the offset sums in, reduce the per-lane trackers over the head's lanes
#pragma unroll
  for (int gs = 0; gs < 2; ++gs) {
    offacc[gs] += __shfl_xor(offacc[gs], 16);
    offacc[gs] += __shfl_xor(offacc[gs], 32);
  }
#pragma unroll
  for (int m = 1; m <= 2; m <<= 1) {
    dmax = fmaxf(dmax, __shfl_xor(dmax, m));
    vmax = fmaxf(vmax, __shfl_xor(vmax, m));
    const float u1 = __shfl_xor(t1, m), u2 = __shfl_xor(t2, m);
    const int j1 = __shfl_xor(i1, m);
    top2_merge_m(t1, i1, t2, u1, j1, u2);
  }
  __syncthreads();
#pragma unroll
  for (int g = 0; g < 8; ++g) {
    const float off = __shfl(offacc[g >> 2], kg * 4 + (g & 3));
    const float val = (g & 3) == 0 ? acc[g][0] : ((g & 3) == 1 ? acc[g][1] : ((g & 3) == 2 ? acc[g][2] : acc[g][3]));
    if (kg < G) mo[w][kg < G ? kg : 0][g * 16 + n] = val + off;
  }
  if (kg == 0 && j == 0 && hvalid) {
    ms[w][h][0] = m_run;
    ms[w][h][1] = l_run;
    ms[w][h][2] = ev;
    ms[w][h][3] = evmax;
    ms[w][h][4] = dmax;
    ms[w][h][5] = vmax;
    ms[w][h][6] = t1;
    ms[w][h][7] = t2;
    ms[w][h][8] = __int_as_float(i1);
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * D; idx += 256) {
    const int hh = idx / D, c = idx % D;
    float M = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) M = fmaxf(M, ms[ww][hh][0]);
    float o = 0.0f;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) o += __expf(ms[ww][hh][0] - M) * mo[ww][hh][c];
    a.partials[(((int64_t)b * a.n_q + kvh * G + hh) * a.nsplit + split) * PART_FLOATS + P_O + c] = o;
  }
  if (threadIdx.x < G) {
    const int hh = threadIdx.x;
    float M = -INFINITY;
    for (int ww = 0; ww < 4; ++ww) M = fmaxf(M, ms[ww][hh][0]);
    float L = 0.0f, EV = 0.0f, EVM = 0.0f, DM = 0.0f, VM = 0.0f, T1 = -INFINITY, T2 = -INFINITY;
    int I1 = -1;
    for (int ww = 0; ww < 4; ++ww) {
      const float fw = __expf(ms[ww][hh][0] - M);
      L += fw * ms[ww][hh][1];
      EV += fw * ms[ww][hh][2];
      EVM = fmaxf(EVM, fw * ms[ww][hh][3]);
      DM = fmaxf(DM, ms[ww][hh][4]);
      VM = fmaxf(VM, ms[ww][hh][5]);
      top2_merge_m(T1, I1, T2, ms[ww][hh][6], __float_as_int(ms[ww][hh][8]), ms[ww][hh][7]);
    }
    float* pp = a.partials + (((int64_t)b * a.n_q + kvh * G + hh) * a.nsplit + split) * PART_FLOATS;
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

int32_t launch_split_mfma(const DecodeArgs& a, int group, dim3 grid, hipStream_t st) {
  switch (group) {
    case 1: hipLaunchKernelGGL(certified_split_mfma_kernel<1>, grid, dim3(256), 0, st, a); break;
    case 2: hipLaunchKernelGGL(certified_split_mfma_kernel<2>, grid, dim3(256), 0, st, a); break;
    case 4: hipLaunchKernelGGL(certified_split_mfma_kernel<4>, grid, dim3(256), 0, st, a); break;
    default: return CQA_ERR_UNSUPPORTED;
  }
  return CQA_OK;
}

}  // namespace cqa
