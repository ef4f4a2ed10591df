// Dense FP16 decode attention, softmax(q K^T / sqrt d) V with FP32 accumulation:
// the O_dense the paper's Rung 3 / Rung 4 return (its "Fallback Ladder" section).
// One launch serves the G query heads of one KV group over device-resident
// FP16 K, V of [n_tokens][128]; split over the sequence, merged by a second
// kernel that also rewrites the served heads' certificates.
#include "cqa_internal.h"

namespace cqa {

constexpr int DP_FLOATS = 4 + D;  // m, l, pad, pad, o[128]
constexpr int DENSE_TILES_PER_SPLIT = 8;
constexpr int DENSE_MAX_SPLITS = 1024;

__device__ __forceinline__ void wave_sync_d() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

int dense_splits(int64_t n_tokens) {
  const int64_t tiles = (n_tokens + BLK - 1) / BLK;
  int64_t s = (tiles + DENSE_TILES_PER_SPLIT - 1) / DENSE_TILES_PER_SPLIT;
  if (s > DENSE_MAX_SPLITS) s = DENSE_MAX_SPLITS;
  if (s < 1) s = 1;
  const int64_t tps = (tiles + s - 1) / s;
  return (int)((tiles + tps - 1) / tps);
}

int64_t dense_ws_floats(int group, int64_t n_tokens) {
  return (int64_t)group * dense_splits(n_tokens) * DP_FLOATS;
}

template <int G>
__global__ __launch_bounds__(256) void dense_split_kernel(const __half* __restrict__ q,
                                                          const __half* __restrict__ k,
                                                          const __half* __restrict__ v,
                                                          int64_t n_tokens, int tiles_per_split,
                                                          int nsplit, float* __restrict__ ws) {
  const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int tok = l & 15, kg = l >> 4;   // score phase: token of the tile, 32-channel slice
  const int vc = l & 15, vt = l >> 4;    // value phase: 8-channel slice, 4-token slice
  const int split = blockIdx.x;
  const int64_t tiles = (n_tokens + BLK - 1) / BLK;
  const int64_t t0 = (int64_t)split * tiles_per_split;
  const int64_t t1 = min(t0 + (int64_t)tiles_per_split, tiles);
  const float inv_sqrt_d = 0.08838834764831845f;

  __shared__ __align__(16) float qf[G][D];
  __shared__ __align__(16) float ps[4][BLK][G];
  __shared__ __align__(16) float mo[4][G][D];
  __shared__ float ms[4][G][2];

  for (int i = threadIdx.x; i < G * D; i += 256) qf[i / D][i % D] = __half2float(q[i]);
  __syncthreads();

  float m_run[G], l_run[G], acc[8][G];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m_run[h] = -INFINITY;
    l_run[h] = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j][h] = 0.0f;
  }

  for (int64_t tile = t0 + w; tile < t1; tile += 4) {
    const int64_t t = tile * BLK + tok;
    const bool valid = t < n_tokens;
    const int64_t tc = valid ? t : n_tokens - 1;
    const uint4* kp = reinterpret_cast<const uint4*>(k + tc * D + kg * 32);
    float dot[G];
#pragma unroll
    for (int h = 0; h < G; ++h) dot[h] = 0.0f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint4 x = kp[u];
      const __half2* hh = reinterpret_cast<const __half2*>(&x);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float k0 = __low2float(hh[j]), k1 = __high2float(hh[j]);
        const int c = kg * 32 + u * 8 + j * 2;
#pragma unroll
        for (int h = 0; h < G; ++h) dot[h] = fmaf(qf[h][c + 1], k1, fmaf(qf[h][c], k0, dot[h]));
      }
    }
    float alpha[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      dot[h] += __shfl_xor(dot[h], 16);
      dot[h] += __shfl_xor(dot[h], 32);
      const float s = valid ? dot[h] * inv_sqrt_d : -INFINITY;
      float mb = s;
#pragma unroll
      for (int m = 1; m < 16; m <<= 1) mb = fmaxf(mb, __shfl_xor(mb, m));
      const float m_new = fmaxf(m_run[h], mb);
      alpha[h] = __expf(m_run[h] - m_new);
      const float p = __expf(s - m_new);
      float sb = p;
#pragma unroll
      for (int m = 1; m < 16; m <<= 1) sb += __shfl_xor(sb, m);
      l_run[h] = l_run[h] * alpha[h] + sb;
      m_run[h] = m_new;
      if (kg == 0) ps[w][tok][h] = p;
    }
    wave_sync_d();
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int h = 0; h < G; ++h) acc[j][h] *= alpha[h];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int tt = vt * 4 + i;
      int64_t tv = tile * BLK + tt;
      if (tv >= n_tokens) tv = n_tokens - 1;  // its probability is exactly 0
      const uint4 x = *reinterpret_cast<const uint4*>(v + tv * D + vc * 8);
      const __half2* hh = reinterpret_cast<const __half2*>(&x);
      float pr[G];
#pragma unroll
      for (int h = 0; h < G; ++h) pr[h] = ps[w][tt][h];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float v0 = __low2float(hh[j]), v1 = __high2float(hh[j]);
#pragma unroll
        for (int h = 0; h < G; ++h) {
          acc[2 * j][h] = fmaf(pr[h], v0, acc[2 * j][h]);
          acc[2 * j + 1][h] = fmaf(pr[h], v1, acc[2 * j + 1][h]);
        }
      }
    }
    wave_sync_d();
  }

#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float x = acc[j][h];
      x += __shfl_xor(x, 16);
      x += __shfl_xor(x, 32);
      if (vt == 0) mo[w][h][vc * 8 + j] = x;
    }
  if (l == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      ms[w][h][0] = m_run[h];
      ms[w][h][1] = l_run[h];
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
    for (int ww = 0; ww < 4; ++ww) o += __expf(ms[ww][h][0] - M) * mo[ww][h][c];
    ws[((int64_t)h * nsplit + split) * DP_FLOATS + 4 + c] = o;
  }
  if (threadIdx.x < G) {
    const int h = threadIdx.x;
    float M = -INFINITY;
    for (int ww = 0; ww < 4; ++ww) M = fmaxf(M, ms[ww][h][0]);
    float L = 0.0f;
    for (int ww = 0; ww < 4; ++ww) L += __expf(ms[ww][h][0] - M) * ms[ww][h][1];
    ws[((int64_t)h * nsplit + split) * DP_FLOATS + 0] = M;
    ws[((int64_t)h * nsplit + split) * DP_FLOATS + 1] = L;
  }
}

__global__ __launch_bounds__(128) void dense_reduce_kernel(const float* __restrict__ ws, int nsplit,
                                                           float* __restrict__ O,
                                                           const uint32_t* __restrict__ select,
                                                           cqa_head_cert* cert, uint32_t* flags,
                                                           int rung) {
  const int h = blockIdx.x, c = threadIdx.x;
  if (select != nullptr && select[h] == 0) return;
  const float* part = ws + (int64_t)h * nsplit * DP_FLOATS;
  float M = -INFINITY;
  for (int s = 0; s < nsplit; ++s) M = fmaxf(M, part[s * DP_FLOATS]);
  float L = 0.0f, o = 0.0f;
  for (int s = 0; s < nsplit; ++s) {
    const float f = __expf(part[s * DP_FLOATS] - M);
    L += f * part[s * DP_FLOATS + 1];
    o += f * part[s * DP_FLOATS + 4 + c];
  }
  O[(int64_t)h * D + c] = o / L;
  if (c == 0) {
    if (cert != nullptr) {
      cert[h].E_key = 0.0f;
      cert[h].E_val = 0.0f;
      cert[h].served_rung = rung;
    }
    if (flags != nullptr)
      flags[h] = (flags[h] & ~(7u << CQA_RUNG_SHIFT)) | ((uint32_t)rung << CQA_RUNG_SHIFT);
  }
}

int32_t launch_dense_group(const __half* q_group, const __half* k, const __half* v, int group,
                           int64_t n_tokens, float* O_group, const uint32_t* select_group,
                           cqa_head_cert* cert_group, uint32_t* flags_group, int rung,
                           float* ws, hipStream_t st) {
  if (n_tokens <= 0) return CQA_ERR_INVALID_ARG;
  const int nsplit = dense_splits(n_tokens);
  const int64_t tiles = (n_tokens + BLK - 1) / BLK;
  const int tps = (int)((tiles + nsplit - 1) / nsplit);
  switch (group) {
    case 1:
      hipLaunchKernelGGL(dense_split_kernel<1>, dim3(nsplit), dim3(256), 0, st, q_group, k, v,
                         n_tokens, tps, nsplit, ws);
      break;
    case 2:
      hipLaunchKernelGGL(dense_split_kernel<2>, dim3(nsplit), dim3(256), 0, st, q_group, k, v,
                         n_tokens, tps, nsplit, ws);
      break;
    case 4:
      hipLaunchKernelGGL(dense_split_kernel<4>, dim3(nsplit), dim3(256), 0, st, q_group, k, v,
                         n_tokens, tps, nsplit, ws);
      break;
    default:
      return CQA_ERR_UNSUPPORTED;
  }
  CQA_HIP(hipGetLastError());
  hipLaunchKernelGGL(dense_reduce_kernel, dim3(group), dim3(128), 0, st, ws, nsplit, O_group,
                     select_group, cert_group, flags_group, rung);
  CQA_HIP(hipGetLastError());
  return CQA_OK;
}

}  // namespace cqa
