// Dense FP16 decode attention, softmax(q K^T / sqrt d) V with FP32 accumulation:
// the O_dense the paper's Rung 3 / Rung 4 return (its "Fallback Ladder" section).
// One launch serves the G query heads of one KV group over device-resident
// FP16 K, V of [n_tokens][128]; split over the sequence, merged by a second
// kernel that also rewrites the served heads' certificates.
#include "cqa_internal.h"
#include "reduce_inl.h"

namespace cqa {

constexpr int DP_FLOATS = 4 + D;  // m, l, pad, pad, o[128]
constexpr int DENSE_TILES_PER_SPLIT = 8;
constexpr int DENSE_MAX_SPLITS = 1024;

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

// One split of the dense pass for the G heads of one KV group: tiles [split * tiles_per_split, ...)
// of k, v ([n_tokens][128], device or mapped host memory); writes (m, l, o) per head to
// ws[h][split].  Called by all 256 threads of a workgroup.
template <int G>
__device__ __forceinline__ void dense_split_work(const __half* __restrict__ q,
                                                 const __half* __restrict__ k,
                                                 const __half* __restrict__ v, int64_t n_tokens,
                                                 int tiles_per_split, int nsplit, int split,
                                                 float* __restrict__ ws) {
  const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int tok = l & 15, kg = l >> 4;   // score phase: token of the tile, 32-channel slice
  const int vc = l & 15, vt = l >> 4;    // value phase: 8-channel slice, 4-token slice
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
    wave_sync();
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
    wave_sync();
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

template <int G>
__global__ __launch_bounds__(256) void dense_split_kernel(const __half* __restrict__ q,
                                                          const __half* __restrict__ k,
                                                          const __half* __restrict__ v,
                                                          int64_t n_tokens, int tiles_per_split,
                                                          int nsplit, float* __restrict__ ws) {
  dense_split_work<G>(q, k, v, n_tokens, tiles_per_split, nsplit, (int)blockIdx.x, ws);
}

// The fallback ladder resolved on the device (the paper's "Fallback Ladder": Rung 3 returns the
// dense FP16 result for the flagged heads, Rung 4 for every head of the layer-step).  Launched
// behind the reduction on every step, grid (splits, batch * kv heads).  Every workgroup reads
// the step's flag words and takes the ladder decision itself -- no head flagged: nothing to do;
// a PRECOND flag anywhere, or at least rung4_min_groups (> 0) flagged KV groups: all groups
// are served (Rung 4); else the flagged groups (Rung 3) -- and leaves at once unless its KV
// group is served.  The workgroups of a served group attend the group's FP16 originals
// straight from the pinned host arrays (the device reads host memory over the link: no copy
// call, no staging buffer, no host decision), and the last of them to arrive merges the
// splits and rewrites O, the certificate and the rung bits of the heads that are served.
template <int G>
__global__ __launch_bounds__(256) void dense_ladder_kernel(LadderArgs a) {
  const int split = blockIdx.x, grp = blockIdx.y;
  __shared__ int s_rung, s_mine, s_last;
  __shared__ int s_cnt[4], s_pre[4], s_my[4];
  {
    // each wave takes every fourth chunk of 64 flag words (a group's heads never straddle a
    // chunk: G divides 64), four chunks per trip with all loads issued first
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    int flagged_groups = 0;
    bool precond = false, mine = false;
    for (int base = 0; base < a.n_rows; base += 1024) {
      uint32_t f[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = base + (j * 4 + w) * 64 + l;
        f[j] = i < a.n_rows ? a.flags[i] : 0u;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i0 = base + (j * 4 + w) * 64;
        const uint64_t m = __ballot((f[j] & CQA_FLAG_ANY) != 0u);
        precond = precond || __ballot((f[j] & CQA_FLAG_PRECOND) != 0u) != 0ull;
        uint64_t gm = m;
#pragma unroll
        for (int jj = 1; jj < G; ++jj) gm |= m >> jj;
        gm &= G == 1 ? ~0ull : (G == 2 ? 0x5555555555555555ull : 0x1111111111111111ull);
        flagged_groups += __popcll(gm);
        const int r0 = grp * G - i0;
        if (r0 >= 0 && r0 < 64) mine = mine || ((m >> r0) & ((1ull << G) - 1ull)) != 0ull;
      }
    }
    if (l == 0) {
      s_cnt[w] = flagged_groups;
      s_pre[w] = precond ? 1 : 0;
      s_my[w] = mine ? 1 : 0;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      const int cnt = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
      const bool pre = (s_pre[0] | s_pre[1] | s_pre[2] | s_pre[3]) != 0;
      const bool my = (s_my[0] | s_my[1] | s_my[2] | s_my[3]) != 0;
      int rung = cnt > 0 ? 3 : 0;
      if (rung != 0 && (pre || (a.rung4_min_groups > 0 && cnt >= a.rung4_min_groups))) rung = 4;
      s_rung = rung;
      s_mine = (rung == 4 || my) ? 1 : 0;
      if (rung != 0 && split == 0 && grp == 0) atomicAdd(a.counts + (rung - 3), 1u);
    }
  }
  __syncthreads();
  const int rung = s_rung;
  if (rung == 0 || s_mine == 0) return;

  const int64_t row0 = (int64_t)grp * G;
  float* ws = a.ws + row0 * a.nsplit * DP_FLOATS;
  dense_split_work<G>(a.q + row0 * D, a.t2_k + (int64_t)grp * a.max_tokens * D,
                      a.t2_v + (int64_t)grp * a.max_tokens * D, a.n_tokens, a.tiles_per_split,
                      a.nsplit, split, ws);
  // every thread publishes its partial stores device-wide before the workgroup draws its ticket
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t* tk = a.tickets + grp;
    const uint32_t t = __hip_atomic_fetch_add(tk, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool last = t == (uint32_t)a.nsplit - 1u;
    if (last) __hip_atomic_store(tk, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next launch
    s_last = last ? 1 : 0;
  }
  __syncthreads();
  if (s_last == 0) return;
  __threadfence();
  for (int idx = threadIdx.x; idx < G * D; idx += 256) {
    const int h = idx / D, c = idx % D;
    const int64_t row = row0 + h;
    if (rung != 4 && (a.flags[row] & CQA_FLAG_ANY) == 0u) continue;   // Rung 3 serves flagged heads only
    const float* part = ws + (int64_t)h * a.nsplit * DP_FLOATS;
    float M = -INFINITY;
    for (int sidx = 0; sidx < a.nsplit; ++sidx) M = fmaxf(M, part[sidx * DP_FLOATS]);
    float L = 0.0f, o = 0.0f;
    for (int sidx = 0; sidx < a.nsplit; ++sidx) {
      const float f = __expf(part[sidx * DP_FLOATS] - M);
      L += f * part[sidx * DP_FLOATS + 1];
      o += f * part[sidx * DP_FLOATS + 4 + c];
    }
    a.O[row * D + c] = o / L;
    if (c == 0) {
      a.cert[row].E_key = 0.0f;
      a.cert[row].E_val = 0.0f;
      a.cert[row].served_rung = rung;
      a.flags[row] = (a.flags[row] & ~(7u << CQA_RUNG_SHIFT)) | ((uint32_t)rung << CQA_RUNG_SHIFT);
    }
  }
}

int ladder_splits(const Cache* c, int64_t n_tokens) {
  const int64_t groups = (int64_t)c->desc.batch * c->desc.n_kv_heads;
  int64_t want = (2 * (int64_t)c->n_cu) / groups;   // the launch's cost does not depend on it
  if (want < 4) want = 4;
  if (want > LADDER_MAX_SPLITS) want = LADDER_MAX_SPLITS;
  const int64_t tiles = (n_tokens + BLK - 1) / BLK;
  if (want > tiles) want = tiles;
  const int64_t tps = (tiles + want - 1) / want;
  return (int)((tiles + tps - 1) / tps);
}

int64_t ladder_ws_floats(int64_t rows) { return rows * LADDER_MAX_SPLITS * DP_FLOATS; }

int32_t launch_dense_ladder(Cache* c, int layer, const __half* q, int rung4_min_groups, float* O,
                            cqa_head_cert* cert, uint32_t* flags, hipStream_t st) {
  if (c->desc.tier2_mode != CQA_TIER2_PINNED) return CQA_ERR_NO_TIER2;
  const int64_t len = c->length[layer];
  if (len <= 0 || q == nullptr || O == nullptr || cert == nullptr || flags == nullptr)
    return CQA_ERR_INVALID_ARG;
  const int bt = c->desc.batch, hq = c->desc.n_q_heads, hkv = c->desc.n_kv_heads;
  const int g = hq / hkv;
  const int64_t layer_head0 = (int64_t)layer * bt * hkv;
  LadderArgs a{};
  a.q = q;
  a.t2_k = c->t2_k + layer_head0 * c->desc.max_tokens * D;
  a.t2_v = c->t2_v + layer_head0 * c->desc.max_tokens * D;
  a.max_tokens = c->desc.max_tokens;
  a.n_tokens = len;
  a.n_rows = bt * hq;
  a.nsplit = ladder_splits(c, len);
  const int64_t tiles = (len + BLK - 1) / BLK;
  a.tiles_per_split = (int)((tiles + a.nsplit - 1) / a.nsplit);
  a.rung4_min_groups = rung4_min_groups;
  a.ws = c->ladder_ws;
  a.tickets = c->ladder_tickets;
  a.counts = c->ladder_counts;
  a.O = O;
  a.cert = cert;
  a.flags = flags;
  const dim3 grid(a.nsplit, bt * hkv);
  switch (g) {
    case 1: hipLaunchKernelGGL(dense_ladder_kernel<1>, grid, dim3(256), 0, st, a); break;
    case 2: hipLaunchKernelGGL(dense_ladder_kernel<2>, grid, dim3(256), 0, st, a); break;
    case 4: hipLaunchKernelGGL(dense_ladder_kernel<4>, grid, dim3(256), 0, st, a); break;
    default: return CQA_ERR_UNSUPPORTED;
  }
  CQA_HIP(hipGetLastError());
  return CQA_OK;
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
