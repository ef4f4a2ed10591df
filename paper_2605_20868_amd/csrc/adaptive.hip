// Adaptive key precision: selector, promoted-set bookkeeping, and the reduction of the attend
// pass with its ranking check.
//
// Follows the paper's "Adaptive Precision Selection" (rank blocks by INT8-estimated mass, K* =
// smallest prefix that covers tau_cov, clamp to [K_min, K_max]), the first rung of its "Fallback
// Ladder" (grow K while the key term is over its threshold), its total error bound with the
// achieved INT8-estimated tail mass, and its "Ranking-Consistency Check" with the boundary
// verification, at depth r <= MAX_RANK_DEPTH.  Key and value precision are chosen per KV group
// (the union of the group's query heads' selections: the paper's per-KV-group selection variant)
// or, with cqa_selector.per_head, per query head over the head's own promoted set (its default).
//
// Sequence on one stream (launch_adaptive): the certified pass over all sealed blocks in INT8 /
// INT4 (it emits the block log-masses, eta_b and the usual partial sets, and its reduction the
// total log-mass, Delta_h and V_max the selector needs) -> select_kernel (per head) ->
// compact_kernel (per group: union bit mask -> per-block flags and ordered list) -> promoted-block
// pass over the listed blocks only: positive partial sets computed with the originals the flags ask
// for (read straight from the pinned Tier-2 arrays over the host link) and negated sets computed as
// the first pass did, so that the merge replaces those blocks' contribution -> adaptive_reduce_kernel.
// Tier-1 is read once per step; the paper's two passes (score, then attend) become one pass plus a
// correction for a few dozen blocks.
#include <algorithm>

#include "cqa_internal.h"
#include "reduce_inl.h"

namespace cqa {

// defined in decode.hip
int32_t launch_promoted_pass(const DecodeArgs& a, int group, dim3 grid, hipStream_t st);

namespace {

// order-preserving map float -> uint32 (larger float <=> larger integer)
__device__ __forceinline__ uint32_t ord32(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

struct SelectArgs {
  const float* lm8;            // [Bt][Hq][nb]: the row that is ranked (log-masses, or contributions)
  const cqa_head_cert* cert;   // first pass: lse, delta_h, v_max
  int32_t* sel;                // [Bt][Hq][MAX_K_LIMIT]
  int32_t* kstar;              // [Bt][Hq]
  uint32_t* umask;             // [Bt][Hq][mask_words]: the head's own selection
  float v_tol, eps_val;        // value selection: local threshold and budget
  float* score_dev;            // [Bt][Hq] canary output, cleared here (null = no canary)
  int v_greedy;
  int64_t mask_words;
  int nb, n_q, n_kv;
  float tau_cov;
  int k_min, k_max, k_limit;
  float eps_key;
  int mass_exp, key_bound_mode;
};

// Strided pass over a row in batches: all loads of a batch are issued before anything is consumed
// (a plain strided loop has one load in flight per thread and is bound by its latency).
constexpr int BATCH = 16;
constexpr int ST = 1024;          // threads of the selector workgroup
constexpr int SBATCH = 8;
#define CQA_ROW_PASS(ROW, N, TID, BODY)                                           \
  for (int base__ = 0; base__ < (N); base__ += ST * SBATCH) {                      \
    float val__[SBATCH];                                                            \
    _Pragma("unroll") for (int j__ = 0; j__ < SBATCH; ++j__) {                      \
      const int i__ = base__ + j__ * ST + (TID);                                  \
      val__[j__] = i__ < (N) ? (ROW)[i__] : 0.0f;                                  \
    }                                                                              \
    _Pragma("unroll") for (int j__ = 0; j__ < SBATCH; ++j__) {                      \
      const int i = base__ + j__ * ST + (TID);                                    \
      const float x = val__[j__];                                                  \
      const bool in = i < (N);                                                     \
      BODY                                                                         \
    }                                                                              \
  }

// The selector walks its row of log-masses several times.  Rows of up to LDS_KEYS blocks are read
// from memory once, as order-preserving integer keys kept in LDS; longer rows are re-read.
constexpr int LDS_KEYS = 10240;   // 40 KB: contexts up to 160K tokens
#define CQA_KEY_PASS(ROW, N, TID, CACHED, KEYS, BODY)                             \
  for (int base__ = 0; base__ < (N); base__ += ST * SBATCH) {                      \
    uint32_t key__[SBATCH];                                                         \
    _Pragma("unroll") for (int j__ = 0; j__ < SBATCH; ++j__) {                      \
      const int i__ = base__ + j__ * ST + (TID);                                  \
      key__[j__] = i__ < (N) ? ((CACHED) ? (KEYS)[i__] : ord32((ROW)[i__])) : 0u;  \
    }                                                                              \
    _Pragma("unroll") for (int j__ = 0; j__ < SBATCH; ++j__) {                      \
      const int i = base__ + j__ * ST + (TID);                                    \
      const uint32_t k = key__[j__];                                               \
      const bool in = i < (N);                                                     \
      BODY                                                                         \
    }                                                                              \
  }

// E_key / (1) from Delta_h, the estimated tail mass and V_max, in double (decision only)
__device__ double key_term_d(double delta, double alpha, double vmax, int mass_exp, int mode) {
  double t_tail = 0.0;
  if (alpha > 0.0 && delta != 0.0) {
    const double grow = exp(fmin((double)mass_exp * delta, 700.0));
    const double widen = expm1(fmin(2.0 * delta, 700.0));
    t_tail = fmin(1.0, grow * alpha) * widen;
  }
  const double t_full = tanh(delta);
  const double tv = mode == 0 ? fmin(t_full, t_tail) : (mode == 1 ? t_tail : t_full);
  return 2.0 * vmax * tv;
}

// Histogram increment for a whole wave.  Log-masses of one head share their leading bits, so in
// the first passes most lanes hit the same bin and plain LDS atomics would serialise 64 ways: up
// to two bins are first counted by ballot (one atomic each), the rest go one by one.
__device__ __forceinline__ void hist_add(uint32_t* hist, uint32_t bin, bool pred) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const unsigned long long active = __ballot(pred);
    if (active == 0ull) return;
    const int leader = __ffsll((long long)active) - 1;
    const uint32_t lb = (uint32_t)__shfl((int)bin, leader);
    const bool same = pred && bin == lb;
    const unsigned long long votes = __ballot(same);
    if (lane == leader) atomicAdd(&hist[lb], (uint32_t)__popcll(votes));
    if (same) pred = false;
  }
  if (pred) atomicAdd(&hist[bin], 1u);
}

// Inclusive scan over the threads of a workgroup with two barriers: shuffles inside each wave,
// then the preceding waves' totals.  `tot` = one word of LDS scratch per wave.
template <typename T>
__device__ __forceinline__ T block_scan_incl(T v, T* tot, int tid) {
  const int l = tid & 63, w = tid >> 6;
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) {
    const T u = __shfl_up(v, s);
    if (l >= s) v += u;
  }
  __syncthreads();            // protects `tot` against the previous use
  if (l == 63) tot[w] = v;
  __syncthreads();
  T off = 0;
  for (int j = 0; j < w; ++j) off += tot[j];
  return v + off;
}

// One workgroup per (batch, query head).  Finds the KL = min(k_limit, nb) best blocks under the
// total order (larger value first, equal values: lower index first) by radix selection over the
// row, ranks them, and takes a prefix.
//   VALUES = false: the row holds INT8 block log-masses; the prefix is the smallest one whose
//                   estimated masses cover tau_cov, clamped, then grown by Rung 1.
//   VALUES = true : the row holds estimated contributions c_b = p_b eta_b (second rung of the
//                   ladder); the prefix is every block with c_b > v_tol and, in the hard-budget
//                   variant, as many more as bring the estimate left under eps_val; cap k_limit.
template <bool VALUES>
__global__ __launch_bounds__(ST) void select_kernel(SelectArgs a) {
  const int tid = threadIdx.x;
  const int hq = blockIdx.x, b = blockIdx.y;
  const int64_t row = (int64_t)b * a.n_q + hq;
  const float* lm = a.lm8 + row * a.nb;
  const int nb = a.nb;
  const int KL = min(max(a.k_limit, a.k_max), min(nb, MAX_K_LIMIT));

  __shared__ uint32_t hist[256];
  __shared__ uint32_t keys[LDS_KEYS];
  const bool cached = nb <= LDS_KEYS;
  __shared__ unsigned long long cand[MAX_K_LIMIT];     // winners, unordered
  __shared__ int sorted_idx[MAX_K_LIMIT];              // their block indices, best first
  __shared__ double pm[MAX_K_LIMIT];                   // prefix sums of their masses
  __shared__ double dtot[ST / 64];
  __shared__ uint32_t utot[ST / 64];
  __shared__ uint32_t s_prefix, s_want, s_cnt;
  __shared__ uint32_t s_idx_prefix, s_idx_want;
  __shared__ int s_k, s_first;

  if (KL == 0) {
    if (tid == 0) a.kstar[row] = 0;
    return;
  }
  const double lse = (double)a.cert[row].lse;
  const float lse_f = a.cert[row].lse;

  // ---- radix selection of the KL-th largest key, 8 bits at a time from the top.  The first pass
  //      also keeps the keys in LDS and sums the estimated mass of the sealed blocks (single-
  //      precision exponentials, accumulated in double; the rest of 1 is the exact trailing tokens).
  double part = 0.0;
  __shared__ int s_done;
  if (tid == 0) {
    s_prefix = 0u;
    s_want = (uint32_t)KL;
    s_done = 0;
  }
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t himask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
    if (tid < 256) hist[tid] = 0u;
    __syncthreads();
    const uint32_t prefix = s_prefix;
    const uint32_t want = s_want;
    if (pass == 0) {
      CQA_ROW_PASS(lm, nb, tid, {
        const uint32_t k = ord32(x);
        if (in) {
          part += VALUES ? (double)x : (double)__expf(x - lse_f);
          if (cached) keys[i] = k;
        }
        hist_add(hist, k >> 24, in);
      })
    } else {
      CQA_KEY_PASS(lm, nb, tid, cached, keys, {
        hist_add(hist, (k >> shift) & 255u, in && (k & himask) == prefix);
      })
    }
    __syncthreads();
    // thread t looks at bin 255 - t, so an inclusive scan over threads counts from the top bin down;
    // the bin to descend into is the one where that count first reaches `want`
    const uint32_t mine = tid < 256 ? hist[255 - tid] : 0u;
    const uint32_t upto = block_scan_incl<uint32_t>(mine, utot, tid);
    if (upto >= want && upto - mine < want) {
      s_want = want - (upto - mine);               // still to take inside the chosen bin
      s_prefix = prefix | ((uint32_t)(255 - tid) << shift);
      // every block of the chosen bin is taken: its lower edge already is the threshold (with
      // distinct log-masses this happens once a bin holds a single block, usually a pass early)
      if (want - (upto - mine) == mine) s_done = 1;
    }
    __syncthreads();
    if (s_done != 0) break;
  }
  const double total_blocks = block_scan_incl<double>(part, dtot, tid);   // last thread: the total
  __shared__ double s_total;
  if (tid == ST - 1) s_total = total_blocks;
  const uint32_t T = s_prefix;                   // key of the KL-th best block
  // blocks with key == T: s_want of them are needed, the ones with the lowest indices.  The last
  // histogram still holds how many there are: when all of them are wanted, which is the rule
  // unless log-masses tie exactly, no index needs to be selected.
  const bool all_ties = s_done != 0 || hist[T & 255u] == s_want;
  __syncthreads();
  if (tid == 0) {
    s_idx_prefix = all_ties ? 0xFFFFFFFFu : 0u;
    s_idx_want = s_want;
    s_cnt = 0u;
    s_first = MAX_K_LIMIT + 1;
  }
  for (int pass = 0; pass < (all_ties ? 0 : 4); ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t himask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
    if (tid < 256) hist[tid] = 0u;
    __syncthreads();
    const uint32_t prefix = s_idx_prefix;
    const uint32_t want = s_idx_want;
    CQA_KEY_PASS(lm, nb, tid, cached, keys, {
      hist_add(hist, (((uint32_t)i) >> shift) & 255u, in && k == T && (((uint32_t)i) & himask) == prefix);
    })
    __syncthreads();
    const uint32_t mine = tid < 256 ? hist[tid] : 0u;   // ascending: the lowest indices are taken first
    const uint32_t upto = block_scan_incl<uint32_t>(mine, utot, tid);
    if (upto >= want && upto - mine < want) {
      s_idx_want = want - (upto - mine);
      s_idx_prefix = prefix | ((uint32_t)tid << shift);
    }
    __syncthreads();
  }
  __syncthreads();
  const uint32_t Tidx = s_idx_prefix;            // largest index taken among the ties
  const double total = s_total;

  // ---- collect the KL winners as composite keys (log-mass order, then lower index first)
  CQA_KEY_PASS(lm, nb, tid, cached, keys, {
    if (in && (k > T || (k == T && (uint32_t)i <= Tidx))) {
      const uint32_t pos = atomicAdd(&s_cnt, 1u);
      if (pos < (uint32_t)MAX_K_LIMIT)
        cand[pos] = ((unsigned long long)k << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)i);
    }
  })
  __syncthreads();
  const int n = (int)min(s_cnt, (uint32_t)KL);
  // ---- rank sort: a winner's place is the number of winners that precede it (keys are distinct)
  for (int i = tid; i < n; i += ST) {
    const unsigned long long mine = cand[i];
    int rank = 0;
    for (int j = 0; j < n; ++j) rank += cand[j] > mine ? 1 : 0;
    sorted_idx[rank] = (int)(0xFFFFFFFFu - (uint32_t)(mine & 0xFFFFFFFFull));
  }
  __syncthreads();
  // ---- masses of the winners, best first, and their inclusive prefix sums: thread t owns place t
  const double m0 = tid < n ? (VALUES ? (double)lm[sorted_idx[tid]] : exp((double)lm[sorted_idx[tid]] - lse)) : 0.0;
  const double upto1 = block_scan_incl<double>(m0, dtot, tid);
  if (tid < MAX_K_LIMIT) pm[tid] = upto1;
  __syncthreads();
  if (!VALUES) {
    // ---- covering prefix: C_k = rho_trail + (mass of the k best); K* never exceeds k_max, so
    //      the search stops there; then clamps and Rung-1 growth
    const double rho_trail = 1.0 - total;
    const int look = min(n, a.k_max);
    for (int kk = tid; kk <= look; kk += ST) {
      const double covered = rho_trail + (kk > 0 ? pm[kk - 1] : 0.0);
      if (covered >= (double)a.tau_cov) atomicMin(&s_first, kk);
    }
    __syncthreads();
    if (tid == 0) {
      int k = s_first <= look ? s_first : nb;             // no prefix up to k_max covers tau_cov
      k = max(a.k_min, min(k, a.k_max));
      k = min(k, nb);
      k = min(k, n);
      // Rung 1
      const double delta = (double)a.cert[row].delta_h, vmax = (double)a.cert[row].v_max;
      const int cap = min(max(a.k_limit, a.k_max), n);
      while (k < cap) {
        const double tail = total - (k > 0 ? pm[k - 1] : 0.0);
        if (!(key_term_d(delta, tail, vmax, a.mass_exp, a.key_bound_mode) > (double)a.eps_key)) break;
        k = min(max(2 * k, 1), cap);
      }
      s_k = k;
      a.kstar[row] = k;
      if (a.score_dev != nullptr) a.score_dev[row] = 0.0f;
    }
  } else {
    // ---- value selection: the blocks over the local threshold form a prefix of the ranking
    //      (count them), the hard-budget rule asks for the smallest prefix that leaves at most
    //      eps_val of the estimate; the longer of the two, capped
    __shared__ int s_over;
    if (tid == 0) s_over = 0;
    __syncthreads();
    for (int kk = tid; kk < n; kk += ST)
      if (lm[sorted_idx[kk]] > a.v_tol) atomicAdd(&s_over, 1);
    if (a.v_greedy) {
      for (int kk = tid; kk <= n; kk += ST) {
        const double left = total - (kk > 0 ? pm[kk - 1] : 0.0);
        if (left <= (double)a.eps_val) atomicMin(&s_first, kk);
      }
    }
    __syncthreads();
    if (tid == 0) {
      int k = s_over;
      if (a.v_greedy) k = max(k, s_first <= n ? s_first : nb);
      k = min(k, min(n, nb));
      s_k = k;
      a.kstar[row] = k;
    }
  }
  __syncthreads();
  const int k = s_k;
  uint32_t* um = a.umask + row * a.mask_words;
  for (int i = tid; i < k; i += ST) {
    const int idx = sorted_idx[i];
    a.sel[row * MAX_K_LIMIT + i] = idx;
    if (idx >= 0 && idx < nb) atomicOr(&um[idx >> 5], 1u << (idx & 31));
  }
}

// Estimated contribution of every block to a head's value term: c_b = exp(l_b - lse) eta_b
// (the paper's rho_hat_b eta_b of its value-promotion rule), one thread per (head, block).
__global__ __launch_bounds__(256) void contrib_kernel(const float* lm8, const float* eta_blk,
                                                      const cqa_head_cert* cert, float* contrib,
                                                      int nb, int n_q, int n_kv) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  const int hq = blockIdx.y, b = blockIdx.z;
  if (i >= nb) return;
  const int64_t row = (int64_t)b * n_q + hq;
  const int64_t grp = (int64_t)b * n_kv + hq / (n_q / n_kv);
  contrib[row * nb + i] = __expf(lm8[row * nb + i] - cert[row].lse) * eta_blk[grp * nb + i];
}

// The exploration draw: 32-bit multiply-xorshift mixer over (block, KV group, seed).
__device__ __forceinline__ uint32_t explore_mix(uint32_t blk, uint32_t grp, uint32_t seed) {
  uint32_t x = blk * 0x9E3779B1u ^ grp * 0x85EBCA77u ^ seed * 0xC2B2AE3Du;
  x ^= x >> 16;
  x *= 0x7FEB352Du;
  x ^= x >> 15;
  x *= 0x846CA68Bu;
  x ^= x >> 16;
  return x;
}

struct CompactArgs {
  uint32_t explore_threshold;   // a block is explored (key-promoted) when its draw is below this; 0 = off
  uint32_t explore_seed;
  uint32_t* vmask;     // [Bt][Hq][mask_words] value selections per head (null = none); cleared likewise
  uint32_t* umask;     // [Bt][Hq][mask_words] key selections per head; cleared on the way out
  int64_t mask_words;
  int group;           // query heads per KV group
  int per_head;        // 1: a head's promoted sets are its own selections; 0: the group's unions
  int32_t* slot;       // [Bt][Hkv][slot_stride]
  int64_t slot_stride;
  int32_t* ulist;      // [Bt][Hkv][MAX_UNION]
  int32_t* ucount;     // [Bt][Hkv]
  int nb;
  // FP16 scratch of the layer (sc_slots = 0: off)
  int32_t* sc_map;     // [Bt][Hkv][sc_map_stride]
  int64_t sc_map_stride;
  int32_t* sc_tag;     // [Bt][Hkv][sc_cap]
  uint32_t* sc_age;    // [Bt][Hkv][sc_cap]
  int32_t* sc_have;    // [Bt][Hkv][sc_cap]
  uint32_t* sc_stats;  // [2]
  int sc_cap, sc_slots;
  uint32_t sc_step;    // stamp of this step (larger than every stamp before it, never 0)
};

// One workgroup per KV group: the heads' bit masks (FP16 keys, FP16 values) -> per-block flags
// (bit 0: some head scores the block with FP16 keys, bit 1: some head attends its FP16 values,
// bits 24-27 / 28-31: which heads; 0 = neither) and the ascending list of blocks with any flag.
// Per-group promotion gives every head the union's bits.  Clears the masks.
__global__ __launch_bounds__(256) void compact_kernel(CompactArgs a) {
  const int tid = threadIdx.x;
  const int64_t grp = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
  uint32_t* um = a.umask + grp * a.group * a.mask_words;        // the group's heads are consecutive rows
  uint32_t* vm = a.vmask != nullptr ? a.vmask + grp * a.group * a.mask_words : nullptr;
  int32_t* slot = a.slot + grp * a.slot_stride;
  int32_t* ulist = a.ulist + grp * MAX_UNION;
  const int words = (a.nb + 31) >> 5;
  __shared__ int itot_c[4];
  __shared__ int s_base;
  // The flag words of the previous call are taken back through its list (the words of all other
  // blocks are zero already: at creation every word is, and only listed blocks are ever set), so
  // a call touches a few dozen words per group instead of one per block.
  {
    const int n_prev = min(a.ucount[grp], MAX_UNION);
    for (int i = tid; i < n_prev; i += 256) {
      const int blk = ulist[i];
      if (blk >= 0 && blk < a.slot_stride) slot[blk] = 0;
    }
  }
  __syncthreads();                       // (with its fence) before the same words are set again
  // thread t owns the contiguous run of mask words [t wpt, (t + 1) wpt): the list comes out ascending
  constexpr int WPT_MAX = 8;             // up to 256 x 8 x 32 blocks (1M tokens) in one sweep
  const int wpt = (words + 255) >> 8;
  int base_total = 0;
  for (int w00 = 0; w00 < words; w00 += 256 * WPT_MAX) {
    const int wpt_here = min(wpt, WPT_MAX);
    uint32_t kb[WPT_MAX], vb[WPT_MAX], khh[WPT_MAX][4], vhh[WPT_MAX][4];
    int cnt = 0;
#pragma unroll
    for (int u = 0; u < WPT_MAX; ++u) {
      const int w = w00 + tid * wpt_here + u;
      uint32_t kbits = 0u, vbits = 0u;
      uint32_t kh[4] = {0u, 0u, 0u, 0u}, vh[4] = {0u, 0u, 0u, 0u};   // per head
      if (u < wpt_here && w < words) {
        for (int i = 0; i < a.group; ++i) {
          kh[i] = um[i * a.mask_words + w];
          if (kh[i] != 0u) um[i * a.mask_words + w] = 0u;
          kbits |= kh[i];
          if (vm != nullptr) {
            vh[i] = vm[i * a.mask_words + w];
            if (vh[i] != 0u) vm[i * a.mask_words + w] = 0u;
            vbits |= vh[i];
          }
        }
        if (a.explore_threshold != 0u) {
          uint32_t ebits = 0u;
#pragma unroll 4
          for (int j = 0; j < 32; ++j)
            if (explore_mix((uint32_t)(w * 32 + j), (uint32_t)grp, a.explore_seed) < a.explore_threshold)
              ebits |= 1u << j;
          kbits |= ebits;                          // explored blocks are promoted for every head
          for (int i = 0; i < a.group; ++i) kh[i] |= ebits;
        }
        if (w == words - 1 && (a.nb & 31)) {      // nothing past nb
          kbits &= (1u << (a.nb & 31)) - 1u;
          vbits &= (1u << (a.nb & 31)) - 1u;
        }
        for (int i = 0; i < 4; ++i) {
          kh[i] = i < a.group ? (a.per_head ? kh[i] & kbits : kbits) : 0u;
          vh[i] = i < a.group ? (a.per_head ? vh[i] & vbits : vbits) : 0u;
        }
      }
      kb[u] = kbits;
      vb[u] = vbits;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        khh[u][i] = kh[i];
        vhh[u][i] = vh[i];
      }
      cnt += __popc(kbits | vbits);
    }
    int pos = base_total + block_scan_incl<int>(cnt, itot_c, tid) - cnt;   // slot of my run's first promoted block
    if (tid == 255) s_base = pos + cnt;
#pragma unroll
    for (int u = 0; u < WPT_MAX; ++u) {
      const int w = w00 + tid * wpt_here + u;
      uint32_t bits = kb[u] | vb[u];
      while (bits != 0u) {
        const int j = __ffs((int)bits) - 1;
        bits &= bits - 1u;
        const int blk = w * 32 + j;
        // the list cannot overflow (4 heads x MAX_K_LIMIT for keys and as many for values);
        // a block that did not fit would simply stay unpromoted
        if (pos < MAX_UNION) {
          uint32_t f = ((kb[u] >> j) & 1u) | (((vb[u] >> j) & 1u) << 1);
#pragma unroll
          for (int i = 0; i < 4; ++i)
            f |= (((khh[u][i] >> j) & 1u) << (SLOT_HK_SHIFT + i)) | (((vhh[u][i] >> j) & 1u) << (SLOT_HV_SHIFT + i));
          slot[blk] = (int)f;
          ulist[pos] = blk;
        }
        ++pos;
      }
    }
    __syncthreads();
    base_total = s_base;
  }
  const int s_base_final = base_total;
  if (tid == 0) a.ucount[grp] = min(s_base_final, MAX_UNION);
  if (a.sc_slots <= 0) return;

  // ---- FP16 scratch: which listed blocks are held on the device, and where the others go.
  // A promoted block found in the map keeps its slot (stamped with this step); a half of it (keys,
  // values) that this step needs and the slot does not hold yet is filled on the way.  The others
  // take over the least recently used slots -- found by a radix selection over the slots' stamps,
  // only in steps that miss -- never one used in this step; the pass that reads their originals
  // from the host stores them into the slot (SLOT_FILL for the keys, SLOT_VFILL for the values).
  // Misses beyond the free slots are read from the host without being kept.
  const int n = min(s_base_final, MAX_UNION);
  int32_t* map = a.sc_map + grp * a.sc_map_stride;
  int32_t* tag = a.sc_tag + grp * (int64_t)a.sc_cap;
  uint32_t* age = a.sc_age + grp * (int64_t)a.sc_cap;
  int32_t* have = a.sc_have + grp * (int64_t)a.sc_cap;
  __shared__ int s_hits, s_part, s_nmiss, s_elig;
  __shared__ int misslist[SC_MAX_SLOTS];
  if (tid == 0) {
    s_hits = 0;
    s_part = 0;
    s_nmiss = 0;
    s_elig = 0;
  }
  __syncthreads();
  for (int i = tid; i < n; i += 256) {
    const int blk = ulist[i];
    const int f = slot[blk];
    const int need = f & (SLOT_KEYS | SLOT_VALUES);
    if (need) {
      const int m = map[blk];
      if (m > 0 && m <= a.sc_slots && tag[m - 1] == blk) {
        const int missing = need & ~have[m - 1];
        age[m - 1] = a.sc_step;
        have[m - 1] |= need;
        slot[blk] = f | (m << SLOT_SC_SHIFT) | ((missing & SLOT_KEYS) ? SLOT_FILL : 0) |
                    ((missing & SLOT_VALUES) ? SLOT_VFILL : 0);
        atomicAdd(missing ? &s_part : &s_hits, 1);
      } else {
        const int k = atomicAdd(&s_nmiss, 1);
        if (k < SC_MAX_SLOTS) misslist[k] = blk;
      }
    }
  }
  __syncthreads();
  const int nmiss = min(s_nmiss, SC_MAX_SLOTS);
  if (tid == 0) {
    atomicAdd(a.sc_stats + 0, (uint32_t)s_hits);
    atomicAdd(a.sc_stats + 1, (uint32_t)(s_nmiss + s_part));
  }
  if (nmiss == 0) return;
  // The `usable` least recently used slots, ties to the lower slot index: radix selection over
  // the 32-bit stamps of the slots that this step does not use (four 8-bit passes: histogram,
  // scan, descend), then two scans in slot order rank the chosen slots.  Thread t owns slots
  // 4t .. 4t+3.
  __shared__ uint32_t hist[256];
  __shared__ uint32_t s_prefix, s_need;
  __shared__ int itot[4];
  __shared__ uint32_t utot[4];
  uint32_t st4[4];
  bool el4[4];
  int elig = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int i = tid * 4 + j;
    st4[j] = i < a.sc_slots ? age[i] : 0xFFFFFFFFu;
    el4[j] = i < a.sc_slots && st4[j] != a.sc_step;
    elig += el4[j] ? 1 : 0;
  }
  atomicAdd(&s_elig, elig);
  __syncthreads();
  const int usable = min(nmiss, s_elig);
  if (usable == 0) return;
  if (tid == 0) {
    s_prefix = 0u;
    s_need = (uint32_t)usable;
  }
  for (int shift = 24; shift >= 0; shift -= 8) {
    hist[tid] = 0u;
    __syncthreads();
    const uint32_t prefix = s_prefix, need = s_need;
    const uint32_t himask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (el4[j] && (st4[j] & himask) == prefix) atomicAdd(&hist[(st4[j] >> shift) & 255u], 1u);
    __syncthreads();
    const uint32_t mine = hist[tid];
    const uint32_t upto = block_scan_incl<uint32_t>(mine, utot, tid);
    if (upto >= need && upto - mine < need) {      // the bin where the count first reaches `need`
      s_need = need - (upto - mine);
      s_prefix = prefix | ((uint32_t)tid << shift);
    }
    __syncthreads();
  }
  const uint32_t T = s_prefix;          // stamp of the last slot taken
  const int need_eq = (int)s_need;      // how many slots with exactly that stamp are taken
  int eq = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) eq += (el4[j] && st4[j] == T) ? 1 : 0;
  int eq_before = block_scan_incl<int>(eq, itot, tid) - eq;
  bool take[4];
  int nt = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const bool is_eq = el4[j] && st4[j] == T;
    take[j] = el4[j] && (st4[j] < T || (is_eq && eq_before < need_eq));
    eq_before += is_eq ? 1 : 0;
    nt += take[j] ? 1 : 0;
  }
  int rank = block_scan_incl<int>(nt, itot, tid) - nt;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (!take[j]) continue;
    if (rank < usable) {
      const int v = tid * 4 + j;
      const int blk = misslist[rank];
      const int old = tag[v];
      if (old >= 0 && old < a.nb && map[old] == v + 1) map[old] = 0;
      tag[v] = blk;
      map[blk] = v + 1;
      age[v] = a.sc_step;
      const int need = slot[blk] & (SLOT_KEYS | SLOT_VALUES);
      have[v] = need;
      slot[blk] |= ((v + 1) << SLOT_SC_SHIFT) | ((need & SLOT_KEYS) ? SLOT_FILL : 0) |
                   ((need & SLOT_VALUES) ? SLOT_VFILL : 0);
    }
    ++rank;
  }
}

struct AdaptiveReduceArgs {
  ReduceArgs ra{};
  const float* lm8;      // [Bt][Hq][nb]
  const float* lmx;      // [Bt][Hq][nb]
  const int32_t* slot;   // [Bt][Hkv][slot_stride]
  int64_t slot_stride;
  float* alpha_out;      // [Bt][Hq]
  const float* score_dev;  // [Bt][Hq] canary deviations, or null
  const float* eta;      // [Bt][Hkv][nb] value annotations eta_b written by the pass over all blocks
  int pos_set0, pos_set1;  // the promoted-block pass's positive partial sets
  const int32_t* ulist;  // [Bt][Hkv][MAX_UNION] listed blocks of the group (ranking depth > 1)
  const int32_t* ucount; // [Bt][Hkv]
};

// One workgroup per (batch, query head): all threads scan the block log-masses of both passes
// (estimated mass left in INT8, best promoted block under either ranking, best unpromoted
// block), then the first wave merges the partial sets of the pass over all blocks and of the
// promoted-block pass and finalises the
// certificate with these substituted.
constexpr int ART = 512;   // threads of the adaptive reduction: 8192 blocks in one trip of 16 per thread
__global__ __launch_bounds__(ART) void adaptive_reduce_kernel(AdaptiveReduceArgs a) {
  const int tid = threadIdx.x;
  const int hq = blockIdx.x, b = blockIdx.y;
  const ReduceArgs& ra = a.ra;
  const int64_t row = (int64_t)b * ra.n_q + hq;
  const int64_t grp = (int64_t)b * ra.n_kv + hq / (ra.n_q / ra.n_kv);
  const float* l8 = a.lm8 + row * ra.nb;
  const float* lx = a.lmx + row * ra.nb;
  const int32_t* slot = a.slot + grp * a.slot_stride;
  // the first pass left its certificate in the caller's array; read what is needed before
  // the first wave overwrites it
  const float lse8 = ra.cert[row].lse;
  const float delta = ra.cert[row].delta_h;

  const float* eta = a.eta + grp * ra.nb;
  const int kbit = 1 << (SLOT_HK_SHIFT + hq % (ra.n_q / ra.n_kv));   // this head scores the block with FP16 keys
  float best_x = -INFINITY, best_8 = -INFINITY, tail_max = -INFINITY, maxc8 = 0.0f;
  int ix = -1, i8 = -1;
  double tail_mass = 0.0, l8u = 0.0, ev8u = 0.0;
  for (int base = 0; base < ra.nb; base += ART * BATCH) {
    float b8[BATCH], bx[BATCH], be[BATCH];
    int bs[BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {       // all loads of the batch first
      const int i = base + j * ART + tid;
      const bool in = i < ra.nb;
      b8[j] = in ? l8[i] : 0.0f;
      bs[j] = in ? slot[i] : 0;
      bx[j] = in ? lx[i] : 0.0f;            // written for listed blocks only; used for key-promoted ones
      be[j] = in ? eta[i] : 0.0f;
    }
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const int i = base + j * ART + tid;
      if (i >= ra.nb) continue;
      const float v8 = b8[j];
      if (bs[j] & kbit) {
        const float vx = bx[j];
        if (vx > best_x) {      // ascending scan per thread: strict > keeps the lowest index
          best_x = vx;
          ix = i;
        }
        if (v8 > best_8) {
          best_8 = v8;
          i8 = i;
        }
      } else {
        const float mass = expf(v8 - lse8);
        tail_max = fmaxf(tail_max, v8);
        tail_mass += (double)mass;
        if (bs[j] == 0) {
          // not listed: the promoted-block pass does not revisit it, it keeps its INT8 mass
          // and its eta_b
          l8u += (double)mass;
          ev8u += (double)(mass * be[j]);
          maxc8 = fmaxf(maxc8, mass * be[j]);
        }
      }
    }
  }
  // reduce over the workgroup: shuffles inside each wave, then the waves' results through LDS
  constexpr int NW = ART / 64;
  __shared__ float s_bx[ART], s_b8[ART];     // (the full-size arrays serve the deeper places below)
  __shared__ int s_ix[ART], s_i8[ART];
  __shared__ float w_bx[NW], w_b8[NW], w_tm[NW], w_mc[NW];
  __shared__ int w_ix[NW], w_i8[NW];
  __shared__ double w_mass[NW], w_l8u[NW], w_ev8u[NW];
  __shared__ float s_top[4];
  __shared__ int s_topi[2];
  __shared__ double s_sum[3];
  __shared__ float wsm[64];
  __shared__ AdaptiveIn s_ad;
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    // larger value wins; equal values: the lower block index (-1 = nothing seen loses)
    const float ox = __shfl_xor(best_x, m);
    const int oix = __shfl_xor(ix, m);
    if (oix >= 0 && (ix < 0 || ox > best_x || (ox == best_x && oix < ix))) {
      best_x = ox;
      ix = oix;
    }
    const float o8 = __shfl_xor(best_8, m);
    const int oi8 = __shfl_xor(i8, m);
    if (oi8 >= 0 && (i8 < 0 || o8 > best_8 || (o8 == best_8 && oi8 < i8))) {
      best_8 = o8;
      i8 = oi8;
    }
    tail_max = fmaxf(tail_max, __shfl_xor(tail_max, m));
    maxc8 = fmaxf(maxc8, __shfl_xor(maxc8, m));
    tail_mass += __shfl_xor(tail_mass, m);
    l8u += __shfl_xor(l8u, m);
    ev8u += __shfl_xor(ev8u, m);
  }
  if ((tid & 63) == 0) {
    const int w = tid >> 6;
    w_bx[w] = best_x;
    w_ix[w] = ix;
    w_b8[w] = best_8;
    w_i8[w] = i8;
    w_tm[w] = tail_max;
    w_mc[w] = maxc8;
    w_mass[w] = tail_mass;
    w_l8u[w] = l8u;
    w_ev8u[w] = ev8u;
  }
  __syncthreads();
  if (tid == 0) {
    float bx = w_bx[0], b8 = w_b8[0], tm = w_tm[0], mc = w_mc[0];
    int jx = w_ix[0], j8 = w_i8[0];
    double ms = w_mass[0], lu = w_l8u[0], eu = w_ev8u[0];
    for (int w = 1; w < NW; ++w) {
      if (w_ix[w] >= 0 && (jx < 0 || w_bx[w] > bx || (w_bx[w] == bx && w_ix[w] < jx))) {
        bx = w_bx[w];
        jx = w_ix[w];
      }
      if (w_i8[w] >= 0 && (j8 < 0 || w_b8[w] > b8 || (w_b8[w] == b8 && w_i8[w] < j8))) {
        b8 = w_b8[w];
        j8 = w_i8[w];
      }
      tm = fmaxf(tm, w_tm[w]);
      mc = fmaxf(mc, w_mc[w]);
      ms += w_mass[w];
      lu += w_l8u[w];
      eu += w_ev8u[w];
    }
    s_top[0] = bx;
    s_top[1] = b8;
    s_top[2] = tm;
    s_top[3] = mc;
    s_topi[0] = jx;
    s_topi[1] = j8;
    s_sum[0] = ms;
    s_sum[1] = lu;
    s_sum[2] = eu;
  }
  __syncthreads();
  // ---- ranking check (the paper's "Ranking-Consistency Check" with its boundary verification)
  //      at depth r: the r best promoted blocks under the FP16 and under the INT8 log-masses must
  //      be the same blocks in the same order, and no unpromoted block may reach the r-th FP16
  //      log-mass with its upper-bounded one.  Depth 1 is what the scan has found; each further
  //      place is one more arg-max over the group's listed blocks (a few dozen, held in registers),
  //      restricted to what comes after the previous place in the order (larger log-mass first,
  //      equal log-masses by lower index).  Fewer promoted blocks than r: the depth is their number.
  const float top_x = s_top[0], top_8 = s_top[1];
  const int top_ix = s_topi[0], top_i8 = s_topi[1];
  bool disagree = top_ix >= 0 && top_ix != top_i8;
  float kth_x = top_x;
  const int depth = min(ra.tol.rank_depth, MAX_RANK_DEPTH);
  if (depth > 1 && top_ix >= 0) {          // uniform over the workgroup
    constexpr int CAND = MAX_UNION / ART;
    float cx[CAND], c8[CAND];
    int cb[CAND];
    const int n = min(a.ucount[grp], MAX_UNION);
    const int32_t* ulist = a.ulist + grp * MAX_UNION;
#pragma unroll
    for (int j = 0; j < CAND; ++j) {
      const int i = j * ART + tid;
      const int blk = i < n ? ulist[i] : -1;
      const bool keyp = blk >= 0 && blk < ra.nb && (slot[blk] & kbit);
      cb[j] = keyp ? blk : -1;
      cx[j] = keyp ? lx[blk] : 0.0f;
      c8[j] = keyp ? l8[blk] : 0.0f;
    }
    float px = top_x, p8 = top_8;
    int pix = top_ix, pi8 = top_i8;
    __syncthreads();                        // every thread has read the depth-1 results
    for (int k = 1; k < depth; ++k) {
      float bx = -INFINITY, b8 = -INFINITY;
      int jx = -1, j8 = -1;
#pragma unroll
      for (int j = 0; j < CAND; ++j) {
        if (cb[j] < 0) continue;
        if ((cx[j] < px || (cx[j] == px && cb[j] > pix)) &&
            (jx < 0 || cx[j] > bx || (cx[j] == bx && cb[j] < jx))) {
          bx = cx[j];
          jx = cb[j];
        }
        if ((c8[j] < p8 || (c8[j] == p8 && cb[j] > pi8)) &&
            (j8 < 0 || c8[j] > b8 || (c8[j] == b8 && cb[j] < j8))) {
          b8 = c8[j];
          j8 = cb[j];
        }
      }
      s_bx[tid] = bx;
      s_ix[tid] = jx;
      s_b8[tid] = b8;
      s_i8[tid] = j8;
      __syncthreads();
      for (int st = ART / 2; st > 0; st >>= 1) {
        if (tid < st) {
          const float ox = s_bx[tid + st];
          const int oix = s_ix[tid + st];
          if (oix >= 0 && (s_ix[tid] < 0 || ox > s_bx[tid] || (ox == s_bx[tid] && oix < s_ix[tid]))) {
            s_bx[tid] = ox;
            s_ix[tid] = oix;
          }
          const float o8 = s_b8[tid + st];
          const int oi8 = s_i8[tid + st];
          if (oi8 >= 0 && (s_i8[tid] < 0 || o8 > s_b8[tid] || (o8 == s_b8[tid] && oi8 < s_i8[tid]))) {
            s_b8[tid] = o8;
            s_i8[tid] = oi8;
          }
        }
        __syncthreads();
      }
      const float nx = s_bx[0], n8 = s_b8[0];
      const int nix = s_ix[0], ni8 = s_i8[0];
      __syncthreads();                      // read before the next round overwrites
      if (nix < 0) break;                   // fewer promoted blocks than the depth (uniform)
      disagree = disagree || nix != ni8;
      kth_x = nx;
      px = nx;
      pix = nix;
      p8 = n8;
      pi8 = ni8;
    }
  }
  if (tid == 0) {
    AdaptiveIn ad;
    ad.alpha = (float)s_sum[0];
    ad.delta = delta;
    ad.top_block = top_ix;
    ad.top_fp16 = top_ix >= 0 ? top_x : -INFINITY;
    ad.kth_fp16 = top_ix >= 0 ? kth_x : -INFINITY;
    const float tmax = s_top[2];
    const bool has_tail = tmax > -INFINITY;
    ad.tail_ub = has_tail ? tmax + delta : -INFINITY;
    const bool boundary = top_ix >= 0 && has_tail && tmax + delta + ra.tol.eps_guard > kth_x;
    ad.rank_fail = (disagree || boundary) ? 1 : 0;
    ad.precond = (a.score_dev != nullptr && a.score_dev[row] > delta + ra.tol.eps_guard) ? 1 : 0;
    ad.pos_set0 = a.pos_set0;
    ad.pos_set1 = a.pos_set1;
    ad.L8u = (float)s_sum[1];
    ad.EV8u = (float)s_sum[2];
    ad.maxc8 = s_top[3];
    ad.lse8 = lse8;
    s_ad = ad;
    a.alpha_out[row] = ad.alpha;
  }
  __syncthreads();
  if (tid < 64) reduce_head_wave(ra, b, hq, wsm, &s_ad);
}

}  // namespace

int32_t launch_adaptive(Cache* c, int layer, const __half* q, const cqa_tolerances& tol,
                        const cqa_selector& sel, float* O, cqa_head_cert* cert, uint32_t* flags,
                        uint32_t* flags_mirror, uint32_t mirror_tag, hipStream_t st) {
  // quantised-query scoring: the pass over all blocks scores on the INT8 matrix cores, the
  // promoted-block pass reproduces those scores for the blocks (and heads) that stay in INT8
  if (tol.int8_query != 0 && c->variant != 0) return CQA_ERR_UNSUPPORTED;
  const int bt = c->desc.batch, hq = c->desc.n_q_heads, hkv = c->desc.n_kv_heads;
  const int g = hq / hkv;
  const int64_t len = c->length[layer];
  const int64_t nb = len / BLK;
  const int r = (int)(len % BLK);
  AdaptiveWs& w = c->ad;

  // ---- 1. one pass over all sealed blocks in INT8 / INT4 (the ordinary certified pass): block
  //         log-masses, eta_b and the partial sets the promoted-block pass will correct.  Every
  //         threshold is off: its certificate only feeds the selector (lse, Delta_h, V_max) and
  //         is overwritten below.
  int nsplit = 0, bps = 0;
  split_geometry(c, nb, &nsplit, &bps);
  const int total = nsplit + 2 * PROM_SPLITS;
  cqa_tolerances loose = tol;
  loose.eps_total = loose.eps_key = loose.eps_val = loose.v_tol = INFINITY;
  loose.rank_depth = 0;
  loose.force_flags = 0;
  if (nb == 0) {
    // nothing sealed: the exact trailing tokens are the answer, with the caller's thresholds
    return launch_certified(c, layer, q, tol, O, cert, flags, flags_mirror, mirror_tag, nullptr, st);
  }
  int32_t rc = launch_certified(c, layer, q, loose, O, cert, flags, nullptr, 0u, w.lm8, st, nullptr, nullptr,
                                total, w.eta_blk);
  if (rc != CQA_OK) return rc;

  // ---- 2. selection per head (+ Rung 1), union bit mask per group
  SelectArgs sa{};
  sa.lm8 = w.lm8;
  sa.cert = cert;
  sa.sel = w.sel;
  sa.kstar = w.kstar;
  sa.umask = w.umask;
  sa.mask_words = w.mask_words;
  sa.nb = (int)nb;
  sa.n_q = hq;
  sa.n_kv = hkv;
  sa.tau_cov = sel.tau_cov;
  sa.k_min = sel.k_min;
  sa.k_max = sel.k_max;
  sa.k_limit = sel.k_limit;
  sa.eps_key = tol.eps_key;
  sa.mass_exp = tol.mass_exp;
  sa.key_bound_mode = tol.key_bound_mode;
  sa.v_tol = tol.v_tol;
  sa.eps_val = tol.eps_val;
  sa.v_greedy = sel.v_greedy;
  sa.score_dev = sel.canary ? w.score_dev : nullptr;
  hipLaunchKernelGGL(select_kernel<false>, dim3(hq, bt), dim3(ST), 0, st, sa);
  CQA_HIP(hipGetLastError());
  const bool values = sel.v_limit > 0;
  if (values) {
    // value promotion: rank the estimated contributions p_b eta_b
    hipLaunchKernelGGL(contrib_kernel, dim3((unsigned)((nb + 255) / 256), hq, bt), dim3(256), 0, st,
                       w.lm8, w.eta_blk, cert, w.contrib, (int)nb, hq, hkv);
    CQA_HIP(hipGetLastError());
    SelectArgs va = sa;
    va.lm8 = w.contrib;
    va.sel = w.vsel;
    va.kstar = w.vcount;
    va.umask = w.vmask;
    va.k_min = 0;
    va.k_max = sel.v_limit;
    va.k_limit = sel.v_limit;
    va.score_dev = nullptr;
    hipLaunchKernelGGL(select_kernel<true>, dim3(hq, bt), dim3(ST), 0, st, va);
    CQA_HIP(hipGetLastError());
  }

  // ---- 3. slot map and ordered list per group
  CompactArgs ca{};
  {
    const double thr = (double)sel.explore_frac * 4294967296.0;
    ca.explore_threshold = sel.explore_frac > 0.0f ? (uint32_t)std::min(thr, 4294967295.0) : 0u;
    ca.explore_seed = sel.explore_seed;
  }
  ca.vmask = values ? w.vmask : nullptr;
  ca.umask = w.umask;
  ca.group = g;
  ca.per_head = sel.per_head;
  ca.mask_words = w.mask_words;
  ca.slot = w.slot;
  ca.slot_stride = c->nq_cap * 4;
  ca.ulist = w.ulist;
  ca.ucount = w.ucount;
  ca.nb = (int)nb;
  const int64_t layer_head0 = head_index(c, layer, 0, 0);
  ca.sc_slots = w.sc_slots;
  if (w.sc_slots > 0) {
    w.sc_step += 1u;
    ca.sc_map = w.sc_map + layer_head0 * c->nb_cap;
    ca.sc_map_stride = c->nb_cap;
    ca.sc_tag = w.sc_tag + layer_head0 * w.sc_cap;
    ca.sc_age = w.sc_age + layer_head0 * w.sc_cap;
    ca.sc_have = w.sc_have + layer_head0 * w.sc_cap;
    ca.sc_stats = w.sc_stats;
    ca.sc_cap = w.sc_cap;
    ca.sc_step = w.sc_step;
  }
  hipLaunchKernelGGL(compact_kernel, dim3(hkv, bt), dim3(256), 0, st, ca);
  CQA_HIP(hipGetLastError());

  // ---- 4. promoted-block pass: the listed blocks once more with the originals their flags ask
  //         for (positive sets) and once as the first pass saw them (negated sets)
  ReduceArgs ra{};
  ra.partials = c->partials;
  ra.q = q;
  ra.trail_k = c->trail_k + layer_head0 * BLK * D;
  ra.trail_v = c->trail_v + layer_head0 * BLK * D;
  ra.O = O;
  ra.cert = cert;
  ra.flags = flags;
  ra.flags_mirror = flags_mirror;
  ra.mirror_tag = mirror_tag;
  ra.tol = tol;
  ra.nsplit = total;
  ra.nb = (int)nb;
  ra.r = r;
  ra.n_q = hq;
  ra.n_kv = hkv;
  DecodeArgs a{};   // every field starts null / zero
  a.t1 = c->t1 + layer_head0 * c->nq_cap * QUAD_BYTES;
  a.sigmax = c->sigmax + layer_head0;
  a.q = q;
  a.partials = c->partials;
  a.blk_logmass = w.lmx;
  a.nq_cap = c->nq_cap;
  a.nb = (int)nb;
  a.nsplit = nsplit;
  a.pstride = total;
  a.bps = bps;
  a.n_q = hq;
  a.n_kv = hkv;
  a.slot = w.slot;
  a.sc_k = w.sc_slots > 0 ? w.sc_k + layer_head0 * w.sc_cap * BLK * D : nullptr;
  a.sc_v = w.sc_slots > 0 ? w.sc_v + layer_head0 * w.sc_cap * BLK * D : nullptr;
  a.sc_cap = w.sc_cap;
  a.ulist = w.ulist;
  a.ucount = w.ucount;
  a.t2_k = c->t2_k + layer_head0 * c->desc.max_tokens * D;
  a.t2_v = c->t2_v + layer_head0 * c->desc.max_tokens * D;
  a.eta_out = nullptr;
  a.score_dev = sel.canary ? w.score_dev : nullptr;
  a.int8_query = tol.int8_query;
  a.max_tokens = c->desc.max_tokens;
  a.split0 = nsplit;
  rc = launch_promoted_pass(a, g, dim3(2 * PROM_SPLITS, hkv, bt), st);
  if (rc != CQA_OK) return rc;

  // ---- 5. merge, certificate with the achieved tail, ranking check
  AdaptiveReduceArgs ar{};
  ar.ra = ra;
  ar.lm8 = w.lm8;
  ar.lmx = w.lmx;
  ar.slot = w.slot;
  ar.slot_stride = c->nq_cap * 4;
  ar.alpha_out = w.alpha;
  ar.score_dev = sel.canary ? w.score_dev : nullptr;
  ar.eta = w.eta_blk;
  ar.pos_set0 = nsplit;
  ar.pos_set1 = nsplit + PROM_SPLITS;
  ar.ulist = w.ulist;
  ar.ucount = w.ucount;
  hipLaunchKernelGGL(adaptive_reduce_kernel, dim3(hq, bt), dim3(ART), 0, st, ar);
  CQA_HIP(hipGetLastError());
  return CQA_OK;
}

}  // namespace cqa
