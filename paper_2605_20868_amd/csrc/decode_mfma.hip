// Certified decode, split-K pass on the matrix cores (gfx950 MFMA, 64-wide waves).
//
// Same mathematics as the paper's Algorithm 1 with no promoted blocks and its
// scaled-query identity  q . k_hat = sum_c (q_c sigma_c) code_c + sum_c q_c z_c;
// the two contractions run as 16x16x32 MFMAs with FP32 accumulation:
//
//  scores   S[(h, j)][token] = sum_c q~[(h, j)][c] * code[token][c]            (FP16 inputs)
//           One wave takes four consecutive blocks (a "quad") per iteration.
//           B = the 16 tokens of block i as the exact FP16 integers 1152 + code (the stored byte
//           dropped into the mantissa of 1024.0: one operation per two codes); the bias leaves
//           through one more product of the same A operand with a column of ones, which yields
//           sum_c q~[(h, j)][c] for every row, so it cancels exactly whatever A was rounded to;
//           A = 16 rows = 4 query heads x the 4 blocks of the quad, each row holding that
//           block's scaled query q~ = q (.) sigma as TWO FP16 terms (hi + lo, 22 significant
//           bits), q pre-scaled per head by a power of two so that q~ cannot overflow FP16;
//           only the rows of block i are kept from B_i's product.  Forming A once per quad
//           keeps every lane busy: lane (n, kg) owns row n, channels of slice kg.
//  values   O[(h, g')][c] = sum_t w[t][(h, g')] * (16 + code[t][c])               (bf16 inputs)
//           w = p_t * scale_{t,g} as TWO bf16 terms, K = 32 tokens (two blocks),
//           one 16-channel value group per tile; the bias 16 (which makes the
//           4-bit code an exact bf16 by bit insertion) leaves through a product of the same
//           weights with a column of ones (sum_t w[t][(h, g')], so it cancels exactly), and the
//           group offsets are added as  sum_t p_t offset_{t,g},  accumulated on the VALU.
//
// Lane roles (l = lane, n = l & 15, kg = l >> 4, h = n >> 2, j = g' = n & 3):
//   operand forming: scaled query of row (head h, block j), channels of slice kg;
//                    value weights of row (head h, group g'), 8-token slice kg
//   score results  : C_i[row 4 kg + v][col n] -> head kg, block v (v == i kept), token n, so the
//                    softmax state of head kg lives in row kg and token reductions are DPP row ops
//   accumulators   : acc_g[row 4 kg + v][col n] -> head kg, group set member v = g & 3, channel n
// The raw data of the next quad is loaded while the current one is processed; the per-block
// metadata (sigma, z, scale, offset) is staged through wave-private LDS so that each byte is
// fetched once although four heads consume it.
#include <hip/hip_ext.h>

#include "cqa_internal.h"
#include "reduce_inl.h"

namespace cqa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

union BF8 {
  bf16x8 v;
  uint32_t u[4];
};
union HF8 {
  f16x8 v;
  uint32_t u[4];
};

// Loads of Tier-1 records, which a launch reads exactly once.  NT = with the non-temporal hint.
// Measured on a pure read stream of this shape: when every launch reads memory that no recent
// launch has touched (a layer stack, or one layer beyond ~500 MB) the hinted loads reach
// 6.9 TB/s against 6.1 TB/s for plain ones; when one 300 MB layer is read over and over, plain
// loads find part of it in the memory-side cache (7.1 against 7.0 TB/s).  The host picks.
template <bool NT>
__device__ __forceinline__ u32x4 ld_stream(const uint8_t* p) {
  if (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return *reinterpret_cast<const u32x4*>(p);
}
template <bool NT>
__device__ __forceinline__ uint4 ld_stream4(const uint8_t* p) {
  const u32x4 v = ld_stream<NT>(p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// two FP32 values -> packed FP16, round toward zero (never overflows to infinity); x0 in the low half
__device__ __forceinline__ f16x2 pack_f16_rtz(float x0, float x1) {
  return __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(x0, x1));
}
// stored bytes (b_lo, b_hi) of a dword, b = code + 128 -> FP16 pair (1152 + code_lo, 1152 + code_hi):
// the byte is dropped into the mantissa of 1024.0 (0x6400 | b = 1024 + b exactly)
template <uint32_t SEL>
__device__ __forceinline__ uint32_t bytes_to_f16_biased(uint32_t d) {
  return __builtin_amdgcn_perm(0x64646464u, d, SEL);
}
constexpr float K_BIAS = 1152.0f;

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
// (mask & a) | (~mask & b) in one VALU operation (v_bfi_b32)
__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(r) : "s"(mask), "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float trunc_bf16(float x) {
  return __uint_as_float(__float_as_uint(x) & 0xffff0000u);
}

constexpr int KM_ROW = 2 * D + 4;       // floats per staged K-meta block (+4: bank spread over blocks)
constexpr int VM_ROW = 2 * BLK * NG + 32;  // halves per staged V-meta block (+32: bank spread)
constexpr int P_HEAD = 4 * BLK + 16;    // floats per head in the probability buffer

// LM: also writes the block log-masses (and, when asked, eta_b per block) for callers that rank
// blocks afterwards.  NT: Tier-1 loads carry the non-temporal hint.
// Q8: INT8 x INT8 scoring (the paper's optional tensor-core scoring mode): per block the scaled
//     query is quantised to 8 bits with one scale per (head, block) row, s_q = max_c |q~_c| / 127,
//     and scored against the stored key codes by mfma_i32_16x16x64_i8; the block's score bound
//     grows by the explicit term (128 / sqrt d) sum_c |q~_c - s_q T_c|.
// W: waves per workgroup, 8 (one workgroup per compute unit) or 4 (two); either way a SIMD holds two waves.
template <int G, bool LM, bool NT, bool Q8, int W>
__global__ __launch_bounds__(64 * W, 8 / W) void certified_split_mfma_kernel(DecodeArgs a) {
  const int l = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = l & 15, kg = l >> 4;
  const int h = n >> 2, j = n & 3;   // operand-forming role: (head, block of quad) / (head, group)
  // Workgroup -> (head, partial set) and this wave's quads: the head's quads are dealt round-robin
  // over its W * nsplit waves (wave ci takes quads ci, ci + nw, ...), so counts differ by at most one
  // and, the waves advancing at about the same pace, the launch reads a window of consecutive
  // records that moves through the head (measured against contiguous runs per wave: the same with
  // one layer read over and over, 0.5 us faster when nothing is left in the caches).  A wave still
  // meets its blocks in increasing order.
  // (Measured and not adopted: handing the quads out from per-head counters, so that faster XCDs
  // and earlier workgroups take more -- per-wave clock stamps show the waves of a launch finishing
  // up to 10 us apart.  Atomics on one address are served at ~130 ns each across XCDs, far too
  // slow for one draw per quad, and a simulation on the measured per-wave speeds showed that at
  // a granularity of one quad (~4.5 us of work) even an ideal greedy schedule gains < 1 us.
  // Likewise uneven static deals -- longer runs for the first workgroup of every compute unit,
  // shares weighted by XCD -- measured no faster.)
  const int nquads = (a.nb + 3) >> 2;
  const int L = blockIdx.x;
  const int head = L / a.nsplit, split = L - head * a.nsplit;
  // a SIMD holds two waves: w and w + 4 of the one workgroup on its compute unit (W = 8), or wave w
  // of each of the two (W = 4; the second half of the launch order presumably arrives later);
  // "younger" names the second of them in the priority scheme below
  const bool younger = W == 8 ? w >= 4 : 2 * L >= (int)gridDim.x;
  constexpr int Q_NONE = 0x40000000;   // "no quad": larger than any quad index
  int q_cur, q_next, q_stop;
  const int q_step = W * a.nsplit;     // waves of the head
  {
    const int ci = W * split + w;
    q_stop = nquads;
    q_cur = ci < nquads ? ci : Q_NONE;
    q_next = ci + q_step < nquads ? ci + q_step : Q_NONE;
  }
  const int b = head / a.n_kv, kvh = head - b * a.n_kv;
  const int64_t head_rec = (int64_t)head * a.nq_cap;
  const float inv_sqrt_d = 0.08838834764831845f;

  __shared__ __align__(16) float kmbuf[W][4][KM_ROW];    // [wave][block of quad][sigma | z]
  __shared__ __align__(16) __half vmbuf[W][4][VM_ROW];   // [wave][block of quad][scale | offset]
  __shared__ __align__(16) float pbuf[W][4][P_HEAD];     // [wave][head][block of quad][token]
  __shared__ __align__(16) float cbuf[W][3][4][4];       // [wave][c_b | Delta_b | s_q][head][block]
  __shared__ float abuf[W][4];                           // [wave][head] rescale factor of the step
  __shared__ __align__(16) float qbuf[4][D + 4];         // [head][channel], FP32 query times S_h
  __shared__ float sbuf[4];                              // [head] 1 / S_h
  __shared__ __align__(16) float mo[W][G][D];
  __shared__ float ms[W][G][12];

  // A one-token append that rides on this launch: the first wave of each KV group's first
  // workgroup stores the group's new key and value (2 x 256 bytes) into the trailing block and
  // the pinned originals.  This pass reads sealed blocks only; the reduction, which attends the
  // trailing tokens, runs after this launch has completed.
  if (a.ap_k_new != nullptr && split == 0 && w == 0) {
    const int64_t grp = (int64_t)b * a.n_kv + kvh;
    const uint32_t kx = reinterpret_cast<const uint32_t*>(a.ap_k_new + grp * D)[l];
    const uint32_t vx = reinterpret_cast<const uint32_t*>(a.ap_v_new + grp * D)[l];
    reinterpret_cast<uint32_t*>(a.ap_trail_k + (grp * BLK + a.ap_slot) * D)[l] = kx;
    reinterpret_cast<uint32_t*>(a.ap_trail_v + (grp * BLK + a.ap_slot) * D)[l] = vx;
    if (a.ap_t2_k != nullptr) {
      reinterpret_cast<uint32_t*>(a.ap_t2_k + (grp * a.ap_max_tokens + a.ap_pos) * D)[l] = kx;
      reinterpret_cast<uint32_t*>(a.ap_t2_v + (grp * a.ap_max_tokens + a.ap_pos) * D)[l] = vx;
    }
  }
  // Wave priorities.  A SIMD holds one wave of each of the two workgroups resident on its CU and,
  // at equal priority, always issues the older wave first: left alone, the older workgroup runs
  // ~25 % faster and the younger one finishes the launch alone on a half-empty CU.  So the short
  // set-up runs at the highest priority (ahead of other waves' main loops), and in the main loop a
  // wave is high while it forms operands for the score product and low during the value product,
  // the presumably younger workgroup (second half of the launch order) one level above the older
  // one in the high phase: of the four phase combinations each wave then wins two.
  __builtin_amdgcn_s_setprio(3);
  // This wave's query row (head w of the group), requested before the bulk loads: loads return in
  // order, so the row arrives first and the set-up below does not wait for a whole quad.
  __half2 q_in = __floats2half2_rn(0.0f, 0.0f);
  if (w < G)
    q_in = *reinterpret_cast<const __half2*>(a.q + ((int64_t)b * a.n_q + kvh * G + w) * D + 2 * l);
  const float sigmax_head = a.sigmax[(int64_t)b * a.n_kv + kvh];

  // Loads of one quad = one Tier-1 record.  Every address is the record's wave-uniform base plus
  // a constant plus a per-lane 32-bit offset that never changes, so the loop carries no vector
  // address arithmetic.  The prefetch issued by a wave's last iteration is never used: it is
  // aimed at one record per head that every wave shares (the head's first), which stays in L2, so
  // it costs no HBM traffic.  A ragged last quad of the head reads the not yet sealed blocks of
  // its record, which hold zeros and are masked out.
  // The prefetch is unconditional on purpose: guarding it with a branch makes every prefetched
  // register a phi and costs dozens of spilled VGPRs.
  //   K codes : block i, channel half cq; lane (token n, kg) takes bytes [16 l, +16) of each KB
  //   V codes : pair P, group set gs; lane (channel n, 8-token slice kg)
  //   metadata: each byte once per wave -- K meta of block i bytes [16 l, +16); V meta of blocks
  //             2P + (l >> 5) bytes [16 (l & 31), +16); (eta, nu) of block i (wave-uniform)
  const uint8_t* const head_base = a.t1 + head_rec * QUAD_BYTES;
  const uint32_t lo16 = (uint32_t)l * 16u;
  const uint32_t vo16 = (uint32_t)kg * 512u + (uint32_t)n * 16u;
// QI: a quad index, or Q_NONE (then the head's first record absorbs the load)
#define CQA_REC(QI) (head_base + (int64_t)((QI) < nquads ? (QI) : 0) * QUAD_BYTES)
#define CQA_LOAD_K(QB, CQ)                                                               \
  {                                                                                      \
    const uint8_t* rec = CQA_REC(QB) + (Q_KC + (CQ) * 1024);                             \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                        \
      kraw[i][CQ] = ld_stream4<NT>(rec + i * KC_BYTES + lo16);                               \
  }
#define CQA_LOAD_V(QB, P)                                                                \
  {                                                                                      \
    const uint8_t* rec = CQA_REC(QB) + (Q_VC + (P) * 2 * VC_BYTES);                      \
    vraw[P][0] = ld_stream4<NT>(rec + vo16);                                                 \
    vraw[P][1] = ld_stream4<NT>(rec + 256 + vo16);                                           \
  }
#define CQA_LOAD_META(QB)                                                                \
  {                                                                                      \
    const uint8_t* rec = CQA_REC(QB);                                                    \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                      \
      km_n[i] = ld_stream<NT>(rec + (Q_KM + i * KM_BYTES) + lo16);                           \
      an_n[i] = *reinterpret_cast<const float2*>(rec + (Q_AN + i * AN_BYTES));           \
    }                                                                                    \
    _Pragma("unroll") for (int P = 0; P < 2; ++P)                                        \
      vm_n[P] = ld_stream<NT>(rec + (Q_VM + P * 2 * VM_BYTES) + lo16);                   \
  }

  // The first quad is requested before anything else, so the query set-up below runs under the
  // latency of these loads.
  // Software pipeline without extra registers: every piece of raw data is re-requested for the
  // NEXT quad right after its last use for the current one, into the registers it has just
  // freed -- K codes per channel half (after slices u = 1 and u = 3), V codes per pair of
  // blocks -- so each load has 70-85 % of an iteration to arrive and the requests are spread
  // evenly over time.  The metadata of quad k+1 is requested at the top of iteration k.
  uint4 kraw[4][2], vraw[2][2];
  u32x4 km_n[4], vm_n[2];
  float2 an_n[4];
  if (q_cur < nquads) {
    CQA_LOAD_META(q_cur)
    CQA_LOAD_K(q_cur, 0)
    CQA_LOAD_K(q_cur, 1)
    CQA_LOAD_V(q_cur, 0)
    CQA_LOAD_V(q_cur, 1)
  }

  // Queries of the group as FP32 in LDS, rows of absent heads zero, each head pre-scaled by a
  // power of two S_h chosen so that |q S_h sigma| <= 2^14 for every sigma of this KV head (its
  // running maximum is kept at seal time): the scaled query then fits FP16 without overflow, and
  // elements too small for a normal FP16 low part are negligible against the largest ones.
  // Wave w prepares the row of head w.
  // Lane (h, kg) reads channels (u>>1)*64 + kg*16 + (u&1)*8 + e of head h when it forms slice u.
  if (w < 4) {   // qbuf has four rows; the other waves of the workgroup have none to prepare
    float2 qq = __half22float2(q_in);
    float qmax = fmaxf(fabsf(qq.x), fabsf(qq.y));
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) qmax = fmaxf(qmax, __shfl_xor(qmax, m));
    const float bound = qmax * sigmax_head;
    int e = 0;
    (void)frexpf(bound, &e);                       // bound < 2^e
    e = bound > 0.0f ? min(max(14 - e, -100), 100) : 0;
    const float S = ldexpf(1.0f, e);
    qq.x *= S;
    qq.y *= S;
    *reinterpret_cast<float2*>(&qbuf[w][2 * l]) = qq;
    if (l == 0) sbuf[w] = ldexpf(1.0f, -e);
  }
  __syncthreads();
  const float unscale_op = sbuf[h];                // 1 / S of my operand head
  // raw MFMA sum -> logit in units of ln 2 (the softmax state below is kept in base 2: v_exp_f32
  // and v_log_f32 are base-2 instructions), for my softmax head
  const float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;
  const float score_scale = sbuf[kg] * (inv_sqrt_d * LOG2E);
  HF8 ones_h;
  BF8 ones_b;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ones_h.u[i] = 0x3C003C00u;   // FP16 1.0
    ones_b.u[i] = 0x3F803F80u;   // bf16 1.0
  }

  // softmax state of head kg (replicated over the 16 lanes of the row)
  float m_run = -INFINITY, l_run = 0.0f, ev = 0.0f, evmax = 0.0f, dmax = 0.0f, vmax = 0.0f;
  float t1 = -INFINITY, t2 = -INFINITY;
  int i1 = -1;
  float offacc[2] = {0.0f, 0.0f};   // sum_t p_t offset_t of (head h, groups g', 4 + g'), operand role
  f32x4 acc[8], accw[2];             // accw[gs][v]: sum_t w_t of (head kg, group 4 gs + v), every column
#pragma unroll
  for (int g = 0; g < 8; ++g) acc[g] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  accw[0] = accw[1] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

  while (q_cur < nquads) {
    if (younger) __builtin_amdgcn_s_setprio(2); else __builtin_amdgcn_s_setprio(1);
    const int qb = 4 * q_cur;   // first block of the quad
    bool live[4];               // block exists (the head's last quad may be ragged)
#pragma unroll
    for (int i = 0; i < 4; ++i) live[i] = qb + i < a.nb;
    float2 an[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      an[i] = an_n[i];
      reinterpret_cast<u32x4*>(&kmbuf[w][i][0])[l] = km_n[i];
    }
#pragma unroll
    for (int P = 0; P < 2; ++P)
      reinterpret_cast<u32x4*>(&vmbuf[w][2 * P + (l >> 5)][0])[l & 31] = vm_n[P];
    CQA_LOAD_META(q_next)
    wave_sync();

    float craw[4];                  // raw score sum of (head kg, block i, token n), before c_b
    float csum = 0.0f, dsum = 0.0f, qres = 0.0f, sq = 1.0f;
    if constexpr (!Q8) {
      // ---- scores.  A operand: scaled query of row-role (h, j), two FP16 terms (hi + lo);
      //      B operand: the 16 tokens of block i, their signed codes as exact FP16 integers.
      //      C_i[row (head kg, block v)][col token n]: row v == i is the one kept.
      f32x4 C[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) C[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
      f32x4 R = f32x4{0.0f, 0.0f, 0.0f, 0.0f};   // R[v] = sum_c q~ of row (head kg, block v), every column
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c0 = (u >> 1) * 64 + kg * 16 + (u & 1) * 8;
        const float4 s0 = *reinterpret_cast<const float4*>(&kmbuf[w][j][c0]);
        const float4 s1 = *reinterpret_cast<const float4*>(&kmbuf[w][j][c0 + 4]);
        const float4 z0 = *reinterpret_cast<const float4*>(&kmbuf[w][j][D + c0]);
        const float4 z1 = *reinterpret_cast<const float4*>(&kmbuf[w][j][D + c0 + 4]);
        const float4 q0 = *reinterpret_cast<const float4*>(&qbuf[h][c0]);
        const float4 q1 = *reinterpret_cast<const float4*>(&qbuf[h][c0 + 4]);
        const float sg[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
        const float zz[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
        const float qq[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
        float qt[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float qv = qq[e];
          qt[e] = qv * sg[e];
          csum = fmaf(qv, zz[e], csum);
          dsum = fmaf(fabsf(qv), sg[e], dsum);
        }
        HF8 qh2, ql2;   // scaled query = hi + lo, two FP16 terms (22 significant bits)
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const f16x2 hp = pack_f16_rtz(qt[2 * p], qt[2 * p + 1]);
          const f16x2 lp = pack_f16_rtz(qt[2 * p] - (float)hp[0], qt[2 * p + 1] - (float)hp[1]);
          qh2.u[p] = __builtin_bit_cast(uint32_t, hp);
          ql2.u[p] = __builtin_bit_cast(uint32_t, lp);
        }
        HF8 kv[4];      // 1152 + code for the 8 codes of my token and channel slice in each block
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint4 kx = kraw[i][u >> 1];
          const uint32_t d0 = (u & 1) ? kx.z : kx.x, d1 = (u & 1) ? kx.w : kx.y;
          kv[i].u[0] = bytes_to_f16_biased<0x04010400u>(d0);
          kv[i].u[1] = bytes_to_f16_biased<0x04030402u>(d0);
          kv[i].u[2] = bytes_to_f16_biased<0x04010400u>(d1);
          kv[i].u[3] = bytes_to_f16_biased<0x04030402u>(d1);
        }
        // consecutive MFMAs go to different accumulators, so none waits for its predecessor
#pragma unroll
        for (int i = 0; i < 4; ++i)
          C[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(qh2.v, kv[i].v, C[i], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          C[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ql2.v, kv[i].v, C[i], 0, 0, 0);
        R = __builtin_amdgcn_mfma_f32_16x16x32_f16(qh2.v, ones_h.v, R, 0, 0, 0);
        R = __builtin_amdgcn_mfma_f32_16x16x32_f16(ql2.v, ones_h.v, R, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);   // keep the four channel slices apart (register pressure)
        if (u == 1) {
          CQA_LOAD_K(q_next, 0)
          __builtin_amdgcn_sched_barrier(0);
        }
        if (u == 3) {
          CQA_LOAD_K(q_next, 1)
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) craw[i] = fmaf(-K_BIAS, R[i], C[i][i]);
    } else {
      // ---- scores, INT8 x INT8.  Pass 1: the 32 scaled-query elements of my row (h, j), their
      //      sums c_b, Delta_b and the row maximum; pass 2: T = round(q~ * 127 / max), packed
      //      four to a dword in channel order, and the residual sum of the third error term.
      float qt[32];
      float amax = 0.0f;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c0 = (u >> 1) * 64 + kg * 16 + (u & 1) * 8;
        const float4 s0 = *reinterpret_cast<const float4*>(&kmbuf[w][j][c0]);
        const float4 s1 = *reinterpret_cast<const float4*>(&kmbuf[w][j][c0 + 4]);
        const float4 z0 = *reinterpret_cast<const float4*>(&kmbuf[w][j][D + c0]);
        const float4 z1 = *reinterpret_cast<const float4*>(&kmbuf[w][j][D + c0 + 4]);
        const float4 q0 = *reinterpret_cast<const float4*>(&qbuf[h][c0]);
        const float4 q1 = *reinterpret_cast<const float4*>(&qbuf[h][c0 + 4]);
        const float sg[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
        const float zz[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
        const float qq[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float qv = qq[e];
          const float t = qv * sg[e];
          qt[u * 8 + e] = t;
          csum = fmaf(qv, zz[e], csum);
          dsum = fmaf(fabsf(qv), sg[e], dsum);
          amax = fmaxf(amax, fabsf(t));
        }
      }
      amax = fmaxf(amax, __shfl_xor(amax, 16));
      amax = fmaxf(amax, __shfl_xor(amax, 32));
      // binary32, correctly rounded quotients (the power-of-two pre-scale of q commutes with both)
      const float inv = amax > 0.0f ? 127.0f / amax : 0.0f;
      sq = amax / 127.0f;
      const float MAGIC = 12582912.0f;   // 1.5 * 2^23: fl(x + MAGIC) - MAGIC = round-half-even(x), |x| < 2^22
      v4i aq[2];                        // A operand per channel half: 16 codes T, two's complement bytes
#pragma unroll
      for (int g4 = 0; g4 < 8; ++g4) {
        uint32_t bits[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float x = qt[4 * g4 + e];
          const float r = fmaf(x, inv, MAGIC);              // one rounding: the exact product, rounded to an integer
          const float tf = r - MAGIC;
          qres += fabsf(fmaf(-sq, tf, x));
          bits[e] = __float_as_uint(r);                     // low byte = T mod 256
        }
        const uint32_t lo2 = __builtin_amdgcn_perm(bits[1], bits[0], 0x0c0c0400u);
        const uint32_t hi2 = __builtin_amdgcn_perm(bits[3], bits[2], 0x0c0c0400u);
        aq[g4 >> 2][g4 & 3] = (int)__builtin_amdgcn_perm(hi2, lo2, 0x05040100u);
      }
      v4i Ci[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) Ci[i] = v4i{0, 0, 0, 0};
#pragma unroll
      for (int cq = 0; cq < 2; ++cq) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          // stored bytes are code + 128: flipping the top bit gives the two's complement code
          const uint4 kx = kraw[i][cq];
          const v4i kb = {(int)(kx.x ^ 0x80808080u), (int)(kx.y ^ 0x80808080u), (int)(kx.z ^ 0x80808080u),
                          (int)(kx.w ^ 0x80808080u)};
          Ci[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aq[cq], kb, Ci[i], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (cq == 0) {
          CQA_LOAD_K(q_next, 0)
        } else {
          CQA_LOAD_K(q_next, 1)
        }
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) craw[i] = (float)Ci[i][i];
    }
    // per-block constant c_b = q.z and Delta_b (both still times S_h): summed over the four
    // channel slices, then handed to the rows that own head kg
    float cb = csum;
    cb += __shfl_xor(cb, 16);
    cb += __shfl_xor(cb, 32);
    dsum += __shfl_xor(dsum, 16);
    dsum += __shfl_xor(dsum, 32);
    if constexpr (Q8) {
      qres += __shfl_xor(qres, 16);
      qres += __shfl_xor(qres, 32);
      dsum = fmaf(256.0f, qres, dsum);   // Delta_b + Delta^q_b = (sum |q| sigma + 256 sum |q~ - s_q T|) / (2 sqrt d)
      cbuf[w][2][h][j] = sq;
    }
    // (all four kg lanes of a column hold the same sums and store the same words: no branch)
    cbuf[w][0][h][j] = cb;
    cbuf[w][1][h][j] = dsum * (0.5f * inv_sqrt_d) * unscale_op;
    wave_sync();
    const float4 cb4 = *reinterpret_cast<const float4*>(&cbuf[w][0][kg][0]);
    const float4 dl4 = *reinterpret_cast<const float4*>(&cbuf[w][1][kg][0]);
    const float cbs[4] = {cb4.x, cb4.y, cb4.z, cb4.w};
    const float dls[4] = {dl4.x, dl4.y, dl4.z, dl4.w};
    if constexpr (Q8) {
      const float4 sq4 = *reinterpret_cast<const float4*>(&cbuf[w][2][kg][0]);
      craw[0] *= sq4.x;
      craw[1] *= sq4.y;
      craw[2] *= sq4.z;
      craw[3] *= sq4.w;
    }

    // ---- block statistics and online softmax of head kg; this lane is token n of each block.
    //      Branch-free.  Blocks past the end of the head (only in its last quad) hold zeros --
    //      unsealed memory is cleared -- so their eta, nu and Delta_b are already zero; giving
    //      their scores a huge negative value makes every weight and mass they produce vanish.
    float mbv[4], ptv[4], sbv[4];
    float mq = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float s = live[i] ? (craw[i] + cbs[i]) * score_scale : -1.0e30f;
      mbv[i] = row_max(s);
      ptv[i] = __builtin_amdgcn_exp2f(s - mbv[i]);
      sbv[i] = row_sum(ptv[i]);
      mq = fmaxf(mq, mbv[i]);
    }
    const float m_new = fmaxf(m_run, mq);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    l_run *= alpha;
    ev *= alpha;
    evmax *= alpha;
    m_run = m_new;
    float lbv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float f = __builtin_amdgcn_exp2f(mbv[i] - m_new);
      const float sf = sbv[i] * f;
      const float ce = sf * an[i].x;
      const float lb = (mbv[i] + __builtin_amdgcn_logf(sbv[i])) * LN2;   // natural units
      lbv[i] = lb;
      l_run += sf;
      ev += ce;
      evmax = fmaxf(evmax, ce);
      dmax = fmaxf(dmax, dls[i]);
      vmax = fmaxf(vmax, an[i].y);
      // blocks arrive in increasing order: ties keep the lower index; the second largest of
      // (t1, t2, l_b), t1 >= t2, is their median
      i1 = lb > t1 ? qb + i : i1;
      t2 = __builtin_amdgcn_fmed3f(t1, t2, lb);
      t1 = fmaxf(t1, lb);
      pbuf[w][kg][i * BLK + n] = ptv[i] * f;
    }
    if (LM) {
      if (n == 0 && kg < G) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (live[i])
            a.blk_logmass[((int64_t)b * a.n_q + kvh * G + kg) * a.nb + qb + i] = lbv[i];
      }
      if (a.eta_out != nullptr && l == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (live[i]) a.eta_out[((int64_t)b * a.n_kv + kvh) * a.nb + qb + i] = an[i].x;
      }
    }
    abuf[w][kg] = alpha;   // every lane of the row stores the same word
    wave_sync();

    __builtin_amdgcn_s_setprio(0);
    // ---- rescale the accumulators (an accumulator lane's head is kg, its own softmax head)
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int g = 0; g < 8; ++g)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[g][v] *= alpha;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        accw[0][v] *= alpha;
        accw[1][v] *= alpha;
      }
    }
    const float alpha_op = abuf[w][h];
    offacc[0] *= alpha_op;
    offacc[1] *= alpha_op;

    // ---- values: two pairs of blocks, K = 32 tokens each; operand role (head h, group g' = j)
#pragma unroll
    for (int P = 0; P < 2; ++P) {
      const int bi = 2 * P + (kg >> 1);
      const float4 pa = *reinterpret_cast<const float4*>(&pbuf[w][h][bi * BLK + (kg & 1) * 8]);
      const float4 pb = *reinterpret_cast<const float4*>(&pbuf[w][h][bi * BLK + (kg & 1) * 8 + 4]);
      const float p8[8] = {pa.x, pa.y, pa.z, pa.w, pb.x, pb.y, pb.z, pb.w};
#pragma unroll
      for (int gs = 0; gs < 2; ++gs) {
        const __half* vmp = &vmbuf[w][bi][(kg & 1) * 64 + (4 * gs + j) * 8];
        const uint4 sraw = *reinterpret_cast<const uint4*>(vmp);
        const uint4 oraw = *reinterpret_cast<const uint4*>(vmp + BLK * NG);
        const __half2* sh = reinterpret_cast<const __half2*>(&sraw);
        const __half2* oh = reinterpret_cast<const __half2*>(&oraw);
        float wv[8], wr[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float sc0 = __low2float(sh[e]), sc1 = __high2float(sh[e]);
          const float of0 = __low2float(oh[e]), of1 = __high2float(oh[e]);
          wv[2 * e] = p8[2 * e] * sc0;
          wv[2 * e + 1] = p8[2 * e + 1] * sc1;
          offacc[gs] = fmaf(p8[2 * e], of0, offacc[gs]);
          offacc[gs] = fmaf(p8[2 * e + 1], of1, offacc[gs]);
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
        BF8 bv[4];   // bf16(16 + code): exponent bits 0x4180, code in mantissa bits 6..3
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint32_t x = xs[t];
          bv[t].u[0] = bfi(0x00780078u, x << 3, 0x41804180u);
          bv[t].u[1] = bfi(0x00780078u, x >> 1, 0x41804180u);
          bv[t].u[2] = bfi(0x00780078u, x >> 5, 0x41804180u);
          bv[t].u[3] = bfi(0x00780078u, x >> 9, 0x41804180u);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
          acc[4 * gs + t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah.v, bv[t].v, acc[4 * gs + t], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 4; ++t)
          acc[4 * gs + t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al.v, bv[t].v, acc[4 * gs + t], 0, 0, 0);
        accw[gs] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah.v, ones_b.v, accw[gs], 0, 0, 0);
        accw[gs] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al.v, ones_b.v, accw[gs], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (P == 0) {
        CQA_LOAD_V(q_next, 0)
      } else {
        CQA_LOAD_V(q_next, 1)
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    wave_sync();
    // advance: the quad whose data was requested during this iteration becomes current
    q_cur = q_next;
    q_next = q_next + q_step < q_stop ? q_next + q_step : Q_NONE;
  }

  // ---- per-wave epilogue: fold the offset sums in; the softmax state of head kg is already
  //      complete in every lane of row kg
#pragma unroll
  for (int gs = 0; gs < 2; ++gs) {
    offacc[gs] += __shfl_xor(offacc[gs], 16);
    offacc[gs] += __shfl_xor(offacc[gs], 32);
  }
#pragma unroll
  for (int g = 0; g < 8; ++g) {
    const float off = __shfl(offacc[g >> 2], kg * 4 + (g & 3));
    const float val = (g & 3) == 0 ? acc[g][0] : ((g & 3) == 1 ? acc[g][1] : ((g & 3) == 2 ? acc[g][2] : acc[g][3]));
    const f32x4 ws = accw[g >> 2];
    const float wsum = (g & 3) == 0 ? ws[0] : ((g & 3) == 1 ? ws[1] : ((g & 3) == 2 ? ws[2] : ws[3]));
    // sum_t w_t (16 + code) - 16 sum_t w_t + sum_t p_t offset_t
    if (kg < G) mo[w][kg < G ? kg : 0][g * 16 + n] = fmaf(-16.0f, wsum, val) + off;
  }
  if (n == 0 && kg < G) {
    float* m = ms[w][kg < G ? kg : 0];
    m[0] = m_run * LN2;   // the running maximum was kept in base 2
    m[1] = l_run;
    m[2] = ev;
    m[3] = evmax;
    m[4] = dmax;
    m[5] = vmax;
    m[6] = t1;
    m[7] = t2;
    m[8] = __int_as_float(i1);
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * D; idx += 64 * W) {
    const int hh = idx / D, c = idx % D;
    float M = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < W; ++ww) M = fmaxf(M, ms[ww][hh][0]);
    const float Mr = (M == -INFINITY) ? 0.0f : M;   // a workgroup that drew no quad writes zeros
    float o = 0.0f;
#pragma unroll
    for (int ww = 0; ww < W; ++ww) o += __expf(ms[ww][hh][0] - Mr) * mo[ww][hh][c];
    a.partials[(((int64_t)b * a.n_q + kvh * G + hh) * a.pstride + split) * PART_FLOATS + P_O + c] = o;
  }
  if (threadIdx.x < G) {
    const int hh = threadIdx.x;
    float M = -INFINITY;
    for (int ww = 0; ww < W; ++ww) M = fmaxf(M, ms[ww][hh][0]);
    const float Mr = (M == -INFINITY) ? 0.0f : M;
    float L = 0.0f, EV = 0.0f, EVM = 0.0f, DM = 0.0f, VM = 0.0f, T1 = -INFINITY, T2 = -INFINITY;
    int I1 = -1;
    for (int ww = 0; ww < W; ++ww) {
      const float fw = __expf(ms[ww][hh][0] - Mr);
      L += fw * ms[ww][hh][1];
      EV += fw * ms[ww][hh][2];
      EVM = fmaxf(EVM, fw * ms[ww][hh][3]);
      DM = fmaxf(DM, ms[ww][hh][4]);
      VM = fmaxf(VM, ms[ww][hh][5]);
      top2_merge(T1, I1, T2, ms[ww][hh][6], __float_as_int(ms[ww][hh][8]), ms[ww][hh][7]);
    }
    float* pp = a.partials + (((int64_t)b * a.n_q + kvh * G + hh) * a.pstride + split) * PART_FLOATS;
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

#undef CQA_REC
#undef CQA_LOAD_K
#undef CQA_LOAD_V
#undef CQA_LOAD_META

// Measurement only: reads the same Tier-1 records with the same launch shape, dealing of quads
// and load instructions as the split kernel (18 x 16 bytes per lane and quad, the next quad
// requested while the current one is consumed) and does nothing else with them.  Its duration is
// the ceiling the memory system sets for this access pattern.
template <bool NT, int W>
__global__ __launch_bounds__(64 * W, 8 / W) void stream_read_kernel(const uint8_t* t1, int64_t nq_cap, int nb,
                                                             int nsplit, uint32_t* sink) {
  const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int split = blockIdx.x;
  const int64_t head = (int64_t)blockIdx.z * gridDim.y + blockIdx.y;
  const int nquads = (nb + 3) >> 2;
  const int gw = split * W + w, nw = nsplit * W;
  const int q0 = gw, q1 = nquads;       // round-robin over the head's waves, as the split kernel deals
  if (q0 >= q1) return;
  const uint8_t* base = t1 + head * nq_cap * QUAD_BYTES;
  u32x4 buf[18], acc = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int i = 0; i < 18; ++i) buf[i] = ld_stream<NT>(base + (int64_t)q0 * QUAD_BYTES + i * 1024 + l * 16);
  for (int q = q0; q < q1; q += nw) {
    const uint8_t* nxt = base + (int64_t)(q + nw < q1 ? q + nw : q0) * QUAD_BYTES;
#pragma unroll
    for (int i = 0; i < 18; ++i) {
      acc ^= buf[i];
      buf[i] = ld_stream<NT>(nxt + i * 1024 + l * 16);
    }
  }
  // keeps the loads alive: a 128-bit coincidence that does not occur in practice
  if (acc.x == 0x9E3779B9u && acc.y == 0x85EBCA6Bu && acc.z == 0xC2B2AE35u && acc.w == 0x27D4EB2Fu)
    sink[0] = acc.x;
}

int32_t launch_stream_read(const uint8_t* t1, int64_t nq_cap, int nb, dim3 grid, bool nt, int wpb,
                           uint32_t* sink, hipStream_t st) {
  if (wpb != 4 && wpb != 8) return CQA_ERR_INVALID_ARG;
#define CQA_LAUNCH_SR(NTV, WV) \
  hipLaunchKernelGGL((stream_read_kernel<NTV, WV>), grid, dim3(64 * WV), 0, st, t1, nq_cap, nb, (int)grid.x, sink)
  if (nt) {
    if (wpb == 8) CQA_LAUNCH_SR(true, 8); else CQA_LAUNCH_SR(true, 4);
  } else {
    if (wpb == 8) CQA_LAUNCH_SR(false, 8); else CQA_LAUNCH_SR(false, 4);
  }
#undef CQA_LAUNCH_SR
  CQA_HIP(hipGetLastError());
  return CQA_OK;
}

// ev0 / ev1 (both or neither): HIP events attached to the dispatch itself, so their elapsed time
// is the kernel's own execution time (what a kernel trace reports), not launch overhead.
int32_t launch_split_mfma(const DecodeArgs& a, int group, dim3 grid, hipEvent_t ev0, hipEvent_t ev1,
                          hipStream_t st) {
  const bool lm = a.blk_logmass != nullptr;
  if (a.wpb != 4 && a.wpb != 8) return CQA_ERR_INVALID_ARG;
#define CQA_LAUNCH_W(GG, NTV, Q8V, WV)                                                             \
  if (lm)                                                                                          \
    hipExtLaunchKernelGGL((certified_split_mfma_kernel<GG, true, NTV, Q8V, WV>), grid, dim3(64 * WV), 0, st, \
                          ev0, ev1, 0, a);                                                         \
  else                                                                                             \
    hipExtLaunchKernelGGL((certified_split_mfma_kernel<GG, false, NTV, Q8V, WV>), grid, dim3(64 * WV), 0,   \
                          st, ev0, ev1, 0, a);
#define CQA_LAUNCH_Q(GG, NTV, Q8V)                                                                 \
  if (a.wpb == 8) { CQA_LAUNCH_W(GG, NTV, Q8V, 8) } else { CQA_LAUNCH_W(GG, NTV, Q8V, 4) }
#define CQA_LAUNCH_NT(GG, NTV)                                                                     \
  if (a.int8_query) { CQA_LAUNCH_Q(GG, NTV, true) } else { CQA_LAUNCH_Q(GG, NTV, false) }
#define CQA_LAUNCH(GG)                                                                             \
  if (a.stream_nt) { CQA_LAUNCH_NT(GG, true) } else { CQA_LAUNCH_NT(GG, false) }
  switch (group) {
    case 1: CQA_LAUNCH(1) break;
    case 2: CQA_LAUNCH(2) break;
    case 4: CQA_LAUNCH(4) break;
    default: return CQA_ERR_UNSUPPORTED;
  }
#undef CQA_LAUNCH
#undef CQA_LAUNCH_NT
#undef CQA_LAUNCH_Q
#undef CQA_LAUNCH_W
  return CQA_OK;
}

}  // namespace cqa
