// Cache-write kernels: seal a block of 16 tokens into Tier-1.
//
// Follows the paper's "Quantization Schemes" section: per-block per-channel INT8
// keys with sigma_c = (u_c - l_c)/255, z_c = l_c + 128 sigma_c, code =
// clamp(round((k - z_c)/sigma_c), -128, 127); per-token per-16-channel-group INT4
// values with an FP16 scale and offset; and the block annotations eta_b =
// max_t ||v_hat_t - v_t||_2, nu_b = max_t ||v_t||_2.
//
// All quantizer arithmetic is IEEE binary32 with one rounding per operation in
// the order written (subtract, divide; multiply, add; subtract, divide,
// round-half-even, clamp): contraction into fused multiply-adds is switched off
// for this file so codes and scales have exactly one correct value.
// Inputs are assumed finite.
#pragma clang fp contract(off)

#include "cqa_internal.h"

namespace cqa {

struct SealArgs {
  const __half* k_in;   // [Bt][Hkv][n_new][128]
  const __half* v_in;
  const __half* trail_k;  // [heads][16][128]
  const __half* trail_v;
  uint8_t* t1;          // Tier-1 quad records
  float* sigmax;        // [heads]: running max of sigma per (layer, batch, kv-head)
  int64_t nq_cap;
  int64_t nb_old;       // sealed blocks before this append
  int64_t n_new;
  int r;                // tokens in the trailing block before this append
  int layer, batch, n_kv;
  // short appends that end on a block boundary: the kernel also stores the FP16 originals of the
  // new tokens into the pinned Tier-2 arrays (null = Tier 2 is written elsewhere)
  __half* t2_k;         // [heads][t2_cap][128]
  __half* t2_v;
  int64_t t2_cap;
  int64_t len_before;
};

// Quotient x / d for the quantizers, where only  round-half-even(fl(x / d))  is needed (fl = the
// correctly rounded binary32 quotient the definition asks for) and |x / d| < 2^8.  One IEEE division
// costs ten instructions and a block needs 4096 of them, so the quotient is first approximated as
// x * r with r = 1/d refined by one Newton step: the hardware reciprocal is within one unit in the
// last place, so after the step r is the rounded value of a number within 2^-44 of 1/d (relative
// error <= 2^-24), x * r carries one more rounding (2^-24), and |x r - x/d| <= 2^8 * 2^-23 = 2^-15;
// the exact quotient's own rounding moves it by at most 2^-17.  Unless the approximation lies
// within 2^-13 of a half-integer, both therefore round to the same integer; the rare lanes that
// are closer -- and anything not finite -- take the exact division.  Bit-identical to
// rintf(x / d) by construction.
__device__ __forceinline__ float refined_rcp(float d) {
  const float r0 = __builtin_amdgcn_rcpf(d);
  return fmaf(fmaf(-d, r0, 1.0f), r0, r0);
}
__device__ __forceinline__ float rint_quotient(float x, float d, float r) {
  const float qa = x * r;
  float q = rintf(qa);
  if (!(fabsf(qa - q) <= 0.5f - 0.0001220703125f)) q = rintf(x / d);
  return q;
}

// DPP moves for the few cross-lane sums of FP64 annotations (lanes of one token are adjacent)
template <int CTRL>
__device__ __forceinline__ double dpp_d(double x) {
  const unsigned long long u = (unsigned long long)__double_as_longlong(x);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, CTRL, 0xf, 0xf, true);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), CTRL, 0xf, 0xf, true);
  return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
// sum over the 8 lanes of an aligned octet: quad xor 1, quad xor 2, half-row mirror
__device__ __forceinline__ double octet_sum_d(double x) {
  x += dpp_d<0xB1>(x);
  x += dpp_d<0x4E>(x);
  x += dpp_d<0x141>(x);
  return x;
}

// One workgroup of 128 threads seals one block of 16 tokens.  Two thread roles, so that every
// reduction the quantizers need runs inside one thread's registers:
//   keys   : thread = channel c; its 16 values (one per token) give l_c, u_c, sigma_c, z_c and
//            the 16 codes of the channel;
//   values : thread = (token t, group g) = (tid >> 3, tid & 7); its 16 values (32 contiguous
//            bytes) give lo, hi, the FP16 scale and offset, the 16 codes of the group and the
//            group's share of the token's squared reconstruction error and squared norm (FP64).
// Codes pass through LDS to reach the physical layout of the Tier-1 record.
// (Measured and not adopted: fetching the keys as whole rows with 128-bit loads too and handing
// the columns to the channel threads through LDS -- 0.28 ms against 0.25 ms for the 128K prefill.)
__global__ __launch_bounds__(128) void seal_kernel(SealArgs a) {
  const int tid = threadIdx.x;
  const int j = blockIdx.x;             // new block index
  const int kvh = blockIdx.y, b = blockIdx.z;
  const int64_t head = ((int64_t)a.layer * a.batch + b) * a.n_kv + kvh;
  const int64_t blk = a.nb_old + j;
  const int64_t in_head = ((int64_t)b * a.n_kv + kvh) * a.n_new;

  __shared__ __align__(16) uint8_t kbuf[KC_BYTES];
  __shared__ __align__(16) uint8_t vnib[BLK][D];
  __shared__ __align__(16) __half vmeta[2 * BLK * NG];
  __shared__ double red[BLK][2];        // [token][err^2 | norm^2]

  // token i of this block: one of the r tokens waiting in the trailing block, or a new one
  const int64_t i0 = (int64_t)j * BLK;
  // ---- values first (their loads are the wide ones): thread (t, g)
  {
    const int t = tid >> 3, g = tid & 7;
    const int64_t i = i0 + t;
    const __half* src = i < a.r ? a.trail_v + (head * BLK + i) * D : a.v_in + (in_head + (i - a.r)) * D;
    const uint4 x0 = *reinterpret_cast<const uint4*>(src + g * VG);
    const uint4 x1 = *reinterpret_cast<const uint4*>(src + g * VG + 8);
    if (a.t2_v != nullptr && i >= a.r) {
      __half* dst = a.t2_v + (head * a.t2_cap + a.len_before + (i - a.r)) * D + g * VG;
      *reinterpret_cast<uint4*>(dst) = x0;
      *reinterpret_cast<uint4*>(dst + 8) = x1;
    }
    const __half2* h0 = reinterpret_cast<const __half2*>(&x0);
    const __half2* h1 = reinterpret_cast<const __half2*>(&x1);
    float vf[VG];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      vf[2 * e] = __low2float(h0[e]);
      vf[2 * e + 1] = __high2float(h0[e]);
      vf[8 + 2 * e] = __low2float(h1[e]);
      vf[8 + 2 * e + 1] = __high2float(h1[e]);
    }
    float vlo = vf[0], vhi = vf[0];
#pragma unroll
    for (int e = 1; e < VG; ++e) {
      vlo = fminf(vlo, vf[e]);
      vhi = fmaxf(vhi, vf[e]);
    }
    const __half sh = __float2half_rn((vhi - vlo) / 15.0f);
    const float sc = __half2float(sh);
    const float rs = refined_rcp(sc);
    uint32_t packed[4] = {0u, 0u, 0u, 0u};   // the group's 16 codes, one per byte, channel order
    double e2 = 0.0, n2 = 0.0;
    const double dlo = (double)vlo;
#pragma unroll
    for (int e = 0; e < VG; ++e) {
      float q = 0.0f;
      if (sc != 0.0f) {
        q = rint_quotient(vf[e] - vlo, sc, rs);
        q = fminf(fmaxf(q, 0.0f), 15.0f);
      }
      packed[e >> 2] |= (uint32_t)(int)q << (8 * (e & 3));
      // v_hat - v = code * scale + (lo - v): the product is exact in binary32 (4 x 11 bits), the
      // difference and the sum are taken in double
      const double dv = (double)vf[e];
      const double err = (double)(q * sc) + (dlo - dv);
      e2 += err * err;
      n2 += dv * dv;
    }
    *reinterpret_cast<uint4*>(&vnib[t][g * VG]) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
    vmeta[vm_index(t, g)] = sh;
    vmeta[BLK * NG + vm_index(t, g)] = __float2half_rn(vlo);  // exact: vlo is an FP16 input
    e2 = octet_sum_d(e2);
    n2 = octet_sum_d(n2);
    if (g == 0) {
      red[t][0] = e2;
      red[t][1] = n2;
    }
  }

  // ---- keys: thread = channel c, per-channel affine INT8 over the block's 16 tokens
  {
    const int c = tid;
    float kf[BLK];
#pragma unroll
    for (int t = 0; t < BLK; ++t) {
      const int64_t i = i0 + t;
      const __half kh = i < a.r ? a.trail_k[(head * BLK + i) * D + c] : a.k_in[(in_head + (i - a.r)) * D + c];
      kf[t] = __half2float(kh);
      if (a.t2_k != nullptr && i >= a.r) a.t2_k[(head * a.t2_cap + a.len_before + (i - a.r)) * D + c] = kh;
    }
    float lo = kf[0], hi = kf[0];
#pragma unroll
    for (int t = 1; t < BLK; ++t) {
      lo = fminf(lo, kf[t]);
      hi = fmaxf(hi, kf[t]);
    }
    const float sigma = (hi - lo) / 255.0f;
    const float z = lo + 128.0f * sigma;
    const float rsig = refined_rcp(sigma);
#pragma unroll
    for (int t = 0; t < BLK; ++t) {
      int code = 0;
      if (sigma != 0.0f) {
        float q = rint_quotient(kf[t] - z, sigma, rsig);
        q = fminf(fmaxf(q, -128.0f), 127.0f);
        code = (int)q;
      }
      kbuf[kc_offset(t, c)] = (uint8_t)(code + 128);
    }
    float* km = reinterpret_cast<float*>(a.t1 + t1_offset(head * a.nq_cap, blk, Q_KM, KM_BYTES));
    km[c] = sigma;
    km[D + c] = z;
    // running maximum of sigma over the head's blocks (used by the decode pass to pick an
    // overflow-free power-of-two scaling); sigma >= 0, so its bit pattern orders like an int
    float smax = sigma;
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) smax = fmaxf(smax, __shfl_xor(smax, m));
    // thousands of blocks of one head would queue up on the same word: the running maximum is
    // read first (it only grows, so a stale value merely costs a redundant atomic) and the atomic
    // is issued only by a block that raises it
    if ((c & 63) == 0 && __float_as_int(smax) > __hip_atomic_load(reinterpret_cast<int*>(a.sigmax + head),
                                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
      atomicMax(reinterpret_cast<int*>(a.sigmax + head), __float_as_int(smax));
  }
  __syncthreads();

  // ---- write out, 16 bytes per thread where possible
  const int c = tid;
  uint8_t* kc = a.t1 + t1_offset(head * a.nq_cap, blk, Q_KC, KC_BYTES);
  reinterpret_cast<uint4*>(kc)[c] = reinterpret_cast<const uint4*>(kbuf)[c];

  uint32_t* vc = reinterpret_cast<uint32_t*>(a.t1 + t1_offset(head * a.nq_cap, blk, Q_VC, VC_BYTES));
#pragma unroll
  for (int rep = 0; rep < 2; ++rep) {
    const int dw = c + rep * 128;
    const int o = dw >> 7, gh = (dw >> 6) & 1, n = (dw >> 2) & 15, gq = dw & 3;
    const int ch = (gh * 4 + gq) * 16 + n;
    uint32_t x = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) x |= (uint32_t)vnib[o * 8 + i][ch] << (4 * i);
    vc[dw] = x;
  }
  __half* vm = reinterpret_cast<__half*>(a.t1 + t1_offset(head * a.nq_cap, blk, Q_VM, VM_BYTES));
  reinterpret_cast<uint32_t*>(vm)[c] = reinterpret_cast<const uint32_t*>(vmeta)[c];

  if (c == 0) {
    double eta2 = 0.0, nu2 = 0.0;
    for (int t = 0; t < BLK; ++t) {
      eta2 = fmax(eta2, red[t][0]);
      nu2 = fmax(nu2, red[t][1]);
    }
    float* an = reinterpret_cast<float*>(a.t1 + t1_offset(head * a.nq_cap, blk, Q_AN, AN_BYTES));
    an[0] = (float)sqrt(eta2);
    an[1] = (float)sqrt(nu2);
  }
}

// Moves the tokens that stay unsealed into the trailing FP16 block and, for short appends,
// stores the FP16 originals of ALL new tokens straight into the pinned Tier-2 arrays (device
// stores to mapped host memory: a decode-time append of one token per head is then a single
// small launch instead of two strided copies).
// src_first: index (within this append's input) of the first token to keep in the trailing
// block; dst_first: its slot there; count tokens.  t2_k / t2_v: null = Tier-2 handled elsewhere.
__global__ __launch_bounds__(128) void trail_kernel(const __half* k_in, const __half* v_in,
                                                    __half* trail_k, __half* trail_v,
                                                    int64_t n_new, int64_t src_first,
                                                    int dst_first, int count, int layer, int batch,
                                                    int n_kv, __half* t2_k, __half* t2_v,
                                                    int64_t t2_cap, int64_t len_before) {
  const int c = threadIdx.x;
  const int kvh = blockIdx.x, b = blockIdx.y;
  const int64_t head = ((int64_t)layer * batch + b) * n_kv + kvh;
  const int64_t in_head = ((int64_t)b * n_kv + kvh) * n_new;
  for (int t = 0; t < count; ++t) {
    trail_k[(head * BLK + dst_first + t) * D + c] = k_in[(in_head + src_first + t) * D + c];
    trail_v[(head * BLK + dst_first + t) * D + c] = v_in[(in_head + src_first + t) * D + c];
  }
  if (t2_k != nullptr) {
    for (int64_t t = 0; t < n_new; ++t) {
      t2_k[(head * t2_cap + len_before + t) * D + c] = k_in[(in_head + t) * D + c];
      t2_v[(head * t2_cap + len_before + t) * D + c] = v_in[(in_head + t) * D + c];
    }
  }
}

int32_t launch_seal(Cache* c, int layer, const __half* k_in, const __half* v_in, int64_t n_new,
                    int64_t len_before, bool tier2_by_kernel, hipStream_t st) {
  const int r = (int)(len_before % BLK);
  const int64_t nb_old = len_before / BLK;
  const int64_t n_seal = (r + n_new) / BLK;
  const int r_new = (int)((r + n_new) % BLK);
  const int bt = c->desc.batch, hkv = c->desc.n_kv_heads;
  if (n_seal > 0) {
    SealArgs a;
    a.k_in = k_in;
    a.v_in = v_in;
    a.trail_k = c->trail_k;
    a.trail_v = c->trail_v;
    a.t1 = c->t1;
    a.sigmax = c->sigmax;
    a.nq_cap = c->nq_cap;
    a.nb_old = nb_old;
    a.n_new = n_new;
    a.r = r;
    a.layer = layer;
    a.batch = bt;
    a.n_kv = hkv;
    // an append that ends on a block boundary leaves nothing for the trailing block: its Tier-2
    // stores ride on the seal launch and the second launch is saved
    const bool t2_here = tier2_by_kernel && r_new == 0;
    a.t2_k = t2_here ? c->t2_k : nullptr;
    a.t2_v = t2_here ? c->t2_v : nullptr;
    a.t2_cap = c->desc.max_tokens;
    a.len_before = len_before;
    // grid.x is limited to 2^31-1 blocks; n_seal <= nb_cap is far below that
    hipLaunchKernelGGL(seal_kernel, dim3((unsigned)n_seal, hkv, bt), dim3(128), 0, st, a);
    CQA_HIP(hipGetLastError());
  }
  int64_t src_first;
  int dst_first, count;
  if (n_seal == 0) {
    src_first = 0;
    dst_first = r;
    count = (int)n_new;
  } else {
    src_first = n_new - r_new;
    dst_first = 0;
    count = r_new;
  }
  if (count > 0 || (tier2_by_kernel && n_seal == 0)) {
    hipLaunchKernelGGL(trail_kernel, dim3(hkv, bt), dim3(128), 0, st, k_in, v_in, c->trail_k,
                       c->trail_v, n_new, src_first, dst_first, count, layer, bt, hkv,
                       tier2_by_kernel ? c->t2_k : nullptr, tier2_by_kernel ? c->t2_v : nullptr,
                       (int64_t)c->desc.max_tokens, len_before);
    CQA_HIP(hipGetLastError());
  }
  return CQA_OK;
}

}  // namespace cqa
