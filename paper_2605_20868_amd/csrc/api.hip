// C ABI of the library: cache lifetime, append, decode, fallback ladder, export.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include <chrono>

#include "cqa_internal.h"

struct cqa_cache {
  cqa::Cache impl;
};

namespace cqa {
thread_local int g_last_hip_error = 0;

static int32_t check_desc(const cqa_cache_desc* d) {
  if (d == nullptr) return CQA_ERR_INVALID_ARG;
  if (d->n_layers < 1 || d->batch < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 ||
      d->max_tokens < 1)
    return CQA_ERR_INVALID_ARG;
  if (d->head_dim != D || d->block_tokens != BLK || d->v_group != VG) return CQA_ERR_UNSUPPORTED;
  if (d->n_q_heads % d->n_kv_heads != 0) return CQA_ERR_INVALID_ARG;
  const int g = d->n_q_heads / d->n_kv_heads;
  if (g != 1 && g != 2 && g != 4) return CQA_ERR_UNSUPPORTED;
  if (d->tier2_mode != CQA_TIER2_PINNED && d->tier2_mode != CQA_TIER2_NONE)
    return CQA_ERR_INVALID_ARG;
  if (d->batch > 65535 || d->n_kv_heads > 65535) return CQA_ERR_UNSUPPORTED;  // grid.y / grid.z
  if (d->max_tokens > ((int64_t)1 << 30)) return CQA_ERR_UNSUPPORTED;
  return CQA_OK;
}

struct Sizes {
  int64_t nb_cap, nq_cap, heads, t1, trail, t2, partials, dense_ws, stage, select, ladder_ws;
  int64_t ad_lm, ad_sel, ad_head, ad_mask_words, ad_mask, ad_slot, ad_group, ad_ulist, ad_eta;
  int64_t sc_k, sc_map, sc_tag;
  int sc_cap;
  int max_splits;
};

static Sizes compute_sizes(const cqa_cache_desc* d, int n_cu) {
  Sizes s;
  s.nb_cap = (d->max_tokens + BLK - 1) / BLK;
  s.heads = (int64_t)d->n_layers * d->batch * d->n_kv_heads;
  s.nq_cap = (s.nb_cap + 3) / 4;
  s.t1 = s.heads * s.nq_cap * QUAD_BYTES;
  s.trail = s.heads * BLK * D * 2;
  s.t2 = d->tier2_mode == CQA_TIER2_PINNED ? s.heads * d->max_tokens * D * 2 : 0;
  int64_t ms = (4 * (int64_t)n_cu) / ((int64_t)d->batch * d->n_kv_heads);
  if (ms < 64) ms = 64;
  if (ms > MAX_SPLITS) ms = MAX_SPLITS;
  if (ms > s.nb_cap) ms = s.nb_cap;
  if (ms < 1) ms = 1;
  s.max_splits = (int)ms;
  s.partials = (int64_t)d->batch * d->n_q_heads * (s.max_splits + 2 * PROM_SPLITS) * PART_FLOATS * 4;
  s.dense_ws = dense_ws_floats(d->n_q_heads / d->n_kv_heads, d->max_tokens) * 4;
  s.stage = d->tier2_mode == CQA_TIER2_PINNED ? d->max_tokens * D * 2 : 0;
  s.select = (int64_t)d->batch * d->n_q_heads * 4;
  s.ladder_ws = d->tier2_mode == CQA_TIER2_PINNED ? ladder_ws_floats((int64_t)d->batch * d->n_q_heads) * 4 : 0;
  // adaptive key precision (needs the originals): log-masses of the pass over all blocks and of the promoted-block pass, selections, masks,
  // slot maps and lists, for one layer-step at a time
  const bool ad = d->tier2_mode == CQA_TIER2_PINNED;
  const int64_t rows = (int64_t)d->batch * d->n_q_heads, groups = (int64_t)d->batch * d->n_kv_heads;
  s.ad_lm = ad ? rows * s.nb_cap * 4 : 0;
  s.ad_sel = ad ? rows * MAX_K_LIMIT * 4 : 0;
  s.ad_head = ad ? rows * 4 : 0;
  s.ad_mask_words = (s.nb_cap + 31) / 32;
  s.ad_mask = ad ? rows * s.ad_mask_words * 4 : 0;
  s.ad_slot = ad ? groups * s.nq_cap * 4 * 4 : 0;
  s.ad_group = ad ? groups * 4 : 0;
  s.ad_ulist = ad ? groups * MAX_UNION * 4 : 0;
  s.ad_eta = ad ? groups * s.nb_cap * 4 : 0;
  // FP16 scratch: a power of two of slots per head, at most SC_MAX_SLOTS, no more than needed
  int cap = 1;
  while (cap < SC_MAX_SLOTS && cap < s.nb_cap) cap <<= 1;
  s.sc_cap = ad ? cap : 0;
  s.sc_k = ad ? s.heads * cap * (int64_t)BLK * D * 2 : 0;
  s.sc_map = ad ? s.heads * s.nb_cap * 4 : 0;
  s.sc_tag = ad ? s.heads * cap * 4 : 0;
  return s;
}

static void release(cqa_cache* h) {
  if (h == nullptr) return;
  Cache* c = &h->impl;
  (void)hipSetDevice(c->device);
  (void)hipDeviceSynchronize();
  (void)hipFree(c->t1);
  (void)hipFree(c->sigmax);
  (void)hipFree(c->trail_k);
  (void)hipFree(c->trail_v);
  (void)hipFree(c->partials);
  (void)hipFree(c->dense_ws);
  (void)hipFree(c->select_dev);
  (void)hipFree(c->ladder_ws);
  (void)hipFree(c->ladder_tickets);
  (void)hipFree(c->ladder_counts);
  (void)hipFree(c->ad.lm8);
  (void)hipFree(c->ad.lmx);
  (void)hipFree(c->ad.sel);
  (void)hipFree(c->ad.kstar);
  (void)hipFree(c->ad.alpha);
  (void)hipFree(c->ad.umask);
  (void)hipFree(c->ad.slot);
  (void)hipFree(c->ad.ucount);
  (void)hipFree(c->ad.ulist);
  (void)hipFree(c->ad.vmask);
  (void)hipFree(c->ad.eta_blk);
  (void)hipFree(c->ad.contrib);
  (void)hipFree(c->ad.vsel);
  (void)hipFree(c->ad.vcount);
  (void)hipFree(c->ad.score_dev);
  (void)hipFree(c->ad.sc_k);
  (void)hipFree(c->ad.sc_v);
  (void)hipFree(c->ad.sc_have);
  (void)hipFree(c->ad.sc_map);
  (void)hipFree(c->ad.sc_tag);
  (void)hipFree(c->ad.sc_age);
  (void)hipFree(c->ad.sc_stats);
  for (int i = 0; i < 2; ++i)
    for (int j = 0; j < 2; ++j) (void)hipFree(c->stage[i][j]);
  if (c->t2_k && !c->t2_borrowed) (void)hipHostFree(c->t2_k);
  if (c->t2_v && !c->t2_borrowed) (void)hipHostFree(c->t2_v);
  if (c->flags_host) (void)hipHostFree(c->flags_host);
  delete[] c->need;
  if (c->side) (void)hipStreamDestroy(c->side);
  for (int i = 0; i < 2; ++i) {
    if (c->ev_ready[i]) (void)hipEventDestroy(c->ev_ready[i]);
    if (c->ev_free[i]) (void)hipEventDestroy(c->ev_free[i]);
  }
  if (c->ev_main) (void)hipEventDestroy(c->ev_main);
  if (c->ev_copy) (void)hipEventDestroy(c->ev_copy);
  if (c->ev_t0) (void)hipEventDestroy(c->ev_t0);
  if (c->ev_t1) (void)hipEventDestroy(c->ev_t1);
  if (c->prof_ev) {
    for (int i = 0; i < 2 * c->prof_cap; ++i)
      if (c->prof_ev[i]) (void)hipEventDestroy(c->prof_ev[i]);
    delete[] c->prof_ev;
  }
  delete[] c->prof_ms;
  delete[] c->length;
  delete h;
}

#define CQA_ALLOC_DEV(ptr, bytes)                                         \
  do {                                                                    \
    hipError_t e__ = hipMalloc((void**)&(ptr), (size_t)((bytes) > 0 ? (bytes) : 16)); \
    if (e__ != hipSuccess) {                                              \
      g_last_hip_error = (int)e__;                                        \
      (void)hipGetLastError();                                            \
      release(h);                                                         \
      return e__ == hipErrorOutOfMemory ? CQA_ERR_OOM_DEVICE : CQA_ERR_HIP; \
    }                                                                     \
  } while (0)

#define CQA_ALLOC_PIN(ptr, bytes)                                         \
  do {                                                                    \
    hipError_t e__ = hipHostMalloc((void**)&(ptr), (size_t)(bytes), hipHostMallocDefault); \
    if (e__ != hipSuccess) {                                              \
      g_last_hip_error = (int)e__;                                        \
      (void)hipGetLastError();                                            \
      release(h);                                                         \
      return CQA_ERR_OOM_PINNED;                                          \
    }                                                                     \
  } while (0)

#define CQA_TRY(expr)                    \
  do {                                   \
    hipError_t e__ = (expr);             \
    if (e__ != hipSuccess) {             \
      g_last_hip_error = (int)e__;       \
      release(h);                        \
      return CQA_ERR_HIP;                \
    }                                    \
  } while (0)

}  // namespace cqa

using namespace cqa;

extern "C" {

int32_t cqa_version(void) { return CQA_VERSION; }

int32_t cqa_last_hip_error(void) { return g_last_hip_error; }

const char* cqa_strerror(int32_t status) {
  switch (status) {
    case CQA_OK: return "ok";
    case CQA_ERR_INVALID_ARG: return "invalid argument";
    case CQA_ERR_OOM_DEVICE: return "out of device memory";
    case CQA_ERR_OOM_PINNED: return "out of pinned host memory";
    case CQA_ERR_NO_TIER2: return "FP16 originals (Tier 2) unavailable: cannot fall back";
    case CQA_ERR_CAPACITY: return "cache capacity exceeded";
    case CQA_ERR_HIP: return "HIP runtime error (see cqa_last_hip_error)";
    case CQA_ERR_UNSUPPORTED: return "unsupported geometry";
    case CQA_ERR_SCRATCH: return "shape exceeds the fixed scratch of the no-allocation call";
    default: return "unknown status";
  }
}

int32_t cqa_workspace_bytes(const cqa_cache_desc* desc, int64_t* device_bytes,
                            int64_t* pinned_bytes) {
  const int32_t st = check_desc(desc);
  if (st != CQA_OK) return st;
  const Sizes s = compute_sizes(desc, 256);
  const bool t2 = desc->tier2_mode == CQA_TIER2_PINNED;
  const int64_t groups = (int64_t)desc->batch * desc->n_kv_heads;
  if (device_bytes) {
    // every device allocation of create_cache, in its order ...
    int64_t n = s.t1 + s.heads * 4 + 2 * s.trail + s.partials + 2 * s.dense_ws + s.select;
    if (t2) {
      n += 3 * s.ad_lm + 2 * s.ad_sel + 4 * s.ad_head + 2 * s.ad_mask + s.ad_slot + s.ad_group + s.ad_ulist +
           s.ad_eta + 8;
      n += 4 * s.stage + s.ladder_ws + groups * 4 + 8;
      // ... and what the first cqa_set_scratch_slots(n > 0) adds: key and value halves, map, three words per slot
      n += 2 * s.sc_k + s.sc_map + 3 * s.sc_tag;
    }
    *device_bytes = n;
  }
  if (pinned_bytes) *pinned_bytes = 2 * s.t2 + s.select;
  return CQA_OK;
}

// Range checks of a tolerance set.  The one-pass path tests the ranking at depth 1 (the paper's
// default) and the adaptive path up to MAX_RANK_DEPTH; a larger depth is refused rather than
// silently served by a shallower test.
static int32_t check_tolerances(const cqa_tolerances* tol, int max_rank_depth = 1) {
  if (tol->mass_exp < 0 || tol->key_bound_mode < 0 || tol->key_bound_mode > 2 || tol->rank_depth < 0 ||
      (tol->int8_query != 0 && tol->int8_query != 1))
    return CQA_ERR_INVALID_ARG;
  if (tol->rank_depth > max_rank_depth) return CQA_ERR_UNSUPPORTED;
  return CQA_OK;
}

// caller_k / caller_v: pinned host arrays the caller provides for the originals (and keeps
// alive until the cache is destroyed), or null for library-owned ones.
static int32_t create_cache(const cqa_cache_desc* desc, __half* caller_k, __half* caller_v,
                            cqa_cache** out) {
  if (out == nullptr) return CQA_ERR_INVALID_ARG;
  const int32_t st = check_desc(desc);
  if (st != CQA_OK) return st;
  cqa_cache* h = new (std::nothrow) cqa_cache;
  if (h == nullptr) return CQA_ERR_INVALID_ARG;
  Cache* c = &h->impl;
  memset(c, 0, sizeof(Cache));
  c->desc = *desc;
  c->t2_borrowed = caller_k != nullptr;
  c->length = new (std::nothrow) int64_t[desc->n_layers];
  if (c->length == nullptr) {
    delete h;
    return CQA_ERR_INVALID_ARG;
  }
  for (int i = 0; i < desc->n_layers; ++i) c->length[i] = 0;
  // from here on release() frees whatever has been set, and the handle itself
  CQA_TRY(hipGetDevice(&c->device));
  CQA_TRY(hipDeviceGetAttribute(&c->n_cu, hipDeviceAttributeMultiprocessorCount, c->device));
  if (c->n_cu < 1) c->n_cu = 256;
  const Sizes s = compute_sizes(desc, c->n_cu);
  c->nb_cap = s.nb_cap;
  c->nq_cap = s.nq_cap;
  c->heads_total = s.heads;
  c->max_splits = s.max_splits;
  CQA_ALLOC_DEV(c->t1, s.t1);
  // blocks that are not sealed yet must read as zeros: the decode pass loads whole records and
  // only masks the scores of the unsealed blocks of a head's last record
  CQA_TRY(hipMemset(c->t1, 0, (size_t)s.t1));
  CQA_ALLOC_DEV(c->sigmax, s.heads * 4);
  CQA_TRY(hipMemset(c->sigmax, 0, (size_t)s.heads * 4));
  CQA_ALLOC_DEV(c->trail_k, s.trail);
  CQA_ALLOC_DEV(c->trail_v, s.trail);
  CQA_ALLOC_DEV(c->partials, s.partials);
  CQA_ALLOC_DEV(c->dense_ws, 2 * s.dense_ws);
  CQA_ALLOC_DEV(c->select_dev, s.select);
  if (desc->tier2_mode == CQA_TIER2_PINNED) {
    CQA_ALLOC_DEV(c->ad.lm8, s.ad_lm);
    CQA_ALLOC_DEV(c->ad.lmx, s.ad_lm);
    CQA_ALLOC_DEV(c->ad.sel, s.ad_sel);
    CQA_ALLOC_DEV(c->ad.kstar, s.ad_head);
    CQA_ALLOC_DEV(c->ad.alpha, s.ad_head);
    CQA_ALLOC_DEV(c->ad.umask, s.ad_mask);
    CQA_ALLOC_DEV(c->ad.slot, s.ad_slot);
    CQA_ALLOC_DEV(c->ad.ucount, s.ad_group);
    CQA_ALLOC_DEV(c->ad.ulist, s.ad_ulist);
    CQA_ALLOC_DEV(c->ad.vmask, s.ad_mask);
    CQA_ALLOC_DEV(c->ad.eta_blk, s.ad_eta);
    CQA_ALLOC_DEV(c->ad.contrib, s.ad_lm);
    CQA_ALLOC_DEV(c->ad.vsel, s.ad_sel);
    CQA_ALLOC_DEV(c->ad.vcount, s.ad_head);
    CQA_ALLOC_DEV(c->ad.score_dev, s.ad_head);
    CQA_TRY(hipMemset(c->ad.score_dev, 0, (size_t)s.ad_head));
    c->ad.mask_words = s.ad_mask_words;
    CQA_TRY(hipMemset(c->ad.umask, 0, (size_t)s.ad_mask));       // the selector ORs into it
    CQA_TRY(hipMemset(c->ad.vmask, 0, (size_t)s.ad_mask));
    CQA_TRY(hipMemset(c->ad.slot, 0, (size_t)s.ad_slot));        // 0: no block is promoted
    CQA_TRY(hipMemset(c->ad.vcount, 0, (size_t)s.ad_head));
    CQA_TRY(hipMemset(c->ad.ucount, 0, (size_t)s.ad_group));
    CQA_TRY(hipMemset(c->ad.kstar, 0, (size_t)s.ad_head));
    // FP16 scratch: off until cqa_set_scratch_slots asks for it (allocated then)
    CQA_ALLOC_DEV(c->ad.sc_stats, 8);
    CQA_TRY(hipMemset(c->ad.sc_stats, 0, 8));
    c->ad.sc_cap = s.sc_cap;
    c->ad.sc_slots = 0;
    c->ad.sc_step = 0u;
  }
  CQA_ALLOC_PIN(c->flags_host, s.select);
  memset(c->flags_host, 0, s.select);
  c->need = new (std::nothrow) uint32_t[(size_t)desc->batch * desc->n_q_heads];
  if (c->need == nullptr) {
    release(h);
    return CQA_ERR_INVALID_ARG;
  }
  if (desc->tier2_mode == CQA_TIER2_PINNED) {
    for (int i = 0; i < 2; ++i)
      for (int j = 0; j < 2; ++j) CQA_ALLOC_DEV(c->stage[i][j], s.stage);
    CQA_ALLOC_DEV(c->ladder_ws, s.ladder_ws);
    CQA_ALLOC_DEV(c->ladder_tickets, (int64_t)desc->batch * desc->n_kv_heads * 4);
    CQA_TRY(hipMemset(c->ladder_tickets, 0, (size_t)desc->batch * desc->n_kv_heads * 4));
    CQA_ALLOC_DEV(c->ladder_counts, 8);
    CQA_TRY(hipMemset(c->ladder_counts, 0, 8));
    if (c->t2_borrowed) {
      c->t2_k = caller_k;
      c->t2_v = caller_v;
    } else {
      CQA_ALLOC_PIN(c->t2_k, s.t2);
      CQA_ALLOC_PIN(c->t2_v, s.t2);
      // The copy engines' first access to a pinned page is slow (measured: the first 512 MB
      // device-to-host copy into new pinned memory runs at 35 GB/s, every later one at 57 GB/s;
      // touching the pages from the host or from a kernel does not change that, a strided copy
      // of 4 bytes per page does).  Paid here, once, instead of during the first bulk append.
      const int64_t n_pages = s.t2 / 4096;
      for (int64_t p0 = 0; p0 < n_pages; p0 += 65536) {
        const size_t rows = (size_t)std::min<int64_t>(65536, n_pages - p0);
        CQA_TRY(hipMemcpy2DAsync((char*)c->t2_k + p0 * 4096, 4096, c->t1, 4, 4, rows,
                                 hipMemcpyDeviceToHost, nullptr));
        CQA_TRY(hipMemcpy2DAsync((char*)c->t2_v + p0 * 4096, 4096, c->t1, 4, 4, rows,
                                 hipMemcpyDeviceToHost, nullptr));
      }
      CQA_TRY(hipDeviceSynchronize());
    }
  }
  {
    // this device's copy of the fixed scratch of the no-allocation decode: resolve its address now,
    // so that the call itself only looks it up
    void* p = nullptr;
    const int32_t src = static_scratch(c->device, &p);
    if (src != CQA_OK) {
      release(h);
      return src;
    }
  }
  CQA_TRY(hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking));
  for (int i = 0; i < 2; ++i) {
    CQA_TRY(hipEventCreateWithFlags(&c->ev_ready[i], hipEventDisableTiming));
    CQA_TRY(hipEventCreateWithFlags(&c->ev_free[i], hipEventDisableTiming));
  }
  CQA_TRY(hipEventCreateWithFlags(&c->ev_main, hipEventDisableTiming));
  CQA_TRY(hipEventCreateWithFlags(&c->ev_copy, hipEventDisableTiming));
  CQA_TRY(hipEventCreate(&c->ev_t0));
  CQA_TRY(hipEventCreate(&c->ev_t1));
  *out = h;
  return CQA_OK;
}

int32_t cqa_cache_create(const cqa_cache_desc* desc, cqa_cache** out) {
  return create_cache(desc, nullptr, nullptr, out);
}

int32_t cqa_cache_create_caller_tier2(const cqa_cache_desc* desc, void* t2_k_host, void* t2_v_host,
                                      int64_t bytes_each, cqa_cache** out) {
  if (desc == nullptr || t2_k_host == nullptr || t2_v_host == nullptr) return CQA_ERR_INVALID_ARG;
  if (desc->tier2_mode != CQA_TIER2_PINNED) return CQA_ERR_INVALID_ARG;
  const int32_t st = check_desc(desc);
  if (st != CQA_OK) return st;
  const int64_t need = (int64_t)desc->n_layers * desc->batch * desc->n_kv_heads * desc->max_tokens * D * 2;
  if (bytes_each < need) return CQA_ERR_INVALID_ARG;
  // both arrays must be pinned host memory the device can address (hipHostMalloc, or a framework's
  // pinned allocation): the kernels read and write them in place
  for (void* p : {t2_k_host, t2_v_host}) {
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
      (void)hipGetLastError();
      return CQA_ERR_INVALID_ARG;
    }
    if (attr.type != hipMemoryTypeHost || attr.devicePointer == nullptr) return CQA_ERR_INVALID_ARG;
  }
  return create_cache(desc, (__half*)t2_k_host, (__half*)t2_v_host, out);
}

int32_t cqa_cache_destroy(cqa_cache* h) {
  if (h == nullptr) return CQA_ERR_INVALID_ARG;
  release(h);
  return CQA_OK;
}

int32_t cqa_cache_length(const cqa_cache* h, int32_t layer, int64_t* n_tokens) {
  if (h == nullptr || n_tokens == nullptr || layer < 0 || layer >= h->impl.desc.n_layers)
    return CQA_ERR_INVALID_ARG;
  *n_tokens = h->impl.length[layer];
  return CQA_OK;
}

int32_t cqa_cache_reset(cqa_cache* h, int32_t layer) {
  if (h == nullptr || layer < 0 || layer >= h->impl.desc.n_layers) return CQA_ERR_INVALID_ARG;
  Cache* c = &h->impl;
  CQA_HIP(hipDeviceSynchronize());
  CQA_HIP(hipMemset(c->sigmax + head_index(c, layer, 0, 0), 0,
                    (size_t)c->desc.batch * c->desc.n_kv_heads * 4));
  // unsealed blocks must read as zeros (the decode pass loads whole records and relies on it)
  CQA_HIP(hipMemset(c->t1 + head_index(c, layer, 0, 0) * c->nq_cap * QUAD_BYTES, 0,
                    (size_t)c->desc.batch * c->desc.n_kv_heads * c->nq_cap * QUAD_BYTES));
  if (c->ad.sc_map != nullptr) {
    // the layer's blocks are gone: nothing of it stays in the FP16 scratch
    const int64_t h0 = head_index(c, layer, 0, 0), nh = (int64_t)c->desc.batch * c->desc.n_kv_heads;
    CQA_HIP(hipMemset(c->ad.sc_map + h0 * c->nb_cap, 0, (size_t)(nh * c->nb_cap) * 4));
    CQA_HIP(hipMemset(c->ad.sc_tag + h0 * c->ad.sc_cap, 0xFF, (size_t)(nh * c->ad.sc_cap) * 4));
    CQA_HIP(hipMemset(c->ad.sc_age + h0 * c->ad.sc_cap, 0, (size_t)(nh * c->ad.sc_cap) * 4));
    CQA_HIP(hipMemset(c->ad.sc_have + h0 * c->ad.sc_cap, 0, (size_t)(nh * c->ad.sc_cap) * 4));
  }
  c->length[layer] = 0;
  return CQA_OK;
}

int32_t cqa_set_scratch_slots(cqa_cache* h, int32_t n_slots) {
  if (h == nullptr || n_slots < 0) return CQA_ERR_INVALID_ARG;
  Cache* c = &h->impl;
  if (c->desc.tier2_mode != CQA_TIER2_PINNED) return CQA_ERR_NO_TIER2;
  if (n_slots > c->ad.sc_cap) return CQA_ERR_INVALID_ARG;
  CQA_HIP(hipDeviceSynchronize());
  const int64_t cap = c->ad.sc_cap;
  if (n_slots > 0 && c->ad.sc_k == nullptr) {
    // first use: the scratch and its maps
    __half *k = nullptr, *v = nullptr;
    int32_t *map = nullptr, *tag = nullptr, *have = nullptr;
    uint32_t* age = nullptr;
    hipError_t e = hipMalloc((void**)&k, (size_t)(c->heads_total * cap) * BLK * D * 2);
    if (e == hipSuccess) e = hipMalloc((void**)&v, (size_t)(c->heads_total * cap) * BLK * D * 2);
    if (e == hipSuccess) e = hipMalloc((void**)&have, (size_t)(c->heads_total * cap) * 4);
    if (e == hipSuccess) e = hipMalloc((void**)&map, (size_t)(c->heads_total * c->nb_cap) * 4);
    if (e == hipSuccess) e = hipMalloc((void**)&tag, (size_t)(c->heads_total * cap) * 4);
    if (e == hipSuccess) e = hipMalloc((void**)&age, (size_t)(c->heads_total * cap) * 4);
    if (e != hipSuccess) {
      g_last_hip_error = (int)e;
      (void)hipGetLastError();
      (void)hipFree(k);
      (void)hipFree(v);
      (void)hipFree(have);
      (void)hipFree(map);
      (void)hipFree(tag);
      (void)hipFree(age);
      return e == hipErrorOutOfMemory ? CQA_ERR_OOM_DEVICE : CQA_ERR_HIP;
    }
    c->ad.sc_k = k;
    c->ad.sc_v = v;
    c->ad.sc_have = have;
    c->ad.sc_map = map;
    c->ad.sc_tag = tag;
    c->ad.sc_age = age;
  }
  if (c->ad.sc_k != nullptr) {
    CQA_HIP(hipMemset(c->ad.sc_map, 0, (size_t)(c->heads_total * c->nb_cap) * 4));
    CQA_HIP(hipMemset(c->ad.sc_tag, 0xFF, (size_t)(c->heads_total * cap) * 4));   // -1: empty
    CQA_HIP(hipMemset(c->ad.sc_age, 0, (size_t)(c->heads_total * cap) * 4));
    CQA_HIP(hipMemset(c->ad.sc_have, 0, (size_t)(c->heads_total * cap) * 4));
  }
  c->ad.sc_slots = n_slots;
  return CQA_OK;
}

int32_t cqa_scratch_stats(cqa_cache* h, int32_t* slots_per_head, int64_t* hits, int64_t* misses) {
  if (h == nullptr) return CQA_ERR_INVALID_ARG;
  Cache* c = &h->impl;
  uint32_t n[2] = {0u, 0u};
  if (c->ad.sc_stats != nullptr) {
    CQA_HIP(hipDeviceSynchronize());
    CQA_HIP(hipMemcpy(n, c->ad.sc_stats, 8, hipMemcpyDeviceToHost));
  }
  if (slots_per_head) *slots_per_head = c->ad.sc_slots;
  if (hits) *hits = n[0];
  if (misses) *misses = n[1];
  return CQA_OK;
}

int32_t cqa_set_splits(cqa_cache* h, int32_t n_splits) {
  if (h == nullptr || n_splits < 0) return CQA_ERR_INVALID_ARG;
  h->impl.forced_splits = n_splits;
  return CQA_OK;
}

int32_t cqa_set_stream_hint(cqa_cache* h, int32_t mode) {
  if (h == nullptr || mode < 0 || mode > 2) return CQA_ERR_INVALID_ARG;
  h->impl.stream_hint = mode;
  return CQA_OK;
}

int32_t cqa_set_kernel_variant(cqa_cache* h, int32_t variant) {
  if (h == nullptr || variant < 0 || variant > 1) return CQA_ERR_INVALID_ARG;
  h->impl.variant = variant;
  return CQA_OK;
}

int32_t cqa_decode_splits(const cqa_cache* h, int32_t layer, int32_t* n_splits) {
  if (h == nullptr || n_splits == nullptr || layer < 0 || layer >= h->impl.desc.n_layers)
    return CQA_ERR_INVALID_ARG;
  *n_splits = pick_splits(&h->impl, h->impl.length[layer] / BLK);
  return CQA_OK;
}

int32_t cqa_cache_append(cqa_cache* h, int32_t layer, const void* k_fp16_dev,
                         const void* v_fp16_dev, int64_t n_new, void* stream) {
  if (h == nullptr || layer < 0 || layer >= h->impl.desc.n_layers || k_fp16_dev == nullptr ||
      v_fp16_dev == nullptr || n_new < 0)
    return CQA_ERR_INVALID_ARG;
  if (n_new == 0) return CQA_OK;
  Cache* c = &h->impl;
  const int64_t len = c->length[layer];
  if (len + n_new > c->desc.max_tokens) return CQA_ERR_CAPACITY;
  hipStream_t st = (hipStream_t)stream;
  const __half* k = (const __half*)k_fp16_dev;
  const __half* v = (const __half*)v_fp16_dev;
  // short appends (the decode-time case) store their originals from the kernel that also fills
  // the trailing block; long ones (prefill) use the copy engines
  const bool t2_by_kernel = c->desc.tier2_mode == CQA_TIER2_PINNED && n_new <= BLK;
  if (c->desc.tier2_mode == CQA_TIER2_PINNED && !t2_by_kernel) {
    // one strided copy per tensor: row = one (batch, kv-head) sequence
    const int64_t head0 = head_index(c, layer, 0, 0);
    const size_t rows = (size_t)c->desc.batch * c->desc.n_kv_heads;
    const size_t width = (size_t)n_new * D * 2;
    const size_t dpitch = (size_t)c->desc.max_tokens * D * 2;
    // on the side stream, so that the copy engines run while the seal kernel quantizes: the side
    // stream starts when the caller's stream has reached this point (the inputs are ready), and
    // the caller's stream goes on past the seal only when the copies are done (the caller may
    // then reuse k and v, and later kernels may read the originals)
    CQA_HIP(hipEventRecord(c->ev_main, st));
    CQA_HIP(hipStreamWaitEvent(c->side, c->ev_main, 0));
    CQA_HIP(hipMemcpy2DAsync(c->t2_k + (head0 * c->desc.max_tokens + len) * D, dpitch, k, width,
                             width, rows, hipMemcpyDeviceToHost, c->side));
    CQA_HIP(hipMemcpy2DAsync(c->t2_v + (head0 * c->desc.max_tokens + len) * D, dpitch, v, width,
                             width, rows, hipMemcpyDeviceToHost, c->side));
    CQA_HIP(hipEventRecord(c->ev_copy, c->side));
  }
  const int32_t rc = launch_seal(c, layer, k, v, n_new, len, t2_by_kernel, st);
  if (c->desc.tier2_mode == CQA_TIER2_PINNED && !t2_by_kernel)
    CQA_HIP(hipStreamWaitEvent(st, c->ev_copy, 0));
  if (rc != CQA_OK) return rc;
  c->length[layer] = len + n_new;
  return CQA_OK;
}

int32_t cqa_cache_export_block(const cqa_cache* h, int32_t layer, int32_t batch, int32_t kv_head,
                               int64_t block, int8_t* kcodes, float* sigma, float* z,
                               uint8_t* vcodes, uint16_t* vscale_bits, uint16_t* voffset_bits,
                               float* eta, float* nu) {
  if (h == nullptr) return CQA_ERR_INVALID_ARG;
  const Cache* c = &h->impl;
  if (layer < 0 || layer >= c->desc.n_layers || batch < 0 || batch >= c->desc.batch ||
      kv_head < 0 || kv_head >= c->desc.n_kv_heads || block < 0 ||
      block >= c->length[layer] / BLK)
    return CQA_ERR_INVALID_ARG;
  CQA_HIP(hipDeviceSynchronize());
  const int64_t head_rec = head_index(c, layer, batch, kv_head) * c->nq_cap;
  uint8_t kc[KC_BYTES];
  float km[KM_BYTES / 4];
  uint32_t vc[VC_BYTES / 4];
  uint16_t vm[VM_BYTES / 2];
  float an[2];
  CQA_HIP(hipMemcpy(kc, c->t1 + t1_offset(head_rec, block, Q_KC, KC_BYTES), KC_BYTES, hipMemcpyDeviceToHost));
  CQA_HIP(hipMemcpy(km, c->t1 + t1_offset(head_rec, block, Q_KM, KM_BYTES), KM_BYTES, hipMemcpyDeviceToHost));
  CQA_HIP(hipMemcpy(vc, c->t1 + t1_offset(head_rec, block, Q_VC, VC_BYTES), VC_BYTES, hipMemcpyDeviceToHost));
  CQA_HIP(hipMemcpy(vm, c->t1 + t1_offset(head_rec, block, Q_VM, VM_BYTES), VM_BYTES, hipMemcpyDeviceToHost));
  CQA_HIP(hipMemcpy(an, c->t1 + t1_offset(head_rec, block, Q_AN, AN_BYTES), AN_BYTES, hipMemcpyDeviceToHost));
  for (int t = 0; t < BLK; ++t)
    for (int ch = 0; ch < D; ++ch) {
      if (kcodes) kcodes[t * D + ch] = (int8_t)((int)kc[kc_offset(t, ch)] - 128);
      if (vcodes)
        vcodes[t * D + ch] =
            (uint8_t)((vc[vc_dword_offset(t >> 3, ch) / 4] >> (4 * (t & 7))) & 15u);
    }
  for (int ch = 0; ch < D; ++ch) {
    if (sigma) sigma[ch] = km[ch];
    if (z) z[ch] = km[D + ch];
  }
  for (int t = 0; t < BLK; ++t)
    for (int g = 0; g < NG; ++g) {
      if (vscale_bits) vscale_bits[t * NG + g] = vm[vm_index(t, g)];
      if (voffset_bits) voffset_bits[t * NG + g] = vm[BLK * NG + vm_index(t, g)];
    }
  if (eta) *eta = an[0];
  if (nu) *nu = an[1];
  return CQA_OK;
}

int32_t cqa_certified_decode(cqa_cache* h, int32_t layer, const void* q_fp16_dev,
                             const cqa_tolerances* tol, float* O_dev, cqa_head_cert* cert_dev,
                             uint32_t* flags_dev, float* blk_logmass_dev, void* stream) {
  if (h == nullptr || layer < 0 || layer >= h->impl.desc.n_layers || q_fp16_dev == nullptr ||
      tol == nullptr || O_dev == nullptr || cert_dev == nullptr || flags_dev == nullptr)
    return CQA_ERR_INVALID_ARG;
  if (h->impl.length[layer] <= 0) return CQA_ERR_INVALID_ARG;
  if (const int32_t trc = check_tolerances(tol)) return trc;
  return launch_certified(&h->impl, layer, (const __half*)q_fp16_dev, *tol, O_dev, cert_dev,
                          flags_dev, nullptr, 0u, blk_logmass_dev, (hipStream_t)stream);
}

int32_t cqa_certified_decode_noalloc(cqa_cache* h, int32_t layer, const void* q_fp16_dev,
                                     const cqa_tolerances* tol, float* O_dev,
                                     cqa_head_cert* cert_dev, uint32_t* flags_dev, void* stream) {
  if (h == nullptr || layer < 0 || layer >= h->impl.desc.n_layers || q_fp16_dev == nullptr ||
      tol == nullptr || O_dev == nullptr || cert_dev == nullptr || flags_dev == nullptr)
    return CQA_ERR_INVALID_ARG;
  Cache* c = &h->impl;
  if (c->length[layer] <= 0) return CQA_ERR_INVALID_ARG;
  if (const int32_t trc = check_tolerances(tol)) return trc;
  int cur = -1;
  CQA_HIP(hipGetDevice(&cur));
  if (cur != c->device) return CQA_ERR_INVALID_ARG;
  // the partial sets of this launch: [batch * q heads][splits][PART_FLOATS] floats
  const int64_t nsplit = pick_splits(c, c->length[layer] / BLK);
  const int64_t need = (int64_t)c->desc.batch * c->desc.n_q_heads * std::max<int64_t>(nsplit, 1) * PART_FLOATS * 4;
  if (need > CQA_STATIC_SCRATCH_BYTES) return CQA_ERR_SCRATCH;
  void* sp = nullptr;
  const int32_t src = static_scratch(c->device, &sp);   // resolved at cache creation: a lookup
  if (src != CQA_OK) return src;
  return launch_certified(c, layer, (const __half*)q_fp16_dev, *tol, O_dev, cert_dev, flags_dev,
                          nullptr, 0u, nullptr, (hipStream_t)stream, nullptr, nullptr, 0, nullptr,
                          (float*)sp);
}

int32_t cqa_time_certified_decode(cqa_cache* h, int32_t layer, const void* q_fp16_dev,
                                  const cqa_tolerances* tol, float* O_dev,
                                  cqa_head_cert* cert_dev, uint32_t* flags_dev,
                                  float* blk_logmass_dev, int32_t iters, float* ms_per_step,
                                  void* stream) {
  if (h == nullptr || iters < 1 || ms_per_step == nullptr) return CQA_ERR_INVALID_ARG;
  Cache* c = &h->impl;
  hipStream_t st = (hipStream_t)stream;
  CQA_HIP(hipEventRecord(c->ev_t0, st));
  for (int i = 0; i < iters; ++i) {
    const int32_t rc = cqa_certified_decode(h, layer, q_fp16_dev, tol, O_dev, cert_dev, flags_dev,
                                            blk_logmass_dev, stream);
    if (rc != CQA_OK) return rc;
  }
  CQA_HIP(hipEventRecord(c->ev_t1, st));
  CQA_HIP(hipEventSynchronize(c->ev_t1));
  float ms = 0.0f;
  CQA_HIP(hipEventElapsedTime(&ms, c->ev_t0, c->ev_t1));
  *ms_per_step = ms / (float)iters;
  return CQA_OK;
}

int32_t cqa_time_stream_read(cqa_cache* h, int32_t layer, int32_t iters, float* ms_per_launch,
                             int64_t* bytes_per_launch, void* stream) {
  if (h == nullptr || layer < 0 || layer >= h->impl.desc.n_layers || iters < 1 ||
      ms_per_launch == nullptr)
    return CQA_ERR_INVALID_ARG;
  Cache* c = &h->impl;
  const int64_t nb = c->length[layer] / BLK;
  if (nb < 1) return CQA_ERR_INVALID_ARG;
  int nsplit = 0, bps = 0;
  split_geometry(c, nb, &nsplit, &bps);
  hipStream_t st = (hipStream_t)stream;
  const dim3 grid(nsplit, c->desc.n_kv_heads, c->desc.batch);
  const uint8_t* t1 = c->t1 + head_index(c, layer, 0, 0) * c->nq_cap * QUAD_BYTES;
  const bool nt = stream_nt(c, nb) != 0;
  // the select flags buffer doubles as the (never written) sink
  int32_t rc = launch_stream_read(t1, c->nq_cap, (int)nb, grid, nt, waves_per_workgroup(c), c->select_dev, st);   // warm-up
  if (rc != CQA_OK) return rc;
  CQA_HIP(hipEventRecord(c->ev_t0, st));
  for (int i = 0; i < iters; ++i) {
    rc = launch_stream_read(t1, c->nq_cap, (int)nb, grid, nt, waves_per_workgroup(c), c->select_dev, st);
    if (rc != CQA_OK) return rc;
  }
  CQA_HIP(hipEventRecord(c->ev_t1, st));
  CQA_HIP(hipEventSynchronize(c->ev_t1));
  float ms = 0.0f;
  CQA_HIP(hipEventElapsedTime(&ms, c->ev_t0, c->ev_t1));
  *ms_per_launch = ms / (float)iters;
  if (bytes_per_launch)
    *bytes_per_launch = (int64_t)c->desc.batch * c->desc.n_kv_heads * ((nb + 3) / 4) * (18 * 1024);
  return CQA_OK;
}

int32_t cqa_profile_begin(cqa_cache* h, int32_t max_launches) {
  if (h == nullptr || max_launches < 1 || max_launches > 65536) return CQA_ERR_INVALID_ARG;
  Cache* c = &h->impl;
  if (c->prof_ev != nullptr && c->prof_cap < max_launches) {
    for (int i = 0; i < 2 * c->prof_cap; ++i)
      if (c->prof_ev[i]) (void)hipEventDestroy(c->prof_ev[i]);
    delete[] c->prof_ev;
    c->prof_ev = nullptr;
    c->prof_cap = 0;
  }
  if (c->prof_ev == nullptr) {
    c->prof_ev = new (std::nothrow) hipEvent_t[2 * (size_t)max_launches];
    if (c->prof_ev == nullptr) return CQA_ERR_INVALID_ARG;
    for (int i = 0; i < 2 * max_launches; ++i) c->prof_ev[i] = nullptr;
    c->prof_cap = max_launches;
    for (int i = 0; i < 2 * max_launches; ++i) CQA_HIP(hipEventCreate(&c->prof_ev[i]));
  }
  c->prof_n = 0;
  return CQA_OK;
}

int32_t cqa_profile_end(cqa_cache* h, float* mean_ms, float* min_ms, int32_t* n_launches) {
  if (h == nullptr) return CQA_ERR_INVALID_ARG;
  Cache* c = &h->impl;
  if (c->prof_ev == nullptr) return CQA_ERR_INVALID_ARG;
  const int n = c->prof_n;
  double sum = 0.0;
  float mn = 0.0f;
  delete[] c->prof_ms;
  c->prof_ms = new (std::nothrow) float[(size_t)(n > 0 ? n : 1)];
  c->prof_ms_n = 0;
  if (c->prof_ms == nullptr) return CQA_ERR_INVALID_ARG;
  for (int i = 0; i < n; ++i) {
    CQA_HIP(hipEventSynchronize(c->prof_ev[2 * i + 1]));
    float ms = 0.0f;
    CQA_HIP(hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]));
    c->prof_ms[i] = ms;
    c->prof_ms_n = i + 1;
    sum += ms;
    mn = (i == 0 || ms < mn) ? ms : mn;
  }
  if (mean_ms) *mean_ms = n > 0 ? (float)(sum / n) : 0.0f;
  if (min_ms) *min_ms = mn;
  if (n_launches) *n_launches = n;
  c->prof_n = c->prof_cap;  // stop recording until the next begin
  return CQA_OK;
}

int32_t cqa_profile_durations(cqa_cache* h, float* ms_host, int32_t cap, int32_t* n_launches) {
  if (h == nullptr || cap < 0 || (cap > 0 && ms_host == nullptr)) return CQA_ERR_INVALID_ARG;
  Cache* c = &h->impl;
  const int n = c->prof_ms != nullptr ? c->prof_ms_n : 0;
  for (int i = 0; i < n && i < cap; ++i) ms_host[i] = c->prof_ms[i];
  if (n_launches) *n_launches = n;
  return CQA_OK;
}

int32_t cqa_dense_fallback(cqa_cache* h, int32_t layer, const void* q_fp16_dev,
                           const uint32_t* head_select_host, int32_t all_heads, int32_t rung,
                           float* O_dev, cqa_head_cert* cert_dev, uint32_t* flags_dev,
                           void* stream) {
  if (h == nullptr || layer < 0 || layer >= h->impl.desc.n_layers || q_fp16_dev == nullptr ||
      O_dev == nullptr || (!all_heads && head_select_host == nullptr) || rung < 0 || rung > 7)
    return CQA_ERR_INVALID_ARG;
  Cache* c = &h->impl;
  if (c->desc.tier2_mode != CQA_TIER2_PINNED) return CQA_ERR_NO_TIER2;
  const int64_t len = c->length[layer];
  if (len <= 0) return CQA_ERR_INVALID_ARG;
  const int bt = c->desc.batch, hq = c->desc.n_q_heads, hkv = c->desc.n_kv_heads;
  const int g = hq / hkv;
  hipStream_t st = (hipStream_t)stream;
  const __half* q = (const __half*)q_fp16_dev;

  std::vector<int> groups;
  for (int b = 0; b < bt; ++b)
    for (int kh = 0; kh < hkv; ++kh) {
      bool any = all_heads != 0;
      for (int i = 0; i < g && !any; ++i) any = head_select_host[b * hq + kh * g + i] != 0;
      if (any) groups.push_back(b * hkv + kh);
    }
  if (groups.empty()) return CQA_OK;
  if (!all_heads)
    CQA_HIP(hipMemcpyAsync(c->select_dev, head_select_host, (size_t)bt * hq * 4,
                           hipMemcpyHostToDevice, st));
  // the side stream must see every Tier-2 write queued on the caller's stream so far
  CQA_HIP(hipEventRecord(c->ev_main, st));
  CQA_HIP(hipStreamWaitEvent(c->side, c->ev_main, 0));
  const int64_t ws_floats = dense_ws_floats(g, c->desc.max_tokens);
  const size_t bytes = (size_t)len * D * 2;
  for (size_t i = 0; i < groups.size(); ++i) {
    const int buf = (int)(i & 1);
    const int b = groups[i] / hkv, kh = groups[i] % hkv;
    const int64_t head = head_index(c, layer, b, kh);
    if (c->free_valid[buf]) CQA_HIP(hipStreamWaitEvent(c->side, c->ev_free[buf], 0));
    CQA_HIP(hipMemcpyAsync(c->stage[buf][0], c->t2_k + head * c->desc.max_tokens * D, bytes,
                           hipMemcpyHostToDevice, c->side));
    CQA_HIP(hipMemcpyAsync(c->stage[buf][1], c->t2_v + head * c->desc.max_tokens * D, bytes,
                           hipMemcpyHostToDevice, c->side));
    CQA_HIP(hipEventRecord(c->ev_ready[buf], c->side));
    CQA_HIP(hipStreamWaitEvent(st, c->ev_ready[buf], 0));
    const int64_t row = (int64_t)b * hq + kh * g;
    const int32_t rc = launch_dense_group(
        q + row * D, c->stage[buf][0], c->stage[buf][1], g, len, O_dev + row * D,
        all_heads ? nullptr : c->select_dev + row, cert_dev ? cert_dev + row : nullptr,
        flags_dev ? flags_dev + row : nullptr, rung, c->dense_ws + buf * ws_floats, st);
    if (rc != CQA_OK) return rc;
    CQA_HIP(hipEventRecord(c->ev_free[buf], st));
    c->free_valid[buf] = true;
  }
  return CQA_OK;
}

// Flag read-back and ladder shared by the one-call steps.  `adaptive` selects which decode runs.
static int32_t step_with_ladder(cqa_cache* h, int32_t layer, const void* q_fp16_dev,
                                const cqa_tolerances* tol, const cqa_selector* sel, float* O_dev,
                                cqa_head_cert* cert_dev, uint32_t* flags_dev,
                                float* blk_logmass_dev, int32_t* rung_served, void* stream,
                                const __half* k_new = nullptr, const __half* v_new = nullptr) {
  Cache* c = &h->impl;
  hipStream_t st = (hipStream_t)stream;
  // The reduction also writes each head's flag word, tagged with this step's sequence number,
  // into mapped pinned host memory as its last store.  The host polls those words instead of
  // waiting for the stream: the ladder decision needs nothing else on the host, and everything
  // enqueued afterwards is ordered behind the reduction by the stream itself.  The poll is
  // bounded; when the tags do not all show up in time it falls back to a stream synchronisation.
  c->step_seq = (c->step_seq % 0xFFFFu) + 1u;            // 1 .. 65535, never 0
  const uint32_t tag = c->step_seq << 16;
  int32_t rc;
  if (sel != nullptr)
    rc = launch_adaptive(c, layer, (const __half*)q_fp16_dev, *tol, *sel, O_dev, cert_dev, flags_dev,
                         c->flags_host, tag, st);
  else
    rc = launch_certified(c, layer, (const __half*)q_fp16_dev, *tol, O_dev, cert_dev, flags_dev,
                          c->flags_host, tag, blk_logmass_dev, st, k_new, v_new);
  if (rc != CQA_OK) return rc;
  const int bt = c->desc.batch, hq = c->desc.n_q_heads, hkv = c->desc.n_kv_heads;
  const int g = hq / hkv;
  const int n = bt * hq;
  {
    volatile const uint32_t* mirror = c->flags_host;
    const auto t_start = std::chrono::steady_clock::now();
    bool seen = false;
    for (uint32_t spin = 0; !seen; ++spin) {
      seen = true;
      for (int i = 0; i < n; ++i)
        if ((mirror[i] & 0xFFFF0000u) != tag) {
          seen = false;
          break;
        }
      if (!seen && (spin & 1023u) == 1023u &&
          std::chrono::steady_clock::now() - t_start > std::chrono::milliseconds(20))
        break;
    }
    if (!seen) {
      CQA_HIP(hipStreamSynchronize(st));
      for (int i = 0; i < n; ++i)
        if ((mirror[i] & 0xFFFF0000u) != tag) return CQA_ERR_HIP;
    }
  }
  // ladder policy: PRECOND anywhere, or enough flagged KV groups, escalates to the whole layer
  bool any = false, precond = false;
  int flagged_groups = 0;
  uint32_t* need = c->need;
  memset(need, 0, sizeof(uint32_t) * n);
  for (int b = 0; b < bt; ++b)
    for (int kh = 0; kh < hkv; ++kh) {
      bool grp = false;
      for (int i = 0; i < g; ++i) {
        const int idx = b * hq + kh * g + i;
        const uint32_t f = c->flags_host[idx] & 0xFFFFu;
        if (f & CQA_FLAG_ANY) {
          need[idx] = 1u;
          grp = true;
        }
        if (f & CQA_FLAG_PRECOND) precond = true;
      }
      if (grp) {
        any = true;
        ++flagged_groups;
      }
    }
  int rung = 0;
  if (any) {
    rung = 3;
    if (precond || (tol->rung4_min_groups > 0 && flagged_groups >= tol->rung4_min_groups)) rung = 4;
  }
  if (rung_served) *rung_served = rung;
  if (rung == 0) return CQA_OK;
  return cqa_dense_fallback(h, layer, q_fp16_dev, need, rung == 4, rung, O_dev, cert_dev,
                            flags_dev, stream);
}

static int32_t check_decode_args(cqa_cache* h, int32_t layer, const void* q, const cqa_tolerances* tol,
                                 float* O, cqa_head_cert* cert, uint32_t* flags,
                                 int max_rank_depth = 1) {
  if (h == nullptr || layer < 0 || layer >= h->impl.desc.n_layers || q == nullptr ||
      tol == nullptr || O == nullptr || cert == nullptr || flags == nullptr)
    return CQA_ERR_INVALID_ARG;
  if (h->impl.length[layer] <= 0) return CQA_ERR_INVALID_ARG;
  if (const int32_t trc = check_tolerances(tol, max_rank_depth)) return trc;
  return CQA_OK;
}

static int32_t check_selector(const cqa_cache* h, const cqa_selector* sel) {
  if (sel == nullptr || !(sel->tau_cov == sel->tau_cov) || sel->k_min < 0 || sel->k_max < sel->k_min ||
      sel->k_limit < sel->k_max || sel->k_limit > MAX_K_LIMIT || sel->v_limit < 0 ||
      sel->v_limit > MAX_K_LIMIT || (sel->v_greedy != 0 && sel->v_greedy != 1) ||
      (sel->canary != 0 && sel->canary != 1) || !(sel->explore_frac >= 0.0f && sel->explore_frac <= 1.0f) ||
      (sel->per_head != 0 && sel->per_head != 1))
    return CQA_ERR_INVALID_ARG;
  if (h->impl.desc.tier2_mode != CQA_TIER2_PINNED) return CQA_ERR_NO_TIER2;
  return CQA_OK;
}

int32_t cqa_decode_step(cqa_cache* h, int32_t layer, const void* q_fp16_dev,
                        const cqa_tolerances* tol, float* O_dev, cqa_head_cert* cert_dev,
                        uint32_t* flags_dev, float* blk_logmass_dev, int32_t* rung_served,
                        void* stream) {
  const int32_t rc = check_decode_args(h, layer, q_fp16_dev, tol, O_dev, cert_dev, flags_dev);
  if (rc != CQA_OK) return rc;
  return step_with_ladder(h, layer, q_fp16_dev, tol, nullptr, O_dev, cert_dev, flags_dev,
                          blk_logmass_dev, rung_served, stream);
}

// Appends one token per sequence ahead of a decode launch.  The new token rides on the decode
// launch itself (*ride_k / *ride_v set, length already counted) when it neither completes a block
// (the seal must run first then) nor finds the cache without a sealed block (no split pass is
// launched then), and the matrix-core kernel is in use; otherwise it is appended here.
static int32_t append_or_ride(cqa_cache* h, int32_t layer, const void* k, const void* v, void* stream,
                              const __half** ride_k, const __half** ride_v) {
  Cache* c = &h->impl;
  const int64_t len = c->length[layer];
  *ride_k = nullptr;
  *ride_v = nullptr;
  if (len + 1 > c->desc.max_tokens) return CQA_ERR_CAPACITY;
  const bool ride = (len % BLK) != BLK - 1 && len >= BLK && c->variant == 0;
  if (!ride) return cqa_cache_append(h, layer, k, v, 1, stream);
  c->length[layer] = len + 1;
  *ride_k = (const __half*)k;
  *ride_v = (const __half*)v;
  return CQA_OK;
}

int32_t cqa_append_decode_step(cqa_cache* h, int32_t layer, const void* k_fp16_dev,
                               const void* v_fp16_dev, const void* q_fp16_dev,
                               const cqa_tolerances* tol, float* O_dev, cqa_head_cert* cert_dev,
                               uint32_t* flags_dev, int32_t* rung_served, void* stream) {
  if (h == nullptr || layer < 0 || layer >= h->impl.desc.n_layers || k_fp16_dev == nullptr ||
      v_fp16_dev == nullptr || q_fp16_dev == nullptr || tol == nullptr || O_dev == nullptr ||
      cert_dev == nullptr || flags_dev == nullptr)
    return CQA_ERR_INVALID_ARG;
  if (const int32_t trc = check_tolerances(tol)) return trc;
  const __half *rk = nullptr, *rv = nullptr;
  const int32_t rc = append_or_ride(h, layer, k_fp16_dev, v_fp16_dev, stream, &rk, &rv);
  if (rc != CQA_OK) return rc;
  const int64_t len_before = h->impl.length[layer];
  const int32_t src = step_with_ladder(h, layer, q_fp16_dev, tol, nullptr, O_dev, cert_dev, flags_dev,
                                       nullptr, rung_served, stream, rk, rv);
  // a failure before the split launch (the launch that stores a riding token) leaves the cache as
  // it was; later failures (a fallback without originals) keep the token
  if (src == CQA_ERR_INVALID_ARG && rk != nullptr) h->impl.length[layer] = len_before - 1;
  return src;
}

int32_t cqa_decode_step_enqueue(cqa_cache* h, int32_t layer, const void* k_fp16_dev,
                                const void* v_fp16_dev, const void* q_fp16_dev,
                                const cqa_tolerances* tol, float* O_dev, cqa_head_cert* cert_dev,
                                uint32_t* flags_dev, void* stream) {
  if (h == nullptr || layer < 0 || layer >= h->impl.desc.n_layers || q_fp16_dev == nullptr ||
      tol == nullptr || O_dev == nullptr || cert_dev == nullptr || flags_dev == nullptr ||
      (k_fp16_dev == nullptr) != (v_fp16_dev == nullptr))
    return CQA_ERR_INVALID_ARG;
  if (const int32_t trc = check_tolerances(tol)) return trc;
  Cache* c = &h->impl;
  if (c->desc.tier2_mode != CQA_TIER2_PINNED) return CQA_ERR_NO_TIER2;
  const __half *rk = nullptr, *rv = nullptr;
  if (k_fp16_dev != nullptr) {
    const int32_t rc = append_or_ride(h, layer, k_fp16_dev, v_fp16_dev, stream, &rk, &rv);
    if (rc != CQA_OK) return rc;
  }
  if (c->length[layer] <= 0) return CQA_ERR_INVALID_ARG;
  int32_t rc = launch_certified(c, layer, (const __half*)q_fp16_dev, *tol, O_dev, cert_dev, flags_dev,
                                nullptr, 0u, nullptr, (hipStream_t)stream, rk, rv);
  if (rc != CQA_OK) {
    if (rk != nullptr) c->length[layer] -= 1;   // the launch that was to store the token did not happen
    return rc;
  }
  return launch_dense_ladder(c, layer, (const __half*)q_fp16_dev, tol->rung4_min_groups, O_dev,
                             cert_dev, flags_dev, (hipStream_t)stream);
}

int32_t cqa_ladder_counts(cqa_cache* h, int64_t* rung3_steps, int64_t* rung4_steps) {
  if (h == nullptr) return CQA_ERR_INVALID_ARG;
  uint32_t n[2] = {0u, 0u};
  if (h->impl.ladder_counts != nullptr) {
    CQA_HIP(hipDeviceSynchronize());
    CQA_HIP(hipMemcpy(n, h->impl.ladder_counts, 8, hipMemcpyDeviceToHost));
  }
  if (rung3_steps) *rung3_steps = n[0];
  if (rung4_steps) *rung4_steps = n[1];
  return CQA_OK;
}

int32_t cqa_adaptive_decode(cqa_cache* h, int32_t layer, const void* q_fp16_dev,
                            const cqa_tolerances* tol, const cqa_selector* sel, float* O_dev,
                            cqa_head_cert* cert_dev, uint32_t* flags_dev, void* stream) {
  int32_t rc = check_decode_args(h, layer, q_fp16_dev, tol, O_dev, cert_dev, flags_dev, MAX_RANK_DEPTH);
  if (rc != CQA_OK) return rc;
  rc = check_selector(h, sel);
  if (rc != CQA_OK) return rc;
  return launch_adaptive(&h->impl, layer, (const __half*)q_fp16_dev, *tol, *sel, O_dev, cert_dev,
                         flags_dev, nullptr, 0u, (hipStream_t)stream);
}

int32_t cqa_adaptive_step(cqa_cache* h, int32_t layer, const void* q_fp16_dev,
                          const cqa_tolerances* tol, const cqa_selector* sel, float* O_dev,
                          cqa_head_cert* cert_dev, uint32_t* flags_dev, int32_t* rung_served,
                          void* stream) {
  int32_t rc = check_decode_args(h, layer, q_fp16_dev, tol, O_dev, cert_dev, flags_dev, MAX_RANK_DEPTH);
  if (rc != CQA_OK) return rc;
  rc = check_selector(h, sel);
  if (rc != CQA_OK) return rc;
  return step_with_ladder(h, layer, q_fp16_dev, tol, sel, O_dev, cert_dev, flags_dev, nullptr,
                          rung_served, stream);
}

int32_t cqa_adaptive_step_enqueue(cqa_cache* h, int32_t layer, const void* q_fp16_dev,
                                  const cqa_tolerances* tol, const cqa_selector* sel, float* O_dev,
                                  cqa_head_cert* cert_dev, uint32_t* flags_dev, void* stream) {
  int32_t rc = check_decode_args(h, layer, q_fp16_dev, tol, O_dev, cert_dev, flags_dev, MAX_RANK_DEPTH);
  if (rc != CQA_OK) return rc;
  rc = check_selector(h, sel);
  if (rc != CQA_OK) return rc;
  rc = launch_adaptive(&h->impl, layer, (const __half*)q_fp16_dev, *tol, *sel, O_dev, cert_dev,
                       flags_dev, nullptr, 0u, (hipStream_t)stream);
  if (rc != CQA_OK) return rc;
  return launch_dense_ladder(&h->impl, layer, (const __half*)q_fp16_dev, tol->rung4_min_groups,
                             O_dev, cert_dev, flags_dev, (hipStream_t)stream);
}

int32_t cqa_adaptive_state(cqa_cache* h, int32_t layer, int32_t* k_star_host,
                           int32_t* selected_host, uint16_t* promoted_host,
                           float* logmass_int8_host, float* logmass_mixed_host,
                           int32_t* v_count_host, int32_t* v_selected_host, float* contrib_host,
                           float* score_dev_host) {
  if (h == nullptr || layer < 0 || layer >= h->impl.desc.n_layers) return CQA_ERR_INVALID_ARG;
  Cache* c = &h->impl;
  if (c->desc.tier2_mode != CQA_TIER2_PINNED) return CQA_ERR_NO_TIER2;
  CQA_HIP(hipDeviceSynchronize());
  const int64_t rows = (int64_t)c->desc.batch * c->desc.n_q_heads;
  const int64_t groups = (int64_t)c->desc.batch * c->desc.n_kv_heads;
  const int64_t nb = c->length[layer] / BLK;
  if (k_star_host)
    CQA_HIP(hipMemcpy(k_star_host, c->ad.kstar, (size_t)rows * 4, hipMemcpyDeviceToHost));
  if (selected_host)
    CQA_HIP(hipMemcpy(selected_host, c->ad.sel, (size_t)rows * MAX_K_LIMIT * 4, hipMemcpyDeviceToHost));
  if (logmass_int8_host && nb > 0)
    CQA_HIP(hipMemcpy(logmass_int8_host, c->ad.lm8, (size_t)(rows * nb) * 4, hipMemcpyDeviceToHost));
  if (logmass_mixed_host && nb > 0) {
    // the promoted-block pass writes the log-masses of the listed blocks only: every other block
    // keeps the one it got in the pass over all blocks
    std::vector<float> l8((size_t)(rows * nb));
    std::vector<int32_t> slot((size_t)nb);
    CQA_HIP(hipMemcpy(logmass_mixed_host, c->ad.lmx, (size_t)(rows * nb) * 4, hipMemcpyDeviceToHost));
    CQA_HIP(hipMemcpy(l8.data(), c->ad.lm8, (size_t)(rows * nb) * 4, hipMemcpyDeviceToHost));
    const int gsz = c->desc.n_q_heads / c->desc.n_kv_heads;
    for (int64_t gidx = 0; gidx < groups; ++gidx) {
      CQA_HIP(hipMemcpy(slot.data(), c->ad.slot + gidx * c->nq_cap * 4, (size_t)nb * 4,
                        hipMemcpyDeviceToHost));
      for (int i = 0; i < gsz; ++i) {
        const int64_t row = gidx * gsz + i;    // rows are [batch][q-head], groups [batch][kv-head]
        for (int64_t blk = 0; blk < nb; ++blk)
          if (slot[(size_t)blk] == 0) logmass_mixed_host[row * nb + blk] = l8[(size_t)(row * nb + blk)];
      }
    }
  }
  if (score_dev_host)
    CQA_HIP(hipMemcpy(score_dev_host, c->ad.score_dev, (size_t)rows * 4, hipMemcpyDeviceToHost));
  if (v_count_host)
    CQA_HIP(hipMemcpy(v_count_host, c->ad.vcount, (size_t)rows * 4, hipMemcpyDeviceToHost));
  if (v_selected_host)
    CQA_HIP(hipMemcpy(v_selected_host, c->ad.vsel, (size_t)rows * MAX_K_LIMIT * 4, hipMemcpyDeviceToHost));
  if (contrib_host && nb > 0)
    CQA_HIP(hipMemcpy(contrib_host, c->ad.contrib, (size_t)(rows * nb) * 4, hipMemcpyDeviceToHost));
  if (promoted_host && nb > 0) {
    std::vector<int32_t> slot((size_t)nb);
    for (int64_t gidx = 0; gidx < groups; ++gidx) {
      CQA_HIP(hipMemcpy(slot.data(), c->ad.slot + gidx * c->nq_cap * 4, (size_t)nb * 4,
                        hipMemcpyDeviceToHost));
      for (int64_t i = 0; i < nb; ++i) {
        const uint32_t f = (uint32_t)slot[(size_t)i];
        promoted_host[gidx * nb + i] =
            (uint16_t)((f & 3u) | (((f >> SLOT_HK_SHIFT) & 15u) << 4) | (((f >> SLOT_HV_SHIFT) & 15u) << 8));
      }
    }
  }
  return CQA_OK;
}

int64_t cqa_dense_workspace_bytes(int32_t batch, int32_t n_q_heads, int64_t n_tokens) {
  (void)batch;
  (void)n_q_heads;
  if (n_tokens < 1) return 0;
  return dense_ws_floats(4, n_tokens) * 4;
}

int32_t cqa_dense_attention(const void* q_fp16_dev, const void* k_fp16_dev,
                            const void* v_fp16_dev, int32_t batch, int32_t n_q_heads,
                            int32_t n_kv_heads, int64_t n_tokens, float* O_dev,
                            void* workspace_dev, void* stream) {
  if (q_fp16_dev == nullptr || k_fp16_dev == nullptr || v_fp16_dev == nullptr ||
      O_dev == nullptr || workspace_dev == nullptr || batch < 1 || n_q_heads < 1 ||
      n_kv_heads < 1 || n_tokens < 1 || n_q_heads % n_kv_heads != 0)
    return CQA_ERR_INVALID_ARG;
  const int g = n_q_heads / n_kv_heads;
  if (g != 1 && g != 2 && g != 4) return CQA_ERR_UNSUPPORTED;
  const __half* q = (const __half*)q_fp16_dev;
  const __half* k = (const __half*)k_fp16_dev;
  const __half* v = (const __half*)v_fp16_dev;
  for (int b = 0; b < batch; ++b)
    for (int kh = 0; kh < n_kv_heads; ++kh) {
      const int64_t row = (int64_t)b * n_q_heads + kh * g;
      const int64_t kv = ((int64_t)b * n_kv_heads + kh) * n_tokens * D;
      const int32_t rc =
          launch_dense_group(q + row * D, k + kv, v + kv, g, n_tokens, O_dev + row * D, nullptr,
                             nullptr, nullptr, 0, (float*)workspace_dev, (hipStream_t)stream);
      if (rc != CQA_OK) return rc;
    }
  return CQA_OK;
}

}  // extern "C"
