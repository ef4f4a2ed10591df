/*
 * cqa -- certified quantized decode attention for AMD MI355X (gfx950).
 *
 * C ABI of the library.  Everything here is plain C: opaque handle, plain
 * pointers and sizes.  "dev" pointers are HIP device memory, "host" pointers are
 * ordinary host memory; streams are hipStream_t passed as void* (NULL = the
 * default stream).  Every call returns a status (CQA_OK = 0, negative = error);
 * no C++ exception crosses this boundary.  The library never returns an
 * uncertified output silently: when a fallback is required and the FP16
 * originals or the staging buffer are unavailable, the call fails with
 * CQA_ERR_NO_TIER2 / CQA_ERR_OOM_* and leaves the outputs of the affected heads
 * untouched (the paper's precondition P4 and its contract).
 *
 * Fixed geometry (the paper's defaults): head_dim d = 128, block B = 16 tokens,
 * value group g = 16 channels.  Other values are rejected with
 * CQA_ERR_UNSUPPORTED.
 *
 * Ownership: the handle owns Tier-1 (packed INT8 keys / INT4 values and their
 * metadata, in HBM), Tier-2 (FP16 originals in pinned host memory), the trailing
 * FP16 partial blocks, the split workspace, the fallback staging buffer and one
 * side stream with its events.  The caller owns q, O, cert, flags, blk_logmass
 * and the main stream.  All kernels are enqueued on the caller's stream; only
 * the host-resolved steps (cqa_decode_step, cqa_append_decode_step,
 * cqa_adaptive_step), which read the flag words back, and the statistics getters
 * wait for the device (as do the test hooks of cqa_test.h); cqa_decode_step_enqueue and
 * cqa_adaptive_step_enqueue never do.
 *
 * Concurrency: the decode calls of one handle share its workspaces (split
 * partials, fallback partials and arrival counters, selector state), whatever
 * the layer.  Calls on one handle must therefore be ordered -- issue them on one
 * stream, or order the streams with events; two handles are independent.
 */
#ifndef CQA_H
#define CQA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CQA_VERSION 100

enum {
  CQA_OK = 0,
  CQA_ERR_INVALID_ARG = -1,
  CQA_ERR_OOM_DEVICE = -2,
  CQA_ERR_OOM_PINNED = -3,
  CQA_ERR_NO_TIER2 = -4,
  CQA_ERR_CAPACITY = -5,
  CQA_ERR_HIP = -6,
  CQA_ERR_UNSUPPORTED = -7,
  CQA_ERR_SCRATCH = -8   /* the shape needs more than the fixed scratch of a no-allocation call */
};

/* Where the FP16 originals live (the paper's Tier 2). */
enum {
  CQA_TIER2_PINNED = 0, /* library-owned pinned host memory (hipHostMalloc)      */
  CQA_TIER2_NONE = 1    /* not retained: any call that needs a fallback fails   */
};

/* Flag word written per (batch, query head) by cqa_certified_decode.
 * Bits 0-4 request more precision; bits 8-10 record the rung that served the
 * head (0 = fast path, 3 = per-head dense recompute, 4 = whole-layer recompute). */
#define CQA_FLAG_KEY 0x01u     /* E_key > eps_key                                */
#define CQA_FLAG_VAL 0x02u     /* E_val > eps_val or max_b rho_b eta_b > v_tol   */
#define CQA_FLAG_RANK 0x04u    /* top-1 block not certified by the interval test */
#define CQA_FLAG_PRECOND 0x08u /* a non-finite certificate quantity              */
#define CQA_FLAG_TOTAL 0x10u   /* E_key + E_val > eps_total                      */
#define CQA_FLAG_ANY 0x1Fu
#define CQA_RUNG_SHIFT 8

typedef struct cqa_cache cqa_cache;

typedef struct cqa_cache_desc {
  int32_t n_layers;
  int32_t batch;        /* Bt sequences, all of the same length                 */
  int32_t n_q_heads;    /* Hq, a multiple of n_kv_heads; Hq / Hkv in {1,2,4}     */
  int32_t n_kv_heads;   /* Hkv                                                  */
  int32_t head_dim;     /* must be 128                                          */
  int32_t block_tokens; /* must be 16                                           */
  int32_t v_group;      /* must be 16                                           */
  int32_t tier2_mode;   /* CQA_TIER2_*                                          */
  int64_t max_tokens;   /* capacity per sequence                                */
} cqa_cache_desc;

/* Thresholds of the runtime certificate policy (the paper's policy table).
 * +inf disables a threshold; comparisons are strict (>). */
typedef struct cqa_tolerances {
  float eps_total;          /* on E_key + E_val                                  */
  float eps_key;            /* on E_key                                          */
  float eps_val;            /* on E_val                                          */
  float v_tol;              /* on max_b rho_b eta_b (per-block value test)       */
  float rank_min_mass;      /* ranking test only if the top block holds >= this  */
  float eps_guard;          /* additive slack of the ranking test                */
  int32_t rank_depth;       /* r: 0 = ranking test off, 1 = top-1 block (the      */
                            /* paper's default); the adaptive calls take r <= 8,  */
                            /* the one-pass calls r <= 1 (else UNSUPPORTED)       */
  int32_t mass_exp;         /* c in e^{c Delta}: 2 (theorems) or 3 (paper impl.)  */
  int32_t key_bound_mode;   /* 0 min(tanh, tail), 1 tail form only, 2 tanh only  */
  int32_t rung4_min_groups; /* >0: that many flagged KV groups => Rung 4         */
  uint32_t force_flags;     /* OR-ed into every head's flag word (test hook)     */
  int32_t int8_query;       /* 1: INT8 x INT8 scoring (the paper's optional tensor-core scoring
                               mode): per sealed block the scaled query q~ = q . sigma is
                               quantised to 8 bits, one scale s_q = max_c |q~_c| / 127 per
                               (head, block), T_c = round(q~_c / s_q), and scored against the
                               stored key codes on the INT8 matrix cores.  The paper budgets
                               "one more Delta" for this third error source (mass_exp = 3);
                               here the block's score bound also gets the explicit term
                               (128 / sqrt d) sum_c |q~_c - s_q T_c|, so delta_h, E_key and the
                               ranking test stay valid with mass_exp = 2.  In the adaptive
                               calls the pass over all blocks scores this way, blocks left in
                               INT8 keep those scores and promoted blocks are scored exactly
                               from their FP16 keys.  (The vector-ALU cross-check kernel, a
                               test hook, returns CQA_ERR_UNSUPPORTED.)  0: the scaled query
                               is used unquantised (default).                            */
} cqa_tolerances;

/* Per-(batch, query head) certificate of one decode step.  40 bytes. */
typedef struct cqa_head_cert {
  float E_key;             /* 2 V_max * TV bound (key-quantization term)         */
  float E_val;             /* sum_b rho_b eta_b (value-reconstruction term)      */
  float delta_h;           /* max_b Delta_b over sealed blocks                   */
  float v_max;             /* max value norm over all attended tokens            */
  float alpha_tail_hat;    /* INT8-estimated mass on INT8-keyed tokens           */
  float lse;               /* log sum_t exp(s'_t)                                */
  float max_block_contrib; /* max_b rho_b eta_b                                  */
  float rank_margin;       /* l_(1) - l_(2) of the block log-masses (+inf if <2) */
  int32_t top_block;       /* argmax_b l_b (-1 if no sealed block)               */
  int32_t served_rung;     /* 0, 3 or 4                                          */
} cqa_head_cert;

/* ---- cache lifetime ------------------------------------------------------ */

/* As cqa_cache_create with tier2_mode = CQA_TIER2_PINNED, but the FP16 originals
 * live in two pinned host arrays the CALLER provides and keeps alive until the
 * cache is destroyed (e.g. one pinned pool shared with the rest of a serving
 * stack): t2_k_host, t2_v_host, each of at least bytes_each >= n_layers * batch *
 * n_kv_heads * max_tokens * 256 bytes, laid out [layer][batch][kv_head][max_tokens]
 * [128] FP16.  They must be pinned host memory that the device can address
 * (hipHostMalloc or a framework's pinned allocation; checked with
 * hipPointerGetAttributes): the library's kernels read and write them in place.
 * The library never frees them and writes to them only what it appends (with its
 * own arrays it also gives every page a first copy-engine access at creation;
 * arrays that no copy has touched yet make the first bulk append slower).
 * Errors: INVALID_ARG (null, too small, not pinned
 * host memory, wrong tier2_mode), otherwise as cqa_cache_create. */
int32_t cqa_cache_create_caller_tier2(const cqa_cache_desc* desc, void* t2_k_host, void* t2_v_host,
                                      int64_t bytes_each, cqa_cache** out);

/* Allocates every buffer up front on the current HIP device (the paper's
 * "allocated at load, never released"): Tier-1, Tier-2 (unless NONE), trailing
 * blocks, split workspace, staging for one layer.  *out is set only on success.
 * Errors: INVALID_ARG, UNSUPPORTED (geometry), OOM_DEVICE, OOM_PINNED, HIP. */
int32_t cqa_cache_create(const cqa_cache_desc* desc, cqa_cache** out);
int32_t cqa_cache_destroy(cqa_cache* c);

/* Bytes a cache of this shape allocates on a 256-compute-unit device:
 * *device_bytes in HBM -- every buffer of the create call plus, with Tier 2, what
 * the first cqa_set_scratch_slots(n > 0) adds at its largest -- and *pinned_bytes
 * in pinned host memory (library-owned Tier 2 and the flag mirror).  Not counted:
 * the library's fixed 4 MiB scratch of the no-allocation decode, which every
 * device holds once per process.  Either pointer may be NULL. */
int32_t cqa_workspace_bytes(const cqa_cache_desc* desc, int64_t* device_bytes,
                            int64_t* pinned_bytes);

/* ---- cache write: the paper's quantize-at-block-fill path ---------------- */

/* Appends n_new tokens to every (batch, kv-head) sequence of `layer`.
 * k_fp16_dev, v_fp16_dev: device, FP16, layout [batch][n_kv_heads][n_new][128]
 * (post-RoPE keys).  New tokens join the trailing FP16 partial block; every
 * block that reaches 16 tokens is sealed: per-channel INT8 keys with FP32
 * (sigma, z) per block, per-token per-16-channel-group INT4 values with FP16
 * (scale, offset), and the block annotations eta_b, nu_b.  Sealed blocks are
 * immutable.  The FP16 originals are copied to Tier-2 (pinned host) on the same
 * stream unless tier2_mode is NONE.  Asynchronous on `stream`; the inputs must
 * stay valid until the stream has passed this call.
 * Errors: INVALID_ARG, CAPACITY (length + n_new > max_tokens), HIP. */
int32_t cqa_cache_append(cqa_cache* c, int32_t layer, const void* k_fp16_dev,
                         const void* v_fp16_dev, int64_t n_new, void* stream);

/* Tokens currently held per sequence of `layer` (host-side counter). */
int32_t cqa_cache_length(const cqa_cache* c, int32_t layer, int64_t* n_tokens);

/* Drops every token of `layer` (host counter only; buffers are reused). */
int32_t cqa_cache_reset(cqa_cache* c, int32_t layer);

/* Canonical logical view of one sealed block, independent of the physical
 * packing, written to HOST buffers (synchronises the device):
 *   kcodes[16*128] int8 [token][channel]; sigma[128], z[128] float;
 *   vcodes[16*128] uint8 in 0..15 [token][channel];
 *   vscale_bits[16*8], voffset_bits[16*8] raw FP16 bits [token][group];
 *   *eta, *nu the block annotations.
 * Errors: INVALID_ARG (indices out of range or block not sealed), HIP. */
int32_t cqa_cache_export_block(const cqa_cache* c, int32_t layer, int32_t batch,
                               int32_t kv_head, int64_t block, int8_t* kcodes, float* sigma,
                               float* z, uint8_t* vcodes, uint16_t* vscale_bits,
                               uint16_t* voffset_bits, float* eta, float* nu);

/* ---- decode: the paper's fused certified attention + certificate --------- */

/* One decode step of `layer` on the quantized cache, for all (batch, q-head):
 * split-K pass over Tier-1 (scaled-query scoring identity, block statistics
 * m_b, S_b, l_b, FP32 online softmax, in-register INT8/INT4 dequantization,
 * both bound terms accumulated in the same pass; the trailing FP16 tokens are
 * attended exactly) followed by the cross-split reduction that finalises
 *   O_dev     float [batch][n_q_heads][128]      (O_quant for EVERY head),
 *   cert_dev  cqa_head_cert [batch][n_q_heads]   (served_rung = 0),
 *   flags_dev uint32 [batch][n_q_heads]          (bits 0-4 only),
 *   blk_logmass_dev float [batch][n_q_heads][n_sealed_blocks], may be NULL.
 * q_fp16_dev: device FP16 [batch][n_q_heads][128].  tol: host pointer, copied.
 * Flags only REQUEST a fallback; see cqa_dense_fallback / cqa_decode_step.
 * Asynchronous on `stream`.  Calls on the same handle must not overlap (they
 * share the split workspace).  Errors: INVALID_ARG (incl. an empty cache), HIP. */
int32_t cqa_certified_decode(cqa_cache* c, int32_t layer, const void* q_fp16_dev,
                             const cqa_tolerances* tol, float* O_dev, cqa_head_cert* cert_dev,
                             uint32_t* flags_dev, float* blk_logmass_dev, void* stream);

/* cqa_certified_decode for callers that cannot allocate device memory or have it
 * allocated on their behalf: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same kernels, same results and the same
 * arguments (without the optional log-mass output); the only difference is where
 * the per-split partial results live between the split pass and the reduction:
 * not in the cache's workspace but in a fixed array of CQA_STATIC_SCRATCH_BYTES
 * that is part of the library's device image (each GPU the library runs on holds
 * its own copy from load until the process ends; its address on the cache's GPU
 * is resolved when the cache is created).  The call itself allocates nothing and
 * calls no allocating routine; inputs and outputs are the caller's as before.
 * Limit: batch * n_q_heads * splits * 576 bytes must fit the array, where splits
 * is what cqa_decode_splits reports: about compute units / (batch * n_kv_heads),
 * and 1 once there are more sequences than compute units, so a shape fits up to
 * batch * n_q_heads = 7281 rows (unless a test hook forces more splits); beyond
 * it the call fails with CQA_ERR_SCRATCH and touches nothing.  Every such call on one GPU uses that
 * GPU's one array, whatever the cache: calls that overlap on a GPU (two streams,
 * two caches) race and must be ordered by the caller.  The array keeps the last
 * call's contents; every word a call reads it has written first, so nothing needs
 * clearing.  The current device must be the cache's.
 * Errors: as cqa_certified_decode, plus CQA_ERR_SCRATCH. */
#define CQA_STATIC_SCRATCH_BYTES (4 * 1024 * 1024)
int32_t cqa_certified_decode_noalloc(cqa_cache* c, int32_t layer, const void* q_fp16_dev,
                                     const cqa_tolerances* tol, float* O_dev,
                                     cqa_head_cert* cert_dev, uint32_t* flags_dev, void* stream);

/* The paper's Rung 3 / Rung 4 body: recomputes dense FP16 attention (FP32
 * accumulation) from the Tier-2 originals for the selected heads and overwrites
 * their rows of O_dev; their certificates become E_key = E_val = 0 with
 * served_rung = rung, and bits 8-10 of their flag words are set to `rung`.
 * head_select_host: uint32 [batch][n_q_heads] on the HOST, nonzero = recompute;
 * ignored (may be NULL) if all_heads != 0.  Originals are paged per (batch,
 * kv-head) with pinned hipMemcpyAsync on the library's side stream into the
 * staging buffer, double-buffered against the dense kernel, which runs on
 * `stream` after an event join.  cert_dev / flags_dev may be NULL.
 * Errors: NO_TIER2 (tier2_mode NONE; outputs untouched), INVALID_ARG, HIP. */
int32_t cqa_dense_fallback(cqa_cache* c, int32_t layer, const void* q_fp16_dev,
                           const uint32_t* head_select_host, int32_t all_heads, int32_t rung,
                           float* O_dev, cqa_head_cert* cert_dev, uint32_t* flags_dev,
                           void* stream);

/* certified_decode, then the ladder: reads the flag words back (one D2H copy
 * and a stream synchronise), serves flagged heads by Rung 3, or the whole layer
 * by Rung 4 when any head has PRECOND set or when rung4_min_groups > 0 and at
 * least that many (batch, kv-head) groups hold a flagged head.  On return O_dev
 * is final.  *rung_served (host, may be NULL) receives 0, 3 or 4.
 * Errors: as the two calls above. */
int32_t cqa_decode_step(cqa_cache* c, int32_t layer, const void* q_fp16_dev,
                        const cqa_tolerances* tol, float* O_dev, cqa_head_cert* cert_dev,
                        uint32_t* flags_dev, float* blk_logmass_dev, int32_t* rung_served,
                        void* stream);

/* cqa_cache_append of ONE token per sequence followed by cqa_decode_step, as a
 * single call (the decode-time pattern: the paper's trailing partial block takes
 * the new token, then the step attends it).  k_fp16_dev, v_fp16_dev: device FP16
 * [batch][n_kv_heads][1][128].  When the token does not complete a block, its
 * stores ride on the decode launch itself (one launch fewer per step); results
 * are identical to the two calls.  Errors as the two calls. */
int32_t cqa_append_decode_step(cqa_cache* c, int32_t layer, const void* k_fp16_dev,
                               const void* v_fp16_dev, const void* q_fp16_dev,
                               const cqa_tolerances* tol, float* O_dev, cqa_head_cert* cert_dev,
                               uint32_t* flags_dev, int32_t* rung_served, void* stream);

/* The decode step as enqueue-only work: the same split pass and reduction as
 * cqa_decode_step, followed by the paper's fallback ladder ("Fallback Ladder":
 * Rung 3 = dense FP16 result for the flagged heads' KV groups, Rung 4 = for every
 * head when a PRECOND flag is raised or at least tol->rung4_min_groups (> 0) groups
 * are flagged) resolved ON THE DEVICE: a kernel launched behind the reduction reads
 * the step's flag words, leaves at once when none is raised, and otherwise attends
 * the FP16 originals straight from the pinned Tier-2 arrays and rewrites O, the
 * certificate (E_key = E_val = 0, served_rung) and the rung bits of the served heads.
 * The call never waits for the GPU and reads nothing back: results are in O_dev,
 * cert_dev, flags_dev once `stream` has passed the enqueued work.
 * k_fp16_dev / v_fp16_dev: device FP16 [batch][n_kv_heads][1][128], the token to
 * append first (as cqa_append_decode_step), or both NULL for no append.
 * Needs the Tier-2 originals (CQA_ERR_NO_TIER2 otherwise); CQA_ERR_CAPACITY when
 * the token does not fit; CQA_ERR_INVALID_ARG for an empty cache or null pointers. */
int32_t cqa_decode_step_enqueue(cqa_cache* c, int32_t layer, const void* k_fp16_dev,
                                const void* v_fp16_dev, const void* q_fp16_dev,
                                const cqa_tolerances* tol, float* O_dev, cqa_head_cert* cert_dev,
                                uint32_t* flags_dev, void* stream);

/* How many cqa_decode_step_enqueue steps of this cache were served by Rung 3 and by
 * Rung 4 so far (device counters; the call waits for the device).  Host pointers, may be NULL. */
int32_t cqa_ladder_counts(cqa_cache* c, int64_t* rung3_steps, int64_t* rung4_steps);

/* ---- adaptive key precision: the paper's "Adaptive Precision Selection",
 *      first rung of its "Fallback Ladder", the total error bound with the
 *      achieved tail mass, and its "Ranking-Consistency Check" ---------------- */

/* Parameters of the selector (the paper's policy table: tau_cov, K_min, K_max). */
typedef struct cqa_selector {
  float tau_cov;   /* coverage threshold on INT8-estimated mass (paper: 0.995)       */
  int32_t k_min;   /* K* is clamped to [k_min, k_max] and to the sealed blocks       */
  int32_t k_max;   /* 0 <= k_min <= k_max <= k_limit <= 512                          */
  int32_t k_limit; /* cap of the Rung-1 doubling                                     */
  int32_t v_limit; /* blocks one head may promote to FP16 VALUES (Rung 2); 0 = off,  */
                   /* at most 512                                                    */
  int32_t v_greedy;/* 0: promote blocks whose estimated contribution p_b eta_b       */
                   /* exceeds tol->v_tol; 1: also keep promoting, largest first,     */
                   /* until the estimated value term left is <= tol->eps_val         */
  int32_t canary;  /* 1: score-consistency check on key-promoted blocks: a head with */
                   /* |s_fp16 - s_int8| > Delta_h + eps_guard on any token gets       */
                   /* PRECOND (the paper's "Instability Detection")                  */
  float explore_frac;    /* exploration budget: this fraction of the blocks (paper:  */
                         /* 0.01-0.05) is key-promoted on top of the selection, so    */
                         /* the check also sees blocks the selector never picks      */
  uint32_t explore_seed; /* counter of the draw, e.g. the decode step: a block is    */
                         /* explored when mix32(block * 0x9E3779B1 ^ group *          */
                         /* 0x85EBCA77 ^ seed * 0xC2B2AE3D) < explore_frac * 2^32,    */
                         /* mix32 = the multiply-xorshift mixer with constants       */
                         /* 0x7FEB352D, 0x846CA68B; group = batch * n_kv_heads + kvh  */
  int32_t per_head;      /* 0: precision is chosen per KV group -- a block is promoted for all  */
                         /* heads of the group when any of them selects it (the paper's       */
                         /* per-KV-group selection variant; one set of FP16 scores serves the  */
                         /* group and every head's tail only shrinks).  1: the paper's         */
                         /* default -- each head's promoted set F is its own selection (plus   */
                         /* the explored blocks), for keys and for values; its achieved tail   */
                         /* and its ranking check run over its own F.  The FP16 originals of a */
                         /* block are still read once per group when any head asks for them.   */
} cqa_selector;

/* One decode step of `layer` with mask-gated key precision, all on `stream`:
 *  1. the certified pass over all sealed blocks (INT8 keys, INT4 values): the
 *     INT8 block log-masses l_b, the total log-mass, Delta_h and V_max of every
 *     head, and the partial results that step 4 corrects;
 *  2. selection per head: blocks ranked by l_b (ties: lower index), K* = the
 *     smallest k whose blocks, with the exact trailing tokens, hold >= tau_cov
 *     of the estimated mass, clamped; Rung 1: K doubles (up to k_limit) while
 *     the key term of the achieved tail exceeds tol->eps_key;
 *  3. the promoted set of a (batch, kv-head) group is the union of its heads'
 *     selections (sel->per_head = 0) or every head keeps its own (sel->per_head
 *     = 1); value promotion (the ladder's second rung, sel->v_limit > 0) is
 *     decided the same way from the estimated contributions p_b eta_b and
 *     follows the same switch;
 *  4. the result is that of cqa_certified_decode with the promoted blocks
 *     scored from their FP16 keys, which the device reads straight from the
 *     pinned Tier-2 originals (no host step, no staging); values are INT4 except
 *     in value-promoted blocks, which are attended from their FP16 originals
 *     and count with eta_b = 0.  It is formed without a second pass over
 *     Tier-1: a small pass revisits the promoted blocks only, adds them with
 *     their originals and takes their step-1 contribution back out.  E_val uses
 *     the masses of the corrected result; E_key uses alpha_hat_T = step 1's
 *     estimated mass of the blocks the group left in INT8, and step 1's Delta_h;
 *  5. ranking check at depth r = tol->rank_depth (1..8; 0 = off): RANK is set
 *     when the r promoted blocks with the largest FP16 log-masses are not, in the
 *     same order, the r with the largest INT8 log-masses (larger first, equal
 *     ones by lower index; fewer than r promoted blocks: r = their number), or
 *     when an unpromoted block has l_b + Delta_h + eps_guard > the r-th largest
 *     FP16 log-mass (gated by tol->rank_min_mass on the top block's mass).
 * Outputs as cqa_certified_decode; cert.alpha_tail_hat is the achieved tail,
 * cert.top_block the promoted block with the largest FP16 log-mass,
 * cert.rank_margin = the r-th largest FP16 log-mass - (largest unpromoted l_b + Delta_h).
 * Flags only REQUEST a fallback (Rung 3 / 4), as in cqa_certified_decode.
 * Needs the Tier-2 originals.  Asynchronous; shares the handle's workspaces.
 * Errors: INVALID_ARG (incl. selector out of range), NO_TIER2, HIP. */
int32_t cqa_adaptive_decode(cqa_cache* c, int32_t layer, const void* q_fp16_dev,
                            const cqa_tolerances* tol, const cqa_selector* sel, float* O_dev,
                            cqa_head_cert* cert_dev, uint32_t* flags_dev, void* stream);

/* cqa_adaptive_decode, then the ladder exactly as in cqa_decode_step. */
int32_t cqa_adaptive_step(cqa_cache* c, int32_t layer, const void* q_fp16_dev,
                          const cqa_tolerances* tol, const cqa_selector* sel, float* O_dev,
                          cqa_head_cert* cert_dev, uint32_t* flags_dev, int32_t* rung_served,
                          void* stream);

/* cqa_adaptive_step as enqueue-only work: the adaptive decode followed by the
 * device-resolved fallback ladder of cqa_decode_step_enqueue (same rules, same
 * outputs); never waits for the GPU. */
int32_t cqa_adaptive_step_enqueue(cqa_cache* c, int32_t layer, const void* q_fp16_dev,
                                  const cqa_tolerances* tol, const cqa_selector* sel, float* O_dev,
                                  cqa_head_cert* cert_dev, uint32_t* flags_dev, void* stream);

/* FP16 scratch (the paper's VRAM scratch cache of promoted originals, LRU); off
 * unless switched on here.  Per (layer, batch, kv-head) it keeps up to n_slots
 * promoted blocks on the device (at most min(1024, capacity in blocks rounded up
 * to a power of two)); a slot has a key half and a value half of 4 KB each, and
 * a half is filled the first time a step needs it.  An adaptive decode then reads
 * a promoted block's FP16 keys / values from there when the slot holds them, else
 * from the pinned originals over the host link, and keeps them in the least
 * recently used slot that the step does not use.  Results do not depend on it (the
 * same FP16 bits either way).  On this hardware the kernel's direct reads of pinned
 * host memory are as fast for the few dozen blocks a step promotes, which is why it
 * is off by default.
 * cqa_set_scratch_slots: 0 = off; the first non-zero call allocates; every call
 * empties the scratch and waits for the device.
 * cqa_scratch_stats: slots per head in use and, since the cache was created, how many
 * promoted blocks found every original they needed in the scratch / did not; waits
 * for the device.
 * Host pointers, may be NULL.  Errors: INVALID_ARG (n_slots out of range), NO_TIER2,
 * OOM_DEVICE, HIP. */
int32_t cqa_set_scratch_slots(cqa_cache* c, int32_t n_slots);
int32_t cqa_scratch_stats(cqa_cache* c, int32_t* slots_per_head, int64_t* hits, int64_t* misses);

/* Dense FP16 decode attention on device-resident K, V (the same kernel the
 * fallback runs after paging): softmax(q K^T / sqrt(128)) V with FP32
 * accumulation.  q [batch][n_q_heads][128] FP16; k, v [batch][n_kv_heads]
 * [n_tokens][128] FP16; O float [batch][n_q_heads][128].  `workspace_dev` must
 * hold cqa_dense_workspace_bytes(batch, n_q_heads, n_tokens) bytes.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP. */
int32_t cqa_dense_attention(const void* q_fp16_dev, const void* k_fp16_dev,
                            const void* v_fp16_dev, int32_t batch, int32_t n_q_heads,
                            int32_t n_kv_heads, int64_t n_tokens, float* O_dev,
                            void* workspace_dev, void* stream);
int64_t cqa_dense_workspace_bytes(int32_t batch, int32_t n_q_heads, int64_t n_tokens);

/* ---- misc ------------------------------------------------------------------ */

/* Split count the decode pass uses for the current length of `layer`
 * (for reporting and for sizing the no-allocation call; chosen from the device's
 * compute-unit count). */
int32_t cqa_decode_splits(const cqa_cache* c, int32_t layer, int32_t* n_splits);

const char* cqa_strerror(int32_t status);
int32_t cqa_version(void);
/* hipError_t of the last failing HIP call on this thread (0 if none). */
int32_t cqa_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CQA_H */
