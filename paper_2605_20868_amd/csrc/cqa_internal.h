// Internal declarations shared by the library's translation units (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "../../include/cqa.h"
#include "../../include/cqa_test.h"

namespace cqa {

// ---- fixed geometry (the paper's defaults: d = 128, B = 16, g = 16) ------------
constexpr int D = 128;          // head dimension
constexpr int BLK = 16;         // tokens per block
constexpr int VG = 16;          // value channels per group
constexpr int NG = D / VG;      // 8 value groups per token

// ---- physical Tier-1 layout, per sealed block ---------------------------------
// Five block-major streams per (layer, batch, kv-head); block b of a head lives at
// offset b * <bytes per block> in each stream, so one split of the decode pass
// reads five contiguous byte ranges.
//
// K codes (2048 B): biased bytes u = code + 128, ordered [cq][kg][token][j] with
//   channel = cq*64 + kg*16 + j  (cq in 0..1, kg in 0..3, j in 0..15), so a wave's
//   lane l = kg*16 + token reads one aligned 16-byte piece and the whole wave reads
//   1 KB contiguously per cq.
// K meta (1024 B): sigma[128] then z[128], FP32, natural channel order.
// V codes (1024 B): dwords ordered [o][gh][n][gq]; the dword of (o, g = gh*4+gq, n)
//   holds channel g*16+n of the eight tokens o*8 .. o*8+7, token i in bits 4i..4i+3.
// V meta (512 B): FP16 scale[o][g][i] (256 B) then FP16 offset[o][g][i] (256 B),
//   token = o*8 + i.
// Annotations (8 B): float eta_b, float nu_b.
constexpr int KC_BYTES = BLK * D;            // 2048
constexpr int KM_BYTES = 2 * D * 4;          // 1024
constexpr int VC_BYTES = BLK * D / 2;        // 1024
constexpr int VM_BYTES = 2 * BLK * NG * 2;   // 512
constexpr int AN_BYTES = 8;

// The five per-block pieces of four consecutive blocks (a "quad") are stored together as one
// contiguous record, piece-major inside the record:
//   [K codes 4 x 2048][K meta 4 x 1024][V codes 4 x 1024][V meta 4 x 512][annotations 4 x 8]
// so that a wave, which works on one quad at a time, streams a single 18464-byte run instead of
// five separate arrays (measured: 7.1 TB/s against 6.5 TB/s for the same bytes in five arrays).
// Blocks that are not sealed (yet) always read as zeros: the memory is cleared at creation and at reset.
constexpr int Q_KC = 0;
constexpr int Q_KM = Q_KC + 4 * KC_BYTES;   //  8192
constexpr int Q_VC = Q_KM + 4 * KM_BYTES;   // 12288
constexpr int Q_VM = Q_VC + 4 * VC_BYTES;   // 16384
constexpr int Q_AN = Q_VM + 4 * VM_BYTES;   // 18432
constexpr int QUAD_DATA_BYTES = Q_AN + 4 * AN_BYTES;            // 18464 = 64 tokens x 288.5 B
// records start on 128-byte lines (96 bytes of padding, 0.5 %): every 1 KB wave load then covers
// exactly 8 lines and no line is shared between two records
constexpr int QUAD_BYTES = (QUAD_DATA_BYTES + 127) / 128 * 128;    // 18560

// address of one piece of block `blk` of head-local numbering; `head_rec` = first record of the head
__host__ __device__ inline int64_t t1_offset(int64_t head_rec, int64_t blk, int piece_off,
                                             int piece_bytes) {
  return (head_rec + (blk >> 2)) * QUAD_BYTES + piece_off + (blk & 3) * piece_bytes;
}

__host__ __device__ inline int kc_offset(int token, int channel) {
  const int cq = channel >> 6, kg = (channel >> 4) & 3, j = channel & 15;
  return cq * 1024 + kg * 256 + token * 16 + j;
}
// byte offset of the dword holding (token octet o, channel c); nibble index = token & 7
__host__ __device__ inline int vc_dword_offset(int o, int channel) {
  const int g = channel >> 4, n = channel & 15;
  return o * 512 + (g >> 2) * 256 + n * 16 + (g & 3) * 4;
}
// index (in halves) of the scale of (token, group) inside the V-meta block; offsets follow at +128
__host__ __device__ inline int vm_index(int token, int g) {
  return (token >> 3) * 64 + g * 8 + (token & 7);
}

// ---- split partial written by the decode pass, merged by the reduction ---------
// Per (batch, q-head, split): PART_FLOATS floats.
constexpr int P_M = 0;      // running max of the split
constexpr int P_L = 1;      // sum of exp(s - m)
constexpr int P_EV = 2;     // sum_b S_b e^{m_b - m} eta_b
constexpr int P_EVMAX = 3;  // max_b S_b e^{m_b - m} eta_b
constexpr int P_DMAX = 4;   // max_b Delta_b
constexpr int P_VMAX = 5;   // max_b nu_b
constexpr int P_T1 = 6;     // largest block log-mass
constexpr int P_T2 = 7;     // second largest
constexpr int P_I1 = 8;     // block index of the largest (int bits)
constexpr int P_O = 16;     // o[128]
constexpr int PART_FLOATS = 16 + D;  // 144
constexpr int MAX_SPLITS = 1024;     // upper bound on splits per (batch, kv-head)

// ---- adaptive key precision ------------------------------------------------------
constexpr int MAX_K_LIMIT = 512;            // blocks one head may promote (Rung-1 growth included)
constexpr int MAX_UNION = 8 * MAX_K_LIMIT;  // blocks one KV group may promote (keys and values, <= 4 heads each)
constexpr int PROM_SPLITS = 16;             // workgroups (= partial sets) per KV group of each half of the promoted-block
                                            // pass: 64 waves, about two blocks per wave for a group that promotes K_max = 128.
                                            // With the 32 sets of the pass over all blocks the adaptive reduction then merges
                                            // 64 sets, one trip of its head wave (measured: 32 per half, two trips, 3.6 us slower;
                                            // 8 per half, 3.5 us slower: too few waves for the large unions)

// Workspace of the adaptive path, shared by all layers (one decode step at a time).
struct AdaptiveWs {
  float* lm8;        // [Bt][Hq][nb_cap]      INT8 block log-masses of the pass over all blocks
  float* lmx;        // [Bt][Hq][nb_cap]      log-masses of the listed blocks as the promoted-block pass computed them (FP16 keys where promoted)
  int32_t* sel;      // [Bt][Hq][MAX_K_LIMIT] the head's own selection, best first
  int32_t* kstar;    // [Bt][Hq]              its size after Rung-1 growth
  float* alpha;      // [Bt][Hq]              estimated mass of the blocks its group left in INT8
  uint32_t* umask;   // [Bt][Hq][mask_words]  the head's key selection, one bit per block
  uint32_t* vmask;   // [Bt][Hq][mask_words]  its value selection
  int32_t* slot;     // [Bt][Hkv][4 nq_cap]   per block: bit 0 = FP16 keys, bit 1 = FP16 values (0 = neither), per-head bits above
  float* eta_blk;    // [Bt][Hkv][nb_cap]     eta_b as read by the pass over all blocks
  float* contrib;    // [Bt][Hq][nb_cap]      estimated contributions p_b eta_b
  int32_t* vsel;     // [Bt][Hq][MAX_K_LIMIT] the head's value selection
  int32_t* vcount;   // [Bt][Hq]
  float* score_dev;  // [Bt][Hq]              canary: largest |s_fp16 - s_int8| on key-promoted tokens
  int32_t* ucount;   // [Bt][Hkv]             promoted blocks of the group
  int32_t* ulist;    // [Bt][Hkv][MAX_UNION]  their indices, ascending
  int64_t mask_words;
  // FP16 scratch (the paper's VRAM scratch cache of promoted originals, LRU): per (layer, batch,
  // kv-head) `sc_cap` slots of one block each, a key half and a value half.  sc_map: block ->
  // slot + 1 (0 = not held); sc_tag: slot -> block (-1 = empty); sc_age: slot -> step stamp of its
  // last use; sc_have: slot -> which halves hold the block's data (SLOT_KEYS | SLOT_VALUES).
  __half* sc_k;      // [heads_total][sc_cap][16][128]
  __half* sc_v;      // [heads_total][sc_cap][16][128]
  int32_t* sc_map;   // [heads_total][nb_cap]
  int32_t* sc_tag;   // [heads_total][sc_cap]
  uint32_t* sc_age;  // [heads_total][sc_cap]
  int32_t* sc_have;  // [heads_total][sc_cap]
  uint32_t* sc_stats;  // [2] promoted blocks whose originals were all in the scratch / were not, over all steps
  int sc_cap;        // allocated slots per head (a power of two <= SC_MAX_SLOTS)
  int sc_slots;      // slots in use (test hook may lower it; 0 = scratch off)
  uint32_t sc_step;  // stamp of the last adaptive step
};

constexpr int MAX_RANK_DEPTH = 8;   // largest depth r of the ranking check (adaptive path)
constexpr int SC_MAX_SLOTS = 1024;
// per-block word of AdaptiveWs::slot: bit 0 FP16 keys, bit 1 FP16 values, bit 2 / bit 3 the keys /
// the values are to be stored into the scratch slot by the pass that reads them from the host,
// bits 8-23 scratch slot + 1 (0 = none)
constexpr int SLOT_KEYS = 1, SLOT_VALUES = 2, SLOT_FILL = 4, SLOT_VFILL = 8, SLOT_SC_SHIFT = 8;
// bits 24-27: query head i of the group (i = 0..3) scores this block with FP16 keys; bits 28-31: it
// attends the block's FP16 values.  With per-group promotion every head's bit follows bits 0 / 1.
constexpr int SLOT_HK_SHIFT = 24, SLOT_HV_SHIFT = 28;

struct Cache {
  cqa_cache_desc desc;
  int device;
  int n_cu;
  int64_t nb_cap;            // blocks of capacity per head
  int64_t heads_total;       // n_layers * batch * n_kv_heads
  int64_t* length;           // host, per layer
  int forced_splits;
  int max_splits;
  // Tier-1: quad records, [heads_total][nq_cap][QUAD_BYTES]
  uint8_t* t1;
  int64_t nq_cap;            // quad records of capacity per head
  float* ladder_ws;          // device-resolved ladder: split partials, arrival counters, rung counters
  uint32_t* ladder_tickets;
  uint32_t* ladder_counts;
  float* sigmax;             // [heads_total] running max of sigma (non-negative: ordered as ints)
  // trailing FP16 partial blocks [heads_total][16][128]
  __half* trail_k;
  __half* trail_v;
  // Tier-2 (pinned host) [heads_total][max_tokens][128]
  __half* t2_k;
  __half* t2_v;
  bool t2_borrowed;           // the originals' arrays belong to the caller (not freed here)
  // workspaces
  float* partials;           // [batch][Hq][max_splits][PART_FLOATS]
  float* dense_ws;           // dense partials for one (batch, kv-head) group x 2 buffers
  __half* stage[2][2];       // [buffer][K|V] : max_tokens * 128 halves each
  uint32_t* select_dev;      // [batch][Hq]
  uint32_t* flags_host;      // pinned [batch][Hq]
  uint32_t step_seq;         // 16-bit tag of the decode step whose flags the mirror must carry
  uint32_t* need;            // host [batch][Hq]: ladder scratch, heads to recompute
  hipStream_t side;
  hipEvent_t ev_ready[2];    // staging buffer filled (recorded on side)
  hipEvent_t ev_free[2];     // staging buffer consumed (recorded on main)
  hipEvent_t ev_main;        // main-stream marker the side stream waits on
  hipEvent_t ev_copy;         // bulk append: the copies of the originals on the side stream are done
  hipEvent_t ev_t0, ev_t1;   // timing
  bool free_valid[2];
  // optional per-launch timing of the split kernel (pairs of events on the launch stream)
  hipEvent_t* prof_ev;
  int prof_cap, prof_n;
  float* prof_ms;            // host: durations of the launches timed by the last begin / end pair
  int prof_ms_n;
  int variant;               // 0 = matrix-core split kernel (default), 1 = vector-ALU split kernel
  int stream_hint;           // Tier-1 loads: 0 = chosen from the footprint, 1 = plain, 2 = non-temporal
  AdaptiveWs ad;             // allocated with the cache when Tier-2 is retained
};

struct DecodeArgs {
  const uint8_t* t1;   // layer base of the Tier-1 quad records
  const float* sigmax; // [Bt * Hkv] of the layer: running max of sigma over sealed blocks and channels
  const __half* q;     // [Bt][Hq][128]
  float* partials;     // [Bt][Hq][nsplit][PART_FLOATS]
  float* blk_logmass;  // [Bt][Hq][nb] or null
  int64_t nq_cap;      // quad records per head
  int nb;              // sealed blocks
  int nsplit;
  int bps;             // blocks per split
  int n_q, n_kv;
  int pstride;         // partial sets per (batch, q-head) row of `partials` (>= nsplit)
  int int8_query;      // matrix-core pass: 1 = INT8 x INT8 scoring of the quantised scaled query
  int wpb;             // matrix-core pass: waves per workgroup, 8 or 4 (waves_per_workgroup)
  // promoted-block pass of the adaptive decode (null slot = not that pass)
  const int32_t* slot;      // [Bt][Hkv][4 nq_cap]: bit 0 = FP16 keys, bit 1 = FP16 values, 0 = neither
  __half* sc_k;             // layer base of the FP16 scratch's key halves [Bt * Hkv][sc_cap][16][128], or null
  __half* sc_v;             // ... and of its value halves (null exactly when sc_k is)
  int sc_cap;
  const int32_t* ulist;     // [Bt][Hkv][MAX_UNION]: promoted blocks of the group, ascending
  const int32_t* ucount;    // [Bt][Hkv]
  const __half* t2_k;       // pinned FP16 key originals of the layer: [Bt * Hkv][max_tokens][128]
  const __half* t2_v;       // value originals, same layout
  int64_t max_tokens;
  int split0;               // promoted-block pass: index of its first partial set
  int stream_nt;            // 1 = Tier-1 loads carry the non-temporal hint (see stream_hint)
  float* eta_out;           // eta_b per (batch, kv-head, block) written alongside the log-masses, or null
  float* score_dev;         // promoted-block pass: canary output per (batch, q-head), or null
  // one-token append carried by the decode launch (null k_new = none): the new (k, v) of every
  // (batch, kv-head) goes to slot `ap_slot` of the trailing FP16 block and, unless ap_t2_k is
  // null, to position ap_pos of the pinned originals
  const __half* ap_k_new;   // [Bt][Hkv][1][128]
  const __half* ap_v_new;
  __half* ap_trail_k;       // layer base: [Bt * Hkv][16][128]
  __half* ap_trail_v;
  __half* ap_t2_k;          // layer base: [Bt * Hkv][max_tokens][128]
  __half* ap_t2_v;
  int ap_slot;
  int64_t ap_pos, ap_max_tokens;
};


inline int64_t head_index(const Cache* c, int layer, int b, int kvh) {
  return ((int64_t)layer * c->desc.batch + b) * c->desc.n_kv_heads + kvh;
}

extern thread_local int g_last_hip_error;
#define CQA_HIP(expr)                                   \
  do {                                                  \
    hipError_t e__ = (expr);                            \
    if (e__ != hipSuccess) {                            \
      cqa::g_last_hip_error = (int)e__;                 \
      return CQA_ERR_HIP;                               \
    }                                                   \
  } while (0)

// ---- launchers implemented in the kernel translation units ---------------------
int32_t launch_seal(Cache* c, int layer, const __half* k_in, const __half* v_in, int64_t n_new,
                    int64_t len_before, bool tier2_by_kernel, hipStream_t st);
int32_t launch_certified(Cache* c, int layer, const __half* q, const cqa_tolerances& tol, float* O,
                         cqa_head_cert* cert, uint32_t* flags, uint32_t* flags_mirror,
                         uint32_t mirror_tag, float* blk_logmass, hipStream_t st,
                         const __half* k_new = nullptr,
                         const __half* v_new = nullptr, int pstride = 0, float* eta_out = nullptr,
                         float* partials = nullptr);   // null = the cache's own split workspace
int32_t static_scratch(int device, void** out);
int pick_splits(const Cache* c, int64_t n_blocks);
int stream_nt(const Cache* c, int64_t n_blocks);
void split_geometry(const Cache* c, int64_t n_blocks, int* nsplit, int* bps);
int waves_per_workgroup(const Cache* c);
int32_t launch_adaptive(Cache* c, int layer, const __half* q, const cqa_tolerances& tol,
                        const cqa_selector& sel, float* O, cqa_head_cert* cert, uint32_t* flags,
                        uint32_t* flags_mirror, uint32_t mirror_tag, hipStream_t st);
int32_t launch_split_mfma(const DecodeArgs& a, int group, dim3 grid, hipEvent_t ev0, hipEvent_t ev1,
                          hipStream_t st);

int32_t launch_stream_read(const uint8_t* t1, int64_t nq_cap, int nb, dim3 grid, bool nt, int wpb,
                           uint32_t* sink, hipStream_t st);

int dense_splits(int64_t n_tokens);
// Dense FP16 attention for the G query heads of ONE kv group: k, v point at [n_tokens][128];
// q_group at the group's first query head.  O rows are written only where select (device,
// indexed from the group's first head; NULL = all) is nonzero.
int32_t launch_dense_group(const __half* q_group, const __half* k, const __half* v, int group,
                           int64_t n_tokens, float* O_group, const uint32_t* select_group,
                           cqa_head_cert* cert_group, uint32_t* flags_group, int rung,
                           float* ws, hipStream_t st);
int64_t dense_ws_floats(int group, int64_t n_tokens);

// Device-resolved fallback ladder (dense_ladder_kernel).
constexpr int LADDER_MAX_SPLITS = 64;
struct LadderArgs {
  const __half* q;          // [Bt][Hq][128]
  const __half* t2_k;       // layer base of the pinned originals: [Bt * Hkv][max_tokens][128]
  const __half* t2_v;
  int64_t max_tokens, n_tokens;
  int n_rows;               // Bt * Hq
  int nsplit, tiles_per_split;
  int rung4_min_groups;
  float* ws;                // [Bt * Hq][nsplit][4 + 128]
  uint32_t* tickets;        // [Bt * Hkv], zero between launches
  uint32_t* counts;         // [2]: steps served by Rung 3, by Rung 4
  float* O;
  cqa_head_cert* cert;
  uint32_t* flags;
};
int ladder_splits(const Cache* c, int64_t n_tokens);
int64_t ladder_ws_floats(int64_t rows);
int32_t launch_dense_ladder(Cache* c, int layer, const __half* q, int rung4_min_groups, float* O,
                            cqa_head_cert* cert, uint32_t* flags, hipStream_t st);

}  // namespace cqa
