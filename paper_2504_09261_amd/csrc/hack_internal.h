// Internal declarations shared by the host side (hack_api.cpp) and the HIP
// kernels of the gfx950 library.  Nothing here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_plan.h"

namespace hack {

// Per-unit launch table entry, built on the host from the caller's host arrays
// and uploaded once per distinct table.  One unit = one (batch, head) pair.
struct alignas(16) UnitDesc {
  int64_t in_off;   // first row of the unit's input rows in the cache arrays
  int64_t out_off;  // first row of its output rows (gather target / attention source)
  int32_t len_in;   // cache rows before this step (L)
  int32_t n_new;    // rows of the current scale that virtually follow them (0 or N_k)
  int32_t n_out;    // rows to produce (gather) or rows attended over
  int32_t keep_a;   // select: rows [0, keep_a) are always kept
  int32_t sel_lo;   // select: ranked segment [sel_lo, sel_hi)
  int32_t sel_hi;
  int32_t sel_m;    // select: how many rows of the ranked segment are kept
  int32_t keep_b;   // select: rows [keep_b, T_in) are always kept
  int32_t mode;     // move kernel: MOVE_* below
  int32_t unit;     // unit id u = b*H + h (rows of q/k_new/out start at u*N_k)
  int32_t pad0;
  int32_t pad1;
};
static_assert(sizeof(UnitDesc) == 64, "UnitDesc must stay 64 bytes");

enum : int32_t { MOVE_NONE = 0, MOVE_APPEND = 1, MOVE_GATHER = 2 };

// One attention work item: a tile of queries of one unit.  It carries copies of the descriptor
// fields the attention kernels read, so that a work-group has one dependent table load in front of
// its first K/V copy instead of two (the small scale steps are pure latency chains).
struct alignas(16) AttnItem {
  int32_t desc;     // index into the UnitDesc table; < 0: padding entry, nothing to do
  int32_t q_tile;   // first query row = q_tile * (rows per tile)
  int32_t unit;     // UnitDesc::unit
  int32_t n_out;    // UnitDesc::n_out
  int64_t out_off;  // UnitDesc::out_off
  int64_t in_off;   // UnitDesc::in_off
  int32_t len_in;   // UnitDesc::len_in
  int32_t pad[3];
};
static_assert(sizeof(AttnItem) == 48, "AttnItem must stay 48 bytes");
inline AttnItem make_attn_item(const UnitDesc& d, int desc, int q_tile) {
  AttnItem it{};
  it.desc = desc; it.q_tile = q_tile; it.unit = d.unit; it.n_out = d.n_out; it.out_off = d.out_off; it.in_off = d.in_off;
  it.len_in = d.len_in;
  return it;
}
inline AttnItem attn_item_padding() { AttnItem it{}; it.desc = -1; return it; }

struct CachePtrs {
  void* k;
  void* v;
  int32_t* pos;
};

constexpr int kScoreChunk = 256;   // keys per score work-group (fp32 path)
constexpr int kMaxObs = 32;        // observation queries (one MFMA column block)

// ---- kernel launchers (each validates nothing: the API layer has done so) ----

// Append / gather K, V (and pos) rows.  `descs` has n_desc entries; every entry
// with mode != MOVE_NONE is processed.  max_rows = max over entries of the rows
// it moves.
void launch_move(hipStream_t s, int elem_bytes, int head_dim, const UnitDesc* descs, int n_desc,
                 int max_rows, CachePtrs in, CachePtrs out, const void* k_new, const void* v_new,
                 int N_k, int pos_new, const int32_t* kept_idx, int64_t idx_stride);

// Subset-attention importance, bf16: one launch over `items`, a DEVICE array with
// one entry per chunk of item_keys keys (32, 64, 128 or 256) of every scored unit, each unit
// padded with empty chunks to a multiple of 4 entries (one work-group takes 4
// consecutive entries, which must belong to one unit).  All items of a unit
// must be in the same launch and n_items must not exceed
// score_fused_capacity(head_dim, item_keys) (the waves the device holds at once: the kernel waits
// inside a launch for a unit's items).  slots is a workspace of slot_groups * 32
// 64-bit words per `pos` (slot_groups >= the work-groups of any unit), every word
// all-ones on entry and left all-ones; counters 2 uint32 per `pos`, zero on entry
// and left zero; q_rows DEVICE int32[32]; fault (host-visible int[2]): [0] is set
// if a wait gave up after spin_limit polls, [1] if a logit exceeded the range of
// the parked format.
struct alignas(16) ScoreItem {
  int64_t in_off;    // first row of the unit's cached keys
  int32_t unit;      // u = b*H + h (rows of q/k_new start at u*N_k)
  int32_t len_in;    // cached keys
  int32_t t_in;      // cached + new keys
  int32_t chunk;     // this item covers keys [chunk*keys, (chunk+1)*keys)
  int32_t pos;       // workspace slot of the unit
  int32_t n_groups;  // work-groups (sets of 4 items) of the unit
};
static_assert(sizeof(ScoreItem) == 32, "ScoreItem must stay 32 bytes");
int score_item_keys(int dtype);
int score_max_groups();   // work-groups per unit the fused kernel's exchange supports
int score_fused_capacity(int head_dim, int item_keys);
// two_pass: two launches (row sums, then importance) that read K twice but never wait inside
// a launch, so n_items may then exceed the resident capacity and other kernels may share the
// device.  abort_flag: DEVICE word, zero in normal operation; a fused launch that gave up its
// wait sets it and later fused launches return at once until the host clears it.
// skip_publish: -1, or (test hook) the work-group of the launch that withholds its sums.
void launch_score_fused(hipStream_t s, int head_dim, int item_keys, bool two_pass, const ScoreItem* items, int n_items,
                        const void* q, const int32_t* q_rows, int n_obs, int N_k, float scale, const void* k_cache,
                        const void* k_new, unsigned long long* slots, int slot_groups, unsigned* counters,
                        float* importance, int64_t imp_stride, int* fault, int spin_limit, const unsigned* abort_flag,
                        int skip_publish);
// The same importance (bf16, two-pass form) with all scratch in a fixed device array of the
// library instead of context memory; no allocation, no host-to-device copy.  At most
// kStaticUnitsMax units per call; the plan travels by value as a kernel argument.
constexpr int kStaticUnitsMax = 64;
struct StaticScorePlan {
  int64_t in_off[kStaticUnitsMax];   // first cached row of each planned unit
  int32_t len_in[kStaticUnitsMax];   // cached rows
  int32_t unit[kStaticUnitsMax];     // u = b*H + h
  int32_t q_rows[kMaxObs];
  int32_t n_units;
  int32_t n_new;                     // rows of k_new that follow the cached ones (0 or N_k)
  int32_t item_keys;                 // keys per wave item: 32, 64, 128 or 256
};
int score_static_units_max();
size_t score_static_scratch_bytes();
int score_static_item_count(const StaticScorePlan& plan);
hipError_t score_static_setup(int device);   // once per device: finds the device address of the array
hipError_t launch_score_static(hipStream_t s, int device, int head_dim, const StaticScorePlan& plan, const void* q, int n_obs,
                               int N_k, float scale, const void* k_cache, const void* k_new, float* importance,
                               int64_t imp_stride, int* fault);
// fp32: two passes over (chunk of 256 keys, listed unit); list[n_list] indexes
// descs; stats is a workspace of n_list * ceil(max_t_in / 256) * 64 doubles.
void launch_score_generic(hipStream_t s, int head_dim, const UnitDesc* descs, const int32_t* list, int n_list,
                          int max_t_in, const void* q, const int32_t* q_rows, int n_obs, int N_k, float scale,
                          const void* k_cache, const void* k_new, double* stats, float* importance,
                          int64_t imp_stride);

// Budgeted selection; one work-group per listed unit.
void launch_select(hipStream_t s, const UnitDesc* descs, const int32_t* list, int n_list,
                   int max_t_in, const float* importance, int64_t imp_stride, int32_t* kept_idx,
                   int64_t idx_stride);
size_t select_lds_bytes(int max_t_in);

// Attention of N_k queries per unit over rows [out_off, out_off + n_out).
// bf16_kernel: which bf16 kernel serves the 128-query work items, 1 = the deeper
// software pipeline (default), 0 = the plain one-block pipeline (kept for A/B timing
// and as a second implementation the tests run over the same shapes).
void launch_attn(hipStream_t s, int dtype, int head_dim, const UnitDesc* descs, const AttnItem* items,
                 int n_items, int q_tile_rows, const void* q, const void* k_cache,
                 const void* v_cache, int N_k, float scale, void* out, int bf16_kernel);
// Streamed form of the 128-query bf16 kernel: work-group i serves segs[seg_begin[i] .. seg_begin[i+1]).
// part_o: n_slots * 128 * head_dim floats, part_ml: n_slots * 256 floats, part_count: one zeroed
// counter per cut work item (left zero).  Launches that share these arrays must not overlap.
int attn_stream_slots(int head_dim);   // work-groups the current device holds at once
void launch_attn_stream(hipStream_t s, int head_dim, const UnitDesc* descs, const AttnSeg* segs, const int32_t* seg_begin,
                        int n_groups, const void* q, const void* k_cache, const void* v_cache, int N_k, float scale,
                        void* out, float* part_o, float* part_ml, unsigned* part_count);
// bf16 attention for steps with few queries: work item = (unit, tile of
// attn_split_q_tile_rows() queries), keys split over the waves of a work-group.
// fuse == 0: attends over rows [out_off, out_off + n_out) of k_cache / v_cache.
// fuse != 0: attends over [rows in_off .. +len_in of the cache | the unit's N_k rows
// of k_new / v_new] (n_out = len_in + N_k) and also writes those rows (and their
// positions pos_new + row, if pos_app != nullptr) behind the cached ones in
// k_app / v_app / pos_app, i.e. it performs the append of the step as well.
int attn_split_q_tile_rows();
void launch_attn_split(hipStream_t s, int head_dim, const UnitDesc* descs, const AttnItem* items, int n_items,
                       const void* q, const void* k_cache, const void* v_cache, const void* k_new, const void* v_new,
                       void* k_app, void* v_app, int32_t* pos_app, int pos_new, int fuse, int N_k, float scale,
                       void* out);
// Attention variance of the listed units (bf16): sigma[desc.unit] = sum over the
// unit's n_out keys of the population variance, across its N_k queries, of the
// softmax probabilities.  stats: workspace of 2 floats per (unit, query).
void launch_head_variance(hipStream_t s, int head_dim, const UnitDesc* descs, int n_desc, int max_len, const void* q,
                          const void* k_cache, int N_k, float scale, float* stats, double* sigma);
// Final-step merge of the listed units (bf16): every row of the unit's uncompressed cache
// [rows in_off .. +len_in of k_in / v_in | its N_k rows of k_new / v_new] that kept_idx does not
// list is folded into its nearest kept row (cosine similarity of keys) by similarity-weighted
// averaging; the kept rows, which the gather has already written to rows [out_off, out_off + n_out)
// of k_out / v_out, are updated in place.  list[n_list] indexes descs.  nearest / weight /
// inv_norm: workspaces of ws_stride entries per unit id (>= the unit's T_in).
void launch_merge(hipStream_t s, int head_dim, const UnitDesc* descs, const int32_t* list, int n_list, int max_t_in,
                  int max_out, const void* k_in, const void* v_in, const void* k_new, const void* v_new, int N_k,
                  const int32_t* kept_idx, int64_t idx_stride, void* k_out, void* v_out, int32_t* nearest, float* weight,
                  float* inv_norm, int64_t ws_stride);
// Query rows per attention work item for this dtype/head_dim and launch size.
int attn_q_tile_rows(int dtype, int head_dim, int n_units, int N_k);

}  // namespace hack
