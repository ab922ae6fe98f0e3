// Host side of the C ABI declared in include/hack.h: argument validation, the
// host planner that turns (head class, budget, N_init, N_k) into per-unit launch
// tables, the launch-table cache, the managed double-slab cache of hack_step,
// and the kernel launches.  No device memory is ever read from the host.
#include <algorithm>
#include <cmath>
#include <climits>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/hack.h"
#include "hack_internal.h"
#include "table_cache.h"

using namespace hack;

// ---------------------------------------------------------------------------
// context
// ---------------------------------------------------------------------------
namespace {

constexpr size_t kTableChunkBytes = 32u << 20;   // launch tables: one chunk (device memory + pinned mirror)
constexpr size_t kTableLimitBytes = 1u << 30;    // ... and all chunks of a context together
// Polls (each an atomic round trip plus a short sleep, ~1 us) a score wave spends waiting for the
// other items of its unit before it gives up; real waits last a few microseconds.
constexpr int kScoreSpinLimit = 1 << 18;

// Launch-table storage in device memory with a pinned host mirror.
struct HipTableBackend {
  bool alloc(size_t bytes, uint8_t** dev, uint8_t** host) {
    if (hipMalloc((void**)dev, bytes) != hipSuccess) return false;
    if (hipHostMalloc((void**)host, bytes, hipHostMallocDefault) != hipSuccess) {
      (void)hipFree(*dev);
      return false;
    }
    return true;
  }
  void release(uint8_t* dev, uint8_t* host) {
    (void)hipFree(dev);
    (void)hipHostFree(host);
  }
  bool upload(uint8_t* dev, const uint8_t* host, size_t bytes, void* stream) {
    return hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, static_cast<hipStream_t>(stream)) == hipSuccess;
  }
  bool may_alloc(void* stream) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    (void)hipStreamIsCapturing(static_cast<hipStream_t>(stream), &cs);
    return cs == hipStreamCaptureStatusNone;
  }
};

}  // namespace

struct hack_ctx {
  hack_config cfg;
  int elem_bytes = 2;
  // workspace
  float* importance = nullptr;   // [max_units, ws_stride]
  int32_t* kept = nullptr;       // [max_units, ws_stride]
  double* stats = nullptr;       // fp32 path: [max_units, max_chunks, 32, 2] softmax partials
  unsigned long long* rowstat = nullptr;  // bf16 path: [max_units, score_groups, 32] row-sum exchange slots, all-ones between launches
  unsigned long long* rowstat_side = nullptr;  // the same for the side branch of hack_step (two-pass form: its slots are not re-armed)
  int score_groups = 0;          // work-groups a unit of max_cache_len keys is scored by
  int spin_limit = 0;            // polls after which a score work-group gives up its wait for the unit's other work-groups
  unsigned* abort_flag = nullptr; // bf16 path: device word behind the counters; set by a fused score launch that gave up
  size_t n_slots = 0;            // 64-bit words in rowstat
  int score_mode = HACK_SCORE_FUSED;   // hack_score_mode: fused single launch / two launches without in-kernel waits
  int skip_publish = -1;         // test hook: work-group of a fused score launch that withholds its sums
  unsigned* counters = nullptr;  // bf16 path: [max_units, 2] reader counters, zero between launches
  float* hv_stats = nullptr;     // head variance: [max_units, max_queries, 2] softmax statistics of every query
  int32_t* merge_nn = nullptr;   // final-step merge (bf16): [max_units, ws_stride] nearest kept row of every cache row
  float* merge_w = nullptr;      //   ... its weight
  float* merge_inv = nullptr;    //   ... inverse key norms of the kept rows
  int* fault = nullptr;          // pinned, device-visible int[2]: [0] a score wave's bounded wait gave up (fatal),
                                 // [1] a logit exceeded the range the bf16 score kernel supports
  int score_capacity[4] = {0, 0, 0, 0};   // bf16 path: score items one fused launch may hold (resident waves) for items of 32, 64, 128, 256 keys
  int split_max_items = 0;       // launches with at most this many 32-query attention items use the key-split kernel
  int attn_kernel = 1;           // bf16 kernel of the 128-query items: 1 = deeper pipeline, 0 = plain (HACK_ATTN_PIPE=0)
  // streamed form of that kernel: the launch is cut into equal runs of key blocks, one per resident work-group
  int attn_stream = -1;          // HACK_ATTN_STREAM; -1 (default): cut single work items where the pair model gains, 0: never, 1: equal runs
                                 // for every launch of the 128-query kernel, 2: A/B aid, 4: every cut the model likes (see use_stream_attention)
  int attn_slots = 0;            // work-groups of the streamed kernel the device holds at once
  float* part_o = nullptr;       // [2 * attn_slots, 128, head_dim] unnormalised partial outputs
  float* part_ml = nullptr;      // [2 * attn_slots, 2, 128] their references and normalisers
  unsigned* part_count = nullptr; // [attn_slots] ticket counters, zero between launches
  // hack_step overlap: the compression chain of one group of units runs beside the attention of the other group
  bool step_overlap = false;     // off by default (measured slower on MI355X, see step_impl); HACK_STEP_OVERLAP=1 switches it on
  hipStream_t aux_stream = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  int64_t ws_stride = 0;
  int max_chunks = 0;
  // launch-table cache: tables keep their device address for the life of the context
  TableCache<HipTableBackend>* tables = nullptr;
  std::string err;
};

struct hack_kvcache {
  hack_ctx* ctx;
  int32_t n_units;
  std::vector<int32_t> cap;
  std::vector<int64_t> slab[2];
  std::vector<uint8_t> cur;
  std::vector<int64_t> off;
  std::vector<int32_t> len;
  void* k;
  void* v;
  int32_t* pos;
  int64_t rows;
  int64_t tokens_seen;
};

namespace {

hack_status fail(hack_ctx* ctx, hack_status s, const char* fmt, ...) {
  if (ctx) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    ctx->err = buf;
  }
  return s;
}

#define HIP_TRY(ctx, call)                                                              \
  do {                                                                                  \
    hipError_t e_ = (call);                                                             \
    if (e_ != hipSuccess)                                                               \
      return fail(ctx, HACK_EHIP, "%s failed: %s", #call, hipGetErrorString(e_));      \
  } while (0)

inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// A launch table under construction: sections are appended 64-byte aligned.
struct Table {
  std::vector<uint8_t> bytes;
  template <typename T>
  size_t add(const T* data, size_t count) {
    const size_t off = (bytes.size() + 63) / 64 * 64;
    bytes.resize(off + std::max<size_t>(count, 1) * sizeof(T), 0);
    if (count) memcpy(bytes.data() + off, data, count * sizeof(T));
    return off;
  }
};

// Returns the device address of a table with these contents, uploading it on
// the given stream the first time it is seen.  Tables are immutable and keep
// their address until the context is destroyed, so queued kernels and captured
// graphs may go on using them.
hack_status table_device(hack_ctx* ctx, const Table& t, hipStream_t stream, const uint8_t** dev) {
  switch (ctx->tables->get(t.bytes.data(), t.bytes.size(), stream, dev)) {
    case TableStatus::kOk: return HACK_OK;
    case TableStatus::kTooLarge:
      return fail(ctx, HACK_ECAPACITY, "launch table of %zu bytes exceeds the %zu-byte table chunk", t.bytes.size(), kTableChunkBytes);
    case TableStatus::kFullDuringCapture:
      return fail(ctx, HACK_ECAPACITY, "launch-table storage is full and cannot grow while the stream is being captured: "
                                       "run the schedule once outside the capture first");
    case TableStatus::kLimit:
      return fail(ctx, HACK_ECAPACITY, "launch tables of this context exceed %zu bytes", kTableLimitBytes);
    case TableStatus::kAllocFailed: return fail(ctx, HACK_EHIP, "allocating launch-table storage failed");
    case TableStatus::kUploadFailed: return fail(ctx, HACK_EHIP, "uploading a launch table failed");
  }
  return HACK_EHIP;
}

// Sec. 4.4 policies as index ranges (see hack_select in hack.h).
void plan_select(int type, int T, int b, int n_init, int n_recent, UnitDesc* d) {
  if (b >= T) {  // identity
    d->keep_a = T; d->sel_lo = T; d->sel_hi = T; d->sel_m = 0; d->keep_b = T;
    return;
  }
  if (type == HACK_CONTEXTUAL) {
    d->keep_a = 0; d->sel_lo = 0; d->sel_hi = T; d->sel_m = b; d->keep_b = T;
    return;
  }
  const int n_rec = std::min(n_recent, T);
  const int n0 = std::max(0, std::min(n_init, T - n_rec));
  const int M = b - n0 - n_rec;
  if (M >= 0) {
    d->keep_a = n0; d->sel_lo = n0; d->sel_hi = T - n_rec; d->sel_m = M; d->keep_b = T - n_rec;
  } else {  // budget below init + recent: init rows, then the best of the recent scale
    const int ka = std::min(n0, b);
    d->keep_a = ka; d->sel_lo = T - n_rec; d->sel_hi = T; d->sel_m = b - ka; d->keep_b = T;
  }
}

// Brings the exchange workspace of the fused score kernel back to its idle state
// (every slot empty, counters and abort word zero).  Synchronises the device.
hipError_t rearm_score_workspace(hack_ctx* ctx) {
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess && ctx->rowstat) e = hipMemset(ctx->rowstat, 0xFF, ctx->n_slots * sizeof(unsigned long long));
  if (e == hipSuccess && ctx->counters) e = hipMemset(ctx->counters, 0, ((size_t)ctx->cfg.max_units * 2 + 64) * sizeof(unsigned));
  if (e == hipSuccess) e = hipDeviceSynchronize();
  return e;
}

// Conditions that kernels of earlier calls found on the device.
hack_status device_report(hack_ctx* ctx) {
  volatile int* f = ctx->fault;
  if (f && f[0]) {
    // A fused score launch gave up its wait (the device did not keep the launch resident as a
    // whole, e.g. because other work held compute units).  Later fused launches have refused to
    // run since.  Recover: drain, re-arm the workspace, and from now on score in two launches
    // that do not wait for each other inside a kernel.
    if (rearm_score_workspace(ctx) != hipSuccess)
      return fail(ctx, HACK_EHIP, "a score launch gave up its wait and the workspace could not be re-armed");
    f[0] = 0;
    ctx->score_mode = HACK_SCORE_TWO_PASS;
    return fail(ctx, HACK_EHIP, "a score launch gave up waiting for a unit's other work-groups: importance (and whatever "
                                "was derived from it) of the calls since the last successful check is incomplete and those "
                                "calls must be issued again; the context has been re-armed and now scores in two passes "
                                "without in-kernel waits");
  }
  if (f && f[1]) {
    f[1] = 0;
    return fail(ctx, HACK_EUNSUPPORTED, "an earlier bf16 score launch met a logit beyond +-354 (scale * q.k); such logits "
                                        "are clamped, so its importance may differ from the definition");
  }
  return HACK_OK;
}

hack_status check_common(hack_ctx* ctx, int32_t B, int32_t N_k, bool need_nk) {
  if (!ctx) return HACK_EINVAL;
  const hack_status dev = device_report(ctx);
  if (dev != HACK_OK) return dev;
  if (B < 1) return fail(ctx, HACK_EINVAL, "B must be >= 1 (got %d)", B);
  if ((int64_t)B * ctx->cfg.heads > ctx->cfg.max_units)
    return fail(ctx, HACK_ECAPACITY, "B*H = %lld exceeds max_units %d", (long long)B * ctx->cfg.heads, ctx->cfg.max_units);
  if (need_nk) {
    if (N_k < 1) return fail(ctx, HACK_EINVAL, "N_k must be >= 1 (got %d)", N_k);
    if (N_k > ctx->cfg.max_queries) return fail(ctx, HACK_ECAPACITY, "N_k = %d exceeds max_queries %d", N_k, ctx->cfg.max_queries);
  }
  return HACK_OK;
}

hack_status check_cache(hack_ctx* ctx, const hack_cache* c, int n_units, const char* name, bool need_v) {
  if (!c) return fail(ctx, HACK_EINVAL, "%s is NULL", name);
  if (!c->k || (need_v && !c->v) || !c->off || !c->len) return fail(ctx, HACK_EINVAL, "%s has a NULL member", name);
  if (!aligned16(c->k) || (c->v && !aligned16(c->v))) return fail(ctx, HACK_EINVAL, "%s k/v must be 16-byte aligned", name);
  if (c->rows < 0) return fail(ctx, HACK_EINVAL, "%s rows < 0", name);
  for (int u = 0; u < n_units; ++u) {
    if (c->len[u] < 0 || c->off[u] < 0 || (c->off[u] & 7) || c->off[u] + c->len[u] > c->rows)
      return fail(ctx, HACK_EINVAL, "%s unit %d: off %lld len %d outside [0, %lld) or off not a multiple of 8", name, u,
                  (long long)c->off[u], c->len[u], (long long)c->rows);
  }
  return HACK_OK;
}

bool scale_ok(float s) { return std::isfinite(s) && s > 0.f; }

// Attention work items: units dealt to the 8 XCDs in order of decreasing length
// (work-group ids are dispatched round-robin over XCDs, so id%8 picks the XCD);
// within an XCD all tiles of a unit are adjacent, so its K/V stay in that XCD's L2.
void build_attn_items(const std::vector<UnitDesc>& descs, int N_k, int tile_rows, std::vector<AttnItem>* items) {
  const int n = (int)descs.size();
  std::vector<int> order(n);
  for (int i = 0; i < n; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return descs[a].n_out > descs[b].n_out; });
  const int tiles = (N_k + tile_rows - 1) / tile_rows;
  constexpr int X = 8;
  std::vector<AttnItem> per[X];
  int64_t load[X] = {0};
  for (int r = 0; r < n; ++r) {
    int x = 0;
    for (int i = 1; i < X; ++i) if (load[i] < load[x]) x = i;   // least-loaded XCD
    load[x] += (int64_t)descs[order[r]].n_out * tiles;
    for (int t = 0; t < tiles; ++t) per[x].push_back(make_attn_item(descs[order[r]], order[r], t));
  }
  size_t longest = 0;
  for (int x = 0; x < X; ++x) longest = std::max(longest, per[x].size());
  items->assign(longest * X, attn_item_padding());
  for (int x = 0; x < X; ++x)
    for (size_t i = 0; i < per[x].size(); ++i) (*items)[i * X + x] = per[x][i];
}

// Steps with few queries (the early scales) go to the key-split kernel (bf16
// only): its 32-query work items fill the chip where 128-query tiles would not,
// and a step that does not compress then needs no separate append launch.  It is
// used while all of its work items are resident at once or nearly so; beyond
// that the 128-query kernel, which shares every K/V block among four times as
// many queries, is faster.  Measured cross-overs on MI355X: head_dim 128 between
// 416 and 576 items (16 heads, batch 2); head_dim 64 between 1920 and 3840 items
// (30 heads, batch 32).
int split_max_items_default(int head_dim) { return head_dim == 64 ? 2048 : 512; }
bool use_split_attention(const hack_ctx* ctx, int n_units, int N_k) {
  if (ctx->cfg.dtype != HACK_BF16) return false;
  const int tile = attn_split_q_tile_rows();
  return (int64_t)n_units * ((N_k + tile - 1) / tile) <= ctx->split_max_items;
}

// The 128-query bf16 kernel in its streamed form: the work items of the launch are cut into one run of
// key blocks per resident work-group (plan_attn_stream), so that every work-group holds the same number of
// blocks whatever the number and the lengths of the work items are; work items that a cut falls into are
// put together from partial results.  OFF by default (HACK_ATTN_STREAM=1 when the context is created
// switches it on for every launch of the 128-query kernel): on MI355X it measured slower than one work
// item per work-group on all but one step of the benchmark workloads (1024^2 schedules, scale steps 9-13,
// us per launch, plain / streamed: 16 heads x batch 2: 34 / 39, 56 / 64, 113 / 104, 136 / 140, 222 / 230;
// 32 heads x batch 2: 51 / 54, 74 / 92, 159 / 175, 253 / 270, 425 / 527).  In-kernel time stamps show why:
// of the two work-groups that share a compute unit the older one is served first and runs the steady
// loop at 0.73-0.76 us per key block, the younger one at 0.97-1.0 (0.55 alone), so equal shares finish
// up to 30 % apart and the launch lasts as long as the slowest; the hardware's own dispatch of whole work
// items absorbs that difference.  On top come about 3 us per extra segment (pipeline fill), 3-4 us per
// partial result written and 3-4 us per part added up.
// `shared` says that another attention launch of the context may run at the same time (the partial-result
// arrays are the context's), which rules the streamed form out.
// What the library does by default (HACK_ATTN_STREAM unset) is narrower: launches whose work items all start
// at once (no more items than resident work-groups) keep whole work items, and plan_attn_cuts halves the few
// whose compute unit would finish last under the measured pair model, if that shortens the modelled launch by
// kCutMinGain.  On the 1024^2 benchmark workloads this fires at scale step 11 with 16 heads x batch 2 (416 work
// items on 256 compute units: the long items that would share a compute unit with another long one are
// halved; 113.7 -> 98.8 us measured, 111.8 -> 89.3 modelled) and at step 9 with 32 heads x batch 2 (50.3 ->
// 42.8 us measured, 45.3 -> 35.0 modelled); launches with more work items than resident work-groups are
// left alone (there the model is 10-15 % off).  HACK_ATTN_STREAM=0 switches it off, =4 applies every cut
// the model likes (tests).
constexpr AttnPairModel kPairModel128{0.55, 0.75, 1.0, 4.0, 14.0};   // us per key block alone / first / second of a pair; fixed costs in blocks
constexpr double kCutMinGain = 0.05;
constexpr int kCutMinBlocks = 8;
constexpr int kStreamOverheadBlocks = 4;   // start and end of a segment, in key blocks of the steady loop
constexpr int kStreamMinBlocks = 4;        // shortest segment a work item is cut into
bool use_stream_attention(const hack_ctx* ctx, const std::vector<UnitDesc>& descs, int N_k, bool shared, AttnStreamPlan* plan) {
  if (ctx->cfg.dtype != HACK_BF16 || ctx->attn_kernel == 0 || ctx->attn_stream == 0 || ctx->attn_slots <= 0 || shared) return false;
  if (descs.empty()) return false;
  const int tile = attn_q_tile_rows(ctx->cfg.dtype, ctx->cfg.head_dim, (int)descs.size(), N_k);
  if (tile != 128) return false;
  std::vector<int32_t> n_keys(descs.size());
  for (size_t i = 0; i < descs.size(); ++i) n_keys[i] = descs[i].n_out;
  if (ctx->attn_stream == 2) {
    // A/B aid: the streamed kernel on uncut work items, one per work-group, in the order of the plain launch
    std::vector<AttnItem> items;
    build_attn_items(descs, N_k, tile, &items);
    plan->segs.clear();
    plan->seg_begin.assign(1, 0);
    for (const AttnItem& it : items) {
      if (it.desc >= 0) plan->segs.push_back(AttnSeg{it.desc, it.q_tile, 0, 0x3fffffff, -1, 0, 0, 0});
      plan->seg_begin.push_back((int32_t)plan->segs.size());
    }
    plan->n_groups = (int)items.size();
    plan->n_parts = plan->n_counters = 0;
    return plan->n_groups > 0;
  }
  if (ctx->attn_stream < 0 || ctx->attn_stream == 4) {
    // whole work items, a few of them cut in two where the pair model says the launch gets shorter (plan_attn_cuts)
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->cfg.device) != hipSuccess || cus < kAttnXcds) return false;
    const bool forced = ctx->attn_stream == 4;
    // the model's constants were measured for head_dim 128, two work-groups per compute unit
    if (!forced && (ctx->cfg.head_dim != 128 || ctx->attn_slots != 2 * cus)) return false;
    std::vector<AttnItem> items;
    build_attn_items(descs, N_k, tile, &items);
    std::vector<AttnLaneItem> lanes[kAttnXcds];
    for (size_t i = 0; i < items.size(); ++i)
      if (items[i].desc >= 0)
        lanes[i % kAttnXcds].push_back(AttnLaneItem{items[i].desc, items[i].q_tile, (items[i].n_out + kAttnKeyBlock - 1) / kAttnKeyBlock});
    double before = 0.0, after = 0.0;
    if (!plan_attn_cuts(lanes, cus / kAttnXcds, kCutMinBlocks, kPairModel128, forced ? 1e-9 : kCutMinGain, plan, &before, &after)) return false;
    return plan->n_groups > 0 && plan->n_parts <= 2 * ctx->attn_slots && plan->n_counters <= ctx->attn_slots;
  }
  plan_attn_stream(n_keys.data(), (int)descs.size(), (N_k + tile - 1) / tile, ctx->attn_slots, kStreamOverheadBlocks,
                   kStreamMinBlocks, plan);
  return plan->n_groups > 0 && plan->n_parts <= 2 * ctx->attn_slots && plan->n_counters <= ctx->attn_slots;
}

int finish_score_plan(const hack_ctx* ctx, const std::vector<UnitDesc>& descs, const std::vector<int32_t>& list, int keys,
                      bool two_pass, std::vector<ScoreItem>* items, std::vector<int>* group_begin);

// One score work item per chunk of every listed unit, longest units first so the
// tail of a launch is made of short units.  All items of a unit go into the same
// launch group and no group exceeds `capacity` items; group_begin gets the first
// item of every group plus the total as its last entry.
void build_score_items(const std::vector<UnitDesc>& descs, const std::vector<int32_t>& list, int item_keys,
                       int capacity, std::vector<ScoreItem>* items, std::vector<int>* group_begin) {
  items->clear();
  group_begin->assign(1, 0);
  std::vector<int> order(list.size());
  for (size_t i = 0; i < list.size(); ++i) order[i] = (int)i;
  auto t_in = [&](int pos) { return descs[list[pos]].len_in + descs[list[pos]].n_new; };
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return t_in(a) > t_in(b); });
  for (int pos : order) {
    const UnitDesc& d = descs[list[pos]];
    const int wgs = ((t_in(pos) + item_keys - 1) / item_keys + 3) / 4;  // 4 items per work-group, same unit
    if ((int)items->size() - group_begin->back() + 4 * wgs > capacity) group_begin->push_back((int)items->size());
    for (int c = 0; c < 4 * wgs; ++c)
      items->push_back(ScoreItem{d.in_off, d.unit, d.len_in, t_in(pos), c, pos, wgs});
  }
  group_begin->push_back((int)items->size());
}

// bf16: builds the score items of the listed units and returns the item size (keys per wave) chosen.
// Smaller items spread a launch over more compute units and shorten every wave's serial tile work, so the
// smallest size is taken whose items all fit one launch (the fused kernel's work-groups wait for each other
// inside a launch, so a launch holds at most what the device keeps resident) and whose work-groups per unit the
// exchange area supports; if no size fits one launch, the size that needs the fewest launches.  The choice
// does not depend on the score mode, so both modes (and the fixed-scratch entry point, which applies the same
// rule) group the keys alike and give the same bits.
int choose_score_item_keys(const hack_ctx* ctx, std::vector<int> t_in) {
  std::stable_sort(t_in.begin(), t_in.end(), [](int a, int b) { return a > b; });   // the order build_score_items fills launches in
  int best_keys = 0;
  long best_launches = 0;
  for (int i = 0; i < 4; ++i) {
    const int keys = 32 << i, cap = ctx->score_capacity[i];
    if (cap <= 0) continue;
    long launches = 1, in_launch = 0;
    bool fits = true;
    for (int t : t_in) {
      const int wgs = ((t + keys - 1) / keys + 3) / 4;
      if (wgs > score_max_groups()) { fits = false; break; }
      if (in_launch + 4 * wgs > cap) { ++launches; in_launch = 0; }
      in_launch += 4 * wgs;
    }
    if (!fits) continue;
    if (launches <= 1) return keys;
    if (best_keys == 0 || launches < best_launches) {
      best_keys = keys;
      best_launches = launches;
    }
  }
  return best_keys ? best_keys : 256;
}

int plan_score_items(const hack_ctx* ctx, const std::vector<UnitDesc>& descs, const std::vector<int32_t>& list, bool two_pass,
                     std::vector<ScoreItem>* items, std::vector<int>* group_begin) {
  std::vector<int> t_in;
  for (int32_t pos : list) t_in.push_back(descs[pos].len_in + descs[pos].n_new);
  return finish_score_plan(ctx, descs, list, choose_score_item_keys(ctx, std::move(t_in)), two_pass, items, group_begin);
}

// Builds the final item list for the chosen size: launch groups for the fused form, one group for the two-pass
// form (no in-kernel wait: one launch pair holds any number of items).
int finish_score_plan(const hack_ctx* ctx, const std::vector<UnitDesc>& descs, const std::vector<int32_t>& list, int keys,
                      bool two_pass, std::vector<ScoreItem>* items, std::vector<int>* group_begin) {
  int idx = 0;
  while ((32 << idx) != keys) ++idx;
  build_score_items(descs, list, keys, two_pass ? INT32_MAX : ctx->score_capacity[idx], items, group_begin);
  return keys;
}

// Scores the listed units of a table that is already on the device.
void run_score(hack_ctx* ctx, hipStream_t s, bool two_pass, unsigned long long* slots, const UnitDesc* ddev, const int32_t* list_dev, int n_list, int max_t,
               const ScoreItem* items_dev, int item_keys, const std::vector<int>& group_begin, const void* q,
               const int32_t* rows_dev, int n_obs, int N_k, float scale, const void* k_cache, const void* k_new,
               float* importance, int64_t imp_stride) {
  if (ctx->cfg.dtype == HACK_F32) {
    launch_score_generic(s, ctx->cfg.head_dim, ddev, list_dev, n_list, max_t, q, rows_dev, n_obs, N_k, scale, k_cache,
                         k_new, ctx->stats, importance, imp_stride);
    return;
  }
  for (size_t g = 0; g + 1 < group_begin.size(); ++g)
    launch_score_fused(s, ctx->cfg.head_dim, item_keys, two_pass, items_dev + group_begin[g],
                       group_begin[g + 1] - group_begin[g], q, rows_dev, n_obs, N_k, scale, k_cache, k_new, slots,
                       ctx->score_groups, ctx->counters, importance, imp_stride, ctx->fault, ctx->spin_limit, ctx->abort_flag,
                       ctx->skip_publish);
}

void fill_q_rows(const int32_t* q_idx, int n_obs, int N_k, int32_t* rows) {
  for (int i = 0; i < kMaxObs; ++i) rows[i] = 0;
  for (int i = 0; i < n_obs; ++i) rows[i] = q_idx ? q_idx[i] : (int32_t)(((int64_t)i * N_k) / n_obs);
}

}  // namespace

// ---------------------------------------------------------------------------
// life cycle
// ---------------------------------------------------------------------------
extern "C" const char* hack_strerror(hack_status s) {
  switch (s) {
    case HACK_OK: return "ok";
    case HACK_EINVAL: return "invalid argument";
    case HACK_ECAPACITY: return "capacity exceeded";
    case HACK_EUNSUPPORTED: return "unsupported";
    case HACK_EHIP: return "HIP runtime error";
  }
  return "unknown status";
}

extern "C" const char* hack_last_error(const hack_ctx* ctx) { return ctx ? ctx->err.c_str() : "NULL context"; }

extern "C" hack_status hack_check(hack_ctx* ctx) {
  if (!ctx) return HACK_EINVAL;
  return device_report(ctx);
}

extern "C" hack_status hack_set_score_mode(hack_ctx* ctx, int32_t mode) {
  if (!ctx) return HACK_EINVAL;
  if (mode != HACK_SCORE_FUSED && mode != HACK_SCORE_TWO_PASS) return fail(ctx, HACK_EINVAL, "unknown score mode %d", mode);
  if (mode == ctx->score_mode) return HACK_OK;
  // the two forms leave the exchange slots in different states: start the other one from a clean workspace
  if (rearm_score_workspace(ctx) != hipSuccess) return fail(ctx, HACK_EHIP, "re-arming the score workspace failed");
  ctx->score_mode = mode;
  return HACK_OK;
}

extern "C" int32_t hack_get_score_mode(const hack_ctx* ctx) { return ctx ? ctx->score_mode : (int32_t)HACK_EINVAL; }

extern "C" hack_status hack_create(hack_ctx** out, const hack_config* cfg) {
  if (!out || !cfg) return HACK_EINVAL;
  *out = nullptr;
  if (cfg->head_dim != 64 && cfg->head_dim != 128) return HACK_EINVAL;
  if (cfg->dtype != HACK_BF16 && cfg->dtype != HACK_F32) return HACK_EINVAL;
  if (cfg->heads < 1 || cfg->max_units < cfg->heads || cfg->max_cache_len < 1 || cfg->max_queries < 1) return HACK_EINVAL;
  if (cfg->n_obs < 1 || cfg->n_obs > kMaxObs) return HACK_EINVAL;
  if (cfg->max_cache_len > 32768) return HACK_EUNSUPPORTED;  // selection keeps a unit's keys in LDS
  hack_ctx* ctx = new (std::nothrow) hack_ctx();
  if (!ctx) return HACK_EHIP;
  ctx->cfg = *cfg;
  ctx->elem_bytes = cfg->dtype == HACK_F32 ? 4 : 2;
  ctx->ws_stride = round_up(cfg->max_cache_len, 64);
  ctx->max_chunks = (cfg->max_cache_len + kScoreChunk - 1) / kScoreChunk;
  ctx->split_max_items = split_max_items_default(cfg->head_dim);
  ctx->spin_limit = kScoreSpinLimit;
  // test hook: a tiny limit makes the score kernel's bounded wait give up (every work-group still exits normally)
  if (const char* v = std::getenv("HACK_SCORE_SPIN_LIMIT")) ctx->spin_limit = std::max(0, std::atoi(v));
  // test hook: this work-group of every fused score launch does not publish its row sums, so the work-groups of its
  // unit run into the (tiny) spin limit deterministically
  if (const char* v = std::getenv("HACK_SCORE_TEST_SKIP_PUBLISH")) ctx->skip_publish = std::atoi(v);
  if (const char* v = std::getenv("HACK_SCORE_MODE")) ctx->score_mode = std::atoi(v) == 1 ? HACK_SCORE_TWO_PASS : HACK_SCORE_FUSED;
  if (const char* v = std::getenv("HACK_ATTN_SPLIT_ITEMS")) ctx->split_max_items = std::atoi(v);   // tuning / test override
  if (const char* v = std::getenv("HACK_STEP_OVERLAP")) ctx->step_overlap = std::atoi(v) != 0;
  if (const char* v = std::getenv("HACK_ATTN_PIPE")) ctx->attn_kernel = std::atoi(v) != 0;   // A/B and test override
  if (const char* v = std::getenv("HACK_ATTN_STREAM")) ctx->attn_stream = std::atoi(v);       // A/B and test override
  hipError_t e = hipSetDevice(cfg->device);
  const size_t n_ws = (size_t)cfg->max_units * ctx->ws_stride;
  if (e == hipSuccess) e = hipMalloc((void**)&ctx->importance, n_ws * sizeof(float));
  if (e == hipSuccess) e = hipMalloc((void**)&ctx->kept, n_ws * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc((void**)&ctx->stats, (size_t)cfg->max_units * ctx->max_chunks * kMaxObs * 2 * sizeof(double));
  ctx->score_groups = score_max_groups();   // exchange slots per unit: enough for every item size
  const size_t n_slots = (size_t)cfg->max_units * ctx->score_groups * kMaxObs;
  ctx->n_slots = n_slots;
  if (e == hipSuccess) e = hipMalloc((void**)&ctx->rowstat, n_slots * sizeof(unsigned long long));
  if (e == hipSuccess && cfg->dtype == HACK_BF16) e = hipMalloc((void**)&ctx->rowstat_side, n_slots * sizeof(unsigned long long));
  const size_t n_counters = (size_t)cfg->max_units * 2 + 64;   // per-unit reader counters, then the abort word
  if (e == hipSuccess) e = hipMalloc((void**)&ctx->counters, n_counters * sizeof(unsigned));
  if (e == hipSuccess) e = hipMemset(ctx->counters, 0, n_counters * sizeof(unsigned));
  if (e == hipSuccess) ctx->abort_flag = ctx->counters + (size_t)cfg->max_units * 2;
  if (e == hipSuccess && cfg->dtype == HACK_BF16)
    e = hipMalloc((void**)&ctx->hv_stats, (size_t)cfg->max_units * cfg->max_queries * 2 * sizeof(float));
  if (e == hipSuccess && cfg->dtype == HACK_BF16) e = hipMalloc((void**)&ctx->merge_nn, n_ws * sizeof(int32_t));
  if (e == hipSuccess && cfg->dtype == HACK_BF16) e = hipMalloc((void**)&ctx->merge_w, n_ws * sizeof(float));
  if (e == hipSuccess && cfg->dtype == HACK_BF16) e = hipMalloc((void**)&ctx->merge_inv, n_ws * sizeof(float));
  if (e == hipSuccess && cfg->dtype == HACK_BF16) {
    ctx->attn_slots = attn_stream_slots(cfg->head_dim);
    const size_t n_part = 2 * (size_t)std::max(ctx->attn_slots, 1);
    e = hipMalloc((void**)&ctx->part_o, n_part * 128 * cfg->head_dim * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->part_ml, n_part * 256 * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->part_count, (n_part / 2) * sizeof(unsigned));
    if (e == hipSuccess) e = hipMemset(ctx->part_count, 0, (n_part / 2) * sizeof(unsigned));
  }
  if (e == hipSuccess) e = hipHostMalloc((void**)&ctx->fault, 2 * sizeof(int), hipHostMallocDefault);
  if (e == hipSuccess) ctx->fault[0] = ctx->fault[1] = 0;
  if (e == hipSuccess) e = hipMemset(ctx->rowstat, 0xFF, n_slots * sizeof(unsigned long long));   // every slot empty
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e == hipSuccess) {
    ctx->tables = new (std::nothrow) TableCache<HipTableBackend>(HipTableBackend{}, kTableChunkBytes, kTableLimitBytes);
    if (!ctx->tables || !ctx->tables->reserve_first_chunk()) e = hipErrorOutOfMemory;
  }
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&ctx->aux_stream, hipStreamNonBlocking);   // default priority
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming);
  if (e == hipSuccess) e = score_static_setup(cfg->device);   // device address of the library's fixed scratch array
  if (e == hipSuccess && cfg->dtype == HACK_BF16) {
    // a unit's score items wait for each other inside one launch, so a launch may
    // hold at most as many items as the device keeps resident at once
    for (int i = 0; i < 4; ++i) ctx->score_capacity[i] = score_fused_capacity(cfg->head_dim, 32 << i);
    // the largest unit must fit one launch with the largest items
    const int per_unit = (cfg->max_cache_len + 255) / 256 + 3;
    if (ctx->score_capacity[3] < per_unit || (per_unit + 3) / 4 > score_max_groups()) e = hipErrorInvalidConfiguration;
  }
  if (e != hipSuccess) {
    hack_destroy(ctx);
    return HACK_EHIP;
  }
  *out = ctx;
  return HACK_OK;
}

extern "C" void hack_destroy(hack_ctx* ctx) {
  if (!ctx) return;
  if (ctx->importance) (void)hipFree(ctx->importance);
  if (ctx->kept) (void)hipFree(ctx->kept);
  if (ctx->stats) (void)hipFree(ctx->stats);
  if (ctx->rowstat) (void)hipFree(ctx->rowstat);
  if (ctx->rowstat_side) (void)hipFree(ctx->rowstat_side);
  if (ctx->counters) (void)hipFree(ctx->counters);
  if (ctx->fault) (void)hipHostFree(ctx->fault);
  if (ctx->hv_stats) (void)hipFree(ctx->hv_stats);
  if (ctx->merge_nn) (void)hipFree(ctx->merge_nn);
  if (ctx->merge_w) (void)hipFree(ctx->merge_w);
  if (ctx->merge_inv) (void)hipFree(ctx->merge_inv);
  if (ctx->part_o) (void)hipFree(ctx->part_o);
  if (ctx->part_ml) (void)hipFree(ctx->part_ml);
  if (ctx->part_count) (void)hipFree(ctx->part_count);
  if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
  if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
  if (ctx->aux_stream) (void)hipStreamDestroy(ctx->aux_stream);
  delete ctx->tables;
  delete ctx;
}

// ---------------------------------------------------------------------------
// a1: score
// ---------------------------------------------------------------------------
extern "C" hack_status hack_score(hack_ctx* ctx, int32_t B, int32_t N_k, const void* q, const int32_t* q_idx,
                                  int32_t n_obs, float scale, const hack_cache* in, const void* k_new,
                                  const uint8_t* active, float* importance, int64_t imp_stride,
                                  hack_stream stream) {
  hack_status st = check_common(ctx, B, N_k, true);
  if (st != HACK_OK) return st;
  const int U = B * ctx->cfg.heads;
  if (!q || !importance) return fail(ctx, HACK_EINVAL, "q and importance must not be NULL");
  if (!aligned16(q) || (k_new && !aligned16(k_new))) return fail(ctx, HACK_EINVAL, "q/k_new must be 16-byte aligned");
  if (n_obs < 1 || n_obs > ctx->cfg.n_obs || n_obs > N_k)
    return fail(ctx, HACK_EINVAL, "n_obs = %d outside [1, min(%d, N_k = %d)]", n_obs, ctx->cfg.n_obs, N_k);
  if (!scale_ok(scale)) return fail(ctx, HACK_EINVAL, "scale must be finite and > 0");
  if (q_idx)
    for (int i = 0; i < n_obs; ++i)
      if (q_idx[i] < 0 || q_idx[i] >= N_k) return fail(ctx, HACK_EINVAL, "q_idx[%d] = %d outside [0, %d)", i, q_idx[i], N_k);
  if ((st = check_cache(ctx, in, U, "in", false)) != HACK_OK) return st;
  const int n_new = k_new ? N_k : 0;
  std::vector<UnitDesc> descs;
  std::vector<int32_t> list;
  int max_t = 0;
  for (int u = 0; u < U; ++u) {
    if (active && !active[u]) continue;
    const int64_t T = (int64_t)in->len[u] + n_new;
    if (T < 1) return fail(ctx, HACK_EINVAL, "unit %d has no keys to score", u);
    if (T > ctx->cfg.max_cache_len) return fail(ctx, HACK_ECAPACITY, "unit %d: T_in = %lld exceeds max_cache_len %d", u, (long long)T, ctx->cfg.max_cache_len);
    if (T > imp_stride) return fail(ctx, HACK_ECAPACITY, "imp_stride %lld < T_in %lld of unit %d", (long long)imp_stride, (long long)T, u);
    UnitDesc d{};
    d.in_off = in->off[u]; d.out_off = in->off[u]; d.len_in = in->len[u]; d.n_new = n_new; d.n_out = (int)T; d.unit = u;
    list.push_back((int32_t)descs.size());
    descs.push_back(d);
    max_t = std::max(max_t, (int)T);
  }
  if (descs.empty()) return HACK_OK;
  int32_t rows[kMaxObs];
  fill_q_rows(q_idx, n_obs, N_k, rows);
  std::vector<ScoreItem> sitems;
  std::vector<int> groups;
  int item_keys = 0;
  const bool two_pass = ctx->score_mode == HACK_SCORE_TWO_PASS;
  if (ctx->cfg.dtype == HACK_BF16) item_keys = plan_score_items(ctx, descs, list, two_pass, &sitems, &groups);
  Table t;
  const size_t o_desc = t.add(descs.data(), descs.size());
  const size_t o_list = t.add(list.data(), list.size());
  const size_t o_rows = t.add(rows, kMaxObs);
  const size_t o_sit = t.add(sitems.data(), sitems.size());
  const uint8_t* dev;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if ((st = table_device(ctx, t, s, &dev)) != HACK_OK) return st;
  run_score(ctx, s, two_pass, ctx->rowstat, (const UnitDesc*)(dev + o_desc), (const int32_t*)(dev + o_list), (int)list.size(), max_t,
            (const ScoreItem*)(dev + o_sit), item_keys, groups, q, (const int32_t*)(dev + o_rows), n_obs, N_k, scale, in->k, k_new,
            importance, imp_stride);
  HIP_TRY(ctx, hipGetLastError());
  return HACK_OK;
}

// The same call for callers that cannot allocate (see hack.h): scratch in the library's fixed device array.
extern "C" hack_status hack_score_static(hack_ctx* ctx, int32_t B, int32_t N_k, const void* q, const int32_t* q_idx,
                                         int32_t n_obs, float scale, const hack_cache* in, const void* k_new,
                                         const uint8_t* active, float* importance, int64_t imp_stride,
                                         hack_stream stream) {
  hack_status st = check_common(ctx, B, N_k, true);
  if (st != HACK_OK) return st;
  if (ctx->cfg.dtype != HACK_BF16) return fail(ctx, HACK_EUNSUPPORTED, "hack_score_static is implemented for bf16 contexts");
  const int U = B * ctx->cfg.heads;
  if (!q || !importance) return fail(ctx, HACK_EINVAL, "q and importance must not be NULL");
  if (!aligned16(q) || (k_new && !aligned16(k_new))) return fail(ctx, HACK_EINVAL, "q/k_new must be 16-byte aligned");
  if (n_obs < 1 || n_obs > ctx->cfg.n_obs || n_obs > N_k)
    return fail(ctx, HACK_EINVAL, "n_obs = %d outside [1, min(%d, N_k = %d)]", n_obs, ctx->cfg.n_obs, N_k);
  if (!scale_ok(scale)) return fail(ctx, HACK_EINVAL, "scale must be finite and > 0");
  if (q_idx)
    for (int i = 0; i < n_obs; ++i)
      if (q_idx[i] < 0 || q_idx[i] >= N_k) return fail(ctx, HACK_EINVAL, "q_idx[%d] = %d outside [0, %d)", i, q_idx[i], N_k);
  if ((st = check_cache(ctx, in, U, "in", false)) != HACK_OK) return st;
  StaticScorePlan plan{};
  plan.n_new = k_new ? N_k : 0;
  for (int u = 0; u < U; ++u) {
    if (active && !active[u]) continue;
    const int64_t T = (int64_t)in->len[u] + plan.n_new;
    if (T < 1) return fail(ctx, HACK_EINVAL, "unit %d has no keys to score", u);
    if (T > ctx->cfg.max_cache_len) return fail(ctx, HACK_ECAPACITY, "unit %d: T_in = %lld exceeds max_cache_len %d", u, (long long)T, ctx->cfg.max_cache_len);
    if (T > imp_stride) return fail(ctx, HACK_ECAPACITY, "imp_stride %lld < T_in %lld of unit %d", (long long)imp_stride, (long long)T, u);
    if (plan.n_units == kStaticUnitsMax)
      return fail(ctx, HACK_ECAPACITY, "hack_score_static scores at most %d units per call", kStaticUnitsMax);
    plan.in_off[plan.n_units] = in->off[u];
    plan.len_in[plan.n_units] = in->len[u];
    plan.unit[plan.n_units] = u;
    ++plan.n_units;
  }
  if (plan.n_units == 0) return HACK_OK;
  {   // the item size hack_score would take for these units: same grouping of the keys, same bits
    std::vector<int> t_in;
    for (int i = 0; i < plan.n_units; ++i) t_in.push_back(plan.len_in[i] + plan.n_new);
    plan.item_keys = choose_score_item_keys(ctx, std::move(t_in));
  }
  fill_q_rows(q_idx, n_obs, N_k, plan.q_rows);
  HIP_TRY(ctx, launch_score_static(static_cast<hipStream_t>(stream), ctx->cfg.device, ctx->cfg.head_dim, plan, q, n_obs, N_k, scale,
                                   in->k, k_new, importance, imp_stride, ctx->fault));
  return HACK_OK;
}

// ---------------------------------------------------------------------------
// a2: select
// ---------------------------------------------------------------------------
extern "C" hack_status hack_select(hack_ctx* ctx, int32_t B, const float* importance, int64_t imp_stride,
                                   const int32_t* t_in, const uint8_t* head_type, const int32_t* budget,
                                   int32_t n_init, int32_t n_recent, int32_t* kept_idx, int64_t idx_stride,
                                   int32_t* len_out, hack_stream stream) {
  hack_status st = check_common(ctx, B, 0, false);
  if (st != HACK_OK) return st;
  const int U = B * ctx->cfg.heads, H = ctx->cfg.heads;
  if (!importance || !t_in || !head_type || !budget || !kept_idx) return fail(ctx, HACK_EINVAL, "NULL argument");
  if (n_init < 0 || n_recent < 0) return fail(ctx, HACK_EINVAL, "n_init and n_recent must be >= 0");
  for (int h = 0; h < H; ++h)
    if (head_type[h] > 1) return fail(ctx, HACK_EINVAL, "head_type[%d] = %d is not a head class", h, head_type[h]);
  std::vector<UnitDesc> descs(U);
  std::vector<int32_t> list(U);
  int max_t = 0;
  for (int u = 0; u < U; ++u) {
    const int T = t_in[u];
    if (T < 1) return fail(ctx, HACK_EINVAL, "t_in[%d] = %d", u, T);
    if (T > ctx->cfg.max_cache_len) return fail(ctx, HACK_ECAPACITY, "t_in[%d] = %d exceeds max_cache_len %d", u, T, ctx->cfg.max_cache_len);
    if (budget[u] < 1) return fail(ctx, HACK_EINVAL, "budget[%d] = %d", u, budget[u]);
    if (head_type[u % H] == HACK_STRUCTURAL && n_recent > T) return fail(ctx, HACK_EINVAL, "n_recent %d > t_in[%d] = %d", n_recent, u, T);
    const int b = std::min(budget[u], T);
    if (T > imp_stride || b > idx_stride) return fail(ctx, HACK_ECAPACITY, "strides too small for unit %d", u);
    UnitDesc d{};
    d.len_in = T; d.n_new = 0; d.n_out = b; d.unit = u;
    plan_select(head_type[u % H], T, b, n_init, n_recent, &d);
    descs[u] = d;
    list[u] = u;
    max_t = std::max(max_t, T);
    if (len_out) len_out[u] = b;
  }
  Table t;
  const size_t o_desc = t.add(descs.data(), descs.size());
  const size_t o_list = t.add(list.data(), list.size());
  const uint8_t* dev;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if ((st = table_device(ctx, t, s, &dev)) != HACK_OK) return st;
  launch_select(s, (const UnitDesc*)(dev + o_desc), (const int32_t*)(dev + o_list), U, max_t, importance, imp_stride,
                kept_idx, idx_stride);
  HIP_TRY(ctx, hipGetLastError());
  return HACK_OK;
}

// ---------------------------------------------------------------------------
// a3: compact
// ---------------------------------------------------------------------------
extern "C" hack_status hack_compact(hack_ctx* ctx, int32_t B, int32_t N_k, const hack_cache* in, const void* k_new,
                                    const void* v_new, int32_t pos_new, const int32_t* kept_idx, int64_t idx_stride,
                                    const hack_cache* out, hack_stream stream) {
  const bool has_new = (k_new != nullptr);
  hack_status st = check_common(ctx, B, N_k, has_new);
  if (st != HACK_OK) return st;
  const int U = B * ctx->cfg.heads;
  if (!kept_idx) return fail(ctx, HACK_EINVAL, "kept_idx is NULL");
  if (has_new != (v_new != nullptr)) return fail(ctx, HACK_EINVAL, "k_new and v_new must both be given or both be NULL");
  if (has_new && (!aligned16(k_new) || !aligned16(v_new))) return fail(ctx, HACK_EINVAL, "k_new/v_new must be 16-byte aligned");
  if ((st = check_cache(ctx, in, U, "in", true)) != HACK_OK) return st;
  if ((st = check_cache(ctx, out, U, "out", true)) != HACK_OK) return st;
  const int n_new = has_new ? N_k : 0;
  std::vector<UnitDesc> descs;
  int max_rows = 0;
  std::vector<std::pair<int64_t, int64_t>> in_iv;
  for (int u = 0; u < U; ++u) {
    const int n = out->len[u];
    if (n == 0) continue;
    if (n > idx_stride) return fail(ctx, HACK_ECAPACITY, "idx_stride %lld < out->len[%d] = %d", (long long)idx_stride, u, n);
    if ((int64_t)n > (int64_t)in->len[u] + n_new) return fail(ctx, HACK_EINVAL, "unit %d keeps %d rows of %lld", u, n, (long long)in->len[u] + n_new);
    UnitDesc d{};
    d.in_off = in->off[u]; d.out_off = out->off[u]; d.len_in = in->len[u]; d.n_new = n_new; d.n_out = n;
    d.mode = MOVE_GATHER; d.unit = u;
    descs.push_back(d);
    max_rows = std::max(max_rows, n);
    if (in->len[u] > 0) in_iv.emplace_back(in->off[u], in->off[u] + in->len[u]);
  }
  if (descs.empty()) return HACK_OK;
  if (out->k == in->k || out->v == in->v || out->k == in->v || out->v == in->k) {
    std::sort(in_iv.begin(), in_iv.end());
    for (const UnitDesc& d : descs) {
      const int64_t a = d.out_off, b = d.out_off + d.n_out;
      auto it = std::lower_bound(in_iv.begin(), in_iv.end(), std::make_pair(b, (int64_t)INT64_MIN));
      // intervals starting before b: the one with the largest end among them may overlap
      for (auto p = in_iv.begin(); p != it; ++p)
        if (p->second > a) return fail(ctx, HACK_EINVAL, "output rows of unit %d overlap input rows that are read", d.unit);
    }
  }
  Table t;
  const size_t o_desc = t.add(descs.data(), descs.size());
  const uint8_t* dev;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if ((st = table_device(ctx, t, s, &dev)) != HACK_OK) return st;
  CachePtrs pin{in->k, in->v, in->pos}, pout{out->k, out->v, out->pos};
  launch_move(s, ctx->elem_bytes, ctx->cfg.head_dim, (const UnitDesc*)(dev + o_desc), (int)descs.size(), max_rows, pin,
              pout, k_new, v_new, N_k, pos_new, kept_idx, idx_stride);
  HIP_TRY(ctx, hipGetLastError());
  return HACK_OK;
}

// ---------------------------------------------------------------------------
// final-step merge of contextual heads
// ---------------------------------------------------------------------------
extern "C" hack_status hack_merge(hack_ctx* ctx, int32_t B, int32_t N_k, const hack_cache* in, const void* k_new,
                                  const void* v_new, const int32_t* kept_idx, int64_t idx_stride, const uint8_t* active,
                                  const hack_cache* out, hack_stream stream) {
  const bool has_new = (k_new != nullptr);
  hack_status st = check_common(ctx, B, N_k, has_new);
  if (st != HACK_OK) return st;
  if (ctx->cfg.dtype != HACK_BF16) return fail(ctx, HACK_EUNSUPPORTED, "the final-step merge is implemented for bf16 contexts");
  const int U = B * ctx->cfg.heads;
  if (!kept_idx) return fail(ctx, HACK_EINVAL, "kept_idx is NULL");
  if (has_new != (v_new != nullptr)) return fail(ctx, HACK_EINVAL, "k_new and v_new must both be given or both be NULL");
  if (has_new && (!aligned16(k_new) || !aligned16(v_new))) return fail(ctx, HACK_EINVAL, "k_new/v_new must be 16-byte aligned");
  if ((st = check_cache(ctx, in, U, "in", true)) != HACK_OK) return st;
  if ((st = check_cache(ctx, out, U, "out", true)) != HACK_OK) return st;
  const int n_new = has_new ? N_k : 0;
  std::vector<UnitDesc> descs;
  std::vector<int32_t> list;
  int max_t = 0, max_out = 0;
  for (int u = 0; u < U; ++u) {
    if (active && !active[u]) continue;
    const int64_t T = (int64_t)in->len[u] + n_new;
    const int n = out->len[u];
    if (n < 1) return fail(ctx, HACK_EINVAL, "unit %d keeps no row", u);
    if (n > T) return fail(ctx, HACK_EINVAL, "unit %d keeps %d rows of %lld", u, n, (long long)T);
    if (T > ctx->cfg.max_cache_len) return fail(ctx, HACK_ECAPACITY, "unit %d: T_in = %lld exceeds max_cache_len %d", u, (long long)T, ctx->cfg.max_cache_len);
    if (n > idx_stride) return fail(ctx, HACK_ECAPACITY, "idx_stride %lld < out->len[%d] = %d", (long long)idx_stride, u, n);
    if (n == T) continue;   // nothing evicted
    // the kept rows are rewritten in place while the evicted ones are still read from `in`
    if ((out->k == in->k || out->v == in->v) && in->len[u] > 0 && out->off[u] < in->off[u] + in->len[u] &&
        in->off[u] < out->off[u] + n)
      return fail(ctx, HACK_EINVAL, "output rows of unit %d overlap its input rows", u);
    UnitDesc d{};
    d.in_off = in->off[u]; d.out_off = out->off[u]; d.len_in = in->len[u]; d.n_new = n_new; d.n_out = n; d.unit = u;
    list.push_back((int32_t)descs.size());
    descs.push_back(d);
    max_t = std::max(max_t, (int)T);
    max_out = std::max(max_out, n);
  }
  if (descs.empty()) return HACK_OK;
  Table t;
  const size_t o_desc = t.add(descs.data(), descs.size());
  const size_t o_list = t.add(list.data(), list.size());
  const uint8_t* dev;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if ((st = table_device(ctx, t, s, &dev)) != HACK_OK) return st;
  launch_merge(s, ctx->cfg.head_dim, (const UnitDesc*)(dev + o_desc), (const int32_t*)(dev + o_list), (int)list.size(), max_t,
               max_out, in->k, in->v, k_new, v_new, N_k, kept_idx, idx_stride, out->k, out->v, ctx->merge_nn, ctx->merge_w,
               ctx->merge_inv, ctx->ws_stride);
  HIP_TRY(ctx, hipGetLastError());
  return HACK_OK;
}

// ---------------------------------------------------------------------------
// a4: attention
// ---------------------------------------------------------------------------
extern "C" hack_status hack_attn(hack_ctx* ctx, int32_t B, int32_t N_k, const void* q, const hack_cache* kv,
                                 float scale, void* out, hack_stream stream) {
  hack_status st = check_common(ctx, B, N_k, true);
  if (st != HACK_OK) return st;
  const int U = B * ctx->cfg.heads;
  if (!q || !out) return fail(ctx, HACK_EINVAL, "q and out must not be NULL");
  if (!aligned16(q) || !aligned16(out)) return fail(ctx, HACK_EINVAL, "q/out must be 16-byte aligned");
  if (!scale_ok(scale)) return fail(ctx, HACK_EINVAL, "scale must be finite and > 0");
  if ((st = check_cache(ctx, kv, U, "kv", true)) != HACK_OK) return st;
  std::vector<UnitDesc> descs(U);
  for (int u = 0; u < U; ++u) {
    if (kv->len[u] < 1) return fail(ctx, HACK_EINVAL, "unit %d has an empty cache", u);
    UnitDesc d{};
    d.in_off = kv->off[u]; d.out_off = kv->off[u]; d.len_in = kv->len[u]; d.n_out = kv->len[u]; d.unit = u;
    descs[u] = d;
  }
  const bool split = use_split_attention(ctx, U, N_k);
  const int tile = split ? attn_split_q_tile_rows() : attn_q_tile_rows(ctx->cfg.dtype, ctx->cfg.head_dim, U, N_k);
  std::vector<AttnItem> items;
  AttnStreamPlan plan;
  const bool streamed = !split && use_stream_attention(ctx, descs, N_k, false, &plan);
  if (!streamed) build_attn_items(descs, N_k, tile, &items);
  Table t;
  const size_t o_desc = t.add(descs.data(), descs.size());
  const size_t o_items = t.add(items.data(), items.size());
  const size_t o_segs = t.add(plan.segs.data(), plan.segs.size());
  const size_t o_segb = t.add(plan.seg_begin.data(), plan.seg_begin.size());
  const uint8_t* dev;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if ((st = table_device(ctx, t, s, &dev)) != HACK_OK) return st;
  if (streamed)
    launch_attn_stream(s, ctx->cfg.head_dim, (const UnitDesc*)(dev + o_desc), (const AttnSeg*)(dev + o_segs),
                       (const int32_t*)(dev + o_segb), plan.n_groups, q, kv->k, kv->v, N_k, scale, out, ctx->part_o,
                       ctx->part_ml, ctx->part_count);
  else if (split)
    launch_attn_split(s, ctx->cfg.head_dim, (const UnitDesc*)(dev + o_desc), (const AttnItem*)(dev + o_items),
                      (int)items.size(), q, kv->k, kv->v, nullptr, nullptr, nullptr, nullptr, nullptr, 0, 0, N_k, scale,
                      out);
  else
    launch_attn(s, ctx->cfg.dtype, ctx->cfg.head_dim, (const UnitDesc*)(dev + o_desc), (const AttnItem*)(dev + o_items),
                (int)items.size(), tile, q, kv->k, kv->v, N_k, scale, out, ctx->attn_kernel);
  HIP_TRY(ctx, hipGetLastError());
  return HACK_OK;
}

extern "C" int32_t hack_attn_variant(const hack_ctx* ctx, int32_t B, int32_t N_k) {
  if (!ctx || B < 1 || N_k < 1) return (int32_t)HACK_EINVAL;
  return use_split_attention(ctx, B * ctx->cfg.heads, N_k) ? 1 : 0;
}

// ---------------------------------------------------------------------------
// offline head classification: attention variance
// ---------------------------------------------------------------------------
extern "C" hack_status hack_head_variance(hack_ctx* ctx, int32_t B, int32_t N_k, const void* q, const hack_cache* kv,
                                          float scale, double* sigma, hack_stream stream) {
  hack_status st = check_common(ctx, B, N_k, true);
  if (st != HACK_OK) return st;
  if (ctx->cfg.dtype != HACK_BF16) return fail(ctx, HACK_EUNSUPPORTED, "head variance is implemented for bf16 contexts");
  const int U = B * ctx->cfg.heads;
  if (!q || !sigma) return fail(ctx, HACK_EINVAL, "q and sigma must not be NULL");
  if (!aligned16(q) || ((uintptr_t)sigma & 7)) return fail(ctx, HACK_EINVAL, "q must be 16-byte and sigma 8-byte aligned");
  if (!scale_ok(scale)) return fail(ctx, HACK_EINVAL, "scale must be finite and > 0");
  if ((st = check_cache(ctx, kv, U, "kv", false)) != HACK_OK) return st;
  std::vector<UnitDesc> descs(U);
  int max_len = 0;
  for (int u = 0; u < U; ++u) {
    if (kv->len[u] < 1) return fail(ctx, HACK_EINVAL, "unit %d has an empty cache", u);
    UnitDesc d{};
    d.in_off = kv->off[u]; d.out_off = kv->off[u]; d.len_in = kv->len[u]; d.n_out = kv->len[u]; d.unit = u;
    descs[u] = d;
    max_len = std::max(max_len, (int)kv->len[u]);
  }
  Table t;
  const size_t o_desc = t.add(descs.data(), descs.size());
  const uint8_t* dev;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if ((st = table_device(ctx, t, s, &dev)) != HACK_OK) return st;
  launch_head_variance(s, ctx->cfg.head_dim, (const UnitDesc*)(dev + o_desc), U, max_len, q, kv->k, N_k, scale,
                       ctx->hv_stats, sigma);
  HIP_TRY(ctx, hipGetLastError());
  return HACK_OK;
}

// ---------------------------------------------------------------------------
// a5: managed cache + fused step
// ---------------------------------------------------------------------------
extern "C" hack_status hack_kvcache_rows_required(int32_t n_units, const int32_t* cap, int64_t* rows) {
  if (n_units < 1 || !cap || !rows) return HACK_EINVAL;
  int64_t r = 0;
  for (int u = 0; u < n_units; ++u) {
    if (cap[u] < 1) return HACK_EINVAL;
    r += 2 * round_up(cap[u], 8);
  }
  *rows = r;
  return HACK_OK;
}

extern "C" hack_status hack_kvcache_create(hack_ctx* ctx, int32_t n_units, const int32_t* cap, void* k_mem,
                                           void* v_mem, int32_t* pos_mem, int64_t mem_rows, hack_kvcache** out) {
  if (!ctx) return HACK_EINVAL;
  if (!out || !cap || !k_mem || !v_mem) return fail(ctx, HACK_EINVAL, "NULL argument");
  *out = nullptr;
  if (n_units < 1 || n_units > ctx->cfg.max_units || n_units % ctx->cfg.heads)
    return fail(ctx, HACK_EINVAL, "n_units = %d must be a multiple of H within max_units", n_units);
  if (!aligned16(k_mem) || !aligned16(v_mem)) return fail(ctx, HACK_EINVAL, "k_mem/v_mem must be 16-byte aligned");
  int64_t need;
  if (hack_kvcache_rows_required(n_units, cap, &need) != HACK_OK) return fail(ctx, HACK_EINVAL, "cap entries must be >= 1");
  if (need > mem_rows) return fail(ctx, HACK_ECAPACITY, "cache needs %lld rows, %lld given", (long long)need, (long long)mem_rows);
  hack_kvcache* c = new (std::nothrow) hack_kvcache();
  if (!c) return fail(ctx, HACK_EHIP, "out of host memory");
  c->ctx = ctx; c->n_units = n_units; c->k = k_mem; c->v = v_mem; c->pos = pos_mem; c->rows = mem_rows; c->tokens_seen = 0;
  c->cap.assign(cap, cap + n_units);
  c->slab[0].resize(n_units); c->slab[1].resize(n_units);
  c->cur.assign(n_units, 0); c->len.assign(n_units, 0); c->off.resize(n_units);
  int64_t r = 0;
  for (int u = 0; u < n_units; ++u) {
    c->slab[0][u] = r; r += round_up(cap[u], 8);
    c->slab[1][u] = r; r += round_up(cap[u], 8);
    c->off[u] = c->slab[0][u];
  }
  *out = c;
  return HACK_OK;
}

extern "C" void hack_kvcache_destroy(hack_kvcache* c) { delete c; }

extern "C" hack_status hack_kvcache_reset(hack_kvcache* c) {
  if (!c) return HACK_EINVAL;
  for (int u = 0; u < c->n_units; ++u) {
    c->len[u] = 0; c->cur[u] = 0; c->off[u] = c->slab[0][u];
  }
  c->tokens_seen = 0;
  return HACK_OK;
}

extern "C" hack_status hack_kvcache_view(const hack_kvcache* c, hack_cache* view) {
  if (!c || !view) return HACK_EINVAL;
  view->k = c->k; view->v = c->v; view->pos = c->pos; view->rows = c->rows;
  view->off = c->off.data(); view->len = c->len.data();
  return HACK_OK;
}

namespace {

// The units of a step that are launched together on one stream, with their launch tables.
struct StepGroup {
  std::vector<UnitDesc> descs;            // copies of the group's unit descriptors
  std::vector<int32_t> comp, merging;     // indices into descs: units that compress / that also merge
  int max_t = 0, max_rows = 0, merge_t = 0, merge_out = 0;
  std::vector<AttnItem> items;
  AttnStreamPlan plan;                    // attention in the streamed form (then `items` stays empty)
  bool streamed = false;
  std::vector<ScoreItem> sitems;
  std::vector<int> launches;
  int item_keys = 0;
  bool two_pass = false;
  unsigned long long* slots = nullptr;    // row-sum exchange area of the group's score launches
  const uint8_t* dev = nullptr;
  size_t o_desc = 0, o_comp = 0, o_merge = 0, o_rows = 0, o_items = 0, o_sit = 0, o_segs = 0, o_segb = 0;
  const UnitDesc* ddev() const { return reinterpret_cast<const UnitDesc*>(dev + o_desc); }
};

struct StepArgs {
  int N_k, n_obs, tile;
  bool split, fuse_append, shared;   // shared: two groups of the step may attend at the same time
  const void *q, *k_new, *v_new;
  void* out;
  float scale;
  int32_t* kept;
  int64_t kstride;
  CachePtrs cp;
  int32_t pos_new;
};

void add_unit(StepGroup* g, const UnitDesc& d, bool merges, int N_k) {
  const int idx = (int)g->descs.size();
  g->descs.push_back(d);
  if (d.mode == MOVE_GATHER) {
    g->comp.push_back(idx);
    g->max_t = std::max(g->max_t, d.len_in + d.n_new);
    g->max_rows = std::max(g->max_rows, d.n_out);
    if (merges) {
      g->merging.push_back(idx);
      g->merge_t = std::max(g->merge_t, d.len_in + d.n_new);
      g->merge_out = std::max(g->merge_out, d.n_out);
    }
  } else {
    g->max_rows = std::max(g->max_rows, N_k);
  }
}

hack_status upload_group(hack_ctx* ctx, StepGroup* g, const StepArgs& a, const int32_t* rows, hipStream_t s) {
  g->streamed = !a.split && use_stream_attention(ctx, g->descs, a.N_k, a.shared, &g->plan);
  if (!g->streamed) build_attn_items(g->descs, a.N_k, a.tile, &g->items);
  if (ctx->cfg.dtype == HACK_BF16 && !g->comp.empty())
    g->item_keys = plan_score_items(ctx, g->descs, g->comp, g->two_pass, &g->sitems, &g->launches);
  Table t;
  g->o_desc = t.add(g->descs.data(), g->descs.size());
  g->o_comp = t.add(g->comp.data(), g->comp.size());
  g->o_merge = t.add(g->merging.data(), g->merging.size());
  g->o_rows = t.add(rows, kMaxObs);
  g->o_items = t.add(g->items.data(), g->items.size());
  g->o_sit = t.add(g->sitems.data(), g->sitems.size());
  g->o_segs = t.add(g->plan.segs.data(), g->plan.segs.size());
  g->o_segb = t.add(g->plan.seg_begin.data(), g->plan.seg_begin.size());
  return table_device(ctx, t, s, &g->dev);
}

// score -> select -> append / gather (-> merge) of a group's units
void launch_chain(hack_ctx* ctx, const StepGroup& g, const StepArgs& a, hipStream_t s) {
  const int32_t* comp_dev = reinterpret_cast<const int32_t*>(g.dev + g.o_comp);
  if (!g.comp.empty()) {
    run_score(ctx, s, g.two_pass, g.slots, g.ddev(), comp_dev, (int)g.comp.size(), g.max_t,
              reinterpret_cast<const ScoreItem*>(g.dev + g.o_sit), g.item_keys, g.launches, a.q,
              reinterpret_cast<const int32_t*>(g.dev + g.o_rows), a.n_obs, a.N_k, a.scale, a.cp.k, a.k_new, ctx->importance,
              ctx->ws_stride);
    launch_select(s, g.ddev(), comp_dev, (int)g.comp.size(), g.max_t, ctx->importance, ctx->ws_stride, a.kept, a.kstride);
  }
  if (!a.fuse_append)
    launch_move(s, ctx->elem_bytes, ctx->cfg.head_dim, g.ddev(), (int)g.descs.size(), g.max_rows, a.cp, a.cp, a.k_new, a.v_new,
                a.N_k, a.pos_new, a.kept, a.kstride);
  if (!g.merging.empty())   // compression, the merge included, precedes the attention of the step
    launch_merge(s, ctx->cfg.head_dim, g.ddev(), reinterpret_cast<const int32_t*>(g.dev + g.o_merge), (int)g.merging.size(),
                 g.merge_t, g.merge_out, a.cp.k, a.cp.v, a.k_new, a.v_new, a.N_k, a.kept, a.kstride, a.cp.k, a.cp.v,
                 ctx->merge_nn, ctx->merge_w, ctx->merge_inv, ctx->ws_stride);
}

void launch_group_attention(hack_ctx* ctx, const StepGroup& g, const StepArgs& a, hipStream_t s) {
  const AttnItem* items = reinterpret_cast<const AttnItem*>(g.dev + g.o_items);
  if (g.streamed)
    launch_attn_stream(s, ctx->cfg.head_dim, g.ddev(), reinterpret_cast<const AttnSeg*>(g.dev + g.o_segs),
                       reinterpret_cast<const int32_t*>(g.dev + g.o_segb), g.plan.n_groups, a.q, a.cp.k, a.cp.v, a.N_k, a.scale,
                       a.out, ctx->part_o, ctx->part_ml, ctx->part_count);
  else if (a.split)
    launch_attn_split(s, ctx->cfg.head_dim, g.ddev(), items, (int)g.items.size(), a.q, a.cp.k, a.cp.v, a.k_new, a.v_new, a.cp.k,
                      a.cp.v, a.cp.pos, a.pos_new, a.fuse_append ? 1 : 0, a.N_k, a.scale, a.out);
  else
    launch_attn(s, ctx->cfg.dtype, ctx->cfg.head_dim, g.ddev(), items, (int)g.items.size(), a.tile, a.q, a.cp.k, a.cp.v, a.N_k,
                a.scale, a.out, ctx->attn_kernel);
}

}  // namespace

// One scale step.  Units are independent, so a step may be issued as two groups: the compression chain
// (score -> select -> gather) is a sequence of short, latency-bound launches that leaves most of the device
// idle, while attention fills it.  With the overlap switched on (HACK_STEP_OVERLAP=1 when the context is
// created), when contextual units compress at this step and other units exist, the others go first on the
// caller's stream (their chain, then their attention, which is the longer one: structural budgets are the
// larger), and the contextual units' chain and attention run beside that attention on a stream of the context,
// forked and joined with events (capturable: a HIP graph gets two parallel branches).  The side chain scores
// in the two-pass form, whose work-groups never wait for each other and can therefore share the device with
// the attention launch.  What is computed per unit is the same; only the grouping of a unit's keys into work
// items (chosen per launch) may differ from a single-group step.
// The overlap is OFF by default: on MI355X it measured slower (1024^2 benchmark workload: 1005 against 841 us
// per layer).  The attention launch of the first group holds every wave slot of the device, so the side chain
// only advances as attention work-groups retire and ends with them; the second group's attention then runs
// on its own, and a lone attention launch takes one work item's full latency (60 to 120 key blocks at half a
// microsecond each) however few items it has.  Splitting a step therefore lengthens its critical path.
static hack_status step_impl(hack_ctx* ctx, hack_kvcache* cache, int32_t B, int32_t N_k, const void* q,
                             const void* k_new, const void* v_new, const uint8_t* head_type,
                             const int32_t* budget, int32_t n_init, float scale, void* out,
                             int32_t* kept_idx_opt, int64_t idx_stride, hack_stream stream, bool final_merge) {
  hack_status st = check_common(ctx, B, N_k, true);
  if (st != HACK_OK) return st;
  if (final_merge && ctx->cfg.dtype != HACK_BF16)
    return fail(ctx, HACK_EUNSUPPORTED, "the final-step merge is implemented for bf16 contexts");
  const int U = B * ctx->cfg.heads, H = ctx->cfg.heads;
  if (!cache || cache->ctx != ctx || cache->n_units != U) return fail(ctx, HACK_EINVAL, "cache does not belong to this context / batch");
  if (!q || !k_new || !v_new || !head_type || !budget || !out) return fail(ctx, HACK_EINVAL, "NULL argument");
  if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(out)) return fail(ctx, HACK_EINVAL, "q/k_new/v_new/out must be 16-byte aligned");
  if (!scale_ok(scale)) return fail(ctx, HACK_EINVAL, "scale must be finite and > 0");
  if (n_init < 0) return fail(ctx, HACK_EINVAL, "n_init must be >= 0");
  for (int h = 0; h < H; ++h)
    if (head_type[h] > 1) return fail(ctx, HACK_EINVAL, "head_type[%d] = %d is not a head class", h, head_type[h]);
  if (cache->tokens_seen + N_k > INT32_MAX) return fail(ctx, HACK_ECAPACITY, "token ids overflow int32");

  StepArgs a{};
  a.kept = kept_idx_opt ? kept_idx_opt : ctx->kept;
  a.kstride = kept_idx_opt ? idx_stride : ctx->ws_stride;
  std::vector<UnitDesc> descs(U);
  int n_comp = 0, n_side = 0;
  for (int u = 0; u < U; ++u) {
    const int L = cache->len[u];
    const int64_t T = (int64_t)L + N_k;
    if (budget[u] < 1) return fail(ctx, HACK_EINVAL, "budget[%d] = %d", u, budget[u]);
    UnitDesc d{};
    d.unit = u; d.in_off = cache->off[u]; d.len_in = L; d.n_new = N_k;
    if (budget[u] < T) {
      if (T > ctx->cfg.max_cache_len) return fail(ctx, HACK_ECAPACITY, "unit %d: T_in = %lld exceeds max_cache_len %d", u, (long long)T, ctx->cfg.max_cache_len);
      if (budget[u] > cache->cap[u]) return fail(ctx, HACK_ECAPACITY, "unit %d: budget %d exceeds its slab of %d rows", u, budget[u], cache->cap[u]);
      if (budget[u] > a.kstride) return fail(ctx, HACK_ECAPACITY, "idx_stride %lld < budget[%d] = %d", (long long)a.kstride, u, budget[u]);
      d.mode = MOVE_GATHER; d.n_out = budget[u]; d.out_off = cache->slab[cache->cur[u] ^ 1][u];
      plan_select(head_type[u % H], (int)T, budget[u], n_init, N_k, &d);
      ++n_comp;
      if (head_type[u % H] == HACK_CONTEXTUAL) ++n_side;
    } else {
      if (T > cache->cap[u]) return fail(ctx, HACK_ECAPACITY, "unit %d: %lld rows do not fit its slab of %d", u, (long long)T, cache->cap[u]);
      d.mode = MOVE_APPEND; d.n_out = (int)T; d.out_off = cache->off[u];
    }
    descs[u] = d;
  }
  a.N_k = N_k;
  a.n_obs = std::min(ctx->cfg.n_obs, N_k);
  int32_t rows[kMaxObs];
  fill_q_rows(nullptr, a.n_obs, N_k, rows);
  a.split = use_split_attention(ctx, U, N_k);
  a.fuse_append = a.split && n_comp == 0;   // no unit compresses: the attention launch appends as well
  a.tile = a.split ? attn_split_q_tile_rows() : attn_q_tile_rows(ctx->cfg.dtype, ctx->cfg.head_dim, U, N_k);
  a.q = q; a.k_new = k_new; a.v_new = v_new; a.out = out; a.scale = scale;
  a.cp = CachePtrs{cache->k, cache->v, cache->pos};
  a.pos_new = (int32_t)cache->tokens_seen;

  // group 0: the caller's stream; group 1 (optional): the compressing contextual units, beside group 0's attention
  const bool two_groups = ctx->step_overlap && ctx->cfg.dtype == HACK_BF16 && n_side > 0 && n_side < U;
  a.shared = two_groups;
  StepGroup g[2];
  g[0].two_pass = ctx->score_mode == HACK_SCORE_TWO_PASS;
  g[0].slots = ctx->rowstat;
  g[1].two_pass = true;          // leaves its sums in the slots, hence an exchange area of its own
  g[1].slots = ctx->rowstat_side;
  for (int u = 0; u < U; ++u) {
    const bool ctxl = head_type[u % H] == HACK_CONTEXTUAL, compresses = descs[u].mode == MOVE_GATHER;
    add_unit(&g[two_groups && ctxl && compresses ? 1 : 0], descs[u], final_merge && ctxl && compresses, N_k);
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if ((st = upload_group(ctx, &g[0], a, rows, s)) != HACK_OK) return st;
  if (two_groups && (st = upload_group(ctx, &g[1], a, rows, s)) != HACK_OK) return st;

  launch_chain(ctx, g[0], a, s);
  if (two_groups) {
    HIP_TRY(ctx, hipEventRecord(ctx->ev_fork, s));
    HIP_TRY(ctx, hipStreamWaitEvent(ctx->aux_stream, ctx->ev_fork, 0));
  }
  launch_group_attention(ctx, g[0], a, s);
  if (two_groups) {
    launch_chain(ctx, g[1], a, ctx->aux_stream);
    launch_group_attention(ctx, g[1], a, ctx->aux_stream);
    HIP_TRY(ctx, hipEventRecord(ctx->ev_join, ctx->aux_stream));
    HIP_TRY(ctx, hipStreamWaitEvent(s, ctx->ev_join, 0));
  }
  HIP_TRY(ctx, hipGetLastError());

  for (int u = 0; u < U; ++u) {
    if (descs[u].mode == MOVE_GATHER) {
      cache->cur[u] ^= 1;
      cache->off[u] = cache->slab[cache->cur[u]][u];
    }
    cache->len[u] = descs[u].n_out;
  }
  cache->tokens_seen += N_k;
  return HACK_OK;
}

extern "C" hack_status hack_step(hack_ctx* ctx, hack_kvcache* cache, int32_t B, int32_t N_k, const void* q,
                                 const void* k_new, const void* v_new, const uint8_t* head_type,
                                 const int32_t* budget, int32_t n_init, float scale, void* out,
                                 int32_t* kept_idx_opt, int64_t idx_stride, hack_stream stream) {
  return step_impl(ctx, cache, B, N_k, q, k_new, v_new, head_type, budget, n_init, scale, out, kept_idx_opt, idx_stride,
                   stream, false);
}

extern "C" hack_status hack_step_final(hack_ctx* ctx, hack_kvcache* cache, int32_t B, int32_t N_k, const void* q,
                                       const void* k_new, const void* v_new, const uint8_t* head_type,
                                       const int32_t* budget, int32_t n_init, float scale, void* out,
                                       int32_t* kept_idx_opt, int64_t idx_stride, hack_stream stream) {
  return step_impl(ctx, cache, B, N_k, q, k_new, v_new, head_type, budget, n_init, scale, out, kept_idx_opt, idx_stride,
                   stream, true);
}
