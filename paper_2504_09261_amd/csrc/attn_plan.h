// Host-side planning of the streamed bf16 attention launch (plain C++, no HIP):
// the work items (unit, tile of 128 queries) of a launch are laid end to end, longest
// units first, and the line is cut into as many runs of 32-key blocks as the device
// holds work-groups at once, so that every work-group gets the same amount of work
// whatever the lengths of the units are.  A work item that a cut falls into is served
// by several work-groups; their partial results are added up by whichever of them
// finishes last (see the kernel).
#pragma once

#include <stdint.h>

#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

namespace hack {

// One segment: the 32-key blocks [blk0, blk1) of the work item (desc, q_tile).
// part < 0: the segment is the whole work item.  Otherwise the work item is cut into
// n_parts segments whose partial results occupy the slots first_part .. first_part +
// n_parts - 1 (this one: part) and which share the ticket counter `counter`.
struct AttnSeg {
  int32_t desc;
  int32_t q_tile;
  int32_t blk0;
  int32_t blk1;
  int32_t part;
  int32_t first_part;
  int32_t n_parts;
  int32_t counter;
};
static_assert(sizeof(AttnSeg) == 32, "AttnSeg must stay 32 bytes");

struct AttnStreamPlan {
  std::vector<AttnSeg> segs;         // in work-group order
  std::vector<int32_t> seg_begin;    // [n_groups + 1]: work-group g serves segs[seg_begin[g] .. seg_begin[g+1])
  int n_groups = 0;                  // work-groups to launch (a multiple of 8)
  int n_parts = 0;                   // partial-result slots used
  int n_counters = 0;                // ticket counters used (= work items that were cut)
};

constexpr int kAttnKeyBlock = 32;    // keys per block
constexpr int kAttnXcds = 8;         // work-group ids go round-robin over this many XCDs

// n_keys[i]: keys of unit descriptor i; tiles: query tiles per unit; slots: work-groups the
// device holds at once; overhead_blocks: what starting and finishing a segment costs, in
// blocks; min_blocks: no segment is shorter than this unless its whole work item is.
// Consecutive runs go to the same XCD (work-group id % 8), so the tiles of a unit, which
// share its K/V, mostly meet in one L2.
inline void plan_attn_stream(const int32_t* n_keys, int n_desc, int tiles, int slots, int overhead_blocks,
                             int min_blocks, AttnStreamPlan* plan) {
  plan->segs.clear();
  plan->seg_begin.assign(1, 0);
  plan->n_groups = plan->n_parts = plan->n_counters = 0;
  if (n_desc <= 0 || tiles <= 0 || slots <= 0) return;
  min_blocks = std::max(1, min_blocks);
  std::vector<int> order(n_desc);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return n_keys[a] > n_keys[b]; });
  // work items in line order; blk_cum / work_cum: blocks / work before item i
  const int64_t n_items = (int64_t)n_desc * tiles;
  std::vector<int64_t> blk_cum(n_items + 1, 0), work_cum(n_items + 1, 0);
  for (int64_t i = 0; i < n_items; ++i) {
    const int nb = (n_keys[order[i / tiles]] + kAttnKeyBlock - 1) / kAttnKeyBlock;
    blk_cum[i + 1] = blk_cum[i] + nb;
    work_cum[i + 1] = work_cum[i] + nb + overhead_blocks;
  }
  const int64_t total_blocks = blk_cum[n_items], W = work_cum[n_items];
  if (total_blocks <= 0) return;
  const int G = (int)std::max<int64_t>(1, std::min<int64_t>(slots, W / (min_blocks + overhead_blocks)));
  // cut j (1 <= j < G) in global block coordinates
  std::vector<int64_t> cut(G + 1, 0);
  cut[G] = total_blocks;
  int64_t it = 0;
  for (int j = 1; j < G; ++j) {
    const double x = (double)W * j / G;
    while (it + 1 < n_items && (double)work_cum[it + 1] <= x) ++it;
    const int64_t nb = blk_cum[it + 1] - blk_cum[it];
    int64_t b = (int64_t)std::llround(x - (double)work_cum[it] - 0.5 * overhead_blocks);
    b = std::max<int64_t>(0, std::min<int64_t>(nb, b));
    if (b < min_blocks) b = 0;
    else if (nb - b < min_blocks) b = nb;
    cut[j] = std::max(cut[j - 1], blk_cum[it] + b);
  }
  // parts per work item: how many runs hold blocks of it
  std::vector<int32_t> first_part(n_items, -1), n_parts(n_items, 0), counter(n_items, -1), seen(n_items, 0);
  {
    int64_t i = 0;
    for (int j = 0; j < G; ++j) {
      int64_t p = cut[j];
      while (p < cut[j + 1]) {
        while (blk_cum[i + 1] <= p) ++i;
        ++n_parts[i];
        p = std::min(cut[j + 1], blk_cum[i + 1]);
      }
    }
    for (i = 0; i < n_items; ++i) {
      if (n_parts[i] > 1) {
        first_part[i] = plan->n_parts;
        plan->n_parts += n_parts[i];
        counter[i] = plan->n_counters++;
      }
    }
  }
  // runs -> work-groups: run j goes to XCD j / per, as that XCD's (j % per)-th work-group
  const int per = (G + kAttnXcds - 1) / kAttnXcds;
  plan->n_groups = per * kAttnXcds;
  std::vector<std::vector<AttnSeg>> of_run(G);
  {
    int64_t i = 0;
    for (int j = 0; j < G; ++j) {
      int64_t p = cut[j];
      while (p < cut[j + 1]) {
        while (blk_cum[i + 1] <= p) ++i;
        const int64_t e = std::min(cut[j + 1], blk_cum[i + 1]);
        AttnSeg s{};
        s.desc = order[i / tiles];
        s.q_tile = (int32_t)(i % tiles);
        s.blk0 = (int32_t)(p - blk_cum[i]);
        s.blk1 = (int32_t)(e - blk_cum[i]);
        if (n_parts[i] > 1) {
          s.part = first_part[i] + seen[i]++;
          s.first_part = first_part[i];
          s.n_parts = n_parts[i];
          s.counter = counter[i];
        } else {
          s.part = -1;
        }
        of_run[j].push_back(s);
        p = e;
      }
    }
  }
  plan->seg_begin.assign(plan->n_groups + 1, 0);
  for (int g = 0; g < plan->n_groups; ++g) {
    const int j = (g % kAttnXcds) * per + g / kAttnXcds;
    if (j < G) plan->segs.insert(plan->segs.end(), of_run[j].begin(), of_run[j].end());
    plan->seg_begin[g + 1] = (int32_t)plan->segs.size();
  }
}

// ---- cutting single work items of a launch that fits the device at once ------------------------
// When a launch has no more work items than the device holds work-groups, every item starts at once
// and the launch lasts as long as its slowest compute unit.  Two work-groups share a compute unit,
// and work-groups are placed one per compute unit first, then a second one each, in launch order
// within an XCD (work-group id % 8); the one that arrived first is served first.  With `solo`,
// `older` and `younger` the time per 32-key block of a work-group alone, of the first and of the
// second of a pair, a compute unit that holds a pieces-long older and a b-long younger work-group
// finishes at pair_time(a, b).  The planner lays an XCD's pieces out so that the largest second
// occupants meet the smallest first occupants, and cuts pieces of the slowest compute unit in two
// while that shortens the modelled launch (each cut costs a pipeline fill, a partial result and its
// share of adding the parts up: ovh_part against ovh_whole, in blocks).
struct AttnPairModel {
  double solo, older, younger;     // us per key block
  double ovh_whole, ovh_part;      // fixed cost of a whole work item / of a piece of a cut one, in key blocks
};

inline double attn_pair_time(double a, double b, const AttnPairModel& m) {
  if (b <= 0) return m.solo * a;
  const double t_old = m.older * a, t_young = m.younger * b;
  if (t_young <= t_old) return t_young + m.solo * (a - t_young / m.older);   // the younger one ends first
  return t_old + m.solo * (b - t_old / m.younger);
}

struct AttnLaneItem {
  int32_t desc, q_tile, n_blocks;
};

namespace attn_plan_detail {
struct Piece {
  int item, b0, b1;
  bool cut;
};
inline double eff(const Piece& p, const AttnPairModel& m) { return (p.b1 - p.b0) + (p.cut ? m.ovh_part : m.ovh_whole); }
// Sorts the pieces by decreasing size and returns the modelled time of the lane and, in *crit, the piece
// to cut next (the second occupant of the slowest compute unit if it can be cut, else the first; -1: none).
inline double lane_time(std::vector<Piece>* L, int cus, int min_blocks, const AttnPairModel& m, int* crit) {
  std::stable_sort(L->begin(), L->end(), [&](const Piece& a, const Piece& b) { return eff(a, m) > eff(b, m); });
  const int n = (int)L->size(), first = std::min(n, cus);
  double worst = -1.0;
  int wa = -1, wb = -1;
  for (int j = 0; j < first; ++j) {           // j-th smallest first occupant, j-th largest second occupant
    const int ia = first - 1 - j, ib = cus + j;
    const double t = attn_pair_time(eff((*L)[ia], m), ib < n ? eff((*L)[ib], m) : 0.0, m);
    if (t > worst) { worst = t; wa = ia; wb = ib < n ? ib : -1; }
  }
  auto cuttable = [&](int i) { return i >= 0 && (*L)[i].b1 - (*L)[i].b0 >= 2 * min_blocks; };
  *crit = cuttable(wb) ? wb : (cuttable(wa) ? wa : -1);
  return worst;
}
}  // namespace attn_plan_detail

// lanes[x]: the work items of XCD x (work-group id % 8 == x) in any order.  Fills *plan (one segment per
// work-group, in the launch order described above) and returns true if cutting shortens the modelled launch
// by at least min_gain (a fraction); *before / *after get the modelled times in us.  Returns false, leaving
// *plan unspecified, when the launch does not fit the device at once or nothing is gained.
inline bool plan_attn_cuts(const std::vector<AttnLaneItem> (&lanes)[kAttnXcds], int cus_per_xcd, int min_blocks,
                           const AttnPairModel& m, double min_gain, AttnStreamPlan* plan, double* before, double* after) {
  using attn_plan_detail::Piece;
  *before = *after = 0.0;
  if (cus_per_xcd <= 0) return false;
  min_blocks = std::max(1, min_blocks);
  for (int x = 0; x < kAttnXcds; ++x)
    if ((int)lanes[x].size() > 2 * cus_per_xcd) return false;
  std::vector<std::vector<Piece>> states[kAttnXcds];   // lane state after k cuts
  std::vector<double> times[kAttnXcds];
  double t0 = 0.0, t_best = 0.0;
  for (int x = 0; x < kAttnXcds; ++x) {
    std::vector<Piece> L;
    for (int i = 0; i < (int)lanes[x].size(); ++i) L.push_back(Piece{i, 0, lanes[x][i].n_blocks, false});
    if (L.empty()) {
      states[x].push_back(L);
      times[x].push_back(0.0);
      continue;
    }
    for (;;) {
      int crit = -1;
      const double t = attn_plan_detail::lane_time(&L, cus_per_xcd, min_blocks, m, &crit);
      states[x].push_back(L);
      times[x].push_back(t);
      if (crit < 0 || (int)L.size() >= 2 * cus_per_xcd) break;
      // all pieces of the item become pieces of a cut item
      const Piece p = L[crit];
      const int mid = p.b0 + (p.b1 - p.b0) / 2;
      for (Piece& q : L) if (q.item == p.item) q.cut = true;
      L[crit] = Piece{p.item, p.b0, mid, true};
      L.push_back(Piece{p.item, mid, p.b1, true});
    }
    t0 = std::max(t0, times[x][0]);
    t_best = std::max(t_best, *std::min_element(times[x].begin(), times[x].end()));
  }
  *before = t0;
  *after = t_best;
  if (!(t_best <= (1.0 - min_gain) * t0) || t_best >= t0) return false;
  // per lane the fewest cuts that reach the launch's best time
  plan->segs.clear();
  plan->n_parts = plan->n_counters = 0;
  std::vector<AttnSeg> out[kAttnXcds];
  bool any_cut = false;
  for (int x = 0; x < kAttnXcds; ++x) {
    size_t k = 0;
    while (times[x][k] > t_best) ++k;
    std::vector<Piece> L = states[x][k];   // sorted by decreasing size
    any_cut = any_cut || k > 0;
    // parts of the cut items, numbered by position inside the item
    const int n_items = (int)lanes[x].size();
    std::vector<std::vector<int>> of_item(n_items);
    for (int i = 0; i < (int)L.size(); ++i) of_item[L[i].item].push_back(i);
    std::vector<AttnSeg> seg(L.size());
    for (int it = 0; it < n_items; ++it) {
      std::vector<int>& v = of_item[it];
      std::sort(v.begin(), v.end(), [&](int a, int b) { return L[a].b0 < L[b].b0; });
      for (size_t j = 0; j < v.size(); ++j) {
        AttnSeg s{};
        s.desc = lanes[x][it].desc;
        s.q_tile = lanes[x][it].q_tile;
        s.blk0 = L[v[j]].b0;
        s.blk1 = L[v[j]].b1;
        if (v.size() > 1) {
          s.part = plan->n_parts + (int)j;
          s.first_part = plan->n_parts;
          s.n_parts = (int)v.size();
          s.counter = plan->n_counters;
        } else {
          s.part = -1;
        }
        seg[v[j]] = s;
      }
      if (v.size() > 1) {
        plan->n_parts += (int)v.size();
        plan->n_counters += 1;
      }
    }
    // launch order: first occupants smallest first, then second occupants largest first
    const int first = std::min((int)L.size(), cus_per_xcd);
    for (int j = 0; j < first; ++j) out[x].push_back(seg[first - 1 - j]);
    for (int j = first; j < (int)L.size(); ++j) out[x].push_back(seg[j]);
  }
  if (!any_cut) return false;
  size_t longest = 0;
  for (int x = 0; x < kAttnXcds; ++x) longest = std::max(longest, out[x].size());
  plan->seg_begin.assign(1, 0);
  for (size_t r = 0; r < longest; ++r)
    for (int x = 0; x < kAttnXcds; ++x) {
      if (r < out[x].size()) plan->segs.push_back(out[x][r]);
      plan->seg_begin.push_back((int32_t)plan->segs.size());
    }
  plan->n_groups = (int)longest * kAttnXcds;
  return true;
}

}  // namespace hack
