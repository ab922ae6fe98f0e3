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

}  // namespace hack
