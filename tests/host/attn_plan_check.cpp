// Host check of the streamed-attention planner: every 32-key block of every work item
// is served exactly once, the parts of a cut work item are numbered consistently, and
// the work-groups get equal work.  No GPU involved.
#include <cstdio>
#include <cstdlib>
#include <cmath>
#include <map>
#include <random>
#include <vector>

#include "../../paper_2504_09261_amd/csrc/attn_plan.h"

using namespace hack;

static int failures = 0;
#define CHECK(c)                                                        \
  do {                                                                  \
    if (!(c)) { std::printf("FAILED line %d: %s\n", __LINE__, #c); ++failures; } \
  } while (0)

static void check_plan(const std::vector<int32_t>& n_keys, int tiles, int slots, int overhead, int min_blocks,
                       bool expect_balanced) {
  AttnStreamPlan p;
  plan_attn_stream(n_keys.data(), (int)n_keys.size(), tiles, slots, overhead, min_blocks, &p);
  CHECK(p.n_groups % kAttnXcds == 0 && p.n_groups >= 1);
  CHECK((int)p.seg_begin.size() == p.n_groups + 1 && p.seg_begin[0] == 0 && p.seg_begin.back() == (int)p.segs.size());
  for (int g = 0; g < p.n_groups; ++g) CHECK(p.seg_begin[g] <= p.seg_begin[g + 1]);
  CHECK(p.n_groups <= (slots + kAttnXcds - 1) / kAttnXcds * kAttnXcds);
  CHECK(p.n_parts <= 2 * p.n_groups && p.n_counters <= p.n_groups);
  // coverage: per work item the segments tile [0, blocks) without gap or overlap
  std::map<std::pair<int, int>, std::vector<AttnSeg>> by_item;
  for (const AttnSeg& s : p.segs) by_item[{s.desc, s.q_tile}].push_back(s);
  CHECK((int)by_item.size() == (int)n_keys.size() * tiles);
  std::vector<int> part_used(p.n_parts, 0), counter_used(p.n_counters, 0);
  for (auto& kv : by_item) {
    std::vector<AttnSeg> v = kv.second;
    std::sort(v.begin(), v.end(), [](const AttnSeg& a, const AttnSeg& b) { return a.blk0 < b.blk0; });
    const int nb = (n_keys[kv.first.first] + 31) / 32;
    int at = 0;
    for (size_t i = 0; i < v.size(); ++i) {
      CHECK(v[i].blk0 == at && v[i].blk1 > v[i].blk0);
      at = v[i].blk1;
      if (v.size() == 1) {
        CHECK(v[i].part < 0);
      } else {
        CHECK(v[i].n_parts == (int)v.size() && v[i].first_part == v[0].first_part && v[i].counter == v[0].counter);
        CHECK(v[i].part == v[i].first_part + (int)i);
        CHECK(v[i].part >= 0 && v[i].part < p.n_parts);
        if (v[i].part >= 0 && v[i].part < p.n_parts) ++part_used[v[i].part];
        CHECK(v[i].blk1 - v[i].blk0 >= std::min(min_blocks, nb));
      }
    }
    CHECK(at == nb);
    if (v.size() > 1) {
      CHECK(v[0].counter >= 0 && v[0].counter < p.n_counters);
      if (v[0].counter >= 0 && v[0].counter < p.n_counters) ++counter_used[v[0].counter];
    }
  }
  for (int u : part_used) CHECK(u == 1);
  for (int u : counter_used) CHECK(u == 1);
  // a work-group never holds two segments of one work item
  for (int g = 0; g < p.n_groups; ++g)
    for (int a = p.seg_begin[g]; a < p.seg_begin[g + 1]; ++a)
      for (int b = a + 1; b < p.seg_begin[g + 1]; ++b)
        CHECK(!(p.segs[a].desc == p.segs[b].desc && p.segs[a].q_tile == p.segs[b].q_tile));
  if (expect_balanced) {
    int64_t lo = INT64_MAX, hi = 0, total = 0;
    int busy = 0;
    for (int g = 0; g < p.n_groups; ++g) {
      int64_t w = 0;
      for (int a = p.seg_begin[g]; a < p.seg_begin[g + 1]; ++a) w += p.segs[a].blk1 - p.segs[a].blk0 + overhead;
      if (w > 0) { lo = std::min(lo, w); hi = std::max(hi, w); total += w; ++busy; }
    }
    CHECK(busy >= slots - 8);
    const double mean = (double)total / busy;
    if (!(hi <= mean + 2 * min_blocks + overhead && lo >= mean - 2 * min_blocks - overhead))
      std::printf("  balance: lo %lld hi %lld mean %.1f\n", (long long)lo, (long long)hi, mean);
    CHECK(hi <= mean + 2 * min_blocks + overhead && lo >= mean - 2 * min_blocks - overhead);
  }
}

// plan_attn_cuts: validity of the plan (every block once, parts numbered consistently, one segment per
// work-group, lanes kept apart) and what the model promises.
static bool check_cuts(const std::vector<int32_t>& n_keys, int tiles, int cus_per_xcd, double min_gain, double* gain) {
  const AttnPairModel m{0.55, 0.75, 1.0, 4.0, 14.0};
  // lanes as the library deals them: units by decreasing length to the least loaded XCD, tiles adjacent
  std::vector<int> order(n_keys.size());
  for (size_t i = 0; i < order.size(); ++i) order[i] = (int)i;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return n_keys[a] > n_keys[b]; });
  std::vector<AttnLaneItem> lanes[kAttnXcds];
  long load[kAttnXcds] = {0};
  for (int u : order) {
    int x = 0;
    for (int i = 1; i < kAttnXcds; ++i) if (load[i] < load[x]) x = i;
    load[x] += (long)n_keys[u] * tiles;
    for (int t = 0; t < tiles; ++t) lanes[x].push_back(AttnLaneItem{u, t, (n_keys[u] + 31) / 32});
  }
  AttnStreamPlan p;
  double before = 0, after = 0;
  const bool ok = plan_attn_cuts(lanes, cus_per_xcd, 8, m, min_gain, &p, &before, &after);
  *gain = before > 0 ? 1.0 - after / before : 0.0;
  if (!ok) return false;
  CHECK(after < before && after <= (1.0 - min_gain) * before);
  CHECK(p.n_groups % kAttnXcds == 0 && (int)p.seg_begin.size() == p.n_groups + 1);
  CHECK(p.n_groups <= 2 * cus_per_xcd * kAttnXcds);                      // still a single round
  CHECK(p.n_counters > 0 && p.n_parts >= 2 * p.n_counters);
  std::map<std::pair<int, int>, std::vector<AttnSeg>> by_item;
  for (int g = 0; g < p.n_groups; ++g) {
    CHECK(p.seg_begin[g + 1] - p.seg_begin[g] <= 1);                      // one segment per work-group
    for (int a = p.seg_begin[g]; a < p.seg_begin[g + 1]; ++a) {
      const AttnSeg& s = p.segs[a];
      by_item[{s.desc, s.q_tile}].push_back(s);
      // an item stays on the XCD the library dealt it to
      bool found = false;
      for (const AttnLaneItem& li : lanes[g % kAttnXcds]) found = found || (li.desc == s.desc && li.q_tile == s.q_tile);
      CHECK(found);
    }
  }
  CHECK(by_item.size() == n_keys.size() * (size_t)tiles);
  std::vector<int> part_used(p.n_parts, 0);
  for (auto& kv : by_item) {
    std::vector<AttnSeg> v = kv.second;
    std::sort(v.begin(), v.end(), [](const AttnSeg& a, const AttnSeg& b) { return a.blk0 < b.blk0; });
    const int nb = (n_keys[kv.first.first] + 31) / 32;
    int at = 0;
    for (size_t i = 0; i < v.size(); ++i) {
      CHECK(v[i].blk0 == at && v[i].blk1 > v[i].blk0);
      at = v[i].blk1;
      if (v.size() == 1) { CHECK(v[i].part < 0); continue; }
      CHECK(v[i].blk1 - v[i].blk0 >= 8);
      CHECK(v[i].n_parts == (int)v.size() && v[i].first_part == v[0].first_part && v[i].counter == v[0].counter);
      CHECK(v[i].part == v[i].first_part + (int)i && v[i].part < p.n_parts);
      if (v[i].part >= 0 && v[i].part < p.n_parts) ++part_used[v[i].part];
    }
    CHECK(at == nb || (v.size() == 1 && v[0].blk1 >= nb));
  }
  for (int u : part_used) CHECK(u == 1);
  return true;
}

int main() {
  {
    const AttnPairModel m{0.55, 0.75, 1.0, 4.0, 14.0};
    // alone; the second one ends first; the first one ends first
    CHECK(std::fabs(attn_pair_time(100, 0, m) - 55.0) < 1e-9);
    CHECK(std::fabs(attn_pair_time(120, 60, m) - (60.0 + 0.55 * (120 - 80))) < 1e-9);
    CHECK(std::fabs(attn_pair_time(100, 100, m) - (75.0 + 0.55 * 25)) < 1e-9);
    double gain = 0;
    // scale step 11 of the benchmark workload: 20 units of 3885 keys, 12 of 1943, 13 query tiles: more long
    // items than compute units, so some compute units hold two of them until those are halved
    std::vector<int32_t> n;
    for (int u = 0; u < 32; ++u) n.push_back(u % 16 < 6 ? 1943 : 3885);
    CHECK(check_cuts(n, 13, 32, 0.05, &gain) && gain > 0.1);
    // the last scale step (32 tiles: 1024 items) does not fit the device at once: left alone
    CHECK(!check_cuts(n, 32, 32, 0.05, &gain));
    // one work item per compute unit at most and equal lengths: nothing to gain from halving all of them
    std::vector<int32_t> eq(32, 1497);
    CHECK(!check_cuts(eq, 8, 32, 0.05, &gain));
    std::mt19937 rng(777);
    int fired = 0;
    for (int rep = 0; rep < 200; ++rep) {
      const int n_desc = 1 + rng() % 48, tiles = 1 + rng() % 6, cus = 1 + rng() % 32;
      std::vector<int32_t> v(n_desc);
      for (int& x : v) x = 1 + rng() % 8000;
      fired += check_cuts(v, tiles, cus, rep % 2 ? 0.05 : 1e-9, &gain) ? 1 : 0;
    }
    CHECK(fired > 20);
  }

  // the benchmark workload's large steps: 12 units of 1943 keys, 20 of 3885 (2521 at the first), tiles 5 .. 32
  for (int tiles : {5, 8, 13, 18, 32}) {
    std::vector<int32_t> n;
    for (int u = 0; u < 32; ++u) n.push_back(u % 16 < 6 ? 1943 : (tiles == 8 ? 2521 : 3885));
    check_plan(n, tiles, 512, 4, 4, true);
  }
  check_plan({10521, 10521, 7, 33}, 32, 512, 4, 4, true);   // very unequal units
  check_plan({1}, 1, 512, 4, 4, false);                     // a single block
  check_plan({64}, 1, 512, 0, 1, false);
  check_plan({320, 320, 320}, 2, 768, 4, 4, false);         // fewer blocks than work-group slots
  std::mt19937 rng(12345);
  for (int rep = 0; rep < 300; ++rep) {
    const int n_desc = 1 + rng() % 40, tiles = 1 + rng() % 9, slots = 8 * (1 + rng() % 96);
    std::vector<int32_t> n(n_desc);
    for (int& x : n) x = 1 + rng() % (rep % 3 == 0 ? 200 : 6000);
    check_plan(n, tiles, slots, rng() % 7, 1 + rng() % 8, false);
  }
  std::printf(failures ? "%d failures\n" : "ok\n", failures);
  return failures ? 1 : 0;
}
