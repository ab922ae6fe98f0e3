// Budgeted selection (Sec. 4.4, f_C and f_S) on gfx950.
//
// One work-group per unit.  The host has already turned (head class, budget,
// N_init, N_k) into: rows [0, keep_a) and [keep_b, T) kept unconditionally and
// the sel_m most important rows of the ranked segment [sel_lo, sel_hi).
// The ranked segment is resolved with an LDS-resident radix select (4 passes of
// 8 bits over order-preserving uint32 keys) that yields the exact threshold
// value tau and how many rows equal to tau are still needed; an index-ordered
// prefix scan then emits kept rows in ascending order, taking the tau-equal
// rows with the lowest indices first (lowest-index tie-break for free).
#include <mutex>

#include "hack_internal.h"

namespace hack {

namespace {

// Work-group size: 1024 threads for long units, 256 for short ones (template parameter).  A unit of a few
// hundred keys leaves most of 1024 threads idle at every barrier, and a launch over many short units (the
// 256^2 schedules: hundreds of units of at most ~600 keys) then needs several rounds of work-groups.
constexpr int kThreadsLong = 1024;
constexpr int kThreadsShort = 256;
constexpr int kShortMaxKeys = 1024;   // units up to this many keys take the short form

__device__ __forceinline__ uint32_t orderable(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int wave_inclusive_scan(int v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int t = __shfl_up(v, o, 64);
    if (lane >= o) v += t;
  }
  return v;
}

// Exclusive prefix of v over the work-group in thread order; total to all threads.
template <int kWaves>
__device__ __forceinline__ int block_exclusive_scan(int v, int* wave_tot, int& total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int incl = wave_inclusive_scan(v);
  __syncthreads();  // wave_tot may still be read from a previous scan
  if (lane == 63) wave_tot[w] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kWaves; ++i) {
    const int t = wave_tot[i];
    if (i < w) base += t;
    tot += t;
  }
  total = tot;
  return base + incl - v;
}

template <int kThreads>
__global__ __launch_bounds__(kThreads) void select_kernel(
    const UnitDesc* __restrict__ descs, const int32_t* __restrict__ list,
    const float* __restrict__ importance, int64_t imp_stride, int32_t* __restrict__ kept_idx,
    int64_t idx_stride) {
  constexpr int kWaves = kThreads / 64;
  extern __shared__ uint32_t keys[];  // ranked segment as orderable keys
  __shared__ uint32_t hist[256];
  __shared__ int wave_tot[kWaves];
  __shared__ uint32_t s_bin;
  __shared__ int s_want;
  __shared__ int s_eq;    // candidates in the chosen bin (after the last pass: keys equal to the threshold)

  const UnitDesc d = descs[list[blockIdx.x]];
  const float* imp = importance + (int64_t)d.unit * imp_stride;
  int32_t* out = kept_idx + (int64_t)d.unit * idx_stride;
  const int T = d.len_in + d.n_new;
  const int n_sel = d.sel_hi - d.sel_lo;
  const int tid = threadIdx.x;

  for (int i = tid; i < n_sel; i += kThreads) keys[i] = orderable(imp[d.sel_lo + i]);

  // ---- threshold of the ranked segment ----
  const bool take_all = (d.sel_m >= n_sel);
  const bool take_none = (d.sel_m <= 0);
  uint32_t tau = 0;
  int want = d.sel_m;  // rows still to take among the candidates matching the prefix
  if (!take_all && !take_none) {
    uint32_t prefix = 0, mask = 0;
    for (int shift = 24; shift >= 0; shift -= 8) {
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      if (shift == 24) {
        // Importance values of one unit mostly share sign and exponent, so in the first pass nearly all
        // keys fall into a handful of bins and per-lane LDS atomics would serialise on them: a wave
        // counts its lanes per distinct bin first (a few rounds) and adds once per bin.
        for (int i0 = 0; i0 < n_sel; i0 += kThreads) {
          const int i = i0 + tid;
          const bool valid = i < n_sel;
          const uint32_t bin = valid ? (keys[i] >> 24) : 0u;
          unsigned long long todo = __ballot(valid);
          while (todo) {
            const uint32_t b0 = __shfl(bin, __builtin_ctzll(todo), 64);
            const unsigned long long same = __ballot(valid && bin == b0);
            if ((tid & 63) == __builtin_ctzll(same)) atomicAdd(&hist[b0], (uint32_t)__builtin_popcountll(same));
            todo &= ~same;
          }
        }
      } else {
        for (int i = tid; i < n_sel; i += kThreads) {
          const uint32_t k = keys[i];
          if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1u);
        }
      }
      __syncthreads();
      if (tid < 64) {
        // lane l owns bins 255-4l .. 252-4l, i.e. bins in descending order over lanes
        int c[4];
        int tot = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          c[e] = (int)hist[255 - 4 * tid - e];
          tot += c[e];
        }
        int running = wave_inclusive_scan(tot) - tot;  // candidates in strictly larger bins
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (running < want && want <= running + c[e]) {
            s_bin = (uint32_t)(255 - 4 * tid - e);
            s_want = want - running;
            s_eq = c[e];
          }
          running += c[e];
        }
      }
      __syncthreads();
      prefix |= s_bin << shift;
      mask |= 255u << shift;
      want = s_want;
      // hist is cleared after the next barrier pair; s_bin/s_want are rewritten
      // only after every thread has passed the barrier below the histogram loop.
    }
    tau = prefix;
  }

  // ---- ordered emission ----
  const int per = (T + kThreads - 1) / kThreads;
  const int j0 = min(tid * per, T), j1 = min(j0 + per, T);

  // The rank of a threshold-equal row among its equals (lowest index first) only
  // matters if some of them are left out; usually the threshold value occurs
  // once and is taken, and the first block scan can be skipped.
  const bool all_equal_kept = take_all || take_none || (want >= s_eq);
  int eq_rank = 0;
  if (!all_equal_kept) {
    int n_eq = 0;
    const int a = max(j0, d.sel_lo), b = min(j1, d.sel_hi);
    for (int j = a; j < b; ++j) n_eq += (keys[j - d.sel_lo] == tau);
    int tot_eq;
    eq_rank = block_exclusive_scan<kWaves>(n_eq, wave_tot, tot_eq);
  }

  auto kept = [&](int j, int& eq_seen) -> bool {
    if (j < d.keep_a || j >= d.keep_b) return true;
    if (j < d.sel_lo || j >= d.sel_hi) return false;
    if (take_all) return true;
    if (take_none) return false;
    const uint32_t k = keys[j - d.sel_lo];
    if (k > tau) return true;
    if (k == tau) return all_equal_kept || (eq_seen++) < want;
    return false;
  };

  int cnt = 0, e = eq_rank;
  for (int j = j0; j < j1; ++j) cnt += kept(j, e) ? 1 : 0;
  int total;
  int pos = block_exclusive_scan<kWaves>(cnt, wave_tot, total);
  e = eq_rank;
  for (int j = j0; j < j1; ++j)
    if (kept(j, e)) out[pos++] = j;
}

}  // namespace

size_t select_lds_bytes(int max_t_in) { return (size_t)max_t_in * sizeof(uint32_t); }

void launch_select(hipStream_t s, const UnitDesc* descs, const int32_t* list, int n_list,
                   int max_t_in, const float* importance, int64_t imp_stride, int32_t* kept_idx,
                   int64_t idx_stride) {
  if (n_list <= 0) return;
  const size_t lds = select_lds_bytes(max_t_in);
  if (lds > 48 * 1024) {
    // larger dynamic LDS has to be allowed once per device: raise the limit to the largest unit the library
    // supports the first time a device needs it
    static std::mutex mu;
    static bool configured[64] = {};
    int dev = -1;
    if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64) {
      std::lock_guard<std::mutex> lock(mu);
      if (!configured[dev]) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel<kThreadsLong>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)select_lds_bytes(32768));
        configured[dev] = true;
      }
    }
  }
  if (max_t_in <= kShortMaxKeys)
    hipLaunchKernelGGL(select_kernel<kThreadsShort>, dim3(n_list), dim3(kThreadsShort), lds, s, descs, list, importance,
                       imp_stride, kept_idx, idx_stride);
  else
    hipLaunchKernelGGL(select_kernel<kThreadsLong>, dim3(n_list), dim3(kThreadsLong), lds, s, descs, list, importance,
                       imp_stride, kept_idx, idx_stride);
}

}  // namespace hack
