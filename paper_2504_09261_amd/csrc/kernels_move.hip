// Row movement for the ragged per-unit KV cache on gfx950: the cache-update
// concatenation (Preliminaries, cache update equation) for units that do not
// compress, and the gather K^ = K[I,:], V^ = V[I,:] (Sec. 4.4) for units that do.
// Pure 16-byte vector copies: HBM-bound and bit-exact by construction.
#include "hack_internal.h"

namespace hack {

namespace {

constexpr int kThreads = 256;
constexpr int kRowsInFlight = 8;  // independent row copies per lane group

// LPR = 16-byte lanes per row (row_bytes / 16).
template <int LPR>
__global__ __launch_bounds__(kThreads) void move_kernel(
    const UnitDesc* __restrict__ descs, CachePtrs in, CachePtrs out, const uint4* __restrict__ k_new,
    const uint4* __restrict__ v_new, int N_k, int pos_new, const int32_t* __restrict__ kept_idx,
    int64_t idx_stride) {
  const UnitDesc d = descs[blockIdx.y];
  if (d.mode == MOVE_NONE) return;
  constexpr int GROUPS = kThreads / LPR;
  constexpr int ROWS_PER_BLOCK = GROUPS * kRowsInFlight;
  const int n_rows = (d.mode == MOVE_APPEND) ? d.n_new : d.n_out;
  const int row0 = blockIdx.x * ROWS_PER_BLOCK;
  if (row0 >= n_rows) return;
  const int g = threadIdx.x / LPR;
  const int lane = threadIdx.x % LPR;

  const uint4* kin = static_cast<const uint4*>(in.k);
  const uint4* vin = static_cast<const uint4*>(in.v);
  uint4* kout = static_cast<uint4*>(out.k);
  uint4* vout = static_cast<uint4*>(out.v);
  const int64_t new_base = (int64_t)d.unit * N_k;
  const int32_t* idx = kept_idx ? kept_idx + (int64_t)d.unit * idx_stride : nullptr;
  const bool with_pos = (out.pos != nullptr);

  // Phase 1: source row of every in-flight copy (one dependent index load each),
  // clamped to a valid row so that phase 2 can load without branches.
  int s[kRowsInFlight];
  bool live[kRowsInFlight];
#pragma unroll
  for (int r = 0; r < kRowsInFlight; ++r) {
    const int i = row0 + r * GROUPS + g;
    live[r] = i < n_rows;
    const int ic = live[r] ? i : n_rows - 1;
    s[r] = (d.mode == MOVE_APPEND) ? d.len_in + ic : idx[ic];
  }
  // Phase 2: all loads in flight before the first store.
  uint4 kr[kRowsInFlight], vr[kRowsInFlight];
  int32_t pr[kRowsInFlight];
#pragma unroll
  for (int r = 0; r < kRowsInFlight; ++r) {
    const bool from_cache = s[r] < d.len_in;
    const int64_t src = from_cache ? d.in_off + s[r] : new_base + (s[r] - d.len_in);
    const uint4* kp = from_cache ? kin : k_new;
    const uint4* vp = from_cache ? vin : v_new;
    kr[r] = kp[src * LPR + lane];
    vr[r] = vp[src * LPR + lane];
    pr[r] = pos_new + (s[r] - d.len_in);
    if (with_pos && from_cache && in.pos) pr[r] = in.pos[src];
  }
  const int64_t dst0 = (d.mode == MOVE_APPEND) ? d.in_off + d.len_in : d.out_off;
#pragma unroll
  for (int r = 0; r < kRowsInFlight; ++r) {
    if (live[r]) {
      const int64_t dst = dst0 + row0 + r * GROUPS + g;
      kout[dst * LPR + lane] = kr[r];
      vout[dst * LPR + lane] = vr[r];
      if (with_pos && lane == 0) out.pos[dst] = pr[r];
    }
  }
}

template <int LPR>
void launch_t(hipStream_t s, const UnitDesc* descs, int n_desc, int max_rows, CachePtrs in,
              CachePtrs out, const void* k_new, const void* v_new, int N_k, int pos_new,
              const int32_t* kept_idx, int64_t idx_stride) {
  constexpr int ROWS_PER_BLOCK = (kThreads / LPR) * kRowsInFlight;
  dim3 grid((max_rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK, n_desc);
  hipLaunchKernelGGL(move_kernel<LPR>, grid, dim3(kThreads), 0, s, descs, in, out,
                     static_cast<const uint4*>(k_new), static_cast<const uint4*>(v_new), N_k,
                     pos_new, kept_idx, idx_stride);
}

}  // namespace

void launch_move(hipStream_t s, int elem_bytes, int head_dim, const UnitDesc* descs, int n_desc,
                 int max_rows, CachePtrs in, CachePtrs out, const void* k_new, const void* v_new,
                 int N_k, int pos_new, const int32_t* kept_idx, int64_t idx_stride) {
  if (n_desc <= 0 || max_rows <= 0) return;
  const int lpr = elem_bytes * head_dim / 16;
  switch (lpr) {
    case 8: launch_t<8>(s, descs, n_desc, max_rows, in, out, k_new, v_new, N_k, pos_new, kept_idx, idx_stride); break;
    case 16: launch_t<16>(s, descs, n_desc, max_rows, in, out, k_new, v_new, N_k, pos_new, kept_idx, idx_stride); break;
    case 32: launch_t<32>(s, descs, n_desc, max_rows, in, out, k_new, v_new, N_k, pos_new, kept_idx, idx_stride); break;
    default: break;  // excluded by hack_create
  }
}

}  // namespace hack
