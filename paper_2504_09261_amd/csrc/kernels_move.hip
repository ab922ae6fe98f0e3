// Row movement for the ragged per-unit KV cache on gfx950: the cache-update
// concatenation (Preliminaries, cache update equation) for units that do not
// compress, and the gather K^ = K[I,:], V^ = V[I,:] (Sec. 4.4) for units that do.
// Pure 16-byte vector copies: HBM-bound and bit-exact by construction.
#include "hack_internal.h"

namespace hack {

namespace {

// One 16-byte piece of one K row and of one V row per thread, no loop: many
// small work-groups whose load and store phases interleave freely keep reads
// and writes both flowing, which measured about 1.7x faster on the gather than
// work-groups that hold several rows per lane in flight and then store them
// all (a read burst followed by a write burst).
constexpr int kThreads = 512;

// LPR = 16-byte lanes per row (row_bytes / 16).
template <int LPR>
__global__ __launch_bounds__(kThreads) void move_kernel(
    const UnitDesc* __restrict__ descs, CachePtrs in, CachePtrs out, const uint4* __restrict__ k_new,
    const uint4* __restrict__ v_new, int N_k, int pos_new, const int32_t* __restrict__ kept_idx,
    int64_t idx_stride) {
  const UnitDesc d = descs[blockIdx.y];
  if (d.mode == MOVE_NONE) return;
  constexpr int ROWS_PER_BLOCK = kThreads / LPR;
  const int n_rows = (d.mode == MOVE_APPEND) ? d.n_new : d.n_out;
  const int i = blockIdx.x * ROWS_PER_BLOCK + threadIdx.x / LPR;
  if (i >= n_rows) return;
  const int lane = threadIdx.x % LPR;

  // source row in the virtual concatenation [cached rows | new rows]
  const int s = (d.mode == MOVE_APPEND) ? d.len_in + i : kept_idx[(int64_t)d.unit * idx_stride + i];
  const bool from_cache = s < d.len_in;
  const int64_t src = from_cache ? d.in_off + s : (int64_t)d.unit * N_k + (s - d.len_in);
  const uint4* kp = from_cache ? static_cast<const uint4*>(in.k) : k_new;
  const uint4* vp = from_cache ? static_cast<const uint4*>(in.v) : v_new;
  const uint4 kr = kp[src * LPR + lane];
  const uint4 vr = vp[src * LPR + lane];
  const int64_t dst = ((d.mode == MOVE_APPEND) ? d.in_off + d.len_in : d.out_off) + i;
  static_cast<uint4*>(out.k)[dst * LPR + lane] = kr;
  static_cast<uint4*>(out.v)[dst * LPR + lane] = vr;
  if (out.pos != nullptr && lane == 0)
    out.pos[dst] = (from_cache && in.pos) ? in.pos[src] : pos_new + (s - d.len_in);
}

template <int LPR>
void launch_t(hipStream_t s, const UnitDesc* descs, int n_desc, int max_rows, CachePtrs in,
              CachePtrs out, const void* k_new, const void* v_new, int N_k, int pos_new,
              const int32_t* kept_idx, int64_t idx_stride) {
  constexpr int ROWS_PER_BLOCK = kThreads / LPR;
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
