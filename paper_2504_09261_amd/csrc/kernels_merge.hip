// Final-step merge of contextual heads (Sec. 4.4, paragraph after the f_C
// equation; supplementary "Compression Setting": only f_C, only the last
// generation step) on gfx950.
//
// The rows a unit discards at its last compression are folded into the rows it
// keeps: every evicted row e goes to its nearest retained counterpart
//     n(e) = argmax_r cos(k_e, k_r)      (r over the kept rows, ties to the lower index)
// with weight w_e = max(cos(k_e, k_n(e)), 0), and every kept row becomes the weighted
// average of itself (weight 1) and the rows that went to it, keys and values alike:
//     K^_r = (k_r + sum_{e: n(e)=r} w_e k_e) / (1 + sum w_e),   V^_r likewise.
// (The paper names the operation and refers to another work for its definition; the
// formulas above are this library's reading of "similarity-weighted averaging into the
// nearest retained counterpart".)
//
// Three launches, after the gather has written K[I], V[I] into the unit's output rows:
//   merge_prep     marks the rows of the uncompressed cache (-1 kept, -2 evicted) and
//                  forms 1/|k_r| of the kept rows;
//   merge_nearest  MFMA pass: a wave holds 32 cache rows (candidates) as the B operand,
//                  the kept keys stream through LDS as the A operand together with
//                  their inverse norms; per lane a running (best, arg-best) over 16
//                  kept rows per block, the lane pair (l, l^32) combined at the end;
//   merge_apply    one wave per kept row: scans the assignment in ascending row order
//                  (so the float32 sums are formed in a fixed order: the result is
//                  reproducible bit for bit) and rewrites the kept row in place.
// bf16 only.  The products of bf16 values are exact in float32; dots accumulate in
// float32 on the matrix core, the averages in float32 on the vector ALU.
#include "device_util.h"
#include "hack_internal.h"

namespace hack {

namespace {

using namespace dev;

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kRing = 4;          // LDS ring slots (32-row blocks of kept keys)
constexpr int kNearTile = kWaves * 32;   // cache rows per work-group in merge_nearest

// One work-group per merging unit.
template <int D>
__global__ __launch_bounds__(kThreads) void merge_prep(
    const UnitDesc* __restrict__ descs, const int32_t* __restrict__ list, const __bf16* __restrict__ k_out,
    const int32_t* __restrict__ kept_idx, int64_t idx_stride, int32_t* __restrict__ nearest,
    float* __restrict__ inv_norm, int64_t ws_stride) {
  const UnitDesc d = descs[list[blockIdx.x]];
  const int T = d.len_in + d.n_new, b = d.n_out;
  int32_t* nn = nearest + (int64_t)d.unit * ws_stride;
  for (int j = threadIdx.x; j < T; j += kThreads) nn[j] = -2;
  __syncthreads();
  const int32_t* kept = kept_idx + (int64_t)d.unit * idx_stride;
  for (int i = threadIdx.x; i < b; i += kThreads) nn[kept[i]] = -1;
  // inverse norms of the kept keys (already gathered into the unit's output rows): 8 lanes per row
  constexpr int CPR = D / 8;
  const int sub = threadIdx.x & 7;
  float* inv = inv_norm + (int64_t)d.unit * ws_stride;
  for (int r0 = 0; r0 < b; r0 += kThreads / 8) {
    const int r = r0 + (threadIdx.x >> 3);
    float ss = 0.f;
    if (r < b) {
      const __bf16* row = k_out + (d.out_off + r) * D;
#pragma unroll
      for (int c = 0; c < CPR / 8; ++c) {
        const bf16x8 x = *reinterpret_cast<const bf16x8*>(row + (sub + 8 * c) * 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) ss = fmaf((float)x[i], (float)x[i], ss);
      }
    }
    ss += __shfl_xor(ss, 1, 64);
    ss += __shfl_xor(ss, 2, 64);
    ss += __shfl_xor(ss, 4, 64);
    if (r < b && sub == 0) inv[r] = ss > 0.f ? 1.f / sqrtf(ss) : 0.f;
  }
}

// Work item = (merging unit, 128 rows of its uncompressed cache): wave w takes rows
// [e0, e0 + 32).  The kept keys K^ (rows [out_off, out_off + b)) stream through LDS.
template <int D>
__global__ __launch_bounds__(kThreads, 2) void merge_nearest(
    const UnitDesc* __restrict__ descs, const int32_t* __restrict__ list, const __bf16* __restrict__ k_in,
    const __bf16* __restrict__ k_new, const __bf16* __restrict__ k_out, int N_k,
    const float* __restrict__ inv_norm, int32_t* __restrict__ nearest, float* __restrict__ weight,
    int64_t ws_stride) {
  using St = BlockStream<D, kWaves>;
  constexpr int KK = D / 16;
  __shared__ __attribute__((aligned(1024))) __bf16 ring[kRing][St::BLK];
  __shared__ __attribute__((aligned(256))) float inv_ring[kRing][kWaves][64];
  const UnitDesc d = descs[list[blockIdx.y]];
  const int T = d.len_in + d.n_new, b = d.n_out;
  if ((int)blockIdx.x * kNearTile >= T) return;        // whole work-group past the end of this unit
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 31, half = lane >> 5;
  const int n_blocks = (b + 31) / 32;
  St st;
  st.init(k_out + d.out_off * D, b, &ring[0][0], lane, w);
  const float* inv_base = inv_norm + (int64_t)d.unit * ws_stride;
  const unsigned inv_lds = lds_addr_of(&inv_ring[0][0][0]);
  // block blk of the kept keys and its 32 inverse norms (every wave copies the norms itself,
  // so all waves issue the same number of copies per block); a row past the end repeats the last one
  auto issue = [&](int blk, int slot) {
    st.issue(blk, slot);
    const int r = min(blk * 32 + (lane & 31), b - 1);
    load_to_lds_dword(inv_base, (unsigned)r * 4u, inv_lds + (unsigned)((slot * kWaves + w) * 256));
  };
  issue(0, 0);
  if (n_blocks > 1) issue(1, 1);

  // this wave's 32 candidate rows of the virtual concatenation [cached rows | new rows] (B operand);
  // a wave whose rows all lie past the end still takes part in the copies and barriers
  const int e0 = blockIdx.x * kNearTile + w * 32;
  const int e = min(e0 + col, T - 1);
  const __bf16* erow = (e < d.len_in) ? k_in + (d.in_off + e) * D : k_new + ((int64_t)d.unit * N_k + (e - d.len_in)) * D;
  bf16x8 ef[KK];
  float ss = 0.f;
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    ef[kk] = *reinterpret_cast<const bf16x8*>(erow + 16 * kk + 8 * half);
#pragma unroll
    for (int i = 0; i < 8; ++i) ss = fmaf((float)ef[kk][i], (float)ef[kk][i], ss);
  }
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) asm volatile("" ::"v"(ef[kk]));   // waited for here, not inside the loop
  ss = pair_sum(ss);
  const float inv_e = ss > 0.f ? 1.f / sqrtf(ss) : 0.f;

  float best = -INFINITY;   // largest dot(k_e, k_r) / |k_r| so far among this lane's kept rows
  int arg = 0;
  for (int blk = 0; blk < n_blocks; ++blk) {
    if (blk + 1 < n_blocks) dma_wait_but<St::IPW + 1>();   // this wave's copies of block blk have landed
    else dma_wait_but<0>();
    __syncthreads();                                        // all of block blk is visible; the slot of block blk-2 is free
    if (blk + 2 < n_blocks) issue(blk + 2, (blk + 2) % kRing);
    const __bf16* slot = &ring[blk % kRing][0];
    floatx16 sc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag<D>(slot, col, half, kk), ef[kk], sc, 0, 0, 0);
    const float* invs = &inv_ring[blk % kRing][w][0];
    const int nv = min(32, b - blk * 32);
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const float4 iv = *reinterpret_cast<const float4*>(invs + 8 * r4 + 4 * half);
      const float ivs[4] = {iv.x, iv.y, iv.z, iv.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = 8 * r4 + 4 * half + i;            // = c_row(4 r4 + i, half): ascending in (r4, i)
        const float v = (row < nv) ? sc[4 * r4 + i] * ivs[i] : -INFINITY;
        if (v > best) {                                   // strict: an equal later row does not displace an earlier one
          best = v;
          arg = blk * 32 + row;
        }
      }
    }
  }
  // the partner lane holds the other 16 rows of every block: larger value wins, equal values go to the lower index
  const float best_o = __builtin_bit_cast(float, pair_other(__builtin_bit_cast(unsigned, best)));
  const int arg_o = (int)pair_other((unsigned)arg);
  if (best_o > best || (best_o == best && arg_o < arg)) {
    best = best_o;
    arg = arg_o;
  }
  const int ej = e0 + col;
  if (half == 0 && ej < T) {
    int32_t* nn = nearest + (int64_t)d.unit * ws_stride;
    if (nn[ej] == -2) {   // evicted row
      nn[ej] = arg;
      weight[(int64_t)d.unit * ws_stride + ej] = fmaxf(best * inv_e, 0.f);
    }
  }
}

// One wave per kept row p of a merging unit.
template <int D>
__global__ __launch_bounds__(kThreads) void merge_apply(
    const UnitDesc* __restrict__ descs, const int32_t* __restrict__ list, const __bf16* __restrict__ k_in,
    const __bf16* __restrict__ v_in, const __bf16* __restrict__ k_new, const __bf16* __restrict__ v_new, int N_k,
    const int32_t* __restrict__ nearest, const float* __restrict__ weight, int64_t ws_stride,
    __bf16* __restrict__ k_out, __bf16* __restrict__ v_out) {
  constexpr int EPL = D / 64;      // elements per lane
  const UnitDesc d = descs[list[blockIdx.y]];
  const int T = d.len_in + d.n_new, b = d.n_out;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int p = blockIdx.x * kWaves + w;
  if (p >= b) return;
  const int32_t* nn = nearest + (int64_t)d.unit * ws_stride;
  const float* wt = weight + (int64_t)d.unit * ws_stride;
  float ak[EPL], av[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) ak[i] = av[i] = 0.f;
  float wsum = 0.f;
  for (int t0 = 0; t0 < T; t0 += 64) {
    const int j = t0 + lane;
    const bool hit = (j < T) && (nn[j] == p);
    unsigned long long mask = __ballot(hit);
    while (mask) {                                        // ascending rows: a fixed summation order
      const int e = t0 + __builtin_ctzll(mask);
      mask &= mask - 1;
      const float we = wt[e];
      const bool cached = e < d.len_in;
      const int64_t row = cached ? d.in_off + e : (int64_t)d.unit * N_k + (e - d.len_in);
      const __bf16* kr = (cached ? k_in : k_new) + row * D + lane * EPL;
      const __bf16* vr = (cached ? v_in : v_new) + row * D + lane * EPL;
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        ak[i] = fmaf(we, (float)kr[i], ak[i]);
        av[i] = fmaf(we, (float)vr[i], av[i]);
      }
      wsum += we;
    }
  }
  if (wsum > 0.f) {      // nothing merged into this row: it stays bit for bit what the gather wrote
    const float inv = 1.f / (1.f + wsum);
    __bf16* ko = k_out + (d.out_off + p) * D + lane * EPL;
    __bf16* vo = v_out + (d.out_off + p) * D + lane * EPL;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      ko[i] = (__bf16)(((float)ko[i] + ak[i]) * inv);
      vo[i] = (__bf16)(((float)vo[i] + av[i]) * inv);
    }
  }
}

template <int D>
void launch_t(hipStream_t s, const UnitDesc* descs, const int32_t* list, int n_list, int max_t_in, int max_out,
              const void* k_in, const void* v_in, const void* k_new, const void* v_new, int N_k, const int32_t* kept_idx,
              int64_t idx_stride, void* k_out, void* v_out, int32_t* nearest, float* weight, float* inv_norm,
              int64_t ws_stride) {
  typedef __bf16 T;
  hipLaunchKernelGGL(merge_prep<D>, dim3(n_list), dim3(kThreads), 0, s, descs, list, (const T*)k_out, kept_idx, idx_stride,
                     nearest, inv_norm, ws_stride);
  hipLaunchKernelGGL(merge_nearest<D>, dim3((max_t_in + kNearTile - 1) / kNearTile, n_list), dim3(kThreads), 0, s, descs,
                     list, (const T*)k_in, (const T*)k_new, (const T*)k_out, N_k, inv_norm, nearest, weight, ws_stride);
  hipLaunchKernelGGL(merge_apply<D>, dim3((max_out + kWaves - 1) / kWaves, n_list), dim3(kThreads), 0, s, descs, list,
                     (const T*)k_in, (const T*)v_in, (const T*)k_new, (const T*)v_new, N_k, nearest, weight, ws_stride,
                     (T*)k_out, (T*)v_out);
}

}  // namespace

void launch_merge(hipStream_t s, int head_dim, const UnitDesc* descs, const int32_t* list, int n_list, int max_t_in,
                  int max_out, const void* k_in, const void* v_in, const void* k_new, const void* v_new, int N_k,
                  const int32_t* kept_idx, int64_t idx_stride, void* k_out, void* v_out, int32_t* nearest, float* weight,
                  float* inv_norm, int64_t ws_stride) {
  if (n_list <= 0 || max_out <= 0) return;
  if (head_dim == 64)
    launch_t<64>(s, descs, list, n_list, max_t_in, max_out, k_in, v_in, k_new, v_new, N_k, kept_idx, idx_stride, k_out,
                 v_out, nearest, weight, inv_norm, ws_stride);
  else
    launch_t<128>(s, descs, list, n_list, max_t_in, max_out, k_in, v_in, k_new, v_new, N_k, kept_idx, idx_stride, k_out,
                  v_out, nearest, weight, inv_norm, ws_stride);
}

}  // namespace hack
