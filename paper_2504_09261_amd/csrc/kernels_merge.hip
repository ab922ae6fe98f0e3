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
// Four launches, after the gather has written K[I], V[I] into the unit's output rows:
//   merge_fill     marks every row of the uncompressed cache "evicted" (-2);
//   merge_mark     marks the kept rows (-1) and forms 1/|k_r| of the kept keys;
//   merge_nearest  MFMA pass: a wave holds 32 cache rows (candidates) as the B operand,
//                  the kept keys stream through LDS as the A operand together with
//                  their inverse norms, two 32-row blocks per barrier; per lane a running
//                  (best, arg-best) over 16 kept rows per block, the lane pair (l, l^32)
//                  combined at the end;
//   merge_apply    a work-group takes 32 kept rows: its waves scan the assignment once,
//                  each a contiguous quarter, and leave the rows that go to one of the 32
//                  in LDS lists (ascending); every wave then folds the listed rows into
//                  its 8 kept rows in ascending row order (so the float32 sums are formed
//                  in a fixed order: the result is reproducible bit for bit) and rewrites
//                  them in place.
// bf16 only.  The products of bf16 values are exact in float32; dots accumulate in
// float32 on the matrix core, the averages in float32 on the vector ALU.
#include <algorithm>

#include "device_util.h"
#include "hack_internal.h"

namespace hack {

namespace {

using namespace dev;

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kRing = 4;          // LDS ring slots (32-row blocks of kept keys): two stages of two blocks

constexpr int kNearBlocks = 1;                      // 32-row candidate blocks per wave in merge_nearest (one keeps the kernel at four
                                                    // work-groups per compute unit: the vector work of one wave then runs beside
                                                    // the MFMAs of the others)
constexpr int kNearTile = kWaves * 32 * kNearBlocks;   // cache rows per work-group in merge_nearest
constexpr int kFillRows = 1024;                     // rows per work-group in merge_fill
constexpr int kMarkRows = kThreads / 8;             // kept rows per work-group in merge_mark (8 lanes per row)
constexpr int kApplyRows = 32;                      // kept rows per work-group in merge_apply
constexpr int kScanPerWave = 2048;                  // cache rows a wave of merge_apply scans per round = capacity of its list

__global__ __launch_bounds__(kThreads) void merge_fill(const UnitDesc* __restrict__ descs, const int32_t* __restrict__ list,
                                                        int32_t* __restrict__ nearest, int64_t ws_stride) {
  const UnitDesc d = descs[list[blockIdx.y]];
  const int T = d.len_in + d.n_new;
  int32_t* nn = nearest + (int64_t)d.unit * ws_stride;
  for (int j = blockIdx.x * kFillRows + threadIdx.x; j < min(T, (int)(blockIdx.x + 1) * kFillRows); j += kThreads) nn[j] = -2;
}

// Work item = (merging unit, 32 kept rows): 8 lanes per row.
template <int D>
__global__ __launch_bounds__(kThreads) void merge_mark(
    const UnitDesc* __restrict__ descs, const int32_t* __restrict__ list, const __bf16* __restrict__ k_out,
    const int32_t* __restrict__ kept_idx, int64_t idx_stride, int32_t* __restrict__ nearest,
    float* __restrict__ inv_norm, int64_t ws_stride) {
  const UnitDesc d = descs[list[blockIdx.y]];
  const int b = d.n_out;
  const int r = blockIdx.x * kMarkRows + (threadIdx.x >> 3), sub = threadIdx.x & 7;
  if (blockIdx.x * kMarkRows >= b) return;
  // inverse norms of the kept keys (already gathered into the unit's output rows)
  constexpr int CPR = D / 8;
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
  if (r < b && sub == 0) {
    inv_norm[(int64_t)d.unit * ws_stride + r] = ss > 0.f ? 1.f / sqrtf(ss) : 0.f;
    nearest[(int64_t)d.unit * ws_stride + kept_idx[(int64_t)d.unit * idx_stride + r]] = -1;
  }
}

// Work item = (merging unit, 32 kWaves kNearBlocks rows of its uncompressed cache): wave w takes rows
// [e0, e0 + 32 kNearBlocks).  The kept keys K^ (rows [out_off, out_off + b)) stream through LDS; a
// fragment read from LDS serves all of the wave's candidate blocks.
template <int D>
__global__ __launch_bounds__(kThreads, 4) void merge_nearest(
    const UnitDesc* __restrict__ descs, const int32_t* __restrict__ list, const __bf16* __restrict__ k_in,
    const __bf16* __restrict__ k_new, const __bf16* __restrict__ k_out, int N_k,
    const float* __restrict__ inv_norm, int32_t* __restrict__ nearest, float* __restrict__ weight,
    int64_t ws_stride) {
  using St = BlockStream<D, kWaves>;
  constexpr int KK = D / 16;
  constexpr int NB = kNearBlocks;
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
    load_to_lds_dword(inv_base, (unsigned)r * 4u, inv_lds + (unsigned)(((blk % kRing) * kWaves + w) * 256));
  };
  issue(0, 0);
  if (n_blocks > 1) issue(1, 1);
  // this wave's candidate rows of the virtual concatenation [cached rows | new rows] (B operands);
  // a wave whose rows all lie past the end still takes part in the copies and barriers
  const int e0 = blockIdx.x * kNearTile + w * (32 * NB);
  bf16x8 ef[NB][KK];
  float inv_e[NB];
#pragma unroll
  for (int c = 0; c < NB; ++c) {
    const int e = min(e0 + 32 * c + col, T - 1);
    const __bf16* erow = (e < d.len_in) ? k_in + (d.in_off + e) * D : k_new + ((int64_t)d.unit * N_k + (e - d.len_in)) * D;
    float ss = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      ef[c][kk] = *reinterpret_cast<const bf16x8*>(erow + 16 * kk + 8 * half);
#pragma unroll
      for (int i = 0; i < 8; ++i) ss = fmaf((float)ef[c][kk][i], (float)ef[c][kk][i], ss);
    }
    ss = pair_sum(ss);
    inv_e[c] = ss > 0.f ? 1.f / sqrtf(ss) : 0.f;
  }
#pragma unroll
  for (int c = 0; c < NB; ++c)
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) asm volatile("" ::"v"(ef[c][kk]));   // waited for here, not inside the loop

  float best[NB];   // largest dot(k_e, k_r) / |k_r| so far among this lane's kept rows
  int arg[NB];
#pragma unroll
  for (int c = 0; c < NB; ++c) {
    best[c] = -INFINITY;
    arg[c] = 0;
  }
  // One block against this lane's 16 kept rows: the block's largest value displaces the running best only if it
  // is strictly larger (an equal later row does not displace an earlier one), and among equal values of the block
  // the lowest row wins.  A short tree of maxima, then the lowest row that attains the maximum.
  auto update = [&](const floatx16& sc, int blk, int nv, bool ragged, float& bst, int& ag) {
    const float* invs = &inv_ring[blk % kRing][w][0];
    float v[16];
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const float4 iv = *reinterpret_cast<const float4*>(invs + 8 * r4 + 4 * half);
      const float ivs[4] = {iv.x, iv.y, iv.z, iv.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = 8 * r4 + 4 * half + i;            // = c_row(4 r4 + i, half): ascending in (r4, i)
        v[4 * r4 + i] = (ragged && row >= nv) ? -INFINITY : sc[4 * r4 + i] * ivs[i];
      }
    }
    float m4[4];
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) m4[g4] = fmaxf(fmaxf(v[4 * g4], v[4 * g4 + 1]), fmaxf(v[4 * g4 + 2], v[4 * g4 + 3]));
    const float vmax = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
    const bool moved = vmax > bst;
    if (__any(moved)) {                                   // the row is only looked for when some lane's best moved
      int first = 0;
#pragma unroll
      for (int q = 15; q >= 0; --q)                       // descending, so the lowest matching row is written last
        first = (v[q] == vmax) ? 8 * (q >> 2) + 4 * half + (q & 3) : first;
      bst = moved ? vmax : bst;
      ag = moved ? blk * 32 + first : ag;
    }
  };
  auto scores = [&](int blk, floatx16& sc) {
    const __bf16* slot = &ring[blk % kRing][0];
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag<D>(slot, col, half, kk), ef[0][kk], sc, 0, 0, 0);
  };
  static_assert(NB == 1, "the loop below is written for one candidate block per wave");
  // A stage is two blocks of kept keys (one barrier per stage); while a stage is worked on, the copies of the
  // next one are in flight into the other two ring slots.
  for (int blk = 0; blk < n_blocks; blk += 2) {
    dma_wait_but<0>();                                      // this wave's copies of blocks blk, blk+1 have landed
    __syncthreads();                                        // ... and everybody's; the slots of blocks blk-2, blk-1 are free
    if (blk + 2 < n_blocks) issue(blk + 2, (blk + 2) % kRing);
    if (blk + 3 < n_blocks) issue(blk + 3, (blk + 3) % kRing);
    floatx16 s0, s1;
    const bool two = blk + 1 < n_blocks;                    // wave-uniform
    scores(blk, s0);
    if (two) scores(blk + 1, s1);
    // the ragged form (rows past the end masked) is a separate instance, taken by the last block only
    const int nv0 = min(32, b - blk * 32);
    if (nv0 == 32) update(s0, blk, 32, false, best[0], arg[0]);
    else update(s0, blk, nv0, true, best[0], arg[0]);
    if (two) {
      const int nv1 = min(32, b - (blk + 1) * 32);
      if (nv1 == 32) update(s1, blk + 1, 32, false, best[0], arg[0]);
      else update(s1, blk + 1, nv1, true, best[0], arg[0]);
    }
  }
#pragma unroll
  for (int c = 0; c < NB; ++c) {
    // the partner lane holds the other 16 rows of every block: larger value wins, equal values go to the lower index
    const float best_o = __builtin_bit_cast(float, pair_other(__builtin_bit_cast(unsigned, best[c])));
    const int arg_o = (int)pair_other((unsigned)arg[c]);
    float bst = best[c];
    int ag = arg[c];
    if (best_o > bst || (best_o == bst && arg_o < ag)) {
      bst = best_o;
      ag = arg_o;
    }
    const int ej = e0 + 32 * c + col;
    if (half == 0 && ej < T) {
      int32_t* nn = nearest + (int64_t)d.unit * ws_stride;
      if (nn[ej] == -2) {   // evicted row
        nn[ej] = ag;
        weight[(int64_t)d.unit * ws_stride + ej] = fmaxf(bst * inv_e[c], 0.f);
      }
    }
  }
}

// Work item = (merging unit, 32 kept rows [r0, r0 + 32)); wave w owns rows r0 + 8 w .. + 8.
template <int D>
__global__ __launch_bounds__(kThreads) void merge_apply(
    const UnitDesc* __restrict__ descs, const int32_t* __restrict__ list, const __bf16* __restrict__ k_in,
    const __bf16* __restrict__ v_in, const __bf16* __restrict__ k_new, const __bf16* __restrict__ v_new, int N_k,
    const int32_t* __restrict__ nearest, const float* __restrict__ weight, int64_t ws_stride,
    __bf16* __restrict__ k_out, __bf16* __restrict__ v_out, int cap) {
  constexpr int EPL = D / 64;                   // elements per lane
  constexpr int RPW = kApplyRows / kWaves;      // kept rows per wave
  static_assert(kApplyRows == 32, "a list entry keeps the row's offset in 5 bits");
  // entry: (cache row - first row of the round) << 5 | (kept row - r0); each wave's list is ascending
  extern __shared__ uint32_t lst[];   // [kWaves][cap]
  __shared__ int cnt[kWaves];
  const UnitDesc d = descs[list[blockIdx.y]];
  const int T = d.len_in + d.n_new, b = d.n_out;
  const int r0 = blockIdx.x * kApplyRows;
  if (r0 >= b) return;
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int32_t* nn = nearest + (int64_t)d.unit * ws_stride;
  const float* wt = weight + (int64_t)d.unit * ws_stride;
  float ak[RPW][EPL], av[RPW][EPL], wsum[RPW];
#pragma unroll
  for (int i = 0; i < RPW; ++i) {
    wsum[i] = 0.f;
#pragma unroll
    for (int x = 0; x < EPL; ++x) ak[i][x] = av[i][x] = 0.f;
  }
  // rows a wave scans per round: a quarter of the cache (in whole 64-row steps), at most its list's capacity
  const int per = min(cap, (T + 64 * kWaves - 1) / (64 * kWaves) * 64);
  for (int seg0 = 0; seg0 < T; seg0 += kWaves * per) {
    // wave w scans cache rows [seg0 + per w, + per): the rows assigned to one of this work-group's kept rows
    int n = 0;
    const int base = seg0 + w * per;
    for (int t0 = 0; t0 < per && base + t0 < T; t0 += 4 * 64) {
      int v[4];                                               // four steps' loads in flight together
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int j = base + t0 + 64 * u + lane;
        v[u] = (t0 + 64 * u < per && j < T) ? nn[j] : -1;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int j = base + t0 + 64 * u + lane;
        const unsigned rl = (unsigned)(v[u] - r0);            // kept (-1) and unassigned rows wrap to large values
        const bool hit = rl < (unsigned)kApplyRows;
        const unsigned long long m = __ballot(hit);
        if (hit) lst[w * cap + n + __builtin_popcountll(m & ((1ull << lane) - 1ull))] = ((unsigned)(j - seg0) << 5) | rl;
        n += __builtin_popcountll(m);
      }
    }
    if (lane == 0) cnt[w] = n;
    __syncthreads();
    // The lists of waves 0..3 one after the other are in ascending row order: a fixed summation order per kept
    // row.  The wave's 8 kept rows advance side by side: per pass each row that has a listed row left takes its
    // next one, the loads of all of them are issued together, then each row adds its own.
    for (int q = 0; q < kWaves; ++q) {
      const int nq = cnt[q];
      for (int t0 = 0; t0 < nq; t0 += 64) {
        const bool in = t0 + lane < nq;
        const unsigned ent = in ? lst[q * cap + t0 + lane] : 0u;
        unsigned long long m[RPW];
        unsigned long long any = 0;
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
          m[i] = __ballot(in && (ent & 31u) == (unsigned)(w * RPW + i));
          any |= m[i];
        }
        while (any) {
          float we[RPW];
          bf16x2 kx[RPW], vx[RPW];
          static_assert(EPL == 1 || EPL == 2, "one or two elements per lane");
          any = 0;
#pragma unroll
          for (int i = 0; i < RPW; ++i) {
            we[i] = -1.f;                                     // no row taken in this pass
            if (m[i]) {                                       // wave-uniform
              const int src = __builtin_ctzll(m[i]);
              m[i] &= m[i] - 1;
              any |= m[i];
              const int e = seg0 + (int)(__shfl(ent, src, 64) >> 5);
              we[i] = wt[e];
              const bool cached = e < d.len_in;
              const int64_t row = cached ? d.in_off + e : (int64_t)d.unit * N_k + (e - d.len_in);
              const __bf16* kr = (cached ? k_in : k_new) + row * D + lane * EPL;
              const __bf16* vr = (cached ? v_in : v_new) + row * D + lane * EPL;
              if (EPL == 2) {
                kx[i] = *reinterpret_cast<const bf16x2*>(kr);
                vx[i] = *reinterpret_cast<const bf16x2*>(vr);
              } else {
                kx[i][0] = kr[0];
                vx[i][0] = vr[0];
              }
            }
          }
#pragma unroll
          for (int i = 0; i < RPW; ++i) {
            if (we[i] >= 0.f) {                               // weights are >= 0; wave-uniform
#pragma unroll
              for (int x = 0; x < EPL; ++x) {
                ak[i][x] = fmaf(we[i], (float)kx[i][x], ak[i][x]);
                av[i][x] = fmaf(we[i], (float)vx[i][x], av[i][x]);
              }
              wsum[i] += we[i];
            }
          }
        }
      }
    }
    __syncthreads();   // the lists are rewritten in the next round
  }
#pragma unroll
  for (int i = 0; i < RPW; ++i) {
    const int p = r0 + w * RPW + i;
    if (p < b && wsum[i] > 0.f) {      // nothing merged into a row: it stays bit for bit what the gather wrote
      const float inv = 1.f / (1.f + wsum[i]);
      __bf16* ko = k_out + (d.out_off + p) * D + lane * EPL;
      __bf16* vo = v_out + (d.out_off + p) * D + lane * EPL;
#pragma unroll
      for (int x = 0; x < EPL; ++x) {
        ko[x] = (__bf16)(((float)ko[x] + ak[i][x]) * inv);
        vo[x] = (__bf16)(((float)vo[x] + av[i][x]) * inv);
      }
    }
  }
}

template <int D>
void launch_t(hipStream_t s, const UnitDesc* descs, const int32_t* list, int n_list, int max_t_in, int max_out,
              const void* k_in, const void* v_in, const void* k_new, const void* v_new, int N_k, const int32_t* kept_idx,
              int64_t idx_stride, void* k_out, void* v_out, int32_t* nearest, float* weight, float* inv_norm,
              int64_t ws_stride) {
  typedef __bf16 T;
  hipLaunchKernelGGL(merge_fill, dim3((max_t_in + kFillRows - 1) / kFillRows, n_list), dim3(kThreads), 0, s, descs, list, nearest,
                     ws_stride);
  hipLaunchKernelGGL(merge_mark<D>, dim3((max_out + kMarkRows - 1) / kMarkRows, n_list), dim3(kThreads), 0, s, descs, list,
                     (const T*)k_out, kept_idx, idx_stride, nearest, inv_norm, ws_stride);
  hipLaunchKernelGGL(merge_nearest<D>, dim3((max_t_in + kNearTile - 1) / kNearTile, n_list), dim3(kThreads), 0, s, descs,
                     list, (const T*)k_in, (const T*)k_new, (const T*)k_out, N_k, inv_norm, nearest, weight, ws_stride);
  // list capacity of a wave of merge_apply: a quarter of the longest cache in whole 64-row steps, at most kScanPerWave
  const int cap = std::min(kScanPerWave, (max_t_in + 64 * kWaves - 1) / (64 * kWaves) * 64);
  hipLaunchKernelGGL(merge_apply<D>, dim3((max_out + kApplyRows - 1) / kApplyRows, n_list), dim3(kThreads),
                     (size_t)kWaves * cap * sizeof(uint32_t), s, descs, list, (const T*)k_in, (const T*)v_in, (const T*)k_new,
                     (const T*)v_new, N_k, nearest, weight, ws_stride, (T*)k_out, (T*)v_out, cap);
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
