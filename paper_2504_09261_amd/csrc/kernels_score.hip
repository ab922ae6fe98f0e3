// Subset-attention importance (Sec. 4.4, "Importance Estimation via Efficient
// Subset Attention") on gfx950:
//     A~ = Softmax(scale * Q~ K^T),   importance[j] = sum_i A~[i, j]
// over the uncompressed keys of the step (cache rows followed by the current
// scale's rows, read from their two homes without materialising the concat).
//
// The column sum needs each row's softmax normaliser before any key's
// importance can be formed, so the work is split in two streaming passes over
// K, both tiled as (unit, chunk of 256 keys):
//   pass 1  per chunk and observation row: max logit and sum of exp(logit - max)
//   pass 2  combine the chunk partials of the unit, recompute the logits and
//           write importance[j] = sum_i exp(s_ij - m_i) / l_i.
// Both passes are bound by reading K (n_obs <= 32 rows against every key is a
// skinny product, ~31 flop per byte), so the spare ALU is spent on accuracy:
// the logit is widened to fp64 before the shift and the exponential is
// range-reduced in fp64, which keeps float32 importance within a few ulp of the
// exact value; the ranking that follows is decided on those float32 numbers.
//
// bf16: one v_mfma_f32_32x32x16_bf16 column block holds all 32 observation
// rows; a wave owns 64 keys (two 32-key tiles), loads its K fragments straight
// from HBM into registers (each key is used once per wave: staging in LDS would
// buy nothing), and reduces over keys in-lane first, across lanes once.
// fp32: plain fp64 FMA dot products, one key per lane.
#include "hack_internal.h"

namespace hack {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int kThreads = 256;
constexpr double kLog2e = 1.4426950408889634074;

// 2^t for a double t with ~1 ulp float32 accuracy: the range reduction is done
// in fp64 so a large |t| does not cost relative accuracy; the result is a float
// (ldexp of the float mantissa part is exact).
__device__ __forceinline__ float exp2_split(double t) {
  const double n = rint(t);
  const float r = (float)(t - n);  // |r| <= 0.5
  return ldexpf(__builtin_amdgcn_exp2f(r), (int)n);
}
__device__ __forceinline__ double exp_neg(double x) { return (double)exp2_split(x * kLog2e); }

// All-reduce over the 32 lanes of a half-wave without touching LDS memory:
// two quad permutes, the two row mirrors, then a swizzle across the 16-lane rows.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float swz_xor16(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));
}
__device__ __forceinline__ float half_max(float v) {
  v = fmaxf(v, dpp_mov<0xB1>(v));
  v = fmaxf(v, dpp_mov<0x4E>(v));
  v = fmaxf(v, dpp_mov<0x141>(v));
  v = fmaxf(v, dpp_mov<0x140>(v));
  return fmaxf(v, swz_xor16(v));
}
__device__ __forceinline__ float half_sum(float v) {
  v += dpp_mov<0xB1>(v);
  v += dpp_mov<0x4E>(v);
  v += dpp_mov<0x141>(v);
  v += dpp_mov<0x140>(v);
  return v + swz_xor16(v);
}

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(__bf16 v) { return (float)v; }

__device__ __forceinline__ double shfl_xor_f64(double v, int m) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_xor(lo, m, 64);
  hi = __shfl_xor(hi, m, 64);
  return __hiloint2double(hi, lo);
}

// Combine the per-chunk (reference, sum) partials of one unit into sm[i]
// (reference) and sinv[i] (1 / normaliser) for the rows i < n_obs.  All 256
// threads take part: thread (g, i) = (tid / 32, tid % 32) folds the chunks
// g, g + 8, ... of row i, then the eight groups are merged through LDS.
// LOG2: the partials are in log2 units (MFMA path) instead of natural units.
// Ends with a barrier: sm / sinv are ready for every thread on return.
template <bool LOG2>
__device__ __forceinline__ void combine_stats(const double* __restrict__ st, int n_chunks, int n_obs,
                                              double* sm, double* sinv, double (*red)[kMaxObs]) {
  const int i = threadIdx.x & 31, g = threadIdx.x >> 5;
  double m = -INFINITY;
  for (int c = g; c < n_chunks; c += 8) m = fmax(m, st[(c * kMaxObs + i) * 2]);
  red[g][i] = m;
  __syncthreads();
  m = red[0][i];
#pragma unroll
  for (int k = 1; k < 8; ++k) m = fmax(m, red[k][i]);
  __syncthreads();
  double l = 0.0;
  for (int c = g; c < n_chunks; c += 8) {
    const double mc = st[(c * kMaxObs + i) * 2], lc = st[(c * kMaxObs + i) * 2 + 1];
    l += lc * (LOG2 ? (double)exp2_split(mc - m) : exp_neg(mc - m));
  }
  red[g][i] = l;
  __syncthreads();
  if (g == 0) {
    l = red[0][i];
#pragma unroll
    for (int k = 1; k < 8; ++k) l += red[k][i];
    sm[i] = (i < n_obs) ? m : 0.0;  // unused rows: finite shift, zero weight
    sinv[i] = (i < n_obs) ? 1.0 / l : 0.0;
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------
// generic path (fp32 inputs; also usable for bf16): one key per lane, fp64 dots
// ---------------------------------------------------------------------------
template <typename T, int D, int PASS>
__global__ __launch_bounds__(kThreads) void score_generic(
    const UnitDesc* __restrict__ descs, const int32_t* __restrict__ list, int max_chunks,
    const T* __restrict__ q, const int32_t* __restrict__ q_rows, int n_obs, int N_k, float scale,
    const T* __restrict__ k_cache, const T* __restrict__ k_new, double* __restrict__ stats,
    float* __restrict__ importance, int64_t imp_stride) {
  const UnitDesc d = descs[list[blockIdx.y]];
  const int T_in = d.len_in + d.n_new;
  const int key0 = blockIdx.x * kScoreChunk;
  if (key0 >= T_in) return;
  const int n_chunks = (T_in + kScoreChunk - 1) / kScoreChunk;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;

  __shared__ float qs[kMaxObs][D];
  __shared__ double red[8][kMaxObs];
  __shared__ double sm[kMaxObs], sinv[kMaxObs];

  for (int e = tid; e < n_obs * D; e += kThreads) {
    const int i = e / D, c = e % D;
    qs[i][c] = to_float(q[((int64_t)d.unit * N_k + q_rows[i]) * D + c]);
  }
  double* st_unit = stats + (int64_t)blockIdx.y * max_chunks * kMaxObs * 2;
  if (PASS == 2) combine_stats<false>(st_unit, n_chunks, n_obs, sm, sinv, red);
  __syncthreads();

  const int j = key0 + tid;
  const bool valid = j < T_in;
  const int jc = valid ? j : T_in - 1;
  const T* krow = (jc < d.len_in) ? k_cache + (d.in_off + jc) * D
                                  : k_new + ((int64_t)d.unit * N_k + (jc - d.len_in)) * D;
  float kr[D];
#pragma unroll
  for (int c = 0; c < D; ++c) kr[c] = to_float(krow[c]);

  if (PASS == 1) {
    for (int i = 0; i < n_obs; ++i) {
      double acc = 0.0;
#pragma unroll
      for (int c = 0; c < D; ++c) acc = fma((double)qs[i][c], (double)kr[c], acc);
      const double s = acc * (double)scale;
      double m = valid ? s : -INFINITY;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) m = fmax(m, shfl_xor_f64(m, o));
      if (lane == 0) red[w][i] = m;
      __syncthreads();
      m = fmax(fmax(red[0][i], red[1][i]), fmax(red[2][i], red[3][i]));
      __syncthreads();
      double l = valid ? exp_neg(s - m) : 0.0;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) l += shfl_xor_f64(l, o);
      if (lane == 0) red[w][i] = l;
      __syncthreads();
      if (tid == 0) {
        double* o2 = st_unit + ((int64_t)blockIdx.x * kMaxObs + i) * 2;
        o2[0] = m;
        o2[1] = red[0][i] + red[1][i] + red[2][i] + red[3][i];
      }
      __syncthreads();
    }
  } else {
    double imp = 0.0;
    for (int i = 0; i < n_obs; ++i) {
      double acc = 0.0;
#pragma unroll
      for (int c = 0; c < D; ++c) acc = fma((double)qs[i][c], (double)kr[c], acc);
      imp += exp_neg(acc * (double)scale - sm[i]) * sinv[i];
    }
    if (valid) importance[(int64_t)d.unit * imp_stride + j] = (float)imp;
  }
}

// ---------------------------------------------------------------------------
// bf16 MFMA path
// ---------------------------------------------------------------------------
// C = Q~ K^T per 32-key tile: A operand = Q~ (row = observation query l%32),
// B operand = K^T (column = key l%32); both take the 8 contiguous head-dim
// elements [16*kk + 8*(l/32), +8) at MFMA step kk.  C register r of lane l is
// query row 8*(r/4) + 4*(l/32) + r%4, key column l%32.
__device__ __forceinline__ int c_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// ---- wave-private tile pipeline -------------------------------------------
// A work item is (unit, chunk of kItemKeys keys) and belongs to ONE wave: the
// wave copies its 32-key tiles HBM -> LDS with global_load_lds (16 B per lane,
// whole rows, fully coalesced), double-buffered in a private LDS region, and
// reads MFMA operands back with ds_read_b128 (XOR-swizzled chunks, conflict
// free on the 64-bank LDS).  No work-group barrier anywhere: waves only wait on
// their own copies (hand-placed s_waitcnt vmcnt), so they drift freely and keep
// HBM busy.  Reading K fragments straight from HBM in operand layout would touch
// 32 rows x 32 bytes per instruction and re-fetch every cache line several times.
constexpr int kItemKeys = 128;                 // keys per wave item
constexpr int kItemTiles = kItemKeys / 32;

template <int D> __device__ __forceinline__ int score_swz(int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); }

__device__ __forceinline__ void score_dma16(const __bf16* src, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(src), "s"(lds_addr) : "memory", "m0");
}
// same copy, source = wave-uniform base (SGPR pair) + per-lane byte offset
__device__ __forceinline__ void score_dma16_base(const __bf16* base, int voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0"
               :: "s"(base), "v"(voff), "s"(lds_addr) : "memory", "m0");
}
template <int N> __device__ __forceinline__ void score_wait_vm() {
  __builtin_amdgcn_sched_barrier(0);
  if (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else if (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

struct ScoreItem {
  int32_t pos;     // position in the active-unit list (indexes the stats rows)
  int32_t chunk;   // chunk index inside the unit
};

// 2^t as a double for any |t| <= 1000 (the float mantissa part is exact to ~1 ulp
// of float32, the exponent is applied in fp64)
__device__ __forceinline__ double exp2_wide(double t) {
  t = fmin(fmax(t, -1000.0), 1000.0);
  const double n = rint(t);
  const float r = (float)(t - n);
  return ldexp((double)__builtin_amdgcn_exp2f(r), (int)n);
}
// sum over the 32 lanes of a half-wave, fp64 (DPP moves of both dwords)
template <int CTRL>
__device__ __forceinline__ double dpp_mov_f64(double v) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, true);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double half_sum_f64(double v) {
  v += dpp_mov_f64<0xB1>(v);
  v += dpp_mov_f64<0x4E>(v);
  v += dpp_mov_f64<0x141>(v);
  v += dpp_mov_f64<0x140>(v);
  const int lo = __builtin_amdgcn_ds_swizzle(__double2loint(v), 0x401F);
  const int hi = __builtin_amdgcn_ds_swizzle(__double2hiint(v), 0x401F);
  return v + __hiloint2double(hi, lo);
}

// PASS 1: per item the sum over its keys of 2^t for every observation row
//         (t = logit in log2 units; no running max is needed because the sums
//         are kept in fp64, whose exponent range covers |t| <= 1000), added to
//         the unit's 32 row sums with device-scope fp64 atomics.
// PASS 2: every wave turns the row sums into (m_i, w_i), m_i an integer near
//         log2(sum_i) and w_i = 2^m_i / sum_i, and writes
//         importance_j = sum_i 2^(t_ij - m_i) * w_i.  The wave that finishes a
//         unit's last chunk (atomic counter, nobody waits) zeroes the row sums
//         and the counter again, so the workspace is clean for the next launch.
template <int D, int PASS>
__global__ __launch_bounds__(kThreads) void score_mfma(
    const UnitDesc* __restrict__ descs, const int32_t* __restrict__ list,
    const ScoreItem* __restrict__ items, int n_items, int max_chunks,
    const __bf16* __restrict__ q, const int32_t* __restrict__ q_rows, int n_obs, int N_k,
    float scale, const __bf16* __restrict__ k_cache, const __bf16* __restrict__ k_new,
    double* __restrict__ rowsum, unsigned* __restrict__ counters,
    float* __restrict__ importance, int64_t imp_stride) {
  constexpr int KK = D / 16;            // MFMA steps over the head dimension
  constexpr int CPR = D / 8;            // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;         // rows per wave-wide copy instruction
  constexpr int IPT = 32 / RPI;         // copy instructions per 32-key tile (8 or 4)
  constexpr int TILE = 32 * D;          // elements per tile

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int item = blockIdx.x * 4 + w;
  if (item >= n_items) return;          // wave-uniform; the kernel has no barriers
  const ScoreItem it = items[item];
  const UnitDesc d = descs[list[it.pos]];
  const int T_in = d.len_in + d.n_new;
  const int key0 = it.chunk * kItemKeys;
  const int n_tiles = min(kItemTiles, (T_in - key0 + 31) / 32);
  const int n_chunks = (T_in + kItemKeys - 1) / kItemKeys;
  const int col = lane & 31, half = lane >> 5;

  __shared__ __attribute__((aligned(1024))) __bf16 tiles[4][2][TILE];
  const unsigned lds0 = (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void*)&tiles[w][0][0];
  double* sum_unit = rowsum + (int64_t)it.pos * kMaxObs;

  // copy of tile t (keys key0 + 32t ..) into buffer t & 1.  A tile that lies
  // wholly inside the cached rows or wholly inside the new rows (the common
  // case) is addressed as wave-uniform base + loop-invariant lane offset; a tile
  // that straddles the seam or the end picks every row's source on its own and
  // repeats the last key past the end.
  int src_off[IPT];
#pragma unroll
  for (int i = 0; i < IPT; ++i) {
    const int r = i * RPI + lane / CPR, c = lane % CPR;
    src_off[i] = (r * D + ((c ^ score_swz<D>(r)) & (CPR - 1)) * 8) * 2;
  }
  auto issue = [&](int t) {
    const int j0 = key0 + t * 32;
    const unsigned dst = lds0 + (unsigned)((t & 1) * TILE * 2);
    const bool in_cache = j0 + 32 <= d.len_in;
    const bool in_new = j0 >= d.len_in && j0 + 32 <= T_in;
    if (in_cache || in_new) {
      const __bf16* base = in_cache ? k_cache + (d.in_off + j0) * D
                                    : k_new + ((int64_t)d.unit * N_k + (j0 - d.len_in)) * D;
#pragma unroll
      for (int i = 0; i < IPT; ++i) score_dma16_base(base, src_off[i], dst + i * 1024);
    } else {
#pragma unroll
      for (int i = 0; i < IPT; ++i) {
        const int r = i * RPI + lane / CPR, c = lane % CPR;
        const int j = min(j0 + r, T_in - 1);
        const __bf16* row = (j < d.len_in) ? k_cache + (d.in_off + j) * D
                                           : k_new + ((int64_t)d.unit * N_k + (j - d.len_in)) * D;
        score_dma16(row + ((c ^ score_swz<D>(r)) & (CPR - 1)) * 8, dst + i * 1024);
      }
    }
  };
  issue(0);

  // Q~ fragments (rows beyond n_obs are zero and get zero weight below).
  bf16x8 qf[KK];
  {
    const bool qv = col < n_obs;
    const __bf16* qrow = q + ((int64_t)d.unit * N_k + (qv ? q_rows[col] : 0)) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      bf16x8 z = {0};
      qf[kk] = qv ? *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * half) : z;
    }
  }
  const double c2 = (double)scale * kLog2e;  // logits in log2 units: t = dot * c2

  double m_i[16], w_i[16];
  if (PASS == 2) {
    // lane col (both halves) folds row col, then every lane fetches its 16 rows
    const double l = sum_unit[col];
    int ex;
    (void)frexp(l, &ex);                       // l = f * 2^ex, f in [0.5, 1)
    const double mm = (double)ex;
    const double ww = (col < n_obs) ? ldexp(1.0, ex) / l : 0.0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int src = c_row(r, half);
      m_i[r] = __hiloint2double(__shfl(__double2hiint(mm), src, 64), __shfl(__double2loint(mm), src, 64));
      w_i[r] = __hiloint2double(__shfl(__double2hiint(ww), src, 64), __shfl(__double2loint(ww), src, 64));
    }
  }
  // everything the compiler loaded itself must have landed before the loop, so
  // that no compiler-placed vmcnt wait inside it also drains the tile copies
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) asm volatile("" ::"v"(qf[kk]));
  if (PASS == 2) {
#pragma unroll
    for (int r = 0; r < 16; ++r) asm volatile("" ::"v"(m_i[r]), "v"(w_i[r]));
  }

  double lsum[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) lsum[r] = 0.0;
  int k_off[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) k_off[kk] = col * D + (((2 * kk + half) ^ score_swz<D>(col)) & (CPR - 1)) * 8;

  for (int t = 0; t < n_tiles; ++t) {
    if (t + 1 < n_tiles) {
      issue(t + 1);
      score_wait_vm<IPT>();   // tile t has landed, tile t+1 stays in flight
    } else {
      score_wait_vm<0>();
    }
    const __bf16* Kt = &tiles[w][t & 1][0];
    // Raw dot products: every MFMA covers 16 head-dim elements and starts from a
    // zero accumulator; the slice results are summed in fp64, so float32 rounding
    // only ever acts on partial sums that are small next to the full dot product.
    double sd[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) sd[r] = 0.0;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Kt[k_off[kk]]);
      floatx16 c = {0};
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[kk], kf, c, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 16; ++r) sd[r] += (double)c[r];
    }
    const int j = key0 + t * 32 + col;
    const bool valid = j < T_in;
    if (PASS == 1) {
      if (valid) {
#pragma unroll
        for (int r = 0; r < 16; ++r) lsum[r] += exp2_wide(sd[r] * c2);
      }
    } else {
      double imp = 0.0;
#pragma unroll
      for (int r = 0; r < 16; ++r) imp = fma((double)exp2_split(fma(sd[r], c2, -m_i[r])), w_i[r], imp);
      imp += shfl_xor_f64(imp, 32);
      if (valid && half == 0) importance[(int64_t)d.unit * imp_stride + j] = (float)imp;
    }
  }

  if (PASS == 1) {
    // lanes of a half-wave hold different keys of the same 16 query rows
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const double l = half_sum_f64(lsum[r]);
      if (col == 0) atomicAdd(&sum_unit[c_row(r, half)], l);
    }
  } else {
    // the wave that finishes the unit's last chunk cleans the workspace (every
    // wave of the unit has read the row sums before it bumps the counter)
    unsigned arrived = 0;
    if (lane == 0) arrived = atomicAdd(&counters[it.pos], 1u);
    arrived = __builtin_amdgcn_readfirstlane(arrived);
    if ((int)arrived == n_chunks - 1) {
      if (lane < kMaxObs) sum_unit[lane] = 0.0;
      if (lane == 0) counters[it.pos] = 0;
    }
  }
}

template <typename T, int D>
void launch_generic(hipStream_t s, dim3 grid, const UnitDesc* descs, const int32_t* list,
                    int max_chunks, const void* q, const int32_t* q_rows, int n_obs, int N_k,
                    float scale, const void* k_cache, const void* k_new, double* stats,
                    float* importance, int64_t imp_stride) {
  hipLaunchKernelGGL((score_generic<T, D, 1>), grid, dim3(kThreads), 0, s, descs, list, max_chunks,
                     (const T*)q, q_rows, n_obs, N_k, scale, (const T*)k_cache, (const T*)k_new,
                     stats, importance, imp_stride);
  hipLaunchKernelGGL((score_generic<T, D, 2>), grid, dim3(kThreads), 0, s, descs, list, max_chunks,
                     (const T*)q, q_rows, n_obs, N_k, scale, (const T*)k_cache, (const T*)k_new,
                     stats, importance, imp_stride);
}

template <int D>
void launch_mfma(hipStream_t s, const UnitDesc* descs, const int32_t* list, const void* items, int n_items,
                 int max_chunks, const void* q, const int32_t* q_rows, int n_obs, int N_k, float scale,
                 const void* k_cache, const void* k_new, double* stats, double* rowstat, unsigned* counters,
                 float* importance, int64_t imp_stride) {
  typedef __bf16 T;
  (void)stats;
  dim3 grid((n_items + 3) / 4);
  hipLaunchKernelGGL((score_mfma<D, 1>), grid, dim3(kThreads), 0, s, descs, list, (const ScoreItem*)items,
                     n_items, max_chunks, (const T*)q, q_rows, n_obs, N_k, scale, (const T*)k_cache,
                     (const T*)k_new, rowstat, counters, importance, imp_stride);
  hipLaunchKernelGGL((score_mfma<D, 2>), grid, dim3(kThreads), 0, s, descs, list, (const ScoreItem*)items,
                     n_items, max_chunks, (const T*)q, q_rows, n_obs, N_k, scale, (const T*)k_cache,
                     (const T*)k_new, rowstat, counters, importance, imp_stride);
}

}  // namespace

int score_item_keys(int dtype) { return dtype == 1 ? kScoreChunk : kItemKeys; }

void launch_score(hipStream_t s, int dtype, int head_dim, const UnitDesc* descs, const int32_t* list,
                  int n_list, int max_t_in, const void* items, int n_items, const void* q,
                  const int32_t* q_rows, int n_obs, int N_k, float scale, const void* k_cache,
                  const void* k_new, double* stats, double* rowstat, unsigned* counters, float* importance,
                  int64_t imp_stride) {
  if (n_list <= 0 || max_t_in <= 0) return;
  if (dtype == 1) {
    const int max_chunks = (max_t_in + kScoreChunk - 1) / kScoreChunk;
    dim3 grid(max_chunks, n_list);
#define HACK_ARGS s, grid, descs, list, max_chunks, q, q_rows, n_obs, N_k, scale, k_cache, k_new, stats, importance, imp_stride
    if (head_dim == 64) launch_generic<float, 64>(HACK_ARGS);
    else launch_generic<float, 128>(HACK_ARGS);
#undef HACK_ARGS
  } else {
    const int max_chunks = (max_t_in + kItemKeys - 1) / kItemKeys;
#define HACK_ARGS s, descs, list, items, n_items, max_chunks, q, q_rows, n_obs, N_k, scale, k_cache, k_new, stats, rowstat, counters, importance, imp_stride
    if (head_dim == 64) launch_mfma<64>(HACK_ARGS);
    else launch_mfma<128>(HACK_ARGS);
#undef HACK_ARGS
  }
}

}  // namespace hack
