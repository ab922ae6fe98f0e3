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

template <int D, int PASS>
__global__ __launch_bounds__(kThreads) void score_mfma(
    const UnitDesc* __restrict__ descs, const int32_t* __restrict__ list, int max_chunks,
    const __bf16* __restrict__ q, const int32_t* __restrict__ q_rows, int n_obs, int N_k,
    float scale, const __bf16* __restrict__ k_cache, const __bf16* __restrict__ k_new,
    double* __restrict__ stats, float* __restrict__ importance, int64_t imp_stride) {
  constexpr int KK = D / 16;           // MFMA steps over the head dimension
  constexpr int TPW = kScoreChunk / (4 * 32);  // 32-key tiles per wave
  const UnitDesc d = descs[list[blockIdx.y]];
  const int T_in = d.len_in + d.n_new;
  const int key0 = blockIdx.x * kScoreChunk;
  if (key0 >= T_in) return;
  const int n_chunks = (T_in + kScoreChunk - 1) / kScoreChunk;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int col = lane & 31, half = lane >> 5;

  __shared__ double sm[kMaxObs], sinv[kMaxObs];
  __shared__ float redm[4][kMaxObs], redl[4][kMaxObs];
  __shared__ double redc[8][kMaxObs];
  double* st_unit = stats + (int64_t)blockIdx.y * max_chunks * kMaxObs * 2;

  // K fragments of this wave's tiles: issue every load before anything else.
  bf16x8 kf[TPW][KK];
  bool valid[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int j = key0 + (w * TPW + t) * 32 + col;
    valid[t] = j < T_in;
    const int jc = valid[t] ? j : T_in - 1;
    const __bf16* krow = (jc < d.len_in)
                                     ? k_cache + (d.in_off + jc) * D
                                     : k_new + ((int64_t)d.unit * N_k + (jc - d.len_in)) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      kf[t][kk] = *reinterpret_cast<const bf16x8*>(krow + 16 * kk + 8 * half);
  }
  // Q~ fragments (rows beyond n_obs are zero and masked out below).
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
  if (PASS == 2) combine_stats<true>(st_unit, n_chunks, n_obs, sm, sinv, redc);

  // Raw dot products: every MFMA covers 16 head-dim elements and starts from a
  // zero accumulator; the slice results are summed in fp64, so float32 rounding
  // only ever acts on partial sums that are small next to the full dot product.
  double sd[TPW][16];
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
#pragma unroll
    for (int r = 0; r < 16; ++r) sd[t][r] = 0.0;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      floatx16 c = {0};
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[kk], kf[t][kk], c, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 16; ++r) sd[t][r] += (double)c[r];
    }
  }
  const double c2 = (double)scale * kLog2e;  // logits in log2 units: t = dot * c2

  if (PASS == 1) {
    // Per query row a float32 reference near the chunk maximum (any common value
    // works: it only keeps the exponentials in range), then the sum of 2^(t - ref).
    float mrow[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float m = -INFINITY;
#pragma unroll
      for (int t = 0; t < TPW; ++t) m = fmaxf(m, valid[t] ? (float)sd[t][r] : -INFINITY);
      mrow[r] = half_max(m);
    }
    if (col == 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) redm[w][c_row(r, half)] = mrow[r];
    }
    __syncthreads();
    float lrow[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int i = c_row(r, half);
      const double ref = (double)fmaxf(fmaxf(redm[0][i], redm[1][i]), fmaxf(redm[2][i], redm[3][i])) * c2;
      float l = 0.f;
#pragma unroll
      for (int t = 0; t < TPW; ++t)
        if (valid[t]) l += exp2_split(fma(sd[t][r], c2, -ref));
      lrow[r] = half_sum(l);
    }
    if (col == 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) redl[w][c_row(r, half)] = lrow[r];
    }
    __syncthreads();
    if (tid < kMaxObs) {
      const int i = tid;
      double* o2 = st_unit + ((int64_t)blockIdx.x * kMaxObs + i) * 2;
      o2[0] = (double)fmaxf(fmaxf(redm[0][i], redm[1][i]), fmaxf(redm[2][i], redm[3][i])) * c2;
      o2[1] = ((double)redl[0][i] + (double)redl[1][i]) + ((double)redl[2][i] + (double)redl[3][i]);
    }
  } else {
    __syncthreads();  // sm / sinv ready
    double m_i[16], inv_i[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int i = c_row(r, half);
      m_i[r] = sm[i];
      inv_i[r] = sinv[i];  // zero for rows beyond n_obs
    }
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      double imp = 0.0;
#pragma unroll
      for (int r = 0; r < 16; ++r) imp = fma((double)exp2_split(fma(sd[t][r], c2, -m_i[r])), inv_i[r], imp);
      imp += shfl_xor_f64(imp, 32);
      const int j = key0 + (w * TPW + t) * 32 + col;
      if (valid[t] && half == 0) importance[(int64_t)d.unit * imp_stride + j] = (float)imp;
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
void launch_mfma(hipStream_t s, dim3 grid, const UnitDesc* descs, const int32_t* list,
                 int max_chunks, const void* q, const int32_t* q_rows, int n_obs, int N_k,
                 float scale, const void* k_cache, const void* k_new, double* stats,
                 float* importance, int64_t imp_stride) {
  typedef __bf16 T;
  hipLaunchKernelGGL((score_mfma<D, 1>), grid, dim3(kThreads), 0, s, descs, list, max_chunks,
                     (const T*)q, q_rows, n_obs, N_k, scale, (const T*)k_cache, (const T*)k_new,
                     stats, importance, imp_stride);
  hipLaunchKernelGGL((score_mfma<D, 2>), grid, dim3(kThreads), 0, s, descs, list, max_chunks,
                     (const T*)q, q_rows, n_obs, N_k, scale, (const T*)k_cache, (const T*)k_new,
                     stats, importance, imp_stride);
}

}  // namespace

void launch_score(hipStream_t s, int dtype, int head_dim, const UnitDesc* descs, const int32_t* list,
                  int n_list, int max_t_in, const void* q, const int32_t* q_rows, int n_obs, int N_k,
                  float scale, const void* k_cache, const void* k_new, double* stats,
                  float* importance, int64_t imp_stride) {
  if (n_list <= 0 || max_t_in <= 0) return;
  const int max_chunks = (max_t_in + kScoreChunk - 1) / kScoreChunk;
  dim3 grid(max_chunks, n_list);
#define HACK_ARGS s, grid, descs, list, max_chunks, q, q_rows, n_obs, N_k, scale, k_cache, k_new, stats, importance, imp_stride
  if (dtype == 1) {
    if (head_dim == 64) launch_generic<float, 64>(HACK_ARGS);
    else launch_generic<float, 128>(HACK_ARGS);
  } else {
    if (head_dim == 64) launch_mfma<64>(HACK_ARGS);
    else launch_mfma<128>(HACK_ARGS);
  }
#undef HACK_ARGS
}

}  // namespace hack
