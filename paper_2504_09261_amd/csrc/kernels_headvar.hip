// Attention variance of a head (Sec. 4.2, "Offline Head Classification via
// Attention Variance") on gfx950:
//     A = Softmax(scale * Q K^T)  (N_K queries x T_K keys, the final step over the
//     full cache),   sigma = sum_j Var_i(A[i, j])   (population variance).
// With c1_j = sum_i A_ij the sum of the column variances is
//     sigma = (1/N) sum_ij A_ij^2 - (1/N^2) sum_j c1_j^2,
// so no per-column state has to leave the chip: a first pass forms every query's
// softmax statistics (running maximum and normaliser), a second pass recomputes
// the scores tile by tile, turns them into probabilities and accumulates the sum
// of squares and each key's column sum.
//
// This is an offline step (run once per model on a small validation set), so the
// kernels are kept simple: S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (a lane then
// owns one query column and 16 key rows), operands straight from global memory /
// L2, no LDS staging, no work-group barriers.  The sums that are subtracted from
// each other are kept in fp64.
#include "hack_internal.h"

namespace hack {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int kThreads = 256;          // 4 waves
constexpr int kRB1 = 4;                // 32-query blocks per wave in pass 1
constexpr int kRB2 = 2;                // 32-key blocks per wave in pass 2 (64 registers of fp64 sums per block)
constexpr int kTile1 = 4 * 32 * kRB1;  // queries per work-group in pass 1
constexpr int kTile2 = 4 * 32 * kRB2;  // keys per work-group in pass 2
constexpr float kLog2eF = 1.4426950408889634f;

__device__ __forceinline__ float pair_max(float v) {   // over the lane pair (l, l ^ 32)
  return fmaxf(v, __shfl_xor(v, 32, 64));
}
__device__ __forceinline__ float pair_sum(float v) { return v + __shfl_xor(v, 32, 64); }

__device__ __forceinline__ double shfl_xor_f64(double v, int m) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_xor(lo, m, 64);
  hi = __shfl_xor(hi, m, 64);
  return __hiloint2double(hi, lo);
}
// sum over the 32 lanes that share a half-wave (lanes differing in bits 0..4)
__device__ __forceinline__ double half_sum_f64(double v) {
#pragma unroll
  for (int m = 1; m < 32; m <<= 1) v += shfl_xor_f64(v, m);
  return v;
}

// C register r of lane l after S^T = K Q^T: key row 8(r/4) + 4(l/32) + r%4, query column l%32
__device__ __forceinline__ int c_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// Operand fragment of a 32-row block starting at `base` (row-major, D elements per
// row): lane l takes row min(l%32, n_valid-1) (rows past the end repeat the last
// valid one), elements [16kk + 8(l/32), +8) at MFMA step kk.
template <int D>
__device__ __forceinline__ void load_frags(const __bf16* base, int n_valid, int lane, bf16x8 (&f)[D / 16]) {
  const int row = min(lane & 31, n_valid - 1);
  const __bf16* p = base + (int64_t)row * D + 8 * (lane >> 5);
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) f[kk] = *reinterpret_cast<const bf16x8*>(p + 16 * kk);
}

template <int D>
__device__ __forceinline__ floatx16 scores_t(const bf16x8 (&kf)[D / 16], const bf16x8 (&qf)[D / 16]) {
  floatx16 sc;
#pragma unroll
  for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], sc, 0, 0, 0);
  return sc;
}

// Pass 1: stats[(u*N_k + i)] = (max_j s_ij, sum_j 2^((s_ij - max) * c2)), s = raw dot product, c2 = scale*log2(e).
// A wave owns kRB1 blocks of 32 queries, so every K fragment it fetches feeds kRB1 MFMAs.
template <int D>
__global__ __launch_bounds__(kThreads) void hv_rowstats(
    const UnitDesc* __restrict__ descs, const __bf16* __restrict__ q, const __bf16* __restrict__ k_cache,
    int N_k, float scale, float2* __restrict__ stats) {
  const UnitDesc d = descs[blockIdx.y];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int q0 = blockIdx.x * kTile1 + w * (32 * kRB1);
  if (q0 >= N_k) return;
  const int len = d.n_out;
  const __bf16* kg = k_cache + d.out_off * D;
  bf16x8 qf[kRB1][D / 16];
#pragma unroll
  for (int j = 0; j < kRB1; ++j) {
    const int qj = min(q0 + 32 * j, N_k - 1);   // a block past the end repeats the last query; it is not stored
    load_frags<D>(q + ((int64_t)d.unit * N_k + qj) * D, min(32, N_k - qj), lane, qf[j]);
  }
  const float c2 = scale * kLog2eF;
  float m[kRB1], l[kRB1];
#pragma unroll
  for (int j = 0; j < kRB1; ++j) {
    m[j] = -INFINITY;
    l[j] = 0.f;
  }
  for (int t0 = 0; t0 < len; t0 += 32) {
    const int nv = min(32, len - t0);
    bf16x8 kf[D / 16];
    load_frags<D>(kg + (int64_t)t0 * D, nv, lane, kf);
#pragma unroll
    for (int j = 0; j < kRB1; ++j) {
      floatx16 sc = scores_t<D>(kf, qf[j]);
      float mx = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (c_row(r, half) >= nv) sc[r] = -INFINITY;
        mx = fmaxf(mx, sc[r]);
      }
      mx = pair_max(mx);                       // finite: the block holds a valid key
      const float m_new = fmaxf(m[j], mx);
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) s += __builtin_amdgcn_exp2f((sc[r] - m_new) * c2);
      l[j] = l[j] * __builtin_amdgcn_exp2f((m[j] - m_new) * c2) + s;   // first block: 0 * exp2(-inf) = 0
      m[j] = m_new;
    }
  }
#pragma unroll
  for (int j = 0; j < kRB1; ++j) {
    const float lj = pair_sum(l[j]);
    const int qi = q0 + 32 * j + col;
    if (half == 0 && qi < N_k) stats[(int64_t)d.unit * N_k + qi] = make_float2(m[j], lj);
  }
}

// Pass 2: sigma[u] += (1/N) sum_ij p_ij^2 - (1/N^2) sum_j (sum_i p_ij)^2 over this work-group's keys.
// A wave owns kRB2 blocks of 32 keys, so every Q fragment it fetches feeds kRB2 MFMAs.
template <int D>
__global__ __launch_bounds__(kThreads) void hv_colmoments(
    const UnitDesc* __restrict__ descs, const __bf16* __restrict__ q, const __bf16* __restrict__ k_cache,
    int N_k, float scale, const float2* __restrict__ stats, double* __restrict__ sigma) {
  const UnitDesc d = descs[blockIdx.y];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int len = d.n_out;
  const int t0 = blockIdx.x * kTile2 + w * (32 * kRB2);
  if (t0 >= len) return;
  bf16x8 kf[kRB2][D / 16];
  int nv[kRB2];
#pragma unroll
  for (int j = 0; j < kRB2; ++j) {
    const int tj = min(t0 + 32 * j, len - 1);   // a block past the end repeats the last key; nv = 0 leaves it out
    nv[j] = max(0, min(32, len - (t0 + 32 * j)));
    load_frags<D>(k_cache + (d.out_off + tj) * D, max(1, min(32, len - tj)), lane, kf[j]);
  }
  const float c2 = scale * kLog2eF;
  const __bf16* qg = q + (int64_t)d.unit * N_k * D;
  const float2* st = stats + (int64_t)d.unit * N_k;
  double c1[kRB2][16], s2[kRB2][16];   // per key row: sum_i p_ij and sum_i p_ij^2 over this lane's queries
#pragma unroll
  for (int j = 0; j < kRB2; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) c1[j][r] = s2[j][r] = 0.0;
  for (int q0 = 0; q0 < N_k; q0 += 32) {
    const int nq = min(32, N_k - q0);
    bf16x8 qf[D / 16];
    load_frags<D>(qg + (int64_t)q0 * D, nq, lane, qf);
    const float2 ml = st[q0 + min(col, nq - 1)];
    const float inv = (col < nq) ? 1.f / ml.y : 0.f;   // queries past the end contribute nothing
    const float mc = ml.x * c2;
#pragma unroll
    for (int j = 0; j < kRB2; ++j) {
      const floatx16 sc = scores_t<D>(kf[j], qf);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const double p = (double)(__builtin_amdgcn_exp2f(fmaf(sc[r], c2, -mc)) * inv);
        c1[j][r] += p;
        s2[j][r] = fma(p, p, s2[j][r]);
      }
    }
  }
  // a half-wave holds 32 different queries of the same 16 key rows; rows past the
  // end of the unit repeat its last key and are left out
  const double inv_n = 1.0 / (double)N_k;
  double acc = 0.0;
#pragma unroll
  for (int j = 0; j < kRB2; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const double c = half_sum_f64(c1[j][r]) * inv_n;
      const double s = half_sum_f64(s2[j][r]) * inv_n;
      if (c_row(r, half) < nv[j]) acc += s - c * c;   // Var_i(A[i, j]) of this key
    }
  if (col == 0) atomicAdd(&sigma[d.unit], acc);
}

__global__ void hv_zero(const UnitDesc* __restrict__ descs, int n, double* __restrict__ sigma) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) sigma[descs[i].unit] = 0.0;
}

}  // namespace

void launch_head_variance(hipStream_t s, int head_dim, const UnitDesc* descs, int n_desc, int max_len, const void* q,
                          const void* k_cache, int N_k, float scale, float* stats, double* sigma) {
  if (n_desc <= 0) return;
  typedef __bf16 T;
  hipLaunchKernelGGL(hv_zero, dim3((n_desc + 63) / 64), dim3(64), 0, s, descs, n_desc, sigma);
  const dim3 g1((N_k + kTile1 - 1) / kTile1, n_desc), g2((max_len + kTile2 - 1) / kTile2, n_desc);
  if (head_dim == 64) {
    hipLaunchKernelGGL(hv_rowstats<64>, g1, dim3(kThreads), 0, s, descs, (const T*)q, (const T*)k_cache, N_k, scale,
                       (float2*)stats);
    hipLaunchKernelGGL(hv_colmoments<64>, g2, dim3(kThreads), 0, s, descs, (const T*)q, (const T*)k_cache, N_k, scale,
                       (const float2*)stats, sigma);
  } else {
    hipLaunchKernelGGL(hv_rowstats<128>, g1, dim3(kThreads), 0, s, descs, (const T*)q, (const T*)k_cache, N_k, scale,
                       (float2*)stats);
    hipLaunchKernelGGL(hv_colmoments<128>, g2, dim3(kThreads), 0, s, descs, (const T*)q, (const T*)k_cache, N_k,
                       scale, (const float2*)stats, sigma);
  }
}

}  // namespace hack
