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
// Both passes stream one operand (the keys in pass 1, the queries in pass 2) in
// 32-row blocks HBM -> LDS (global_load_lds, coalesced whole rows) through a ring
// shared by the four waves of a work-group, one barrier per block, and keep the
// other operand in registers: S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so a
// lane owns one query column and 16 key rows.  (Fetching MFMA operands straight
// from global memory, one row per lane, runs the memory pipeline at a quarter of
// its coalesced rate.)  The sums that are subtracted from each other are kept in
// fp64.
#include "device_util.h"
#include "hack_internal.h"

namespace hack {

namespace {

using namespace dev;

constexpr int kThreads = 256;          // 4 waves
constexpr int kWaves = 4;
constexpr int kRB1 = 2;                // 32-query blocks per wave in pass 1
constexpr int kRB2 = 2;                // 32-key blocks per wave in pass 2 (64 registers of fp64 sums per block)
constexpr int kTile1 = kWaves * 32 * kRB1;  // queries per work-group in pass 1
constexpr int kTile2 = kWaves * 32 * kRB2;  // keys per work-group in pass 2
constexpr int kRing = 4;               // LDS ring slots (32-row blocks)

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
// A wave owns kRB1 blocks of 32 queries (registers); the keys stream through LDS.
template <int D>
__global__ __launch_bounds__(kThreads, 2) void hv_rowstats(
    const UnitDesc* __restrict__ descs, const __bf16* __restrict__ q, const __bf16* __restrict__ k_cache,
    int N_k, float scale, float2* __restrict__ stats) {
  using St = BlockStream<D, kWaves>;
  constexpr int KK = D / 16;
  __shared__ __attribute__((aligned(1024))) __bf16 ring[kRing][St::BLK];
  const UnitDesc d = descs[blockIdx.y];
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 31, half = lane >> 5;
  const int q0 = blockIdx.x * kTile1 + w * (32 * kRB1);   // may lie past N_k: the wave still copies and synchronises
  const int len = d.n_out;
  const int n_blocks = (len + 31) / 32;
  St st;
  st.init(k_cache + d.out_off * D, len, &ring[0][0], lane, w);
  st.issue(0, 0);
  if (n_blocks > 1) st.issue(1, 1);

  bf16x8 qf[kRB1][KK];
#pragma unroll
  for (int j = 0; j < kRB1; ++j) {
    // a block past the end repeats the last query; it is not stored
    const int qj = min(q0 + 32 * j, N_k - 1);
    load_frags<D>(q + ((int64_t)d.unit * N_k + qj) * D, min(32, N_k - qj), lane, qf[j]);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) asm volatile("" ::"v"(qf[j][kk]));   // waited for here, not inside the loop
  }
  const float c2 = scale * kLog2eF;
  float m[kRB1], l[kRB1];
#pragma unroll
  for (int j = 0; j < kRB1; ++j) {
    m[j] = -INFINITY;
    l[j] = 0.f;
  }
  for (int b = 0; b < n_blocks; ++b) {
    if (b + 1 < n_blocks) dma_wait_but<St::IPW>();   // this wave's part of block b has landed
    else dma_wait_but<0>();
    __syncthreads();                                  // all of block b is visible; the slot of block b-2 is free
    if (b + 2 < n_blocks) st.issue(b + 2, (b + 2) % kRing);
    const __bf16* slot = &ring[b % kRing][0];
    const int nv = min(32, len - b * 32);
    bf16x8 kf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[kk] = lds_frag<D>(slot, col, half, kk);
#pragma unroll
    for (int j = 0; j < kRB1; ++j) {
      floatx16 sc = scores_t<D>(kf, qf[j]);
      if (nv < 32) {                           // only the unit's last block is ragged
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (c_row(r, half) >= nv) sc[r] = -INFINITY;
      }
      float mx = sc[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sc[r]);
      mx = pair_max(mx);                       // finite: the block holds a valid key
      const float m_new = fmaxf(m[j], mx);
      const float mc = m_new * c2;
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) s += __builtin_amdgcn_exp2f(fmaf(sc[r], c2, -mc));
      l[j] = l[j] * __builtin_amdgcn_exp2f(fmaf(m[j], c2, -mc)) + s;   // first block: 0 * exp2(-inf) = 0
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
// A wave owns kRB2 blocks of 32 keys (registers); the queries and their pass-1
// statistics stream through LDS (every wave copies the 256 bytes of statistics
// of a block itself, so all waves issue the same number of copies per block).
template <int D>
__global__ __launch_bounds__(kThreads, 2) void hv_colmoments(
    const UnitDesc* __restrict__ descs, const __bf16* __restrict__ q, const __bf16* __restrict__ k_cache,
    int N_k, float scale, const float2* __restrict__ stats, double* __restrict__ sigma) {
  using St = BlockStream<D, kWaves>;
  constexpr int KK = D / 16;
  __shared__ __attribute__((aligned(1024))) __bf16 ring[kRing][St::BLK];
  __shared__ __attribute__((aligned(256))) float2 st_ring[kRing][kWaves][32];
  const UnitDesc d = descs[blockIdx.y];
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 31, half = lane >> 5;
  const int len = d.n_out;
  if ((int)blockIdx.x * kTile2 >= len) return;   // whole work-group past the end of this unit
  const int t0 = blockIdx.x * kTile2 + w * (32 * kRB2);
  const int n_blocks = (N_k + 31) / 32;
  St st;
  st.init(q + (int64_t)d.unit * N_k * D, N_k, &ring[0][0], lane, w);
  const float* stat_base = reinterpret_cast<const float*>(stats + (int64_t)d.unit * N_k);
  const unsigned st_lds = lds_addr_of(&st_ring[0][0][0]);
  // block b of the queries and its statistics: lane l copies float l of the
  // block's 64 (a query past the end repeats the last one; it is masked below)
  auto issue = [&](int b, int slot) {
    st.issue(b, slot);
    const int qi = min(b * 32 + (lane >> 1), N_k - 1);
    load_to_lds_dword(stat_base, (unsigned)(qi * 2 + (lane & 1)) * 4u, st_lds + (unsigned)((slot * kWaves + w) * 256));
  };
  issue(0, 0);
  if (n_blocks > 1) issue(1, 1);

  // a wave whose keys all lie past the end of the unit still takes part in the copies and barriers
  bf16x8 kf[kRB2][KK];
  int nv[kRB2];
#pragma unroll
  for (int j = 0; j < kRB2; ++j) {
    const int tj = min(t0 + 32 * j, len - 1);   // a block past the end repeats the last key; nv = 0 leaves it out
    nv[j] = max(0, min(32, len - (t0 + 32 * j)));
    load_frags<D>(k_cache + (d.out_off + tj) * D, max(1, min(32, len - tj)), lane, kf[j]);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) asm volatile("" ::"v"(kf[j][kk]));   // waited for here, not inside the loop
  }
  const float c2 = scale * kLog2eF;
  double c1[kRB2][16], s2[kRB2][16];   // per key row: sum_i p_ij and sum_i p_ij^2 over this lane's queries
#pragma unroll
  for (int j = 0; j < kRB2; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) c1[j][r] = s2[j][r] = 0.0;
  for (int b = 0; b < n_blocks; ++b) {
    if (b + 1 < n_blocks) dma_wait_but<St::IPW + 1>();   // this wave's copies of block b have landed
    else dma_wait_but<0>();
    __syncthreads();                                      // all of block b is visible; the slot of block b-2 is free
    if (b + 2 < n_blocks) issue(b + 2, (b + 2) % kRing);
    const __bf16* slot = &ring[b % kRing][0];
    const int nq = min(32, N_k - b * 32);
    const float2 ml = st_ring[b % kRing][w][col];
    // p = 2^(s c2 - (m c2 + log2 l)): the normaliser rides in the exponent; queries past the end give 2^-inf = 0
    const float mc = (col < nq) ? fmaf(ml.x, c2, __builtin_amdgcn_logf(ml.y)) : INFINITY;
    // every query fragment feeds the MFMAs of all kRB2 key blocks and is then dropped
    floatx16 sc[kRB2];
#pragma unroll
    for (int j = 0; j < kRB2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[j][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const bf16x8 qf = lds_frag<D>(slot, col, half, kk);
#pragma unroll
      for (int j = 0; j < kRB2; ++j) sc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j][kk], qf, sc[j], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < kRB2; ++j) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const double p = (double)__builtin_amdgcn_exp2f(fmaf(sc[j][r], c2, -mc));
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
  if (col == 0 && t0 < len) atomicAdd(&sigma[d.unit], acc);
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
