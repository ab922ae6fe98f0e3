// Attention of the current scale's queries over the ragged compressed cache
// (Preliminaries, attention equation: O = Softmax(scale * Q K^T) V, no mask
// inside a scale step) on gfx950.
//
// bf16 path (flash-style, one pass over K/V with an online softmax):
//   * work item = (unit, tile of 4 waves x NQB x 32 queries); K/V tiles of 64
//     keys are staged once per work-group in LDS and shared by the four waves.
//   * S^T = K Q^T with v_mfma_f32_32x32x16_bf16: the accumulator then holds,
//     per lane, one query column and 16 key rows, so the softmax row reductions
//     are in-lane plus one exchange with lane^32, and the running max / rescale
//     factor are per-lane scalars.
//   * O^T += V^T P^T: P^T goes from the accumulator registers straight into the
//     B operand (C rows 8(r/4)+4h+r%4 of registers 8s..8s+7 are exactly two runs
//     of four consecutive keys), and V^T comes from row-major V in LDS through
//     the transposing LDS read (ds_read_b64_tr_b16), four keys per read.
//   * LDS rows are padded (K +16 B, V +32 B) so the b128 K reads and the
//     transposing V reads are bank-conflict free.
// fp32 path: one query per lane, fp32 FMA, K/V rows broadcast from LDS; exact
// enough for the 1e-4 bar and only used for the small fp32 configuration.
#include "hack_internal.h"

namespace hack {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short shortx4;

constexpr float kLog2eF = 1.4426950408889634f;

// ---------------------------------------------------------------------------
// fp32 / generic path
// ---------------------------------------------------------------------------
__device__ __forceinline__ float ld_f(const float* p) { return *p; }
__device__ __forceinline__ float ld_f(const __bf16* p) { return (float)(*p); }
__device__ __forceinline__ void st_f(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_f(__bf16* p, float v) { *p = (__bf16)v; }

constexpr int kGenQ = 64;   // queries per work-group (one per lane)
constexpr int kGenKT = 32;  // keys per LDS tile

template <typename T, int D>
__global__ __launch_bounds__(kGenQ) void attn_generic(
    const UnitDesc* __restrict__ descs, const AttnItem* __restrict__ items, const T* __restrict__ q,
    const T* __restrict__ k_cache, const T* __restrict__ v_cache, int N_k, float scale,
    T* __restrict__ out) {
  const AttnItem it = items[blockIdx.x];
  if (it.desc < 0) return;
  const UnitDesc d = descs[it.desc];
  const int len = d.n_out;
  const int qi = it.q_tile * kGenQ + threadIdx.x;
  const bool qvalid = qi < N_k;
  const int64_t qrow = (int64_t)d.unit * N_k + (qvalid ? qi : N_k - 1);

  __shared__ float ks[kGenKT][D];
  __shared__ float vs[kGenKT][D];

  float qr[D], o[D];
#pragma unroll
  for (int c = 0; c < D; ++c) {
    qr[c] = ld_f(q + qrow * D + c) * scale;
    o[c] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  for (int t0 = 0; t0 < len; t0 += kGenKT) {
    const int nk = min(kGenKT, len - t0);
    __syncthreads();
    for (int e = threadIdx.x; e < nk * D; e += kGenQ) {
      const int r = e / D, c = e % D;
      ks[r][c] = ld_f(k_cache + (d.out_off + t0 + r) * D + c);
      vs[r][c] = ld_f(v_cache + (d.out_off + t0 + r) * D + c);
    }
    __syncthreads();
    for (int r = 0; r < nk; ++r) {
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) s = fmaf(qr[c], ks[r][c], s);
      const float mn = fmaxf(m, s);
      const float a = __expf(m - mn), p = __expf(s - mn);
      l = l * a + p;
#pragma unroll
      for (int c = 0; c < D; ++c) o[c] = fmaf(o[c], a, p * vs[r][c]);
      m = mn;
    }
  }
  if (qvalid) {
    const float inv = 1.f / l;
#pragma unroll
    for (int c = 0; c < D; ++c) st_f(out + qrow * D + c, o[c] * inv);
  }
}

// ---------------------------------------------------------------------------
// bf16 MFMA path
// ---------------------------------------------------------------------------
constexpr int kKT = 64;      // keys per LDS tile
constexpr int kKPad = 8;     // bf16 elements of padding per K row (16 B)
constexpr int kVPad = 16;    // bf16 elements of padding per V row (32 B)

__device__ __forceinline__ bf16x4 lds_read_tr(const __bf16* p) {
  shortx4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) shortx4*)(p));
  return __builtin_bit_cast(bf16x4, v);
}

template <int D, int NQB>
__global__ __launch_bounds__(256) void attn_mfma(
    const UnitDesc* __restrict__ descs, const AttnItem* __restrict__ items,
    const __bf16* __restrict__ q, const __bf16* __restrict__ k_cache,
    const __bf16* __restrict__ v_cache, int N_k, float scale,
    __bf16* __restrict__ out) {
  constexpr int KK = D / 16;        // MFMA steps over head_dim for S^T
  constexpr int MB = D / 32;        // 32-row blocks of O^T
  constexpr int KS = D + kKPad;     // LDS row strides in elements
  constexpr int VS = D + kVPad;
  constexpr int QW = 32 * NQB;      // queries per wave
  constexpr int CPR = D / 8;        // 16-byte chunks per row

  const AttnItem it = items[blockIdx.x];
  if (it.desc < 0) return;
  const UnitDesc d = descs[it.desc];
  const int len = d.n_out;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int col = lane & 31, half = lane >> 5;

  __shared__ __attribute__((aligned(16))) __bf16 Ks[kKT * KS];
  __shared__ __attribute__((aligned(16))) __bf16 Vs[kKT * VS];

  // Q fragments (B operand of S^T = K Q^T): query col, head-dim slice [16kk + 8h, +8).
  const int q0 = it.q_tile * (4 * QW) + w * QW;
  bf16x8 qf[NQB][KK];
#pragma unroll
  for (int nb = 0; nb < NQB; ++nb) {
    const int qi = min(q0 + nb * 32 + col, N_k - 1);
    const __bf16* qrow = q + ((int64_t)d.unit * N_k + qi) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      qf[nb][kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * half);
  }

  floatx16 o[NQB][MB];
#pragma unroll
  for (int nb = 0; nb < NQB; ++nb)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[nb][mb][r] = 0.f;
  float m_run[NQB], l_run[NQB];
#pragma unroll
  for (int nb = 0; nb < NQB; ++nb) {
    m_run[nb] = -INFINITY;
    l_run[nb] = 0.f;
  }
  const float c2 = scale * kLog2eF;

  const uint4* kg = reinterpret_cast<const uint4*>(k_cache + d.out_off * D);
  const uint4* vg = reinterpret_cast<const uint4*>(v_cache + d.out_off * D);

  for (int t0 = 0; t0 < len; t0 += kKT) {
    __syncthreads();  // previous tile fully consumed
    // ---- stage K/V tile (rows beyond len are zero) ----
#pragma unroll
    for (int e = tid; e < kKT * CPR; e += 256) {
      const int r = e / CPR, ch = e % CPR;
      uint4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
      if (t0 + r < len) {
        kv = kg[(int64_t)(t0 + r) * CPR + ch];
        vv = vg[(int64_t)(t0 + r) * CPR + ch];
      }
      *reinterpret_cast<uint4*>(&Ks[r * KS + ch * 8]) = kv;
      *reinterpret_cast<uint4*>(&Vs[r * VS + ch * 8]) = vv;
    }
    __syncthreads();
    const bool tail = (t0 + kKT > len);

#pragma unroll
    for (int kb = 0; kb < kKT / 32; ++kb) {
      // ---- S^T block: 32 keys x QW queries ----
      floatx16 s[NQB];
#pragma unroll
      for (int nb = 0; nb < NQB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[nb][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Ks[(kb * 32 + col) * KS + 16 * kk + 8 * half]);
#pragma unroll
        for (int nb = 0; nb < NQB; ++nb)
          s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[nb][kk], s[nb], 0, 0, 0);
      }
      if (tail) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = t0 + kb * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
          if (key >= len) {
#pragma unroll
            for (int nb = 0; nb < NQB; ++nb) s[nb][r] = -INFINITY;
          }
        }
      }
      // ---- online softmax (per lane: one query, 16 keys; partner lane^32 has the other 16) ----
      bf16x8 pf[NQB][2];
#pragma unroll
      for (int nb = 0; nb < NQB; ++nb) {
        float mx = s[nb][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[nb][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run[nb], mx);   // finite: key 0 of the tile is valid
        const float mc = m_new * c2;
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[nb][r], c2, -mc));
          psum += p;
          pf[nb][r >> 3][r & 7] = (__bf16)p;
        }
        if (__any(m_new > m_run[nb])) {
          const float a = __builtin_amdgcn_exp2f((m_run[nb] - m_new) * c2);
          l_run[nb] *= a;
#pragma unroll
          for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[nb][mb][r] *= a;
        }
        l_run[nb] += psum;
        m_run[nb] = m_new;
      }
      // ---- O^T += V^T P^T ----
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int sg = 0; sg < 2; ++sg) {
          // lanes 4e+qd of a 16-lane group address key (16sg + 4h + e), head-dim 32mb + 16(g&1) + 4qd
          const int g = lane >> 4, e = (lane >> 2) & 3, qd = lane & 3;
          const __bf16* vp =
              &Vs[(kb * 32 + 16 * sg + 4 * half + e) * VS + 32 * mb + 16 * (g & 1) + 4 * qd];
          const bf16x4 v0 = lds_read_tr(vp);
          const bf16x4 v1 = lds_read_tr(vp + 8 * VS);
          bf16x8 vf;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            vf[i] = v0[i];
            vf[4 + i] = v1[i];
          }
#pragma unroll
          for (int nb = 0; nb < NQB; ++nb)
            o[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[nb][sg], o[nb][mb], 0, 0, 0);
        }
      }
    }
  }

  // ---- normalise and store: lane holds query col, head-dim rows 32mb + 8(r/4) + 4h + r%4 ----
#pragma unroll
  for (int nb = 0; nb < NQB; ++nb) {
    const float l = l_run[nb] + __shfl_xor(l_run[nb], 32, 64);
    const float inv = 1.f / l;
    const int qi = q0 + nb * 32 + col;
    if (qi < N_k) {
      __bf16* orow = out + ((int64_t)d.unit * N_k + qi) * D;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          bf16x4 pk;
#pragma unroll
          for (int i = 0; i < 4; ++i) pk[i] = (__bf16)(o[nb][mb][4 * r4 + i] * inv);
          *reinterpret_cast<bf16x4*>(orow + 32 * mb + 8 * r4 + 4 * half) = pk;
        }
      }
    }
  }
}

}  // namespace

int attn_q_tile_rows(int dtype, int head_dim) {
  (void)head_dim;
  return dtype == 1 ? kGenQ : 4 * 32 * 1;
}

void launch_attn(hipStream_t s, int dtype, int head_dim, const UnitDesc* descs, const AttnItem* items,
                 int n_items, int q_tile_rows, const void* q, const void* k_cache,
                 const void* v_cache, int N_k, float scale, void* out) {
  if (n_items <= 0) return;
  (void)q_tile_rows;
  if (dtype == 1) {
    if (head_dim == 64)
      hipLaunchKernelGGL((attn_generic<float, 64>), dim3(n_items), dim3(kGenQ), 0, s, descs, items,
                         (const float*)q, (const float*)k_cache, (const float*)v_cache, N_k, scale,
                         (float*)out);
    else
      hipLaunchKernelGGL((attn_generic<float, 128>), dim3(n_items), dim3(kGenQ), 0, s, descs, items,
                         (const float*)q, (const float*)k_cache, (const float*)v_cache, N_k, scale,
                         (float*)out);
  } else {
    typedef __bf16 T;
    if (head_dim == 64)
      hipLaunchKernelGGL((attn_mfma<64, 1>), dim3(n_items), dim3(256), 0, s, descs, items,
                         (const T*)q, (const T*)k_cache, (const T*)v_cache, N_k, scale, (T*)out);
    else
      hipLaunchKernelGGL((attn_mfma<128, 1>), dim3(n_items), dim3(256), 0, s, descs, items,
                         (const T*)q, (const T*)k_cache, (const T*)v_cache, N_k, scale, (T*)out);
  }
}

}  // namespace hack
