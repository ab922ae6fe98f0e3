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
//   * K/V tiles are double-buffered and loaded HBM -> LDS directly (no register
//     round trip), one barrier per tile; an XOR swizzle of 16-byte chunks keeps
//     the b128 K reads and the transposing V reads bank-conflict free.
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

__device__ __forceinline__ bf16x4 lds_read_tr(const __bf16* p) {
  shortx4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) shortx4*)(p));
  return __builtin_bit_cast(bf16x4, v);
}

// K/V tiles go from HBM straight into LDS (global_load_lds, 16 B per lane, one
// contiguous KiB per wave instruction), so LDS rows cannot be padded; bank
// conflicts are avoided by a swizzle instead: the 16-byte chunk at position c of
// LDS row r holds global chunk c ^ f(r).  The LDS moves 256 bytes per clock (64
// banks of 4 bytes), so one phase of a b128 read covers 16 consecutive lanes (16
// key rows at one chunk position) and one phase of a transposing b64 read covers
// 32 lanes (4 key rows x 64 bytes); f spreads those over all 16 chunk slots of
// 256 bytes:  D=128 (256-byte rows): f_K(r) = r & 15,        f_V(r) = 4 (r & 3)
//             D=64  (128-byte rows): f_K(r) = (r >> 1) & 7,  f_V(r) = 4 ((r >> 1) & 1)
// (measured: SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE was exactly 0.5 with the
// 32-bank variants r & 7 and 2 (r & 3)).
template <int D> __device__ __forceinline__ int swz_k(int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); }
template <int D> __device__ __forceinline__ int swz_v(int r) { return D == 128 ? 4 * (r & 3) : 4 * ((r >> 1) & 1); }

// The copy is issued from inline assembly so that the compiler does not wait for
// it before unrelated LDS reads (it would otherwise drain every outstanding LDS
// write of this kind before the next ds_read, which serialises load and
// compute).  The matching wait is dma_wait_all(), placed by hand before the
// barrier that publishes the tile.  lds_addr is the wave-uniform LDS byte
// address of the KiB this wave instruction fills (lane l writes bytes [16l, 16l+16)).
__device__ __forceinline__ void load_to_lds(const __bf16* src, const __bf16* lds_wave_base) {
  const unsigned lds_addr = (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void*)lds_wave_base;
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(src), "s"(lds_addr) : "memory", "m0");
}
__device__ __forceinline__ void dma_wait_all() {
  __builtin_amdgcn_sched_barrier(0);  // keep the tile's compute above the wait
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// max / sum over the lane pair (l, l ^ 32) with one VALU swap instead of an LDS permute
__device__ __forceinline__ float pair_max(float v) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__builtin_bit_cast(float, (unsigned)r[0]), __builtin_bit_cast(float, (unsigned)r[1]));
}
__device__ __forceinline__ float pair_sum(float v) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}

// NW waves per work-group, each wave owns 32 queries; two work-groups share a CU.
template <int D, int NW>
__global__ __launch_bounds__(64 * NW, 2) void attn_mfma(
    const UnitDesc* __restrict__ descs, const AttnItem* __restrict__ items,
    const __bf16* __restrict__ q, const __bf16* __restrict__ k_cache,
    const __bf16* __restrict__ v_cache, int N_k, float scale,
    __bf16* __restrict__ out) {
  constexpr int KK = D / 16;        // MFMA steps over head_dim for S^T
  constexpr int MB = D / 32;        // 32-row blocks of O^T
  constexpr int CPR = D / 8;        // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;     // tile rows covered by one wave-wide load instruction
  constexpr int IPW = (kKT / RPI) / NW;  // load instructions per wave, tile and tensor

  const AttnItem it = items[blockIdx.x];
  if (it.desc < 0) return;
  const UnitDesc d = descs[it.desc];
  const int len = d.n_out;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;

  __shared__ __attribute__((aligned(1024))) __bf16 Ks[2][kKT * D];
  __shared__ __attribute__((aligned(1024))) __bf16 Vs[2][kKT * D];

  // Q fragments (B operand of S^T = K Q^T): query col, head-dim slice [16kk + 8h, +8).
  const int q0 = it.q_tile * (NW * 32) + w * 32;
  bf16x8 qf[KK];
  {
    const int qi = min(q0 + col, N_k - 1);
    const __bf16* qrow = q + ((int64_t)d.unit * N_k + qi) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * half);
    // Consume the fragments here so that their loads are waited for before the
    // main loop: a vmcnt wait inside the loop would also drain the tile copies
    // that are meant to stay in flight.
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) asm volatile("" ::"v"(qf[kk]));
  }

  floatx16 o[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[mb][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c2 = scale * kLog2eF;

  const __bf16* kg = k_cache + d.out_off * D;
  const __bf16* vg = v_cache + d.out_off * D;

  // Rows past the end repeat the last valid row (finite data); their scores are
  // masked to -inf below, so their probabilities are exactly 0.
  auto issue = [&](int t0, int buf) {
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      const int ci = w + i * NW;                       // wave-uniform KiB index inside the tile
      const int r = ci * RPI + lane / CPR, c = lane % CPR;
      const int64_t grow = (int64_t)min(t0 + r, len - 1) * D;
      load_to_lds(kg + grow + ((c ^ swz_k<D>(r)) & (CPR - 1)) * 8, &Ks[buf][ci * 512]);
      load_to_lds(vg + grow + ((c ^ swz_v<D>(r)) & (CPR - 1)) * 8, &Vs[buf][ci * 512]);
    }
  };

  // per-lane LDS element offsets of the operand reads (tile-relative)
  int k_off[KK];           // K operand: row col (+32 kb), chunk 2kk + half
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) k_off[kk] = col * D + (((2 * kk + half) ^ swz_k<D>(col)) & (CPR - 1)) * 8;
  const int g = lane >> 4, e = (lane >> 2) & 3, qd = lane & 3;
  int v_off[MB];           // V^T operand: row 4 half + e (+16 sg, +32 kb, +8), head-dim 32mb + 16(g&1) + 4qd
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
    v_off[mb] = (4 * half + e) * D + (((4 * mb + 2 * (g & 1) + (qd >> 1)) ^ swz_v<D>(e)) & (CPR - 1)) * 8 + 4 * (qd & 1);

  const int n_tiles = (len + kKT - 1) / kKT;
  issue(0, 0);
  dma_wait_all();
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    const int t0 = t * kKT;
    const int buf = t & 1;
    if (t + 1 < n_tiles) issue(t0 + kKT, buf ^ 1);   // lands while this tile is consumed
    const bool tail = (t0 + kKT > len);
    const __bf16* Kt = Ks[buf];
    const __bf16* Vt = Vs[buf];

#pragma unroll
    for (int kb = 0; kb < kKT / 32; ++kb) {
      if (t0 + kb * 32 >= len) break;  // whole block past the end (wave-uniform)
      // ---- S^T block: 32 keys x 32 queries ----
      floatx16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Kt[kb * 32 * D + k_off[kk]]);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s, 0, 0, 0);
      }
      if (tail) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = t0 + kb * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
          if (key >= len) s[r] = -INFINITY;
        }
      }
      // ---- online softmax (per lane: one query, 16 keys; partner lane^32 has the other 16) ----
      float mx = s[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
      mx = pair_max(mx);
      const float m_new = fmaxf(m_run, mx);   // finite: the block holds a valid key
      const float mc = m_new * c2;
      float psum = 0.f;
      bf16x8 pf[2];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[r], c2, -mc));
        psum += p;
        pf[r >> 3][r & 7] = (__bf16)p;
      }
      if (__any(m_new > m_run)) {
        const float a = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
        l_run *= a;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[mb][r] *= a;
      }
      l_run += psum;
      m_run = m_new;
      // ---- O^T += V^T P^T ----
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int sg = 0; sg < 2; ++sg) {
          const __bf16* vp = &Vt[(kb * 32 + 16 * sg) * D + v_off[mb]];
          const bf16x4 v0 = lds_read_tr(vp);
          const bf16x4 v1 = lds_read_tr(vp + 8 * D);
          bf16x8 vf;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            vf[i] = v0[i];
            vf[4 + i] = v1[i];
          }
          o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sg], o[mb], 0, 0, 0);
        }
      }
    }
    dma_wait_all();
    __syncthreads();  // next tile has landed for every wave; this tile is free to overwrite
  }

  // ---- normalise and store: lane holds query col, head-dim rows 32mb + 8(r/4) + 4h + r%4 ----
  const float l = pair_sum(l_run);
  const float inv = 1.f / l;
  const int qi = q0 + col;
  if (qi < N_k) {
    __bf16* orow = out + ((int64_t)d.unit * N_k + qi) * D;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 pk;
#pragma unroll
        for (int i = 0; i < 4; ++i) pk[i] = (__bf16)(o[mb][4 * r4 + i] * inv);
        *reinterpret_cast<bf16x4*>(orow + 32 * mb + 8 * r4 + 4 * half) = pk;
      }
    }
  }
}

}  // namespace

// Queries per work item.
int attn_q_tile_rows(int dtype, int head_dim, int n_units, int N_k) {
  (void)head_dim; (void)n_units; (void)N_k;
  return dtype == 1 ? kGenQ : 128;
}

template <int D, int NW>
static void launch_mfma_t(hipStream_t s, const UnitDesc* descs, const AttnItem* items, int n_items,
                          const void* q, const void* k_cache, const void* v_cache, int N_k,
                          float scale, void* out) {
  typedef __bf16 T;
  hipLaunchKernelGGL((attn_mfma<D, NW>), dim3(n_items), dim3(64 * NW), 0, s, descs, items,
                     (const T*)q, (const T*)k_cache, (const T*)v_cache, N_k, scale, (T*)out);
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
    return;
  }
  if (head_dim == 64) launch_mfma_t<64, 4>(s, descs, items, n_items, q, k_cache, v_cache, N_k, scale, out);
  else launch_mfma_t<128, 4>(s, descs, items, n_items, q, k_cache, v_cache, N_k, scale, out);
}

}  // namespace hack
