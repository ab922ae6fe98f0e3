// Device-side helpers shared by the gfx950 MFMA kernels of this library
// (attention, score, head variance, merge): vector types, the HBM -> LDS copy
// and its wait, the LDS swizzles, lane-pair exchanges and the accumulator
// layout of v_mfma_f32_32x32x16_bf16.  HIP device code only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hack {
namespace dev {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short shortx4;

constexpr float kLog2eF = 1.4426950408889634f;

// ---- LDS layout -------------------------------------------------------------
// Tiles go from HBM straight into LDS (one contiguous KiB per wave instruction),
// so LDS rows cannot be padded; bank conflicts are avoided by a swizzle instead:
// the 16-byte chunk at position c of LDS row r holds global chunk c ^ f(r).  The
// LDS moves 256 bytes per clock (64 banks of 4 bytes), so one phase of a b128
// read covers 16 consecutive lanes (16 rows at one chunk position) and one phase
// of a transposing b64 read covers 32 lanes (4 rows x 64 bytes); f spreads those
// over all 16 chunk slots of 256 bytes:
//   D=128 (256-byte rows): f_K(r) = r & 15,        f_V(r) = 4 (r & 3)
//   D=64  (128-byte rows): f_K(r) = (r >> 1) & 7,  f_V(r) = 4 ((r >> 1) & 1)
// (measured: SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE was exactly 0.5 with the
// 32-bank variants r & 7 and 2 (r & 3), and is 0 with these).
// swz_k: tiles read as MFMA A/B operands with ds_read_b128 (row = lane % 32).
// swz_v: tiles read with the transposing ds_read_b64_tr_b16 (V^T operand).
template <int D> __device__ __forceinline__ int swz_k(int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); }
template <int D> __device__ __forceinline__ int swz_v(int r) { return D == 128 ? 4 * (r & 3) : 4 * ((r >> 1) & 1); }

__device__ __forceinline__ unsigned lds_addr_of(const void* p) {
  return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// Transposing LDS read: four consecutive rows of one 16-bit column group per lane.
__device__ __forceinline__ bf16x4 lds_read_tr(const __bf16* p) {
  shortx4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)(p));
  return __builtin_bit_cast(bf16x4, v);
}

// ---- HBM -> LDS copies ------------------------------------------------------
// One KiB (dwordx4) or 256 bytes (dword) per wave instruction without a register
// round trip: lane l writes LDS bytes [lds_addr + 16 l, +16) resp. [lds_addr + 4 l, +4).
// Issued from inline assembly so that the compiler does not wait for the copy
// before unrelated LDS reads (it would otherwise drain every outstanding copy
// before the next ds_read, which serialises load and compute); dma_wait_but<N>()
// is the matching wait, placed by hand before the barrier that publishes a tile.
// lds_addr is wave-uniform.
// per-lane source address:
__device__ __forceinline__ void load_to_lds(const void* src, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_addr) : "memory", "m0");
}
// wave-uniform base address + per-lane byte offset (no per-lane 64-bit address
// arithmetic: the offsets inside a full tile are loop invariant):
__device__ __forceinline__ void load_to_lds(const void* base, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(base), "s"(lds_addr) : "memory", "m0");
}
__device__ __forceinline__ void load_to_lds_dword(const void* base, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(voff), "s"(base), "s"(lds_addr) : "memory", "m0");
}
// Waits until at most N of this wave's vector-memory loads are outstanding.
// Loads return in order, so everything issued before the newest N has landed.
template <int N> __device__ __forceinline__ void dma_wait_but() {
  __builtin_amdgcn_sched_barrier(0);   // keep the consumers of the tile below the wait, the producers above
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
  __builtin_amdgcn_sched_barrier(0);
}

// ---- lane-pair exchanges ----------------------------------------------------
// The 32x32 accumulator splits a column over the lane pair (l, l ^ 32); one VALU
// swap instead of an LDS permute brings the two halves together.
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
// the partner lane's value
__device__ __forceinline__ unsigned pair_other(unsigned u) {
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // after the swap r[0] holds, in lanes >= 32, what lanes < 32 had, and r[1] the converse
  return (threadIdx.x & 32) ? (unsigned)r[0] : (unsigned)r[1];
}

__device__ __forceinline__ double shfl_xor_f64(double v, int m) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_xor(lo, m, 64);
  hi = __shfl_xor(hi, m, 64);
  return __hiloint2double(hi, lo);
}

// All-reduce sum over the 32 lanes of a half-wave, fp64, without touching LDS
// memory: two quad permutes, the two row mirrors (DPP moves of both dwords),
// then a swizzle across the 16-lane rows.
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

// ---- accumulator layout -----------------------------------------------------
// C = A B with v_mfma_f32_32x32x16_bf16: A operand row = lane % 32, B operand
// column = lane % 32, both holding the 8 contraction elements [16 kk + 8 (lane / 32), +8)
// at step kk.  C register r of lane l is row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32.
__device__ __forceinline__ int c_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// ---- streamed and resident MFMA operands --------------------------------------
// Streams the 32-row blocks of a row-major [n_rows, D] bf16 matrix into an LDS
// ring of 32-row slots (swz_k layout); the WAVES waves of the work-group each copy
// their share of a block (IPW instructions).  Rows past the end repeat the last row.
template <int D, int WAVES>
struct BlockStream {
  static constexpr int CPR = D / 8;               // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;            // rows per copy instruction
  static constexpr int IPW = (32 / RPI) / WAVES; // copy instructions per wave and block
  static constexpr int BLK = 32 * D;              // elements per block
  const __bf16* base;
  int n_rows, lane, w;
  unsigned lds0;
  unsigned src[IPW];
  __device__ __forceinline__ void init(const __bf16* base_, int n_rows_, const __bf16* ring, int lane_, int w_) {
    base = base_; n_rows = n_rows_; lane = lane_; w = w_;
    lds0 = lds_addr_of(ring);
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      const int r = (w + i * WAVES) * RPI + lane / CPR, c = lane % CPR;
      src[i] = (unsigned)(r * D + ((c ^ swz_k<D>(r)) & (CPR - 1)) * 8) * 2u;
    }
  }
  __device__ __forceinline__ void issue(int b, int slot) const {
    const int r0 = b * 32;
    const __bf16* blk = base + (int64_t)r0 * D;
    if (r0 + 32 <= n_rows) {
#pragma unroll
      for (int i = 0; i < IPW; ++i)
        load_to_lds(blk, src[i], lds0 + (unsigned)((slot * BLK + (w + i * WAVES) * 512) * 2));
    } else {
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        const int r = (w + i * WAVES) * RPI + lane / CPR, c = lane % CPR;
        const int rc = min(r, n_rows - 1 - r0);
        load_to_lds(blk, (unsigned)(rc * D + ((c ^ swz_k<D>(r)) & (CPR - 1)) * 8) * 2u,
                       lds0 + (unsigned)((slot * BLK + (w + i * WAVES) * 512) * 2));
      }
    }
  }
};

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

// Operand fragment kk of the block in an LDS slot: row lane%32, chunk 2kk + lane/32
template <int D>
__device__ __forceinline__ bf16x8 lds_frag(const __bf16* slot, int col, int half, int kk) {
  constexpr int CPR = D / 8;
  return *reinterpret_cast<const bf16x8*>(&slot[col * D + (((2 * kk + half) ^ swz_k<D>(col)) & (CPR - 1)) * 8]);
}

}  // namespace dev
}  // namespace hack
