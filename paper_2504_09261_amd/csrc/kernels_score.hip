// Subset-attention importance (Sec. 4.4, "Importance Estimation via Efficient
// Subset Attention") on gfx950:
//     A~ = Softmax(scale * Q~ K^T),   importance[j] = sum_i A~[i, j]
// over the uncompressed keys of the step (cache rows followed by the current
// scale's rows, read from their two homes without materialising the concat).
//
// The column sum needs each row's softmax normaliser l_i before any key's
// importance can be formed.
//
// bf16 (score_fused): one launch that reads K once.  One
// v_mfma_f32_32x32x16_bf16 column block holds all 32 observation rows; a wave
// takes 128 keys as four 32-key tiles copied HBM -> LDS asynchronously, parks
// the logits in registers, publishes its work-group's row sums in a per-unit
// exchange area, collects (bounded wait) those of the unit's other work-groups
// and then writes importance_j = sum_i 2^t_ij / l_i from the parked logits.
// fp32 (score_generic): two streaming passes over (unit, chunk of 256 keys),
// plain fp64 FMA dot products, one key per lane:
//   pass 1  per chunk and observation row: max logit and sum of exp(logit - max)
//   pass 2  combine the chunk partials of the unit, recompute the logits and
//           write importance[j] = sum_i exp(s_ij - m_i) / l_i.
// n_obs <= 32 rows against every key is a skinny product (~31 flop per byte), so
// ALU is spent on accuracy: logits are accumulated in fp64 and the exponential
// is range-reduced exactly, which keeps float32 importance within a few ulp of
// the exact value; the ranking that follows is decided on those float32 numbers.
#include <mutex>

#include "device_util.h"
#include "hack_internal.h"

namespace hack {

namespace {

using namespace dev;

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

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(__bf16 v) { return (float)v; }

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
// C = Q~ K^T per 32-key tile: A operand = Q~ (row = observation query lane%32),
// B operand = K^T (column = key lane%32); see c_row() for where the results sit.

// ---- wave-private tile pipeline -------------------------------------------
// A work item is (unit, chunk of 32 TILES keys, TILES = 1, 2, 4 or 8) and belongs to ONE wave: the
// wave copies its 32-key tiles HBM -> LDS with global_load_lds (16 B per lane,
// whole rows, fully coalesced), double-buffered in a private LDS region, and
// reads MFMA operands back with ds_read_b128 (XOR-swizzled chunks, conflict
// free on the 64-bank LDS).  No work-group barrier while tiles stream: waves only
// wait on their own copies (hand-placed s_waitcnt vmcnt), so they drift freely and
// keep HBM busy.  Reading K fragments straight from HBM in operand layout would touch
// 32 rows x 32 bytes per instruction and re-fetch every cache line several times.
constexpr int kItemKeys = 128;                 // keys per wave item that the workspace sizes of the fp32 path refer to

// Logits are parked in registers between the two halves of the fused kernel as
// 32-bit fixed point, log2 units with 22 fractional bits: the quantisation moves
// 2^t by at most ln2 * 2^-23 = 8.3e-8 relative, and both the normaliser and the
// importance are formed from the same parked value.  |t| is clamped to 511
// (354 nats), far outside anything a float32 importance can resolve.
constexpr double kFixOne = 4194304.0;  // 2^22
constexpr int kFixLimit = 511 << 22;
constexpr int kMaxGroups = 64;                 // work-groups per unit the exchange supports (4 * 128 keys each)
constexpr unsigned long long kEmpty = ~0ull;   // exchange slot not published yet (a NaN pattern no row sum can have)
__device__ __forceinline__ int fix_from(double t_scaled) {  // t_scaled = t * 2^22
  // the conversion saturates at the ends of the int range, far outside the clamp, so clamping the integer gives
  // what clamping the double first would (one three-operand median instead of two fp64 min / max)
  return min(max(__double2int_rn(t_scaled), -kFixLimit), kFixLimit);
}
__device__ __forceinline__ double exp2_fix(int qv) {
  const int n = qv >> 22;
  const float f = (float)(qv & 0x3FFFFF) * (float)(1.0 / kFixOne);  // [0, 1), exact
  return ldexp((double)__builtin_amdgcn_exp2f(f), n);
}
// One launch, K read once.  Every wave
//   A. forms the logits t_ij (log2 units) of its item, 32 observation rows x up
//      to 32 TILES keys, and parks them in registers as fixed point;
//   B. forms the row sums of p_ij = 2^t_ij (doubles: the fp64 exponent range makes
//      a running maximum unnecessary); the four waves of a work-group (always items
//      of one unit) add theirs and publish the 32 sums in the work-group's own slot
//      of the unit's exchange area with device-coherent stores;
//   C. collects the slots of all work-groups of the unit (device-coherent loads,
//      repeated until a slot no longer holds the "empty" bit pattern), adds them in
//      a fixed order, so every work-group gets the same normalisers l_i bit for bit,
//      and writes importance_j = sum_i p_ij / l_i for its keys.
// A slot value carries its own validity (a sum of powers of two is never the
// all-ones NaN pattern), so no ordering between different addresses is needed:
// one store and, normally, one or two rounds of loads replace atomic round trips.
// The wait in C needs every work-group of a unit to be resident at the same time:
// the host never launches more waves than the device holds at once (occupancy x
// compute units), so all of them run concurrently and each publishes without
// depending on anyone else.  The wait is bounded all the same: a thread that runs
// out of polls raises fault[0] (host-visible), the work-group leaves without
// writing, and the host refuses further work on the context.  fault[1] reports
// clamped logits.  Each work-group draws a ticket after it has read; the one that
// draws the unit's last ticket marks the unit's slots empty again for the next launch.
// A work-group that gives up also raises *abort_flag in device memory; every later
// launch that finds it set leaves at once, before it reads any slot, so the sums a
// failed launch left behind are never taken for valid ones.  The host clears the
// flag when it re-arms the workspace.
//
// MODE selects what a launch does:
//   kScoreFused   everything above, one launch;
//   kScoreSums    A and B only: every work-group stores its row sums (pass 1 of 2);
//   kScoreWrite   A again, then C with the sums pass 1 left (no waiting: pass 1 has
//                 completed), pass 2 of 2.  The two-pass form reads K twice but does
//                 not depend on the launch being resident as a whole.
// skip_publish: test hook, index of a work-group of the launch that does not publish its
// sums (-1: none); with a small spin_limit this makes the give-up path run
// deterministically while every work-group still exits normally.
enum : int { kScoreFused = 0, kScoreSums = 1, kScoreWrite = 2 };

template <int D, int TILES, int MODE>
__global__ __launch_bounds__(kThreads, 2) void score_fused(
    const ScoreItem* __restrict__ items, int n_items, const __bf16* __restrict__ q,
    const int32_t* __restrict__ q_rows, int n_obs, int N_k, float scale,
    const __bf16* __restrict__ k_cache, const __bf16* __restrict__ k_new,
    unsigned long long* __restrict__ slots, int slot_groups, unsigned* __restrict__ counters,
    float* __restrict__ importance, int64_t imp_stride, int* __restrict__ fault, int spin_limit,
    const unsigned* __restrict__ abort_flag_in, int skip_publish) {
  unsigned* abort_flag = const_cast<unsigned*>(abort_flag_in);
  // read now, acted upon once the loads of the Q~ fragments have been waited for anyway
  const unsigned aborted = (MODE == kScoreFused) ? __hip_atomic_load(abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
  constexpr int KK = D / 16;            // MFMA steps over the head dimension
  constexpr int CPR = D / 8;            // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;         // rows per wave-wide copy instruction
  constexpr int IPT = 32 / RPI;         // copy instructions per 32-key tile (8 or 4)
  constexpr int TILE = 32 * D;          // elements per tile

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int item = blockIdx.x * 4 + w;  // the host pads every unit to whole work-groups
  const ScoreItem it = items[item];
  const int T_in = it.t_in;
  constexpr int kItemTiles = TILES;
  const int key0 = it.chunk * (32 * TILES);
  const int n_tiles = max(0, min(kItemTiles, (T_in - key0 + 31) / 32));  // 0: padding item
  const int col = lane & 31, half = lane >> 5;

  __shared__ __attribute__((aligned(1024))) __bf16 tiles[4][2][TILE];
  const unsigned lds0 = (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void*)&tiles[w][0][0];
  // exchange area of the unit: [work-group of the unit][observation row], kEmpty = not published yet
  unsigned long long* unit_slots = slots + (int64_t)it.pos * slot_groups * kMaxObs;
  const int group = it.chunk >> 2;         // this work-group's index inside the unit (4 items per work-group)
  unsigned* cnt = counters + 2 * it.pos;   // [1] work-groups that have read the unit's slots

  // copy of tile t (keys key0 + 32t ..) into buffer t & 1.  A tile that lies
  // wholly inside the cached rows or wholly inside the new rows (the common
  // case) is addressed as wave-uniform base + loop-invariant lane offset; a tile
  // that straddles the seam or the end picks every row's source on its own and
  // repeats the last key past the end.
  int src_off[IPT];
#pragma unroll
  for (int i = 0; i < IPT; ++i) {
    const int r = i * RPI + lane / CPR, c = lane % CPR;
    src_off[i] = (r * D + ((c ^ swz_k<D>(r)) & (CPR - 1)) * 8) * 2;
  }
  auto issue = [&](int t) {
    const int j0 = key0 + t * 32;
    const unsigned dst = lds0 + (unsigned)((t & 1) * TILE * 2);
    const bool in_cache = j0 + 32 <= it.len_in;
    const bool in_new = j0 >= it.len_in && j0 + 32 <= T_in;
    if (in_cache || in_new) {
      const __bf16* base = in_cache ? k_cache + (it.in_off + j0) * D
                                    : k_new + ((int64_t)it.unit * N_k + (j0 - it.len_in)) * D;
#pragma unroll
      for (int i = 0; i < IPT; ++i) load_to_lds(base, (unsigned)src_off[i], dst + i * 1024);
    } else {
#pragma unroll
      for (int i = 0; i < IPT; ++i) {
        const int r = i * RPI + lane / CPR, c = lane % CPR;
        const int j = min(j0 + r, T_in - 1);
        const __bf16* row = (j < it.len_in) ? k_cache + (it.in_off + j) * D
                                            : k_new + ((int64_t)it.unit * N_k + (j - it.len_in)) * D;
        load_to_lds(row + ((c ^ swz_k<D>(r)) & (CPR - 1)) * 8, dst + i * 1024);
      }
    }
  };
  if (n_tiles > 0) issue(0);

  // Q~ fragments (rows beyond n_obs are zero and get zero weight below).
  bf16x8 qf[KK];
  {
    const bool qv = col < n_obs;
    const __bf16* qrow = q + ((int64_t)it.unit * N_k + (qv ? q_rows[col] : 0)) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      bf16x8 z = {0};
      qf[kk] = qv ? *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * half) : z;
    }
  }
  const double c2 = (double)scale * kLog2e * kFixOne;  // logits in log2 units, fixed point: t * 2^22 = dot * c2
  // everything the compiler loaded itself must have landed before the tiles are
  // consumed, so that no compiler-placed vmcnt wait also drains the tile copies
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) asm volatile("" ::"v"(qf[kk]));
  if (MODE == kScoreFused && __builtin_amdgcn_readfirstlane(aborted) != 0) {
    // an earlier launch gave up: its sums may still sit in the slots, so nothing here may be trusted
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the first tile's copy must not outlive the wave
    return;
  }

  int k_off[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) k_off[kk] = col * D + (((2 * kk + half) ^ swz_k<D>(col)) & (CPR - 1)) * 8;

  // ---- A: logits of the item's tiles ---------------------------------------
  // Between A and C a logit waits in registers either as its fixed-point value (one register; 2^t is
  // formed again in C) or, for all but the largest items (TILES <= 4, where the registers are there), as the
  // double 2^t of that same fixed-point value (two registers; nothing is recomputed).  Both forms give
  // the same numbers bit for bit.
  constexpr bool kParkP = TILES <= 4;
  int tq[kParkP ? 1 : kItemTiles][16];
  double pq[kParkP ? kItemTiles : 1][16];
  auto p_of = [&](int t, int r) -> double { return kParkP ? pq[t][r] : exp2_fix(tq[t][r]); };
  int q_hi = 0, q_lo = 0;              // extremes of the fixed-point logits, for the clamp report
#pragma unroll
  for (int t = 0; t < kItemTiles; ++t) {
    if (t < n_tiles) {                 // wave-uniform
      if (t + 1 < n_tiles) {
        issue(t + 1);
        dma_wait_but<IPT>();          // tile t has landed, tile t+1 stays in flight
      } else {
        dma_wait_but<0>();
      }
      const __bf16* Kt = &tiles[w][t & 1][0];
      // Raw dot products: every MFMA covers 16 head-dim elements and starts from a
      // zero accumulator; the slice results are summed in fp64, so float32 rounding
      // only ever acts on partial sums that are small next to the full dot product.
      double sd[16];
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Kt[k_off[kk]]);
        floatx16 c = {0};
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[kk], kf, c, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 16; ++r) sd[r] = (kk == 0) ? (double)c[r] : sd[r] + (double)c[r];   // 0.0 + x == x: same bits
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int qv = fix_from(sd[r] * c2);
        q_hi = max(q_hi, qv);
        q_lo = min(q_lo, qv);
        if (kParkP) pq[t][r] = exp2_fix(qv);
        else tq[t][r] = qv;
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (kParkP) pq[t][r] = 0.0;
        else tq[t][r] = 0;
      }
    }
  }

  // A logit that hit the clamp of the parked format makes the result differ from
  // the definition: tell the host (second flag word; the launch still completes).
  if (__any(q_hi >= kFixLimit || q_lo <= -kFixLimit)) {
    if (lane == 0) __hip_atomic_store(fault + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  }

  // ---- B: row sums of the work-group -> its slot ------------------------------
  // Each wave's tile buffers are free by now, so they carry the exchange inside
  // the work-group: every wave leaves its 32 row sums there, wave 0 adds the four
  // and publishes one value per row.
  double* red = reinterpret_cast<double*>(&tiles[w][0][0]);
  if (MODE != kScoreWrite)
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    double lsum = 0.0;
#pragma unroll
    for (int t = 0; t < kItemTiles; ++t)
      if (t < n_tiles && key0 + t * 32 + col < T_in) lsum += p_of(t, r);
    const double l = half_sum_f64(lsum);
    if (col == 0) red[c_row(r, half)] = l;
  }
  __syncthreads();
  if (MODE != kScoreWrite && w == 0 && lane < kMaxObs && (MODE != kScoreFused || (int)blockIdx.x != skip_publish)) {
    double tot = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k) tot += reinterpret_cast<const double*>(&tiles[k][0][0])[lane];
    __hip_atomic_store(&unit_slots[group * kMaxObs + lane], (unsigned long long)__double_as_longlong(tot),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (MODE == kScoreSums) return;
  // ---- C: collect the unit's slots ---------------------------------------------
  // thread (sub, row) = (tid / 32, tid % 32) takes work-groups sub, sub + 8, ... of row `row`
  double* part8 = reinterpret_cast<double*>(&tiles[1][0][0]) + 64;   // [8][32] partial sums, behind wave 1's row sums
  double* inv_s = reinterpret_cast<double*>(&tiles[0][0][0]) + 64;   // [32], behind wave 0's row sums
  int* ok_s = reinterpret_cast<int*>(inv_s + kMaxObs);
  if (tid == 0) *ok_s = 1;
  __syncthreads();
  {
    const int row = tid & 31, sub = tid >> 5;
    // up to kMaxGroups / 8 slots per thread: all loads are issued first, then each is
    // repeated until it is valid (work-groups past the end count as +0.0)
    unsigned long long bits[kMaxGroups / 8];
#pragma unroll
    for (int k = 0; k < kMaxGroups / 8; ++k) {
      const int g2 = sub + 8 * k;
      bits[k] = (g2 < it.n_groups) ? __hip_atomic_load(&unit_slots[g2 * kMaxObs + row], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                   : 0ull;
    }
    double acc = 0.0;
    bool ok = true;
#pragma unroll
    for (int k = 0; k < kMaxGroups / 8; ++k) {
      int polls = 0;
      while (MODE == kScoreFused && bits[k] == kEmpty) {
        if (++polls > spin_limit) { ok = false; break; }
        __builtin_amdgcn_s_sleep(8);
        bits[k] = __hip_atomic_load(&unit_slots[(sub + 8 * k) * kMaxObs + row], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      acc += __longlong_as_double((long long)bits[k]);
    }
    part8[sub * kMaxObs + row] = acc;
    if (!ok) *ok_s = 0;
  }
  __syncthreads();
  if (*ok_s == 0) {
    if (tid == 0) {
      __hip_atomic_store(abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    return;
  }
  unsigned ticket = 0;
  if (MODE == kScoreFused && w == 0) {
    if (lane < kMaxObs) {
      double l = 0.0;
#pragma unroll
      for (int k = 0; k < 8; ++k) l += part8[k * kMaxObs + lane];   // fixed order: the same bits in every work-group
      inv_s[lane] = (lane < n_obs) ? 1.0 / l : 0.0;
    }
    // every slot this work-group needed has been read (the values were used above):
    // whoever draws the last ticket may mark the slots empty without racing a reader
    if (lane == 0) ticket = atomicAdd(&cnt[1], 1u);
  }
  if (MODE == kScoreWrite && w == 0 && lane < kMaxObs) {
    double l = 0.0;
#pragma unroll
    for (int k = 0; k < 8; ++k) l += part8[k * kMaxObs + lane];
    inv_s[lane] = (lane < n_obs) ? 1.0 / l : 0.0;
  }
  __syncthreads();
  double inv_r[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) inv_r[r] = inv_s[c_row(r, half)];

#pragma unroll
  for (int t = 0; t < kItemTiles; ++t) {
    if (t < n_tiles) {
      double imp = 0.0;
#pragma unroll
      for (int r = 0; r < 16; ++r) imp = fma(p_of(t, r), inv_r[r], imp);
      imp += shfl_xor_f64(imp, 32);
      const int j = key0 + t * 32 + col;
      if (j < T_in && half == 0) importance[(int64_t)it.unit * imp_stride + j] = (float)imp;
    }
  }
  if (MODE == kScoreFused && w == 0) {
    // the work-group that drew a unit's last ticket leaves slots and counter as the next launch expects them
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    if ((int)ticket == it.n_groups - 1) {
      for (int e = lane; e < it.n_groups * kMaxObs; e += 64)
        __hip_atomic_store(&unit_slots[e], kEmpty, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (lane == 0) cnt[1] = 0;
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

}  // namespace

int score_item_keys(int dtype) { return dtype == 1 ? kScoreChunk : kItemKeys; }
int score_max_groups() { return kMaxGroups; }

// Items (= waves) of one fused launch the device keeps resident at once, for items of item_keys keys.
int score_fused_capacity(int head_dim, int item_keys) {
  int dev = 0, cus = 0, blocks = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  hipError_t e = hipErrorInvalidValue;
#define HACK_OCC(D_, TILES_) hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, score_fused<D_, TILES_, kScoreFused>, kThreads, 0)
  switch (item_keys) {
    case 32: e = head_dim == 64 ? HACK_OCC(64, 1) : HACK_OCC(128, 1); break;
    case 64: e = head_dim == 64 ? HACK_OCC(64, 2) : HACK_OCC(128, 2); break;
    case 128: e = head_dim == 64 ? HACK_OCC(64, 4) : HACK_OCC(128, 4); break;
    case 256: e = head_dim == 64 ? HACK_OCC(64, 8) : HACK_OCC(128, 8); break;
    default: break;
  }
#undef HACK_OCC
  if (e != hipSuccess) return 0;
  return blocks * cus * (kThreads / 64);
}

template <int D, int TILES>
static void launch_score_t(hipStream_t s, dim3 grid, bool two_pass, const ScoreItem* items, int n_items, const __bf16* q,
                           const int32_t* q_rows, int n_obs, int N_k, float scale, const __bf16* k_cache,
                           const __bf16* k_new, unsigned long long* slots, int slot_groups, unsigned* counters,
                           float* importance, int64_t imp_stride, int* fault, int spin_limit,
                           const unsigned* abort_flag, int skip_publish) {
#define HACK_SCORE_ARGS grid, dim3(kThreads), 0, s, items, n_items, q, q_rows, n_obs, N_k, scale, k_cache, k_new, slots, \
                        slot_groups, counters, importance, imp_stride, fault, spin_limit, abort_flag, skip_publish
  if (two_pass) {
    hipLaunchKernelGGL((score_fused<D, TILES, kScoreSums>), HACK_SCORE_ARGS);
    hipLaunchKernelGGL((score_fused<D, TILES, kScoreWrite>), HACK_SCORE_ARGS);
  } else {
    hipLaunchKernelGGL((score_fused<D, TILES, kScoreFused>), HACK_SCORE_ARGS);
  }
#undef HACK_SCORE_ARGS
}

void launch_score_fused(hipStream_t s, int head_dim, int item_keys, bool two_pass, const ScoreItem* items, int n_items,
                        const void* q, const int32_t* q_rows, int n_obs, int N_k, float scale, const void* k_cache,
                        const void* k_new, unsigned long long* slots, int slot_groups, unsigned* counters,
                        float* importance, int64_t imp_stride, int* fault, int spin_limit, const unsigned* abort_flag,
                        int skip_publish) {
  if (n_items <= 0) return;
  typedef __bf16 T;
  dim3 grid((n_items + 3) / 4);
#define HACK_SCORE_CALL(D_, TILES_)                                                                                   \
  launch_score_t<D_, TILES_>(s, grid, two_pass, items, n_items, (const T*)q, q_rows, n_obs, N_k, scale, (const T*)k_cache, \
                             (const T*)k_new, slots, slot_groups, counters, importance, imp_stride, fault, spin_limit,  \
                             abort_flag, skip_publish)
  if (head_dim == 64) {
    switch (item_keys) {
      case 32: HACK_SCORE_CALL(64, 1); break;
      case 64: HACK_SCORE_CALL(64, 2); break;
      case 256: HACK_SCORE_CALL(64, 8); break;
      default: HACK_SCORE_CALL(64, 4); break;
    }
  } else {
    switch (item_keys) {
      case 32: HACK_SCORE_CALL(128, 1); break;
      case 64: HACK_SCORE_CALL(128, 2); break;
      case 256: HACK_SCORE_CALL(128, 8); break;
      default: HACK_SCORE_CALL(128, 4); break;
    }
  }
#undef HACK_SCORE_CALL
}

// ---------------------------------------------------------------------------
// hack_score_static: the same importance with every scratch buffer in a fixed
// device array of this library, for callers that must not allocate
// ---------------------------------------------------------------------------
// The score kernels' scratch (work items, q-row table, row-sum exchange slots) lives in
// a file-scope device array instead of context memory; the work items are written by a
// small planning kernel from by-value arguments, so nothing is copied from the host.
// The array is one per GPU and shared by every call on that GPU.
namespace {

constexpr int kStaticItemsMax = kStaticUnitsMax * 4 * kMaxGroups;   // 4 items per work-group, kMaxGroups work-groups per unit
struct StaticScratch {
  ScoreItem items[kStaticItemsMax];                                        // 512 KiB
  unsigned long long slots[(size_t)kStaticUnitsMax * kMaxGroups * kMaxObs]; // 1 MiB
  int32_t q_rows[kMaxObs];
  unsigned counters[2 * kStaticUnitsMax + 64];                             // unused by the two-pass form; abort word last
};
static __device__ __align__(256) unsigned char scratch[sizeof(StaticScratch)];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
StaticScratch* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU (its name is not one in host code)

// Writes the work items of the planned units (4 * wgs items per unit, in caller order) and the
// q-row table.  One work-group.
__global__ __launch_bounds__(256) void score_static_plan(StaticScorePlan plan, ScoreItem* __restrict__ items,
                                                          int32_t* __restrict__ q_rows) {
  __shared__ int first[kStaticUnitsMax + 1];
  if (threadIdx.x == 0) {
    int n = 0;
    for (int i = 0; i < plan.n_units; ++i) {
      first[i] = n;
      const int t_in = plan.len_in[i] + plan.n_new;
      n += 4 * (((t_in + plan.item_keys - 1) / plan.item_keys + 3) / 4);
    }
    first[plan.n_units] = n;
  }
  if (threadIdx.x < kMaxObs) q_rows[threadIdx.x] = plan.q_rows[threadIdx.x];
  __syncthreads();
  for (int i = 0; i < plan.n_units; ++i) {
    const int n = first[i + 1] - first[i];
    const int t_in = plan.len_in[i] + plan.n_new;
    for (int c = threadIdx.x; c < n; c += blockDim.x)
      items[first[i] + c] = ScoreItem{plan.in_off[i], plan.unit[i], plan.len_in[i], t_in, c, i, n / 4};
  }
}

}  // namespace

int score_static_units_max() { return kStaticUnitsMax; }
size_t score_static_scratch_bytes() { return sizeof(StaticScratch); }

int score_static_item_count(const StaticScorePlan& plan) {
  int n = 0;
  for (int i = 0; i < plan.n_units; ++i)
    n += 4 * (((plan.len_in[i] + plan.n_new + plan.item_keys - 1) / plan.item_keys + 3) / 4);
  return n;
}

// Looks up (once per device, with that device current) where this GPU keeps its copy of `scratch`.
hipError_t score_static_setup(int device) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[device]) return hipSuccess;
  int cur = -1;
  hipError_t e = hipGetDevice(&cur);
  if (e != hipSuccess) return e;
  if (cur != device && (e = hipSetDevice(device)) != hipSuccess) return e;
  void* p = nullptr;
  e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
  if (cur != device) (void)hipSetDevice(cur);
  if (e != hipSuccess) return e;
  g_scratch_ptr[device] = static_cast<StaticScratch*>(p);
  return hipSuccess;
}

hipError_t launch_score_static(hipStream_t s, int device, int head_dim, const StaticScorePlan& plan, const void* q, int n_obs,
                               int N_k, float scale, const void* k_cache, const void* k_new, float* importance,
                               int64_t imp_stride, int* fault) {
  StaticScratch* sc = (device >= 0 && device < kMaxDevices) ? g_scratch_ptr[device] : nullptr;
  if (!sc) return hipErrorNotInitialized;
  const int n_items = score_static_item_count(plan);
  if (n_items <= 0) return hipSuccess;
  if (n_items > kStaticItemsMax) return hipErrorInvalidValue;
  hipLaunchKernelGGL(score_static_plan, dim3(1), dim3(256), 0, s, plan, sc->items, sc->q_rows);
  // the two-pass form: every slot that pass 2 reads is written by pass 1 of the same call, so the
  // array needs no clearing between calls
  launch_score_fused(s, head_dim, plan.item_keys, true, sc->items, n_items, q, sc->q_rows, n_obs, N_k, scale, k_cache, k_new,
                     sc->slots, kMaxGroups, sc->counters, importance, imp_stride, fault, 0,
                     sc->counters + 2 * kStaticUnitsMax, -1);
  return hipGetLastError();
}

void launch_score_generic(hipStream_t s, int head_dim, const UnitDesc* descs, const int32_t* list, int n_list,
                          int max_t_in, const void* q, const int32_t* q_rows, int n_obs, int N_k, float scale,
                          const void* k_cache, const void* k_new, double* stats, float* importance,
                          int64_t imp_stride) {
  if (n_list <= 0 || max_t_in <= 0) return;
  const int max_chunks = (max_t_in + kScoreChunk - 1) / kScoreChunk;
  dim3 grid(max_chunks, n_list);
#define HACK_ARGS s, grid, descs, list, max_chunks, q, q_rows, n_obs, N_k, scale, k_cache, k_new, stats, importance, imp_stride
  if (head_dim == 64) launch_generic<float, 64>(HACK_ARGS);
  else launch_generic<float, 128>(HACK_ARGS);
#undef HACK_ARGS
}

}  // namespace hack
