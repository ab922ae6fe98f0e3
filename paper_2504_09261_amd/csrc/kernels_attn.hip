// Attention of the current scale's queries over the ragged compressed cache
// (Preliminaries, attention equation: O = Softmax(scale * Q K^T) V, no mask
// inside a scale step) on gfx950.
//
// bf16 path (flash-style, one pass over K/V with an online softmax):
//   * work item = (unit, tile of 4 waves x 32 queries); K/V blocks of 32 keys
//     are staged once per work-group in LDS and shared by the four waves.
//   * S^T = K Q^T with v_mfma_f32_32x32x16_bf16: the accumulator then holds,
//     per lane, one query column and 16 key rows, so the softmax row reductions
//     are in-lane plus one exchange with lane^32, and the running max / rescale
//     factor are per-lane scalars.
//   * O^T += V^T P^T: P^T goes from the accumulator registers straight into the
//     B operand (C rows 8(r/4)+4h+r%4 of registers 8s..8s+7 are exactly two runs
//     of four consecutive keys), and V^T comes from row-major V in LDS through
//     the transposing LDS read (ds_read_b64_tr_b16), four keys per read.
//   * the loop runs over 32-key blocks, software-pipelined by one block: the
//     scores of block b+1 are formed while block b is exponentiated.
//   * K/V blocks travel HBM -> LDS directly (no register round trip) through a
//     ring of four slots per tensor, one barrier per block; an XOR swizzle of
//     16-byte chunks keeps the b128 K reads and the transposing V reads
//     bank-conflict free.
// fp32 path: one query per lane, fp32 FMA, K/V rows broadcast from LDS; exact
// enough for the 1e-4 bar and only used for the small fp32 configuration.
#include <type_traits>

#include "device_util.h"
#include "hack_internal.h"

namespace hack {

namespace {

using namespace dev;

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
  const AttnItem& d = it;   // the item carries the descriptor fields read here
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
constexpr int kKB = 32;      // keys per block (one LDS ring slot)
constexpr float kRescaleAbove = 65536.f;  // a block sum of probabilities at or above this moves the reference

// NW waves per work-group, each wave owns 32 queries; two work-groups share a CU.
//
// The loop runs over 32-key blocks and is software-pipelined by one block: while
// the vector ALU turns the scores of block b into probabilities, the matrix core
// already forms the scores of block b+1; then O^T += V^T P^T for block b.  (A
// wave issues in order, so matrix and vector work only overlap if independent
// instructions of both kinds sit next to each other in its own stream; on this
// chip ~4 simple VALU ops or ~2 exponentials hide under one 32x32x16 MFMA.)
// K and V blocks travel HBM -> LDS through two rings of kRing slots: the copy of
// block b+3 is issued at stage b into the slot block b-1 has just left, so a
// copy has two full stages to land and one barrier per stage both publishes
// block b+1 and frees the slot.
//
// The vector ALU is the scarce unit (per block a wave issues 16 MFMAs but also
// has to exponentiate 16 scores per lane), so the softmax is kept to
// fma + exp2 + bf16 pack + a bf16 dot2 for the row sum:
//   * the running reference m_run is only moved when a probability would leave
//     [0, 2^16): the exponentials are formed optimistically against the current
//     reference, and only if some lane's block sum says "too large" (or inf, as
//     in the very first block) is the max computed and everything rescaled;
//   * the row sum is taken over the bf16-rounded probabilities, the same numbers
//     the PV product uses.
constexpr int kRing = 4;     // LDS ring slots per tensor (32-key blocks)

template <int D, int NW>
__global__ __launch_bounds__(64 * NW, 2) void attn_mfma(
    const UnitDesc* __restrict__ descs, const AttnItem* __restrict__ items,
    const __bf16* __restrict__ q, const __bf16* __restrict__ k_cache,
    const __bf16* __restrict__ v_cache, int N_k, float scale,
    __bf16* __restrict__ out) {
  constexpr int KK = D / 16;        // MFMA steps over head_dim for S^T
  constexpr int MB = D / 32;        // 32-row blocks of O^T
  constexpr int CPR = D / 8;        // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;     // block rows covered by one wave-wide copy instruction
  constexpr int IPW = (kKB / RPI) / NW;  // copy instructions per wave, block and tensor
  constexpr int BLK = kKB * D;      // elements per block and tensor
  static_assert(IPW >= 1, "a block must give every wave at least one copy instruction");

  const AttnItem it = items[blockIdx.x];
  if (it.desc < 0) return;
  const AttnItem& d = it;   // the item carries the descriptor fields read here
  const int len = d.n_out;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;

  __shared__ __attribute__((aligned(1024))) __bf16 Ks[kRing][BLK];
  __shared__ __attribute__((aligned(1024))) __bf16 Vs[kRing][BLK];

  const __bf16* kg = k_cache + d.out_off * D;
  const __bf16* vg = v_cache + d.out_off * D;
  const int n_blocks = (len + kKB - 1) / kKB;

  // Block copies.  Lane l of copy instruction i of this wave fills LDS row
  // r = (w + i NW) RPI + l / CPR, chunk position c = l % CPR, from global chunk
  // c ^ f(r) of block row r; the byte offsets inside a full block are loop invariant.
  unsigned k_src[IPW], v_src[IPW];
#pragma unroll
  for (int i = 0; i < IPW; ++i) {
    const int r = (w + i * NW) * RPI + lane / CPR, c = lane % CPR;
    k_src[i] = (unsigned)(r * D + ((c ^ swz_k<D>(r)) & (CPR - 1)) * 8) * 2u;
    v_src[i] = (unsigned)(r * D + ((c ^ swz_v<D>(r)) & (CPR - 1)) * 8) * 2u;
  }
  const unsigned ks_lds = lds_addr_of(&Ks[0][0]), vs_lds = lds_addr_of(&Vs[0][0]);
  // Rows past the end of a ragged last block repeat the last valid row (finite
  // data); their scores are masked to -inf, so their probabilities are exactly 0.
  auto issue = [&](int b, int slot) {
    const int t0 = b * kKB;
    const __bf16* kb = kg + (int64_t)t0 * D;
    const __bf16* vb = vg + (int64_t)t0 * D;
    if (t0 + kKB <= len) {
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        const unsigned dst = (unsigned)((slot * BLK + (w + i * NW) * 512) * 2);
        load_to_lds(kb, k_src[i], ks_lds + dst);
        load_to_lds(vb, v_src[i], vs_lds + dst);
      }
    } else {
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        const int r = (w + i * NW) * RPI + lane / CPR, c = lane % CPR;
        const int rc = min(r, len - 1 - t0);
        const unsigned dst = (unsigned)((slot * BLK + (w + i * NW) * 512) * 2);
        load_to_lds(kb, (unsigned)(rc * D + ((c ^ swz_k<D>(r)) & (CPR - 1)) * 8) * 2u, ks_lds + dst);
        load_to_lds(vb, (unsigned)(rc * D + ((c ^ swz_v<D>(r)) & (CPR - 1)) * 8) * 2u, vs_lds + dst);
      }
    }
  };
  issue(0, 0);
  if (n_blocks > 1) issue(1, 1);
  if (n_blocks > 2) issue(2, 2);

  // Q fragments (B operand of S^T = K Q^T): query col, head-dim slice [16kk + 8h, +8).
  const int q0 = it.q_tile * (NW * 32) + w * 32;
  bf16x8 qf[KK];
  {
    const int qi = min(q0 + col, N_k - 1);
    const __bf16* qrow = q + ((int64_t)d.unit * N_k + qi) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * half);
    // Consume the fragments here so that their loads are waited for before the
    // main loop: a vmcnt wait inside the loop would also drain the block copies
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
  float mc = -INFINITY;   // m_run * c2

  // per-lane LDS element offsets of the operand reads (block-relative); the ring
  // slot is a compile-time immediate
  int k_off[KK];           // K operand: row col, chunk 2kk + half
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) k_off[kk] = col * D + (((2 * kk + half) ^ swz_k<D>(col)) & (CPR - 1)) * 8;
  const int g = lane >> 4, e = (lane >> 2) & 3, qd = lane & 3;
  int v_off[MB];           // V^T operand: row 4 half + e (+16 sg, +8), head-dim 32mb + 16(g&1) + 4qd
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
    v_off[mb] = (4 * half + e) * D + (((4 * mb + 2 * (g & 1) + (qd >> 1)) ^ swz_v<D>(e)) & (CPR - 1)) * 8 + 4 * (qd & 1);

  const bf16x2 ones2 = {(__bf16)1.0f, (__bf16)1.0f};

  // S^T of block b (32 keys x 32 queries) from ring slot SLOT.
  auto scores = [&](auto slot_tag, int b) -> floatx16 {
    constexpr int SLOT = decltype(slot_tag)::value;
    const __bf16* Kt = &Ks[SLOT][0];
    floatx16 sc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Kt[k_off[kk]]);
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sc, 0, 0, 0);
    }
    return sc;
  };
  // ragged end: keys past the end get -inf
  auto mask_tail = [&](floatx16& sc, int b) {
    if ((b + 1) * kKB > len) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = b * kKB + 8 * (r >> 2) + 4 * half + (r & 3);
        if (key >= len) sc[r] = -INFINITY;
      }
    }
  };
  // probabilities of a block against the current reference (per lane: one query,
  // 16 keys; the partner lane l ^ 32 holds the other 16) and their sum
  auto probs = [&](const floatx16& sc, bf16x8 (&pf)[2]) -> float {
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) pf[r >> 3][r & 7] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sc[r], c2, -mc));
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      const bf16x2 pr = {pf[r >> 3][r & 7], pf[r >> 3][(r & 7) + 1]};
      psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones2, psum, false);
    }
    return psum;
  };
  // Some probability left the safe range (always so in the first block, where the
  // reference is -inf): move the reference to the running max, bring the
  // accumulators to the new scale and redo this block's probabilities.
  auto rescale = [&](const floatx16& sc, bf16x8 (&pf)[2]) -> float {
    float mx = sc[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sc[r]);
    mx = pair_max(mx);
    const float m_new = fmaxf(m_run, mx);   // finite: the block holds a valid key
    const float a = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
    l_run *= a;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[mb][r] *= a;
    m_run = m_new;
    mc = m_new * c2;
    return probs(sc, pf);
  };
  // O^T += V^T P^T for the block in ring slot SLOT
  auto pv = [&](auto slot_tag, const bf16x8 (&pf)[2]) {
    constexpr int SLOT = decltype(slot_tag)::value;
    const __bf16* Vt = &Vs[SLOT][0];
#pragma unroll
    for (int sg = 0; sg < 2; ++sg) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const __bf16* vp = &Vt[16 * sg * D + v_off[mb]];
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
  };

  // Stage b (ring slot S = b % kRing): sc holds the scores of block b on entry
  // and those of block b+1 on exit.  LAST: block b is the unit's last one.
  // TAIL: block b+1 may be the ragged last block (its scores then need the mask,
  // whose branch would keep the scheduler from mixing matrix and vector work).
  auto stage = [&](auto slot_tag, auto last_tag, auto tail_tag, int b, floatx16& sc) {
    constexpr int S = decltype(slot_tag)::value;
    constexpr bool LAST = decltype(last_tag)::value;
    constexpr bool TAIL = decltype(tail_tag)::value;
    using S1 = std::integral_constant<int, (S + 1) % kRing>;
    // everything but the copy group issued one stage ago (block b+2) has landed
    if (b + 2 < n_blocks) dma_wait_but<2 * IPW>();
    else dma_wait_but<0>();
    __syncthreads();   // block b+1 is visible to every wave; the slot of block b-1 is free
    if (b + 3 < n_blocks) issue(b + 3, (S + 3) % kRing);
    __builtin_amdgcn_sched_barrier(0);
    floatx16 sn;
    if (!LAST) sn = scores(S1{}, b + 1);
    bf16x8 pf[2];
    float psum = probs(sc, pf);
    if (!LAST) {
      // the K fragment reads first, then one MFMA of the next block's scores and a
      // slice of this block's softmax arithmetic, and so on
      __builtin_amdgcn_sched_group_barrier(0x100, KK, 0);
#pragma unroll
      for (int i = 0; i < KK; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 48 / KK, 0);
      }
    }
    if (!LAST && TAIL) mask_tail(sn, b + 1);
    if (__any(!(psum < kRescaleAbove))) psum = rescale(sc, pf);
    l_run += psum;
    pv(slot_tag, pf);
    if (!LAST) sc = sn;
  };

  using R0 = std::integral_constant<int, 0>;
  using R1 = std::integral_constant<int, 1>;
  using R2 = std::integral_constant<int, 2>;
  using R3 = std::integral_constant<int, 3>;
  using No = std::false_type;
  using Yes = std::true_type;

  // block 0 has landed -> its scores
  if (n_blocks > 2) dma_wait_but<4 * IPW>();
  else if (n_blocks > 1) dma_wait_but<2 * IPW>();
  else dma_wait_but<0>();
  __syncthreads();
  floatx16 sc = scores(R0{}, 0);
  mask_tail(sc, 0);

  // main loop: four stages whose next blocks are all full
  int b = 0;
  for (; b + 5 < n_blocks; b += 4) {
    stage(R0{}, No{}, No{}, b, sc);
    stage(R1{}, No{}, No{}, b + 1, sc);
    stage(R2{}, No{}, No{}, b + 2, sc);
    stage(R3{}, No{}, No{}, b + 3, sc);
  }
  // the remaining 1..5 blocks, one stage at a time (b is a multiple of 4 here)
  for (; b < n_blocks; ++b) {
    const bool last = (b + 1 == n_blocks);
    switch (b & 3) {
      case 0: if (last) stage(R0{}, Yes{}, Yes{}, b, sc); else stage(R0{}, No{}, Yes{}, b, sc); break;
      case 1: if (last) stage(R1{}, Yes{}, Yes{}, b, sc); else stage(R1{}, No{}, Yes{}, b, sc); break;
      case 2: if (last) stage(R2{}, Yes{}, Yes{}, b, sc); else stage(R2{}, No{}, Yes{}, b, sc); break;
      default: if (last) stage(R3{}, Yes{}, Yes{}, b, sc); else stage(R3{}, No{}, Yes{}, b, sc); break;
    }
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


// ---------------------------------------------------------------------------
// bf16 MFMA path, deeper software pipeline (the kernel that serves the large steps)
// ---------------------------------------------------------------------------
// Same work item, operand layouts, swizzles and softmax as attn_mfma above; what
// differs is what one stage holds.  Stage b (one barrier) is a single branch-free
// region with three independent strands:
//     S(b+1)   the 8 score MFMAs of the next block       (matrix core)
//     PV(b-1)  O^T += V^T P^T of the previous block       (matrix core)
//     softmax(b): exponentials, bf16 packing, row sum    (vector ALU)
// so every MFMA of the loop has vector work of another block beside it and the LDS
// reads of both products are issued ahead of their use.  The probabilities of block
// b wait in registers for one stage; the check "did a probability leave the safe
// range" (and the rare rescale that follows it) sits at the end of the stage, after
// PV(b-1) has been added, so a rescale always meets accumulators that are complete
// up to block b-1.
// LDS: three slots per tensor.  K(j) is read in stage j-1, V(j) in stage j+1; stage
// b issues the copies K(b+3) and V(b+1) right after its opening barrier, into the
// slots of K(b) and V(b-2), which every wave finished reading in stage b-1.  Each
// copy has two full stages to land; one s_waitcnt vmcnt(2 groups) + barrier per stage.
// Scheduling hints for one pipelined stage: N times {one MFMA, VALU_PER vector ops,
// up to two LDS reads while any are left}.
template <int I, int N, int VALU_PER, int DS_LEFT>
__device__ __forceinline__ void sched_interleave() {
  if constexpr (I < N) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, 0);
    if constexpr (DS_LEFT >= 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    else if constexpr (DS_LEFT == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    sched_interleave<I + 1, N, VALU_PER, (DS_LEFT > 2 ? DS_LEFT - 2 : 0)>();
  }
}

// STREAM = false: work-group i serves work item items[i] (one query tile of one unit, all of its keys).
// STREAM = true: work-group i serves the segments segs[seg_begin[i] .. seg_begin[i+1]), one after the
// other.  A segment is a run of 32-key blocks [blk0, blk1) of one work item; the host cuts the
// concatenation of all work items of a launch into as many equal runs as the device holds work-groups
// at once, so every work-group gets the same number of blocks whatever the lengths of the units are.
// A segment that covers its work item completely stores the output rows as usual (part < 0).
// Otherwise it leaves its reference, normaliser and unnormalised O^T (float32) in slot `part` of the
// partial-result arrays and draws a ticket from the work item's counter; the work-group that draws
// the last of the item's n_parts tickets (every other part has been stored and published by then)
// adds the parts first_part .. first_part + n_parts - 1 up and stores the output rows, then leaves the
// counter at zero for the next launch.  Nobody waits for anybody.
template <int D, int NW, bool STREAM>
__global__ __launch_bounds__(64 * NW, 2) void attn_pipe(
    const UnitDesc* __restrict__ descs, const AttnItem* __restrict__ items,
    const AttnSeg* __restrict__ segs, const int32_t* __restrict__ seg_begin,
    const __bf16* __restrict__ q, const __bf16* __restrict__ k_cache,
    const __bf16* __restrict__ v_cache, int N_k, float scale,
    __bf16* __restrict__ out, float* part_o, float* part_ml, unsigned* part_count) {
  constexpr int KK = D / 16;        // MFMA steps over head_dim for S^T
  constexpr int MB = D / 32;        // 32-row blocks of O^T
  constexpr int CPR = D / 8;        // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;     // block rows covered by one wave-wide copy instruction
  constexpr int IPW = (kKB / RPI) / NW;  // copy instructions per wave, block and tensor
  constexpr int BLK = kKB * D;      // elements per block and tensor
  constexpr int NS = 3;             // ring slots per tensor
  static_assert(IPW >= 1, "a block must give every wave at least one copy instruction");
  static_assert(KK == 2 * MB, "as many score MFMAs as PV MFMAs per block");

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

  __shared__ __attribute__((aligned(1024))) __bf16 Ks[NS][BLK];
  __shared__ __attribute__((aligned(1024))) __bf16 Vs[NS][BLK];
  __shared__ int last_ticket;

  int seg_lo = blockIdx.x, seg_hi = blockIdx.x + 1;
  if (STREAM) {
    seg_lo = seg_begin[blockIdx.x];
    seg_hi = seg_begin[blockIdx.x + 1];
  }
  for (int si = seg_lo; si < seg_hi; ++si) {
  // The lane index is re-read per segment behind a compiler barrier: values derived from it that
  // only the ragged paths need are then formed where they are used instead of being carried
  // through the main loop in registers.
  int lane = tid & 63;
  if (STREAM) asm volatile("" : "+v"(lane));
  const int col = lane & 31, half = lane >> 5;
  AttnSeg sg;
  AttnItem d;      // unit, n_out, out_off of the work item
  if (STREAM) {
    sg = segs[si];
    const UnitDesc ud = descs[sg.desc];
    d.unit = ud.unit; d.n_out = ud.n_out; d.out_off = ud.out_off;
  } else {
    d = items[si];
    if (d.desc < 0) return;
    sg = AttnSeg{d.desc, d.q_tile, 0, 0x3fffffff, -1, 0, 0, 0};
  }
  const int key0 = sg.blk0 * kKB;                                               // first key of the segment
  const int len = (int)min((int64_t)sg.blk1 * kKB, (int64_t)d.n_out) - key0;    // its keys

  const __bf16* kg = k_cache + (d.out_off + key0) * D;
  const __bf16* vg = v_cache + (d.out_off + key0) * D;
  const int n_blocks = (len + kKB - 1) / kKB;
  const int n_full = len / kKB;
  unsigned k_src[IPW], v_src[IPW];
#pragma unroll
  for (int i = 0; i < IPW; ++i) {
    const int r = (w + i * NW) * RPI + lane / CPR, c = lane % CPR;
    k_src[i] = (unsigned)(r * D + ((c ^ swz_k<D>(r)) & (CPR - 1)) * 8) * 2u;
    v_src[i] = (unsigned)(r * D + ((c ^ swz_v<D>(r)) & (CPR - 1)) * 8) * 2u;
  }
  const unsigned ks_lds = lds_addr_of(&Ks[0][0]), vs_lds = lds_addr_of(&Vs[0][0]);
  // Copy of block blk of one tensor into ring slot `slot`.  Rows past the end of a
  // ragged last block repeat the last valid row (finite data); their scores are
  // masked to -inf, so their probabilities are exactly 0.
  auto issue_one = [&](const __bf16* g, const unsigned (&src)[IPW], unsigned lds, bool is_v, int blk, int slot, bool full) {
    const int t0 = blk * kKB;
    const __bf16* gb = g + (int64_t)t0 * D;
    if (full || t0 + kKB <= len) {
#pragma unroll
      for (int i = 0; i < IPW; ++i)
        load_to_lds(gb, src[i], lds + (unsigned)((slot * BLK + (w + i * NW) * 512) * 2));
    } else {
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        const int r = (w + i * NW) * RPI + lane / CPR, c = lane % CPR;
        const int rc = min(r, len - 1 - t0);
        const int f = is_v ? swz_v<D>(r) : swz_k<D>(r);
        load_to_lds(gb, (unsigned)(rc * D + ((c ^ f) & (CPR - 1)) * 8) * 2u,
                    lds + (unsigned)((slot * BLK + (w + i * NW) * 512) * 2));
      }
    }
  };
  auto issue_k = [&](int blk, int slot, bool full = false) { issue_one(kg, k_src, ks_lds, false, blk, slot, full); };
  auto issue_v = [&](int blk, int slot, bool full = false) { issue_one(vg, v_src, vs_lds, true, blk, slot, full); };

  issue_k(0, 0);
  if (n_blocks > 1) issue_k(1, 1);
  if (n_blocks > 2) issue_k(2, 2);
  issue_v(0, 0);

  // Q fragments (B operand of S^T = K Q^T): query col, head-dim slice [16kk + 8h, +8).
  const int q0 = sg.q_tile * (NW * 32) + w * 32;
  bf16x8 qf[KK];
  {
    const int qi = min(q0 + col, N_k - 1);
    const __bf16* qrow = q + ((int64_t)d.unit * N_k + qi) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * half);
    // Consumed here so that their loads are waited for before the main loop (a vmcnt
    // wait inside the loop would also drain the block copies meant to stay in flight).
    // The copies issued above are older than these loads and have landed with them.
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
  float mc = -INFINITY;   // m_run * c2

  int k_off[KK];           // K operand: row col, chunk 2kk + half
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) k_off[kk] = col * D + (((2 * kk + half) ^ swz_k<D>(col)) & (CPR - 1)) * 8;
  const int g = lane >> 4, e = (lane >> 2) & 3, qd = lane & 3;
  int v_off[MB];           // V^T operand: row 4 half + e (+16 sg, +8), head-dim 32mb + 16(g&1) + 4qd
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
    v_off[mb] = (4 * half + e) * D + (((4 * mb + 2 * (g & 1) + (qd >> 1)) ^ swz_v<D>(e)) & (CPR - 1)) * 8 + 4 * (qd & 1);

  const bf16x2 ones2 = {(__bf16)1.0f, (__bf16)1.0f};

  auto mask_tail = [&](floatx16& sc, int b) {
    if ((b + 1) * kKB > len) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = b * kKB + 8 * (r >> 2) + 4 * half + (r & 3);
        if (key >= len) sc[r] = -INFINITY;
      }
    }
  };
  auto probs = [&](const floatx16& sc, bf16x8 (&pf)[2]) -> float {
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) pf[r >> 3][r & 7] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sc[r], c2, -mc));
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      const bf16x2 pr = {pf[r >> 3][r & 7], pf[r >> 3][(r & 7) + 1]};
      psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones2, psum, false);
    }
    return psum;
  };
  auto rescale = [&](const floatx16& sc, bf16x8 (&pf)[2]) -> float {
    float mx = sc[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sc[r]);
    mx = pair_max(mx);
    const float m_new = fmaxf(m_run, mx);   // finite: the block holds a valid key
    const float a = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
    l_run *= a;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[mb][r] *= a;
    m_run = m_new;
    mc = m_new * c2;
    return probs(sc, pf);
  };
  auto k_frag = [&](const __bf16* Kt, int kk) -> bf16x8 { return *reinterpret_cast<const bf16x8*>(&Kt[k_off[kk]]); };
  auto v_frag = [&](const __bf16* Vt, int i) -> bf16x8 {   // PV MFMA i: key group sg = i / MB, head-dim block mb = i % MB
    const __bf16* vp = &Vt[16 * (i / MB) * D + v_off[i % MB]];
    const bf16x4 v0 = lds_read_tr(vp);
    const bf16x4 v1 = lds_read_tr(vp + 8 * D);
    bf16x8 vf;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      vf[j] = v0[j];
      vf[4 + j] = v1[j];
    }
    return vf;
  };

  bf16x8 pp[2];   // probabilities of the previous block, waiting for their PV product

  // Stage b, ring slot S = b % 3 (compile time).  On entry sc = scores of block b and
  // pp = probabilities of block b-1; on exit sc = scores of block b+1, pp = those of block b.
  // FIRST: b == 0 (no previous block).  LAST: block b is the unit's last (no next scores).
  // STEADY: every block this stage touches exists and is full, so copies, waits and
  // masks need no tests.
  auto stage = [&](auto slot_tag, auto first_tag, auto last_tag, auto steady_tag, int b, floatx16& sc) {
    constexpr int S = decltype(slot_tag)::value;
    constexpr bool FIRST = decltype(first_tag)::value;
    constexpr bool LAST = decltype(last_tag)::value;
    constexpr bool STEADY = decltype(steady_tag)::value;
    // K(b+1) and V(b-1) have landed: everything but what the previous stage issued, which is V(b) and, if that
    // block exists, K(b+2) (short caches never reach the steady loop: waiting for everything there would put a
    // whole memory latency into every stage)
    if (STEADY || b + 2 < n_blocks) dma_wait_but<2 * IPW>();
    else dma_wait_but<IPW>();
    __syncthreads();   // both are visible to every wave; the slots of K(b) and V(b-2) are free
    if (STEADY || b + 3 < n_blocks) issue_k(b + 3, S, STEADY);
    if (STEADY || b + 1 < n_blocks) issue_v(b + 1, (S + 1) % NS, STEADY);
    __builtin_amdgcn_sched_barrier(0);
    const __bf16* Kt = &Ks[(S + 1) % NS][0];
    const __bf16* Vt = &Vs[(S + 2) % NS][0];
    floatx16 sn;
#pragma unroll
    for (int r = 0; r < 16; ++r) sn[r] = 0.f;
#pragma unroll
    for (int i = 0; i < KK; ++i) {
      if (!LAST) sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(Kt, i), qf[i], sn, 0, 0, 0);
      if (!FIRST) o[i % MB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_frag(Vt, i), pp[i / MB], o[i % MB], 0, 0, 0);
    }
    bf16x8 pf[2];
    float psum = probs(sc, pf);
    {
      // a few operand reads ahead, then per MFMA a slice of the softmax arithmetic and the next reads
      constexpr int N_MFMA = (LAST ? 0 : KK) + (FIRST ? 0 : KK);
      constexpr int N_DS = (LAST ? 0 : KK) + (FIRST ? 0 : 2 * KK);
      constexpr int AHEAD = N_DS < 6 ? N_DS : 6;
      constexpr int VALU_PER = N_MFMA ? (48 + N_MFMA - 1) / N_MFMA : 0;
      if constexpr (N_MFMA > 0) {
        __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
        sched_interleave<0, N_MFMA, VALU_PER, N_DS - AHEAD>();
      }
    }
    if (!STEADY && !LAST) mask_tail(sn, b + 1);
    if (__any(!(psum < kRescaleAbove))) psum = rescale(sc, pf);
    l_run += psum;
    pp[0] = pf[0];
    pp[1] = pf[1];
    if (!LAST) sc = sn;
  };

  using R0 = std::integral_constant<int, 0>;
  using R1 = std::integral_constant<int, 1>;
  using R2 = std::integral_constant<int, 2>;
  using No = std::false_type;
  using Yes = std::true_type;

  // block 0 has landed (see the Q fragments above) -> its scores
  dma_wait_but<0>();
  __syncthreads();
  floatx16 sc;
  {
    const __bf16* Kt = &Ks[0][0];
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(Kt, kk), qf[kk], sc, 0, 0, 0);
  }
  mask_tail(sc, 0);

  // stage 0 on its own (no previous block), then the steady loop: stages whose blocks b-1 .. b+3 all exist and are full
  if (n_blocks == 1) stage(R0{}, Yes{}, Yes{}, No{}, 0, sc);
  else stage(R0{}, Yes{}, No{}, No{}, 0, sc);
  int b = 1;
  for (; b + 5 < n_full; b += 3) {
    stage(R1{}, No{}, No{}, Yes{}, b, sc);
    stage(R2{}, No{}, No{}, Yes{}, b + 1, sc);
    stage(R0{}, No{}, No{}, Yes{}, b + 2, sc);
  }
  // the remaining blocks, one stage at a time (b % 3 == 1 here)
  for (; b < n_blocks; ++b) {
    const bool last = (b + 1 == n_blocks);
    switch (b % 3) {
      case 0: if (last) stage(R0{}, No{}, Yes{}, No{}, b, sc); else stage(R0{}, No{}, No{}, No{}, b, sc); break;
      case 1: if (last) stage(R1{}, No{}, Yes{}, No{}, b, sc); else stage(R1{}, No{}, No{}, No{}, b, sc); break;
      default: if (last) stage(R2{}, No{}, Yes{}, No{}, b, sc); else stage(R2{}, No{}, No{}, No{}, b, sc); break;
    }
  }
  // PV of the last block
  dma_wait_but<0>();
  __syncthreads();
  {
    const __bf16* Vt = &Vs[(n_blocks - 1) % NS][0];
#pragma unroll
    for (int i = 0; i < KK; ++i)
      o[i % MB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_frag(Vt, i), pp[i / MB], o[i % MB], 0, 0, 0);
  }

  // ---- normalise and store: lane holds query col, head-dim rows 32mb + 8(r/4) + 4h + r%4 ----
  float l = pair_sum(l_run);
  bool store = true;
  if (STREAM && sg.part >= 0) {
    // Partial result, register-major (every store instruction of a wave writes 512 contiguous bytes).
    // The parts of a work item come from work-groups on different XCDs, whose L2 caches are not kept
    // coherent with each other, so parts and tickets travel as device-scope relaxed atomics (stores
    // that write through, loads that do not take a stale line), 8 bytes each; a device-scope fence
    // would instead write back and invalidate the whole L2 at every segment end.  Order is kept by
    // hand: a work-group draws its ticket only after every store of its part has been acknowledged.
    constexpr int QT = NW * 32;
    typedef unsigned long long u64;
    auto pack2 = [](float a, float b) -> u64 {
      return (u64)__builtin_bit_cast(unsigned, a) | ((u64)__builtin_bit_cast(unsigned, b) << 32);
    };
    {
      u64* po = reinterpret_cast<u64*>(part_o + (int64_t)sg.part * (QT * D)) + (w * MB * 8) * 64 + lane;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int h2 = 0; h2 < 8; ++h2)
          __hip_atomic_store(po + (mb * 8 + h2) * 64, pack2(o[mb][2 * h2], o[mb][2 * h2 + 1]), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
      if (half == 0)   // reference in log2 units (finite: the segment holds a valid key) and normaliser
        __hip_atomic_store(reinterpret_cast<u64*>(part_ml + (int64_t)sg.part * (2 * QT)) + w * 32 + col, pack2(mc, l),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's stores have been acknowledged
    __syncthreads();                                    // ... and so have the whole work-group's
    if (tid == 0)
      last_ticket = (__hip_atomic_fetch_add(&part_count[sg.counter], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                     (unsigned)(sg.n_parts - 1)) ? 1 : 0;
    __syncthreads();
    store = last_ticket != 0;
    if (store) {
      // every other part was acknowledged before its ticket was drawn, and all tickets before this one
      float M = -INFINITY;
      for (int p = 0; p < sg.n_parts; ++p) {
        const u64 ml = __hip_atomic_load(reinterpret_cast<const u64*>(part_ml + (int64_t)(sg.first_part + p) * (2 * QT)) + w * 32 + col,
                                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        M = fmaxf(M, __builtin_bit_cast(float, (unsigned)ml));
      }
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[mb][r] = 0.f;
      l = 0.f;
      for (int p = 0; p < sg.n_parts; ++p) {   // in slot order: the sum does not depend on who adds it up
        const u64 ml = __hip_atomic_load(reinterpret_cast<const u64*>(part_ml + (int64_t)(sg.first_part + p) * (2 * QT)) + w * 32 + col,
                                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float f = __builtin_amdgcn_exp2f(__builtin_bit_cast(float, (unsigned)ml) - M);
        l = fmaf(f, __builtin_bit_cast(float, (unsigned)(ml >> 32)), l);
        const u64* po = reinterpret_cast<const u64*>(part_o + (int64_t)(sg.first_part + p) * (QT * D)) + (w * MB * 8) * 64 + lane;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int h2 = 0; h2 < 8; ++h2) {
            const u64 v2 = __hip_atomic_load(po + (mb * 8 + h2) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            o[mb][2 * h2] = fmaf(f, __builtin_bit_cast(float, (unsigned)v2), o[mb][2 * h2]);
            o[mb][2 * h2 + 1] = fmaf(f, __builtin_bit_cast(float, (unsigned)(v2 >> 32)), o[mb][2 * h2 + 1]);
          }
      }
      if (tid == 0)   // as the next launch expects it
        __hip_atomic_store(&part_count[sg.counter], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  const float inv = 1.f / l;
  const int qi = q0 + col;
  if (store && qi < N_k) {
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
  if (STREAM && si + 1 < seg_hi) __syncthreads();   // every wave has left the ring before the next segment refills it
  }  // segments
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
                          float scale, void* out, int kernel) {
  typedef __bf16 T;
  if (kernel != 0)
    hipLaunchKernelGGL((attn_pipe<D, NW, false>), dim3(n_items), dim3(64 * NW), 0, s, descs, items, nullptr, nullptr,
                       (const T*)q, (const T*)k_cache, (const T*)v_cache, N_k, scale, (T*)out, nullptr, nullptr, nullptr);
  else
    hipLaunchKernelGGL((attn_mfma<D, NW>), dim3(n_items), dim3(64 * NW), 0, s, descs, items,
                       (const T*)q, (const T*)k_cache, (const T*)v_cache, N_k, scale, (T*)out);
}

void launch_attn(hipStream_t s, int dtype, int head_dim, const UnitDesc* descs, const AttnItem* items,
                 int n_items, int q_tile_rows, const void* q, const void* k_cache,
                 const void* v_cache, int N_k, float scale, void* out, int bf16_kernel) {
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
  if (head_dim == 64) launch_mfma_t<64, 4>(s, descs, items, n_items, q, k_cache, v_cache, N_k, scale, out, bf16_kernel);
  else launch_mfma_t<128, 4>(s, descs, items, n_items, q, k_cache, v_cache, N_k, scale, out, bf16_kernel);
}

// Work-groups of the streamed bf16 kernel that the current device holds at once.
int attn_stream_slots(int head_dim) {
  int dev = 0, cus = 0, blocks = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  const hipError_t e = head_dim == 64
      ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, attn_pipe<64, 4, true>, 256, 0)
      : hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, attn_pipe<128, 4, true>, 256, 0);
  if (e != hipSuccess) return 0;
  return blocks * cus;
}

void launch_attn_stream(hipStream_t s, int head_dim, const UnitDesc* descs, const AttnSeg* segs, const int32_t* seg_begin,
                        int n_groups, const void* q, const void* k_cache, const void* v_cache, int N_k, float scale,
                        void* out, float* part_o, float* part_ml, unsigned* part_count) {
  if (n_groups <= 0) return;
  typedef __bf16 T;
  if (head_dim == 64)
    hipLaunchKernelGGL((attn_pipe<64, 4, true>), dim3(n_groups), dim3(256), 0, s, descs, nullptr, segs, seg_begin,
                       (const T*)q, (const T*)k_cache, (const T*)v_cache, N_k, scale, (T*)out, part_o, part_ml, part_count);
  else
    hipLaunchKernelGGL((attn_pipe<128, 4, true>), dim3(n_groups), dim3(256), 0, s, descs, nullptr, segs, seg_begin,
                       (const T*)q, (const T*)k_cache, (const T*)v_cache, N_k, scale, (T*)out, part_o, part_ml, part_count);
}

}  // namespace hack
