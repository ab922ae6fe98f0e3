// Attention for scale steps with few queries (Preliminaries, attention
// equation: O = Softmax(scale * Q K^T) V, no mask inside a scale step) on gfx950.
//
// The first scale steps of a next-scale schedule have a handful to a few
// hundred queries per unit: tiles of 128 queries leave most of the chip idle
// and every work-group walks the whole cache alone.  Here a work item is
// (unit, 32 queries) and its four waves split the KEYS: wave w takes the 32-key
// blocks w, w+4, ... with a private online softmax, and the four partial
// results (running max, normaliser, unnormalised O) are merged through LDS at
// the end.  There is no work-group barrier inside the loop: K and V blocks
// travel HBM -> LDS directly (global_load_lds, whole rows, so the copies are
// fully coalesced) into one private K slot and one private V slot per wave; the
// copy of the next K block is issued as soon as the score MFMAs have read the
// current one, the copy of the next V block as soon as the PV MFMAs have read
// theirs.  K fragments are read with ds_read_b128, V^T through the transposing
// LDS read, with the same bank-conflict-free swizzles as the large-step kernel.
// Optionally the kernel also performs the cache update of the step (cache-update
// equation of the Preliminaries): keys are then read from the virtual
// concatenation [cached rows | rows of the current scale] and work item t
// copies rows [32t, 32t+32) of the current scale behind the unit's cached rows,
// so a step that does not compress needs a single launch.
#include "device_util.h"
#include "hack_internal.h"

namespace hack {

namespace {

using namespace dev;

constexpr int kKB = 32;        // keys per block
constexpr int kWaves = 4;      // waves per work-group = key splits
constexpr int kQTile = 32;     // queries per work item

// fuse != 0: keys are [rows in_off .. in_off+len_in of the cache | the unit's n_new
// rows of k_new / v_new], and those new rows are also written behind the cached
// ones (k_app / v_app / pos_app are the cache arrays, which k_cache / v_cache then
// alias: reads stay below row len_in, writes at or above it).
// fuse == 0: keys are rows [out_off, out_off + n_out) of the cache.
template <int D>
__global__ __launch_bounds__(64 * kWaves, 2) void attn_split(
    const UnitDesc* __restrict__ descs, const AttnItem* __restrict__ items, const __bf16* __restrict__ q,
    const __bf16* k_cache, const __bf16* v_cache, const __bf16* k_new, const __bf16* v_new, __bf16* k_app,
    __bf16* v_app, int32_t* pos_app, int pos_new, int fuse, int N_k, float scale, __bf16* __restrict__ out) {
  constexpr int KK = D / 16;        // MFMA steps over head_dim for S^T
  constexpr int MB = D / 32;        // 32-row blocks of O^T
  constexpr int CPR = D / 8;        // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;     // block rows covered by one wave-wide copy instruction
  constexpr int IPB = kKB / RPI;    // copy instructions per V block
  constexpr int BLK = kKB * D;      // elements per block

  const AttnItem it = items[blockIdx.x];
  if (it.desc < 0) return;
  const AttnItem& d = it;   // the item carries the descriptor fields read here
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;

  const int total = d.n_out;                       // keys attended over
  const int len_c = fuse ? d.len_in : d.n_out;     // of which come from the cache
  const int64_t base = fuse ? d.in_off : d.out_off;
  const int64_t new_row0 = (int64_t)d.unit * N_k;  // first row of the unit in q / k_new / v_new / out
  const int q0 = it.q_tile * kQTile;

  // per wave one K slot [0] and one V slot [1]; after the loop the pair holds the
  // wave's unnormalised O^T (same size)
  __shared__ __attribute__((aligned(1024))) __bf16 Vs[kWaves][2][BLK];
  __shared__ float m_sh[kWaves][32], l_sh[kWaves][32];

  // ---- cache update of this tile's rows ----
  if (fuse) {
    constexpr int LPR = D / 8;   // 16-byte pieces per row
    const int nr = min(kQTile, N_k - q0);
    const uint4* ks = reinterpret_cast<const uint4*>(k_new) + (new_row0 + q0) * LPR;
    const uint4* vs = reinterpret_cast<const uint4*>(v_new) + (new_row0 + q0) * LPR;
    uint4* kd = reinterpret_cast<uint4*>(k_app) + (d.in_off + d.len_in + q0) * LPR;
    uint4* vd = reinterpret_cast<uint4*>(v_app) + (d.in_off + d.len_in + q0) * LPR;
    for (int e = tid; e < nr * LPR; e += 64 * kWaves) {
      kd[e] = ks[e];
      vd[e] = vs[e];
    }
    if (pos_app != nullptr && tid < nr) pos_app[d.in_off + d.len_in + q0 + tid] = pos_new + q0 + tid;
  }

  // Block b of K (slot 0) or V (slot 1) into this wave's LDS: lane l of copy
  // instruction i fills LDS row r = i RPI + l / CPR, chunk position c = l % CPR, from
  // global chunk c ^ swz(r) of key row b*32 + r.  A block that lies wholly in the
  // cache or wholly in the new rows is a contiguous piece of memory: uniform base
  // plus loop-invariant lane offsets.  The ragged last block and a block that
  // straddles the two sources take per-lane addresses (rows past the end repeat
  // the last key; their scores are masked).
  const unsigned vs_lds = lds_addr_of(&Vs[0][0][0]);
  unsigned k_src[IPB], v_src[IPB];
#pragma unroll
  for (int i = 0; i < IPB; ++i) {
    const int r = i * RPI + lane / CPR, c = lane % CPR;
    k_src[i] = (unsigned)(r * D + ((c ^ swz_k<D>(r)) & (CPR - 1)) * 8) * 2u;
    v_src[i] = (unsigned)(r * D + ((c ^ swz_v<D>(r)) & (CPR - 1)) * 8) * 2u;
  }
  const unsigned k_lds = vs_lds + (unsigned)((w * 2 + 0) * BLK * 2), v_lds = vs_lds + (unsigned)((w * 2 + 1) * BLK * 2);
  auto issue = [&](int b, const __bf16* cache, const __bf16* fresh, const unsigned (&src)[IPB], unsigned lds, bool is_k) {
    const int j0 = b * kKB;
    const __bf16* blk = nullptr;
    if (j0 + kKB <= len_c) blk = cache + (base + j0) * D;
    else if (j0 >= len_c && j0 + kKB <= total) blk = fresh + (new_row0 + (j0 - len_c)) * D;
    if (blk != nullptr) {
#pragma unroll
      for (int i = 0; i < IPB; ++i) load_to_lds(blk, src[i], lds + (unsigned)(i * 1024));
    } else {
#pragma unroll
      for (int i = 0; i < IPB; ++i) {
        const int r = i * RPI + lane / CPR, c = lane % CPR;
        const int j = min(j0 + r, total - 1);
        const int sw = is_k ? swz_k<D>(r) : swz_v<D>(r);
        const __bf16* p = (j < len_c ? cache + (base + j) * D : fresh + (new_row0 + (j - len_c)) * D) + ((c ^ sw) & (CPR - 1)) * 8;
        load_to_lds(p, lds + (unsigned)(i * 1024));
      }
    }
  };
  auto issue_k = [&](int b) { issue(b, k_cache, k_new, k_src, k_lds, true); };
  auto issue_v = [&](int b) { issue(b, v_cache, v_new, v_src, v_lds, false); };

  const int n_blocks = (total + kKB - 1) / kKB;
  if (w < n_blocks) {
    issue_k(w);
    issue_v(w);
  }

  // Q fragments (B operand): query col, head-dim slice [16kk + 8 half, +8)
  bf16x8 qf[KK];
  {
    const __bf16* qrow = q + (new_row0 + min(q0 + col, N_k - 1)) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * half);
    // consumed here so that the compiler's wait for them sits before the loop,
    // whose vector-memory waits are all placed by hand
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) asm volatile("" ::"v"(qf[kk]));
  }
  dma_wait_but<0>();   // first K and V blocks (and everything above) have landed

  floatx16 o[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[mb][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c2 = scale * kLog2eF;

  // V^T operand reads: row 4 half + e (+16 sg, +8), head-dim 32mb + 16(g&1) + 4qd
  const int g = lane >> 4, e = (lane >> 2) & 3, qd = lane & 3;
  int v_off[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
    v_off[mb] = (4 * half + e) * D + (((4 * mb + 2 * (g & 1) + (qd >> 1)) ^ swz_v<D>(e)) & (CPR - 1)) * 8 + 4 * (qd & 1);
  int k_off[KK];   // K operand reads: row col, chunk 2kk + half
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) k_off[kk] = col * D + (((2 * kk + half) ^ swz_k<D>(col)) & (CPR - 1)) * 8;
  const bf16x2 ones2 = {(__bf16)1.0f, (__bf16)1.0f};

  // Vector-memory traffic of a wave inside the loop, all hand-issued copies, in
  // order: ... K(b), V(b) | K(next) after the score MFMAs of b, V(next) after the
  // PV MFMAs of b.  Copies complete in order, so "all but the newest IPB
  // instructions" is K(b) at the top of an iteration and V(b) before its PV.
  const __bf16* Kt = &Vs[w][0][0];
  const __bf16* Vt = &Vs[w][1][0];
  for (int b = w; b < n_blocks; b += kWaves) {
    const bool more = b + kWaves < n_blocks;
    dma_wait_but<IPB>();                 // K(b) has landed (V(b) may still be in flight)
    // S^T of block b: per lane one query column and 16 key rows
    floatx16 sc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Kt[k_off[kk]]);
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sc, 0, 0, 0);
    }
    // the MFMAs above have consumed every K read, so the slot may be refilled;
    // nothing below moves above this point
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    if (more) issue_k(b + kWaves);
    if ((b + 1) * kKB > total) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (b * kKB + 8 * (r >> 2) + 4 * half + (r & 3) >= total) sc[r] = -INFINITY;
    }
    float mx = sc[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sc[r]);
    mx = pair_max(mx);                       // finite: the block holds a valid key
    const float m_new = fmaxf(m_run, mx);
    if (__any(m_new != m_run)) {
      const float a = __builtin_amdgcn_exp2f((m_run - m_new) * c2);   // first block: exp2(-inf) = 0
      l_run *= a;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[mb][r] *= a;
      m_run = m_new;
    }
    const float mc = m_run * c2;
    bf16x8 pf[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) pf[r >> 3][r & 7] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sc[r], c2, -mc));
    // the row sum is taken over the rounded probabilities, the numbers the PV product uses
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      const bf16x2 pr = {pf[r >> 3][r & 7], pf[r >> 3][(r & 7) + 1]};
      psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones2, psum, false);
    }
    l_run += psum;
    if (more) dma_wait_but<IPB>();       // V(b) has landed (K(next) may still be in flight)
    else dma_wait_but<0>();
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
    // every V read has been consumed by an MFMA above: the slot may be refilled
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    if (more) issue_v(b + kWaves);
  }
  dma_wait_but<0>();   // nothing is outstanding when the slots are reused below

  // ---- merge the four partial results ----
  // This wave's copies have all landed and its LDS reads are done: its two slots
  // become its O^T partial, register-major so that lanes are contiguous.
  l_run = pair_sum(l_run);
  float* mine = reinterpret_cast<float*>(&Vs[w][0][0]);
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) mine[(mb * 16 + r) * 64 + lane] = o[mb][r];
  if (half == 0) {
    m_sh[w][col] = m_run;
    l_sh[w][col] = l_run;
  }
  __syncthreads();
  float M = -INFINITY;
#pragma unroll
  for (int x = 0; x < kWaves; ++x) M = fmaxf(M, m_sh[x][col]);   // finite: wave 0 saw block 0
  float f[kWaves], L = 0.f;
#pragma unroll
  for (int x = 0; x < kWaves; ++x) {
    f[x] = __builtin_amdgcn_exp2f((m_sh[x][col] - M) * c2);       // a wave without blocks: exp2(-inf) = 0
    L = fmaf(f[x], l_sh[x][col], L);
  }
  const float inv = 1.f / L;
  // wave w finishes registers [w CH, (w+1) CH) of the 16 MB per lane; register
  // 16 mb + r of lane (col, half) is head-dim 32mb + 8(r/4) + 4 half + r%4 of query col
  constexpr int CH = 16 * MB / kWaves;
  const int qi = q0 + col;
  __bf16* orow = out + (new_row0 + min(qi, N_k - 1)) * D;
#pragma unroll
  for (int i4 = 0; i4 < CH / 4; ++i4) {
    const int reg0 = w * CH + 4 * i4;
    bf16x4 pk;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float acc = 0.f;
#pragma unroll
      for (int x = 0; x < kWaves; ++x)
        acc = fmaf(f[x], reinterpret_cast<const float*>(&Vs[x][0][0])[(reg0 + i) * 64 + lane], acc);
      pk[i] = (__bf16)(acc * inv);
    }
    const int mb = reg0 >> 4, r4 = (reg0 & 15) >> 2;
    if (qi < N_k) *reinterpret_cast<bf16x4*>(orow + 32 * mb + 8 * r4 + 4 * half) = pk;
  }
}

}  // namespace

int attn_split_q_tile_rows() { return kQTile; }

void launch_attn_split(hipStream_t s, int head_dim, const UnitDesc* descs, const AttnItem* items, int n_items,
                       const void* q, const void* k_cache, const void* v_cache, const void* k_new, const void* v_new,
                       void* k_app, void* v_app, int32_t* pos_app, int pos_new, int fuse, int N_k, float scale,
                       void* out) {
  if (n_items <= 0) return;
  typedef __bf16 T;
  if (head_dim == 64)
    hipLaunchKernelGGL(attn_split<64>, dim3(n_items), dim3(64 * kWaves), 0, s, descs, items, (const T*)q,
                       (const T*)k_cache, (const T*)v_cache, (const T*)k_new, (const T*)v_new, (T*)k_app, (T*)v_app,
                       pos_app, pos_new, fuse, N_k, scale, (T*)out);
  else
    hipLaunchKernelGGL(attn_split<128>, dim3(n_items), dim3(64 * kWaves), 0, s, descs, items, (const T*)q,
                       (const T*)k_cache, (const T*)v_cache, (const T*)k_new, (const T*)v_new, (T*)k_app, (T*)v_app,
                       pos_app, pos_new, fuse, N_k, scale, (T*)out);
}

}  // namespace hack
