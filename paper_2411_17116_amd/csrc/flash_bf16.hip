// bf16 row-tiled attention for gfx950 (head_dim 128): the compute-bound kernel
// behind phase 1 (Section 2.1, Algorithm 1: causal attention inside
// [anchor; block]) and behind phase-2 calls with many rows (Eq. 1-2: local
// attention and log-sum-exp of a row tile over one split of the cache).
//
// Shape of the computation
//   * A workgroup is 4 wavefronts; each wavefront owns 32 query rows and the
//     whole head dimension.  The rows of a workgroup are GQA-packed: up to 4
//     query heads of one KV group x 32 tokens, so the K/V tiles a workgroup
//     streams are shared by all of its rows and every wavefront has the same
//     causal frontier.
//   * K/V tiles of 64 keys are DMA'd from HBM/L2 straight into LDS
//     (global_load_lds_dwordx4, no VGPR staging), double-buffered, one barrier
//     per tile.  Inside a 256-byte key row the sixteen 16-byte chunks are
//     XOR-swizzled so that both the K operand reads (ds_read_b128) and the
//     transposing V operand reads (ds_read_b64_tr_b16) are bank-conflict free
//     without padding.
//   * S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (A = K rows from LDS, B = Q^T
//     held in registers for the whole kernel).  Computing the transposed score
//     tile leaves each lane with 16 keys of ONE query row, so the row maximum
//     and sum are in-lane reductions plus a single cross-half exchange, and the
//     exponentiated tile is already laid out as the B operand of the second
//     MFMA: O^T += V^T P^T, with V^T fragments produced by the LDS transposing
//     read.  P never touches LDS.
//   * Softmax runs in the log2 domain in fp32 against a lazily raised reference
//     maximum: the common path is one fma + one exp per score, a packed bf16
//     conversion and a dot2 for the row sum; the row maximum is only searched
//     (and the accumulators rescaled) for the first unit and when a row sum shows
//     that the reference has become stale.  O / l does not depend on the reference.
//   * The key loop is software-pipelined per 32-key unit: the QK MFMAs of unit
//     u+1, the exponentials of unit u and the PV MFMAs of unit u-1 share one
//     scheduling region whose order is pinned with sched_group_barrier.
//   * Only tiles that touch a row's causal frontier or a ragged range end take
//     the masking path.
#include "star_internal.h"

namespace star {

int heads_per_workgroup(int G);   // defined with the split plan

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int D = 128;
constexpr int TKEYS = 64;                  // keys per LDS tile
constexpr int ROWB = D * 2;                // bytes per key row
constexpr int TILEB = TKEYS * ROWB;        // 16 KiB
constexpr int LDS_K0 = 0, LDS_K1 = TILEB, LDS_V0 = 2 * TILEB, LDS_V1 = 3 * TILEB;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

#define LDS_AS __attribute__((address_space(3)))

// chunk swizzle of a key row: chunk c of row r is stored in slot c ^ swz(r)
__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// 16-byte DMA global -> LDS: lane L's data lands at lds_base + 16 * L.  The
// global address is sbase + voff (unsigned 32-bit byte offset per lane).
__device__ __forceinline__ void dma16(const char* sbase, unsigned voff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(sbase), "s"(lds_base) : "memory");
}

__device__ __forceinline__ bf16x8 lds_read_b128(unsigned addr) {
  return *(LDS_AS bf16x8*)(addr);
}

// Transposing LDS read: within each group of 16 lanes, lane i receives element
// i%4 of the four 8-byte rows addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12.
__device__ __forceinline__ bf16x4 lds_read_tr16(unsigned addr) {
  return __builtin_bit_cast(bf16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(addr)));
}

__device__ __forceinline__ float pair_max(float x) {
  // both lanes of a (l, l^32) pair receive max(x[l], x[l^32])
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Waits for the DMAs.  They must be opaque asm: the DMAs themselves are opaque
// to the compiler, which would drop a builtin s_waitcnt it believes redundant.
__device__ __forceinline__ void wait_vmcnt0() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void wait_vmcnt8() { asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); }

// Sequence of key tiles a workgroup walks: first the tiles of [0, a_hi)
// (n_a of them), then the tiles of [loc_lo, loc_hi).
struct TileSeq {
  int n_a;
  int n_tiles;
  int a_hi;
  int loc_lo;
  int loc_hi;
  __device__ __forceinline__ void tile(int idx, int* key0, int* hi) const {
    if (idx < n_a) { *key0 = idx * TKEYS; *hi = a_hi; }
    else { *key0 = loc_lo + (idx - n_a) * TKEYS; *hi = loc_hi; }
  }
};

struct WaveState {
  bf16x8 q[8];        // Q^T fragments: q[t] = Q[row lane%32][16t + 8*(lane/32) .. +7]
  f32x16 o[4];        // O^T accumulators: o[dt][v] = O[row][32dt + 8(v/4) + 4(lane/32) + v%4]
  float m;            // reference maximum of the raw logits (pair-uniform); see softmax_fix
  float neg_mc;       // -m * c (0 while m == -inf)
  float l;            // this lane's share of the running sum of 2^((s-m) c)
  float lmax;         // largest per-unit partial row sum seen by the fast loop
};

// Per-lane LDS addresses and DMA offsets, fixed for the whole kernel.
struct LaneAddr {
  unsigned k[8];       // K operand: row lane%32, chunk 2t + lane/32 (swizzled)
  unsigned v[4][2];    // V^T operand: see attend()
  unsigned dma;        // byte offset of this thread's 16-byte unit in row tid/16
  int tid;
  int half;
};

// Issue the DMA of one 64-key tile of K or V into an LDS tile buffer.  Thread
// `tid` moves the 16-byte unit (row it*16 + tid/16, slot tid%16) for it = 0..3;
// rows at or past `hi` re-read the last valid row (they are masked in the score
// tile, and finite values keep 0 * V finite).
__device__ __forceinline__ void issue_tile(const char* base, int key0, int hi, unsigned lds,
                                           const LaneAddr& la) {
  unsigned wave_base = __builtin_amdgcn_readfirstlane((la.tid & ~63) * 16);
  if (key0 + TKEYS <= hi) {            // full tile: scalar base, constant lane offsets
    const char* sb = base + (size_t)key0 * ROWB;
#pragma unroll
    for (int it = 0; it < 4; ++it) dma16(sb + it * 16 * ROWB, la.dma, lds + it * 4096 + wave_base);
  } else {
    int chunk_off = la.dma & 255;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      int key = key0 + it * 16 + (la.tid >> 4);
      key = key < hi ? key : hi - 1;
      dma16(base, (unsigned)key * ROWB + chunk_off, lds + it * 4096 + wave_base);
    }
  }
}

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// The fast key loop keeps ONE reference maximum per row, taken from the row's
// first 32 keys, and never rescales: p = 2^(s c - m c) against any fixed m gives
// the same O / l.  It only has to stay finite, so the loop tracks the largest
// per-unit row sum and, if one exceeds this limit (a score more than ~40 nats
// above the reference), the workgroup redoes its rows with the exact online
// softmax (SAFE mode), which searches the maximum of every unit.
constexpr float LSUM_LIMIT = 1.152921504606846976e18f;   // 2^60

__device__ __forceinline__ float unit_max(const f32x16& s) {
  float t0 = fmaxf(fmaxf(s[0], s[1]), s[2]);
  float t1 = fmaxf(fmaxf(s[3], s[4]), s[5]);
  float t2 = fmaxf(fmaxf(s[6], s[7]), s[8]);
  float t3 = fmaxf(fmaxf(s[9], s[10]), s[11]);
  float t4 = fmaxf(fmaxf(s[12], s[13]), s[14]);
  return pair_max(fmaxf(fmaxf(fmaxf(t0, t1), fmaxf(t2, t3)), fmaxf(t4, s[15])));
}

// Softmax numerators of one 32-key score tile against the reference w.m:
// p = 2^(s c - m c) rounded to bf16, and the lane's sum of the ROUNDED values
// (v_dot2 with a vector of ones), so numerator and denominator see the same
// rounding.
__device__ __forceinline__ float softmax_unit(const WaveState& w, const f32x16& s, bf16x8 (&p)[2],
                                              float c) {
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  float lsum = 0.f;
#pragma unroll
  for (int v = 0; v < 16; v += 2) {
    bf16x2 pr;
    pr[0] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[v], c, w.neg_mc));
    pr[1] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[v + 1], c, w.neg_mc));
    p[v / 8][v % 8] = pr[0];
    p[v / 8][v % 8 + 1] = pr[1];
    lsum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, lsum, false);
  }
  return lsum;
}

// SAFE mode: raise the reference to the maximum seen so far; returns the factor
// alpha = 2^((m_old - m_new) c) for everything accumulated before (0 while
// nothing was visible yet, 1 if the maximum did not move).
__device__ __forceinline__ float raise_reference(WaveState& w, const f32x16& s, float c) {
  float m_new = fmaxf(w.m, unit_max(s));
  float mm = m_new == -INFINITY ? 0.f : m_new;
  float alpha = __builtin_amdgcn_exp2f((w.m - mm) * c);
  w.m = m_new;
  w.neg_mc = mm * -c;
  return alpha;
}

__device__ __forceinline__ void rescale(WaveState& w, float alpha) {
  if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {   // some row maximum moved
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) w.o[dt][v] *= alpha;
  }
}

// Causal / range-end mask of one 32-key score tile: element v is key
// key0 + 8(v/4) + 4*half + v%4 and is visible iff it is below `lim`.
__device__ __forceinline__ void mask_unit(f32x16& s, int key0, int lim, int half) {
  int x = lim - key0 - 4 * half;
#pragma unroll
  for (int v = 0; v < 16; ++v) s[v] = (8 * (v / 4) + (v % 4)) < x ? s[v] : -INFINITY;
}

// One pipeline stage holds three independent pieces of work:
//   QK  : s_next  = K[unit u+1] Q^T          (8 MFMAs, K fragments from LDS at KOFF)
//   SM  : p_cur   = softmax numerators of s_cur (unit u), updates w.l / w.lmax
//   PV  : O^T    += V[unit u-1]^T p_prev      (8 MFMAs, V^T fragments from LDS at VOFF)
// so that the MFMAs of two units hide the exponentials of the third.  The
// sched_group_barrier sequence at the end pins the instruction order inside the
// stage: operand fragments are read from LDS two MFMA pairs ahead of their use
// and a few VALU instructions sit between consecutive MFMAs.  Returns the
// rescale factor for the accumulators (SAFE mode; 1 otherwise), to be applied
// after the stage, i.e. after the PV MFMAs of unit u-1 and before those of u.
template <bool SAFE, bool QK, bool SM, bool PV, int KOFF, int VOFF>
__device__ __forceinline__ float stage(WaveState& w, const LaneAddr& la, f32x16& s_next,
                                       f32x16& s_cur, bf16x8 (&p_cur)[2],
                                       const bf16x8 (&p_prev)[2], float c) {
  float alpha = 1.0f;
  bf16x8 kf[8], vf[8];
  // Keep this stage's softmax inside the stage: without the anchors the optimizer
  // hoists it above the preceding barrier and sinks the row sums to the loop end.
  if (SM) asm volatile("" : "+v"(s_cur));
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (QK) kf[i] = lds_read_b128(la.k[i] + KOFF);
    if (PV) {
      // B operand p_prev[hf]: slot e of lane half h is key 16hf + 8(e/4) + 4h + e%4,
      // so the A operand needs, for d-row lane%32, keys k0..k0+3 and k0+8..k0+11
      // with k0 = 16hf + 4h: two transposing reads.
      const int hf = i >> 2, dt = i & 3;
      bf16x4 lo = lds_read_tr16(la.v[dt][0] + VOFF + 16 * hf * ROWB);
      bf16x4 hi = lds_read_tr16(la.v[dt][1] + VOFF + 16 * hf * ROWB);
      vf[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
  }
  if (SM) {
    if (SAFE) {
      alpha = raise_reference(w, s_cur, c);
      w.l = __builtin_fmaf(w.l, alpha, softmax_unit(w, s_cur, p_cur, c));
    } else {
      float lsum = softmax_unit(w, s_cur, p_cur, c);
      w.l += lsum;
      w.lmax = fmaxf(w.lmax, lsum);
    }
  }
  if (QK) {
#pragma unroll
    for (int v = 0; v < 16; ++v) s_next[v] = 0.f;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (QK) s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], w.q[i], s_next, 0, 0, 0);
    if (PV) w.o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i], p_prev[i >> 2], w.o[i & 3], 0, 0, 0);
  }
  if (QK && SM && PV) {
    __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, SAFE ? 5 : 3, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < 6) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, SAFE ? 5 : 4, 0);
    }
  }
  if (SM) asm volatile("" : "+v"(w.l), "+v"(w.lmax), "+v"(p_cur[0]), "+v"(p_cur[1]));
  __builtin_amdgcn_sched_barrier(0);
  return alpha;
}

// Everything a wavefront does for key tile t once tile t's scores exist:
//   barrier (K tile t+1 and V tile t have landed; older buffers are free),
//   DMA of K tile t+2 and V tile t+1 into the buffers just released,
//   stage A: scores of unit 2t+2 | softmax of unit 2t+1 | PV of unit 2t,
//   stage B: scores of unit 2t+3 | softmax of unit 2t+2 | PV of unit 2t+1.
// MORE = tile t+1 exists.  KN / VC are the LDS offsets of K tile t+1 and V tile t,
// KF / VF those of the buffers that are refilled (K tile t+2, V tile t+1).
template <bool SAFE, bool MORE, int KN, int VC, int KF, int VF>
__device__ __forceinline__ void tile_step(WaveState& w, const LaneAddr& la, const TileSeq& seq,
                                          const char* Kb, const char* Vb, int t, int row_lim,
                                          int wave_lo, float c, unsigned lds0, f32x16& sA,
                                          f32x16& sB, bf16x8 (&pA)[2], bf16x8 (&pB)[2]) {
  constexpr int H = 32 * ROWB;
  wait_vmcnt0();
  __builtin_amdgcn_s_barrier();
  if (t + 2 < seq.n_tiles) {
    int k2, h2;
    seq.tile(t + 2, &k2, &h2);
    issue_tile(Kb, k2, h2, lds0 + KF, la);
  }
  if (MORE) {
    int nk0, nhi;
    seq.tile(t + 1, &nk0, &nhi);
    issue_tile(Vb, nk0, nhi, lds0 + VF, la);
    const int nlim = row_lim < nhi ? row_lim : nhi;
    float alpha = stage<SAFE, true, true, true, KN, VC>(w, la, sA, sB, pB, pA, c);
    if (SAFE) rescale(w, alpha);
    if (nk0 + 32 > wave_lo || nk0 + 32 > nhi) mask_unit(sA, nk0, nlim, la.half);
    alpha = stage<SAFE, true, true, true, KN + H, VC + H>(w, la, sB, sA, pA, pB, c);
    if (SAFE) rescale(w, alpha);
    if (nk0 + 64 > wave_lo || nk0 + 64 > nhi) mask_unit(sB, nk0 + 32, nlim, la.half);
  } else {
    float alpha = stage<SAFE, false, true, true, 0, VC>(w, la, sA, sB, pB, pA, c);
    if (SAFE) rescale(w, alpha);
    stage<SAFE, false, false, true, 0, VC + H>(w, la, sB, sA, pA, pB, c);
  }
}

// Walk a tile sequence once for the calling wavefront (all four wavefronts of
// the workgroup call this with the same sequence).
//   row_lim     this lane's exclusive causal key bound (0 for an inactive row)
//   wave_lo     smallest row_lim among the wavefront's active rows: key tiles that
//               end at or below it need no causal mask
template <bool SAFE>
__device__ __forceinline__ void key_loop(WaveState& w, const LaneAddr& la, const TileSeq& seq,
                                         const char* Kb, const char* Vb, int row_lim, int wave_lo,
                                         float c, unsigned lds0) {
  const int T = seq.n_tiles;
  constexpr int K0 = LDS_K0, K1 = LDS_K1, V0 = LDS_V0, V1 = LDS_V1, H = 32 * ROWB;
  f32x16 sA, sB;              // score tiles of the even / odd 32-key unit
  bf16x8 pA[2], pB[2];        // their exponentials (bf16)
  int key0, hi;

  // Prologue: K tile 0, V tile 0 and K tile 1 in flight; scores of tile 0.
  seq.tile(0, &key0, &hi);
  issue_tile(Kb, key0, hi, lds0 + K0, la);
  issue_tile(Vb, key0, hi, lds0 + V0, la);
  if (T > 1) {
    int k1, h1;
    seq.tile(1, &k1, &h1);
    issue_tile(Kb, k1, h1, lds0 + K1, la);
    wait_vmcnt8();
  } else {
    wait_vmcnt0();
  }
  __builtin_amdgcn_s_barrier();
  const int lim0 = row_lim < hi ? row_lim : hi;
  stage<SAFE, true, false, false, K0, 0>(w, la, sA, sA, pA, pA, c);
  if (key0 + 32 > wave_lo || key0 + 32 > hi) mask_unit(sA, key0, lim0, la.half);
  stage<SAFE, true, false, false, K0 + H, 0>(w, la, sB, sA, pA, pA, c);
  if (key0 + 64 > wave_lo || key0 + 64 > hi) mask_unit(sB, key0 + 32, lim0, la.half);
  // first unit: its row maximum becomes the reference (nothing to rescale yet)
  raise_reference(w, sA, c);
  w.l = softmax_unit(w, sA, pA, c);

  // Tile t: V tile t is consumed while K tile t+1 produces the next scores.
  // The loop is unrolled by two so that every LDS buffer offset is an immediate
  // and the accumulators flow through straight-line code.
  int t = 0;
  for (; t + 2 < T; t += 2) {
    tile_step<SAFE, true, K1, V0, K0, V1>(w, la, seq, Kb, Vb, t, row_lim, wave_lo, c, lds0, sA, sB, pA, pB);
    tile_step<SAFE, true, K0, V1, K1, V0>(w, la, seq, Kb, Vb, t + 1, row_lim, wave_lo, c, lds0, sA, sB, pA, pB);
  }
  if (T - t == 2) {
    tile_step<SAFE, true, K1, V0, K0, V1>(w, la, seq, Kb, Vb, t, row_lim, wave_lo, c, lds0, sA, sB, pA, pB);
    tile_step<SAFE, false, K0, V1, K1, V0>(w, la, seq, Kb, Vb, t + 1, row_lim, wave_lo, c, lds0, sA, sB, pA, pB);
  } else {
    tile_step<SAFE, false, K1, V0, K0, V1>(w, la, seq, Kb, Vb, t, row_lim, wave_lo, c, lds0, sA, sB, pA, pB);
  }
}

__device__ __forceinline__ void reset_state(WaveState& w) {
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) w.o[dt][v] = 0.f;
  w.m = -INFINITY;
  w.neg_mc = 0.f;
  w.l = 0.f;
  w.lmax = 0.f;
}

// Attention of the workgroup's rows over a tile sequence: the fast loop, and the
// exact loop again if any wavefront's scores left the fast loop's safe range.
__device__ __forceinline__ void attend(WaveState& w, const TileSeq& seq, const char* Kb,
                                       const char* Vb, int row_lim, int wave_lo,
                                       float c, unsigned lds0) {
  LaneAddr la;
  la.tid = threadIdx.x;
  const int lane = la.tid & 63;
  la.half = lane >> 5;
  const int i32 = lane & 31;
  {
    int x = la.half ^ swz(i32);
#pragma unroll
    for (int t = 0; t < 8; ++t) la.k[t] = lds0 + i32 * ROWB + (((2 * t) ^ x) << 4);
    // V^T operand: source lane addresses row 4*half + (lane%16)/4 (+8 for the
    // second read), columns 32dt + 16*((lane/16)%2) + 4*(lane%4) .. +3
    int q4 = (lane & 15) >> 2, gi = (lane >> 4) & 1;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        int r = 4 * la.half + q4 + 8 * u;
        int chunk = 4 * dt + 2 * gi + ((lane & 3) >> 1);
        la.v[dt][u] = lds0 + r * ROWB + ((chunk ^ swz(r)) << 4) + 8 * (lane & 1);
      }
    unsigned chunk_off = ((la.tid & 15) ^ swz(la.tid >> 4)) << 4;
    la.dma = (la.tid >> 4) * ROWB + chunk_off;
  }
  if (seq.n_tiles == 0) return;
  // Consume the Q fragments here so that the compiler places its own wait for
  // their loads before the first DMA is in flight (and none inside the loops).
#pragma unroll
  for (int t = 0; t < 8; ++t) asm volatile("" : "+v"(w.q[t]));
  key_loop<false>(w, la, seq, Kb, Vb, row_lim, wave_lo, c, lds0);

  // Did any row of any wavefront leave the safe range?  One LDS word per
  // wavefront; __syncthreads() (fence + barrier) orders the tile reads before the
  // flag writes, the writes before the reads, and the reads before any new DMA.
  __syncthreads();
  const bool bad = __builtin_amdgcn_ballot_w64(!(w.lmax < LSUM_LIMIT)) != 0;
  LDS_AS int* flags = (LDS_AS int*)(size_t)lds0;
  if (lane == 0) flags[la.tid >> 6] = bad ? 1 : 0;
  __syncthreads();
  const int any_bad = flags[0] | flags[1] | flags[2] | flags[3];
  __syncthreads();
  if (__builtin_expect(any_bad != 0, 0)) {
    reset_state(w);
    key_loop<true>(w, la, seq, Kb, Vb, row_lim, wave_lo, c, lds0);
  }
}

__device__ __forceinline__ void load_q(WaveState& w, const char* qrow, int half) {
#pragma unroll
  for (int t = 0; t < 8; ++t) w.q[t] = *(const bf16x8*)(qrow + (16 * t + 8 * half) * 2);
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) w.o[dt][v] = 0.f;
  w.m = -INFINITY;
  w.neg_mc = 0.f;
  w.l = 0.f;
  w.lmax = 0.f;
}

// ------------------------------------------------------------------ phase 1
// grid.x enumerates (kv head fastest, then work items); see launch_phase1_bf16.
__global__ __launch_bounds__(256, 2) void phase1_bf16_kernel(Phase1Args a, int hpw, int tpb, int n_hs) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const Geom& g = a.g;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int half = lane >> 5, i32 = lane & 31;
  const int tm = 32 * (4 / hpw);                 // tokens per workgroup

  // work decode: kv head fastest (one KV head per XCD when Hkv is a multiple of
  // 8), then batch, head sub-group, tile within block (late = heavy first),
  // block (block 0, the lightest, last)
  int id = blockIdx.x;
  int kvh = id % g.Hkv; id /= g.Hkv;
  int beta = id % g.B; id /= g.B;
  int hs = id % n_hs; id /= n_hs;
  int t = tpb - 1 - (id % tpb); id /= tpb;
  int n = (int)((g.L + g.b - 1) / g.b);
  int i = id + 1 == n ? 0 : id + 1;

  int s = (int)(i * g.b);
  int e = (int)((int64_t)s + g.b < g.L ? s + g.b : g.L);
  int row0 = s + t * tm;
  if (row0 >= e) return;                         // tile beyond a short block

  int head = kvh * g.G + hs * hpw + wave % hpw;
  int tok0 = row0 + 32 * (wave / hpw);
  int tok = tok0 + i32;
  bool active = tok < e;
  int wg_last = row0 + tm < e ? row0 + tm : e;   // exclusive bound of the workgroup's tokens

  const char* Kb = (const char*)a.Kc + ((size_t)beta * g.Hkv + kvh) * (size_t)g.cap * ROWB;
  const char* Vb = (const char*)a.Vc + ((size_t)beta * g.Hkv + kvh) * (size_t)g.cap * ROWB;
  WaveState w;
  int qtok = active ? tok : (tok0 < e ? tok0 : e - 1);
  load_q(w, (const char*)a.Q + (((size_t)beta * g.L + qtok) * g.Hq + head) * ROWB, half);

  TileSeq seq;
  seq.a_hi = i > 0 ? (int)g.a : 0;
  seq.n_a = (seq.a_hi + TKEYS - 1) / TKEYS;
  seq.loc_lo = s;
  seq.loc_hi = wg_last;
  seq.n_tiles = seq.n_a + (wg_last - s + TKEYS - 1) / TKEYS;

  // a row sees key k iff k < tok + 1; anchor keys always qualify (a <= b <= tok)
  int row_lim = active ? tok + 1 : 0;
  int wave_lo = tok0 < e ? tok0 + 1 : 0;
  unsigned lds0 = (unsigned)(size_t)(LDS_AS char*)lds;
  attend(w, seq, Kb, Vb, row_lim, wave_lo, g.scale * LOG2E, lds0);

  float l_tot = pair_sum(w.l);
  if (active) {
    float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    char* orow = (char*)a.O + (((size_t)beta * g.L + tok) * g.Hq + head) * ROWB;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x4 v;
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = (__bf16)(w.o[dt][4 * j + k] * inv);
        *(bf16x4*)(orow + (32 * dt + 8 * j + 4 * half) * 2) = v;
      }
    if (a.LSE && half == 0)
      a.LSE[((size_t)beta * g.Hq + head) * g.L + tok] =
          l_tot > 0.f ? (w.m * g.scale * LOG2E + __builtin_amdgcn_logf(l_tot)) * LN2 : -INFINITY;
  }
}

// ------------------------------------------------------------------ phase 2
// Local attention (Eq. 1) and log-sum-exp (log of Eq. 2) of a row tile over one
// split of the cache.  grid.x = ((batch * s_total + split) * n_hs + hs) * row_tiles + tile,
// grid.y = kv head.
__global__ __launch_bounds__(256, 2) void phase2_rows_bf16_kernel(Phase2Args a, int hpw, int n_hs,
                                                                  int row_tiles) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const Geom& g = a.g;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int half = lane >> 5, i32 = lane & 31;
  const int tm = 32 * (4 / hpw);

  int id = blockIdx.x;
  int tt = id % row_tiles; id /= row_tiles;
  int hs = id % n_hs; id /= n_hs;
  int sp = id % a.plan.s_total;
  int beta = id / a.plan.s_total;
  int kvh = blockIdx.y;

  int head = kvh * g.G + hs * hpw + wave % hpw;
  int j0 = tt * tm + 32 * (wave / hpw);
  int j = j0 + i32;
  bool active = j < a.q_len;
  int total = (int)(a.cache_len + a.q_len);
  int64_t lo64, hi64;
  split_range(a.plan, g.L, g.b, total, sp, &lo64, &hi64);
  int lo = (int)lo64, hi = (int)hi64;

  const char* Kb = (const char*)a.Kc + ((size_t)beta * g.Hkv + kvh) * (size_t)g.cap * ROWB;
  const char* Vb = (const char*)a.Vc + ((size_t)beta * g.Hkv + kvh) * (size_t)g.cap * ROWB;
  WaveState w;
  int qj = active ? j : (j0 < a.q_len ? j0 : a.q_len - 1);
  load_q(w, (const char*)a.Qq + (((size_t)beta * a.q_len + qj) * g.Hq + head) * ROWB, half);

  TileSeq seq;
  seq.a_hi = 0; seq.n_a = 0; seq.loc_lo = lo; seq.loc_hi = hi;
  seq.n_tiles = hi > lo ? (hi - lo + TKEYS - 1) / TKEYS : 0;

  // token j sees cache rows [0, cache_len + j]
  int cl = (int)a.cache_len;
  int row_lim = active ? cl + j + 1 : 0;
  int wave_lo = j0 < a.q_len ? cl + j0 + 1 : 0;
  unsigned lds0 = (unsigned)(size_t)(LDS_AS char*)lds;
  attend(w, seq, Kb, Vb, row_lim, wave_lo, g.scale * LOG2E, lds0);

  float l_tot = pair_sum(w.l);
  if (active) {
    float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    size_t r = (((size_t)beta * a.plan.s_total + sp) * g.Hq + head) * a.q_len + j;
    float* orow = a.O_sub + r * D;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        f32x4 v;
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = w.o[dt][4 * jj + k] * inv;
        *(f32x4*)(orow + 32 * dt + 8 * jj + 4 * half) = v;
      }
    if (half == 0)
      a.LSE_sub[r] = l_tot > 0.f ? (w.m * g.scale * LOG2E + __builtin_amdgcn_logf(l_tot)) * LN2
                                 : -INFINITY;
  }
}

}  // namespace

hipError_t launch_phase1_bf16(const Phase1Args& a, hipStream_t st) {
  const Geom& g = a.g;
  int hpw = heads_per_workgroup(g.G);
  int tm = 32 * (4 / hpw);
  int n_hs = g.G / hpw;
  int64_t n = (g.L + g.b - 1) / g.b;
  int64_t bmax = g.b < g.L ? g.b : g.L;
  int tpb = (int)((bmax + tm - 1) / tm);
  int64_t wgs = (int64_t)g.Hkv * g.B * n_hs * tpb * n;
  if (wgs > 0x7fffffff) return hipErrorInvalidValue;
  hipError_t e = hipFuncSetAttribute((const void*)phase1_bf16_kernel,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 4 * TILEB);
  if (e != hipSuccess) return e;
  phase1_bf16_kernel<<<dim3((unsigned)wgs), 256, 4 * TILEB, st>>>(a, hpw, tpb, n_hs);
  return hipGetLastError();
}

hipError_t launch_phase2_rows_bf16(const Phase2Args& a, hipStream_t st) {
  const Geom& g = a.g;
  int hpw = heads_per_workgroup(g.G);
  int tm = 32 * (4 / hpw);
  int n_hs = g.G / hpw;
  int row_tiles = (a.q_len + tm - 1) / tm;
  int64_t gx = (int64_t)g.B * a.plan.s_total * n_hs * row_tiles;
  if (gx > 0x7fffffff || g.Hkv > 65535) return hipErrorInvalidValue;
  hipError_t e = hipFuncSetAttribute((const void*)phase2_rows_bf16_kernel,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 4 * TILEB);
  if (e != hipSuccess) return e;
  phase2_rows_bf16_kernel<<<dim3((unsigned)gx, (unsigned)g.Hkv), 256, 4 * TILEB, st>>>(a, hpw, n_hs,
                                                                                       row_tiles);
  return hipGetLastError();
}

}  // namespace star
