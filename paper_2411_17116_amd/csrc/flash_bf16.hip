// bf16 row-tiled attention for gfx950 (head_dim 128): the compute-bound kernel
// behind phase 1 (Section 2.1, Algorithm 1: causal attention inside
// [anchor; block]) and behind phase-2 calls with many rows (Eq. 1-2: local
// attention and log-sum-exp of a row tile over one split of the cache).
//
// Shape of the computation
//   * A workgroup is 8 wavefronts (two per SIMD, one workgroup per CU); each
//     wavefront owns 32 query rows (two blocks of 16) and the whole head
//     dimension.  The rows of a workgroup are GQA-packed: up to 8 query heads of
//     one KV group times 32 to 256 tokens, so the K/V tiles a workgroup streams
//     are fetched from L2 once per 256 rows, and the wavefronts' causal
//     frontiers lie within those tokens.
//   * K/V tiles of 64 keys are DMA'd from HBM/L2 straight into LDS
//     (global_load_lds_dwordx4, no VGPR staging), double-buffered, one barrier
//     per tile.  Key rows may sit anywhere a fixed stride apart: phase 1 reads
//     the caller's token-major K/V in place (and files them in the head-major
//     caches when it is done), phase 2 reads the caches.  In LDS, inside a
//     256-byte key row the sixteen 16-byte chunks are
//     XOR-swizzled so that both the K operand reads (ds_read_b128) and the
//     transposing V operand reads (ds_read_b64_tr_b16) are bank-conflict free
//     without padding.
//   * S^T = K Q^T with v_mfma_f32_16x16x32_bf16 (A = K rows from LDS, B = Q^T
//     held in registers for the whole kernel); a wavefront's 32 rows are two
//     column blocks of 16, and every K / V^T fragment read from LDS feeds both.
//     (The 16x16x32 shape moves a quarter of the accumulator registers per
//     instruction of the 32x32x16 one; at this chip's power limit it sustains
//     about 10 % more flops.)  Computing the transposed score tile leaves each
//     lane with keys of ONE query row, so row sums are in-lane and a row
//     maximum is an exchange among four lanes, and the exponentiated tile is
//     already laid out as the B operand of the second MFMA: O^T += V^T P^T,
//     with V^T fragments produced by the LDS transposing read.  P never
//     touches LDS.
//   * Softmax runs in the log2 domain in fp32 against a reference maximum taken
//     from the row's first 32 keys: the common path is one fma + one exp per
//     score and a packed bf16 conversion, with no maximum search and no rescale
//     (O / l does not depend on the reference).  The row sums come out of the
//     matrix pipe as well: one more MFMA per row block and unit multiplies P^T by
//     an operand whose first row is all ones, which leaves the sums of the bf16
//     numerators in row 0 of an accumulator (13 VALU instructions fewer per 32
//     MFMAs than summing on the VALU; what bounds this kernel is the number of
//     instructions a wavefront issues).  If a row sum shows that the reference
//     was too low to be safe, the workgroup redoes its rows with the exact
//     online softmax.
//   * The key loop is software-pipelined per 32-key unit: the QK MFMAs of unit
//     u+1, the exponentials of unit u and the PV MFMAs of unit u-1 share one
//     scheduling region whose order is pinned with sched_group_barrier.
//   * Only tiles that touch a row's causal frontier or a ragged range end take
//     the masking path.
//   * Phase 1 is launched with one workgroup per CU; the workgroups draw their
//     work items (a row tile of one block and KV head) from eight ticket queues,
//     each XCD from its own first (one KV head per XCD's L2 when Hkv is a
//     multiple of 8) and from the others once that is empty.  The queue counters
//     are the launch's own (Phase1Args::tickets).
#include "star_internal.h"

#include <atomic>

namespace star {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int D = 128;
constexpr int TKEYS = 64;                  // keys per LDS tile
constexpr int ROWB = D * 2;                // bytes per key row
constexpr int TILEB = TKEYS * ROWB;        // 16 KiB
constexpr int LDS_K0 = 0, LDS_K1 = TILEB, LDS_V0 = 2 * TILEB, LDS_V1 = 3 * TILEB;
// Wavefronts per workgroup.  All of them walk the same K/V tiles, so the L2 -> LDS
// traffic per flop falls with NW; 8 wavefronts of <= 256 registers are two per SIMD.
#ifndef STAR_FLASH_WAVES
#define STAR_FLASH_WAVES 8
#endif
constexpr int NW = STAR_FLASH_WAVES;
constexpr int NT = 64 * NW;                // threads per workgroup
constexpr int RB = 2;                      // 16-row blocks per wavefront
constexpr int WG_BLOCKS = NW * RB;         // 16-row blocks per workgroup
constexpr int DMA_ROWS = NT / 16;          // key rows one DMA instruction of the workgroup moves
constexpr int DMA_ITERS = TKEYS / DMA_ROWS;
static_assert(NW == 4 || NW == 8, "tile DMA is written for 4 or 8 wavefronts");
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

#define LDS_AS __attribute__((address_space(3)))

// chunk swizzle of a key row: chunk c of row r is stored in slot c ^ swz(r)
// (a rotation of the row's low four bits: conflict-free for the 16-row K operand
// read and for the 4-row transposing V read)
__device__ __forceinline__ int swz(int r) { return ((r << 1) & 15) | ((r >> 3) & 1); }

// 16-byte DMA global -> LDS: lane L's data lands at lds_base + 16 * L.  The
// global address is sbase + voff (unsigned 32-bit byte offset per lane).
__device__ __forceinline__ void dma16(const char* sbase, unsigned voff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(sbase), "s"(lds_base) : "memory");
}

__device__ __forceinline__ bf16x8 lds_read_b128(unsigned addr) {
  return *(LDS_AS bf16x8*)(size_t)(addr);
}

// Transposing LDS read: within each group of 16 lanes, lane i receives element
// i%4 of the four 8-byte rows addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12.
__device__ __forceinline__ bf16x4 lds_read_tr16(unsigned addr) {
  return __builtin_bit_cast(bf16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(size_t)(addr)));
}

// The four lanes l, l^16, l^32, l^48 hold the keys of one query row.
__device__ __forceinline__ float xor16(float x) {
  return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), 0x401F));
}
__device__ __forceinline__ float quad_max(float x) {
  x = fmaxf(x, xor16(x));
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float quad_sum(float x) {
  x += xor16(x);
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Waits for the DMAs.  They must be opaque asm: the DMAs themselves are opaque
// to the compiler, which would drop a builtin s_waitcnt it believes redundant.
__device__ __forceinline__ void wait_vmcnt0() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// all but the two most recent tile DMAs (DMA_ITERS instructions each) have landed
__device__ __forceinline__ void wait_vmcnt_2tiles() {
  if (DMA_ITERS == 4) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
}

// Sequence of key tiles a workgroup walks: first the tiles of the anchor rows
// [a_lo, a_hi) of Ka / Va (n_a of them), then the tiles of rows [loc_lo, loc_hi)
// of Kl / Vl.  All four are bases of one (batch, KV head); consecutive key rows
// are a_stride / l_stride bytes apart (ROWB in a head-major cache, Hkv * ROWB in
// a token-major input tensor).
struct TileSeq {
  int n_a;
  int n_tiles;
  int a_lo;
  int a_hi;
  int loc_lo;
  int loc_hi;
  const char* Ka;
  const char* Va;
  const char* Kl;
  const char* Vl;
  int a_stride;
  int l_stride;
  __device__ __forceinline__ int stride(int idx) const { return idx < n_a ? a_stride : l_stride; }
  __device__ __forceinline__ void tile(int idx, int* key0, int* hi) const {
    if (idx < n_a) { *key0 = a_lo + idx * TKEYS; *hi = a_hi; }
    else { *key0 = loc_lo + (idx - n_a) * TKEYS; *hi = loc_hi; }
  }
  __device__ __forceinline__ const char* kbase(int idx) const { return idx < n_a ? Ka : Kl; }
  __device__ __forceinline__ const char* vbase(int idx) const { return idx < n_a ? Va : Vl; }
};

// A wavefront's state.  Lane (col = lane % 16, j4 = lane / 16) belongs to query
// row `col` of each of the wavefront's RB 16-row blocks.
struct WaveState {
  bf16x8 q[RB][4];    // Q^T fragments: q[rb][t] = Q[row col of block rb][32 j4 + 8t .. +7]
  f32x4 o[RB][8];     // O^T accumulators: o[rb][dt][v] = O[row][16 dt + 4 j4 + v]
  float m[RB];        // reference maximum of the raw logits (uniform over a row's four lanes)
  float neg_mc[RB];   // -m * c (0 while m == -inf)
  float l[RB];        // this lane's share of the running sum of 2^((s-m) c)
  float lmax;         // fast loop: largest row sum of the wavefront's rows (safe-range check)
  f32x4 lacc[RB];     // fast loop: row sums accumulated by MFMA; row 0 of ones * P^T, i.e.
                      // element 0 of the lanes with j4 == 0 holds the sum of the lane's row
  bf16x8 ones;        // that MFMA's A operand: row 0 all ones, the other rows zero
};

// Per-lane LDS addresses and DMA offsets, fixed for the whole kernel.
struct LaneAddr {
  unsigned k[4];       // K operand: row col, chunk 4 j4 + t (swizzled)
  unsigned v[8];       // V^T operand: see lane_addr()
  unsigned dma;        // byte offset of this thread's 16-byte unit inside its key row
  int tid;
  int j4;
  bool upper;          // wave-uniform: the second of the two wavefronts that share a SIMD
};

// Issue the DMA of one 64-key tile of K or V into an LDS tile buffer.  Thread
// `tid` moves the 16-byte unit (row it*DMA_ROWS + tid/16, slot tid%16) for each it;
// rows at or past `hi` re-read the last valid row (they are masked in the score
// tile, and finite values keep 0 * V finite).
__device__ __forceinline__ void issue_tile(const char* base, int stride, int key0, int hi,
                                           unsigned lds, const LaneAddr& la) {
  unsigned wave_base = __builtin_amdgcn_readfirstlane((la.tid & ~63) * 16);
  if (key0 + TKEYS <= hi) {            // full tile: scalar base, loop-invariant lane offsets
    const char* sb = base + (size_t)key0 * stride;
    const unsigned voff = (unsigned)(la.tid >> 4) * stride + la.dma;
#pragma unroll
    for (int it = 0; it < DMA_ITERS; ++it)
      dma16(sb + (size_t)(it * DMA_ROWS) * stride, voff, lds + it * DMA_ROWS * ROWB + wave_base);
  } else {                             // ragged tile: clamp each lane's row below hi
    const char* sb = base + (size_t)key0 * stride;
#pragma unroll
    for (int it = 0; it < DMA_ITERS; ++it) {
      int row = it * DMA_ROWS + (la.tid >> 4);
      row = key0 + row < hi ? row : hi - 1 - key0;
      dma16(sb, (unsigned)row * (unsigned)stride + la.dma, lds + it * DMA_ROWS * ROWB + wave_base);
    }
  }
}

// A 32-key score unit of one row block: s[kt][v] is key 16 kt + 4 j4 + v.
struct Scores {
  f32x4 s[2];
};

// The fast key loop keeps ONE reference maximum per row, taken from the row's
// first 32 keys, and never rescales: p = 2^(s c - m c) against any fixed m gives
// the same O / l.  It only has to stay finite, so the row sums are checked when
// the loop ends and, if one exceeds this limit (a score more than ~40 nats above
// the reference), the workgroup redoes its rows with the exact online softmax
// (SAFE mode), which searches the maximum of every unit.
constexpr float LSUM_LIMIT = 1.152921504606846976e18f;   // 2^60

__device__ __forceinline__ float unit_max(const Scores& x) {
  float t0 = fmaxf(fmaxf(x.s[0][0], x.s[0][1]), fmaxf(x.s[0][2], x.s[0][3]));
  float t1 = fmaxf(fmaxf(x.s[1][0], x.s[1][1]), fmaxf(x.s[1][2], x.s[1][3]));
  return quad_max(fmaxf(t0, t1));
}

// Softmax numerators of one 32-key score unit against a reference maximum:
// p = 2^(s c - m c) rounded to bf16, and the lane's sum of the ROUNDED values
// (v_dot2 with a vector of ones), so numerator and denominator see the same
// rounding.  Slot 4 kt + v of p is key 16 kt + 4 j4 + v.
__device__ __forceinline__ float softmax_unit(const Scores& x, float neg_mc, bf16x8& p, float c) {
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  float lsum = 0.f;
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int v = 0; v < 4; v += 2) {
      bf16x2 pr;
      pr[0] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(x.s[kt][v], c, neg_mc));
      pr[1] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(x.s[kt][v + 1], c, neg_mc));
      p[4 * kt + v] = pr[0];
      p[4 * kt + v + 1] = pr[1];
      lsum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, lsum, false);
    }
  return lsum;
}

// The same numerators without the row sum (the fast loop sums them with an MFMA).
__device__ __forceinline__ void softmax_unit_p(const Scores& x, float neg_mc, bf16x8& p, float c) {
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int v = 0; v < 4; ++v)
      p[4 * kt + v] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(x.s[kt][v], c, neg_mc));
}

// Raise the reference of row block rb to the maximum seen so far; returns the
// factor alpha = 2^((m_old - m_new) c) for everything accumulated before (0 while
// nothing was visible yet, 1 if the maximum did not move).
__device__ __forceinline__ float raise_reference(WaveState& w, int rb, const Scores& x, float c) {
  float m_new = fmaxf(w.m[rb], unit_max(x));
  float mm = m_new == -INFINITY ? 0.f : m_new;
  float alpha = __builtin_amdgcn_exp2f((w.m[rb] - mm) * c);
  w.m[rb] = m_new;
  w.neg_mc[rb] = mm * -c;
  return alpha;
}

__device__ __forceinline__ void rescale(WaveState& w, const float (&alpha)[RB]) {
  bool moved = false;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) moved |= alpha[rb] != 1.0f;
  if (__builtin_amdgcn_ballot_w64(moved) != 0) {   // some row maximum moved
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) w.o[rb][dt] *= alpha[rb];
  }
}

// Causal / range-end mask of one 32-key score unit: element (kt, v) is key
// key0 + 16 kt + 4 j4 + v and is visible iff it is below `lim`.
__device__ __forceinline__ void mask_unit(Scores& x, int key0, int lim, int j4) {
  int y = lim - key0 - 4 * j4;
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int v = 0; v < 4; ++v) x.s[kt][v] = (16 * kt + v) < y ? x.s[kt][v] : -INFINITY;
}

// Mask the score units [key0, key0 + 32) where some row of the wavefront cannot
// see all of it (wave_lo = smallest causal bound in the wave).  Anchor keys are
// visible to every active row whatever their row numbers in the anchor buffer
// are: only the range end and inactive rows (row_lim == 0) mask them.
__device__ __forceinline__ void mask_if_needed(Scores (&s)[RB], int key0, int hi, int wave_lo,
                                               const int (&row_lim)[RB], int j4, bool anchor) {
  if (anchor) wave_lo = 0x7fffffff;
  if (key0 + 32 > wave_lo || key0 + 32 > hi) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      int lim = anchor ? (row_lim[rb] > 0 ? hi : 0) : (row_lim[rb] < hi ? row_lim[rb] : hi);
      mask_unit(s[rb], key0, lim, j4);
    }
  }
}

// PRE_IN: the first two K and V^T fragments were already read by the previous
// stage and arrive in `pre`; PRE_OUT: this stage reads the first two fragment
// pairs of the next stage (LDS offsets NKOFF / NVOFF) into `pre` behind its last
// MFMAs, so that the next stage starts without waiting for LDS.
struct PreFrag {
  bf16x8 k[2], v[2];
};

// K fragment i = 4 kt + t of a 32-key unit: keys 16 kt .. +15, MFMA step t.
__device__ __forceinline__ bf16x8 read_k(const LaneAddr& la, int i, int off) {
  return lds_read_b128(la.k[i & 3] + off + (i >> 2) * 16 * ROWB);
}
// The j-th K fragment a stage reads and uses: step t of both 16-key halves before
// step t + 1, so that four consecutive score MFMAs take their Q^T operands from
// the same two registers.
__device__ __forceinline__ constexpr int k_order(int j) { return (j & 1) * 4 + (j >> 1); }
// V^T fragment dt of a 32-key unit: d 16 dt .. +15; slot e of lane group j4 is key
// 4 j4 + e (e < 4) or 16 + 4 j4 + e - 4, matching the slots of p: two transposing
// reads, 16 key rows apart.
__device__ __forceinline__ bf16x8 read_v(const LaneAddr& la, int dt, int off) {
  bf16x4 lo = lds_read_tr16(la.v[dt] + off);
  bf16x4 hi = lds_read_tr16(la.v[dt] + off + 16 * ROWB);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// One pipeline stage holds three independent pieces of work:
//   QK  : s_next  = K[unit u+1] Q^T          (8 RB MFMAs, K fragments from LDS at KOFF)
//   SM  : p_cur   = softmax numerators of s_cur (unit u)  (SAFE: also w.l, w.m)
//   PV  : O^T    += V[unit u-1]^T p_prev      (8 RB MFMAs, V^T fragments from LDS at VOFF;
//                  fast loop: RB more for the row sums)
// so that the MFMAs of two units hide the exponentials of the third.  The
// sched_group_barrier sequence at the end pins the instruction order inside the
// stage: operand fragments are read from LDS two fragment pairs ahead of their
// use and a few VALU instructions sit between consecutive MFMAs.  `alpha`
// receives the rescale factors for the accumulators (SAFE mode; 1 otherwise), to
// be applied after the stage, i.e. after the PV MFMAs of unit u-1 and before
// those of unit u.
template <bool SAFE, bool QK, bool SM, bool PV, int KOFF, int VOFF, bool PRE_IN = false,
          bool PRE_OUT = false, int NKOFF = 0, int NVOFF = 0>
__device__ __forceinline__ void stage(WaveState& w, const LaneAddr& la, Scores (&s_next)[RB],
                                      Scores (&s_cur)[RB], bf16x8 (&p_cur)[RB],
                                      const bf16x8 (&p_prev)[RB], float c, float (&alpha)[RB],
                                      PreFrag& pre) {
  bf16x8 kf[8], vf[8];
  // Keep this stage's softmax inside the stage: without the anchors the optimizer
  // hoists it above the preceding barrier and sinks the row sums to the loop end.
  if (SM) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) asm volatile("" : "+v"(s_cur[rb].s[0]), "+v"(s_cur[rb].s[1]));
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (PRE_IN && i < 2) {
      kf[i] = pre.k[i];
      vf[i] = pre.v[i];
      continue;
    }
    if (QK) kf[i] = read_k(la, k_order(i), KOFF);
    if (PV) vf[i] = read_v(la, i, VOFF);
  }
  if (PRE_OUT) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      pre.k[i] = read_k(la, k_order(i), NKOFF);
      pre.v[i] = read_v(la, i, NVOFF);
    }
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    alpha[rb] = 1.0f;
    if (SM) {
      if (SAFE) {
        alpha[rb] = raise_reference(w, rb, s_cur[rb], c);
        w.l[rb] = __builtin_fmaf(w.l[rb], alpha[rb], softmax_unit(s_cur[rb], w.neg_mc[rb], p_cur[rb], c));
      } else {
        softmax_unit_p(s_cur[rb], w.neg_mc[rb], p_cur[rb], c);
      }
    }
  }
  // MFMA order: four score MFMAs (two K fragments x two row blocks), then four PV
  // MFMAs (two V^T fragments x two row blocks, the row blocks of the second in
  // reverse).  Runs of MFMAs that read few distinct operand registers draw less
  // power, and the power limit is what bounds this loop: measured 1.3-1.5 %
  // faster than alternating pairs of score and PV MFMAs in fragment order.
#pragma unroll
  for (int j2 = 0; j2 < 8; j2 += 2) {
    if (QK) {
#pragma unroll
      for (int j = j2; j < j2 + 2; ++j) {
        const int i = k_order(j);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          // the first d-chunk of a 16-key sub-unit starts from zero (an inline constant)
          const f32x4 acc = (i & 3) == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : s_next[rb].s[i >> 2];
          s_next[rb].s[i >> 2] =
              __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[j], w.q[rb][i & 3], acc, 0, 0, 0);
        }
      }
    }
    if (PV) {
#pragma unroll
      for (int i = j2; i < j2 + 2; ++i) {
#pragma unroll
        for (int r = 0; r < RB; ++r) {
          const int rb = (i & 1) ? RB - 1 - r : r;
          w.o[rb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[i], p_prev[rb], w.o[rb][i], 0, 0, 0);
        }
      }
    }
  }
  if (PV && !SAFE) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      w.lacc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w.ones, p_prev[rb], w.lacc[rb], 0, 0, 0);
  }
  if (QK && SM && PV) {
    if (!PRE_IN) __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, SAFE ? 3 : 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, SAFE ? 3 : 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, SAFE ? 3 : 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < 6 || PRE_OUT) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, SAFE ? 3 : 2, 0);
    }
    if (!SAFE) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
  }
  if (SM) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      if (SAFE) asm volatile("" : "+v"(w.l[rb]), "+v"(p_cur[rb]));
      else asm volatile("" : "+v"(p_cur[rb]));
    }
  }
  __builtin_amdgcn_sched_barrier(0);
}

// Everything a wavefront does for key tile t once tile t's scores exist:
//   barrier (K tile t+1 and V tile t have landed; older buffers are free),
//   DMA of K tile t+2 and V tile t+1 into the buffers just released,
//   stage A: scores of unit 2t+2 | softmax of unit 2t+1 | PV of unit 2t,
//   stage B: scores of unit 2t+3 | softmax of unit 2t+2 | PV of unit 2t+1.
// MORE = tile t+1 exists.  KN / VC are the LDS offsets of K tile t+1 and V tile t,
// KF / VF those of the buffers that are refilled (K tile t+2, V tile t+1).
struct LoopRegs {
  Scores sA[RB], sB[RB];      // score units of the even / odd 32-key unit
  bf16x8 pA[RB], pB[RB];      // their exponentials (bf16)
};

template <bool SAFE, bool MORE, int KN, int VC, int KF, int VF>
__device__ __forceinline__ void tile_step(WaveState& w, const LaneAddr& la, const TileSeq& seq,
                                          int t, const int (&row_lim)[RB], int wave_lo, float c,
                                          unsigned lds0, LoopRegs& r) {
  constexpr int H = 32 * ROWB;
  float alpha[RB];
  PreFrag pre;
  wait_vmcnt0();
  __builtin_amdgcn_s_barrier();
  if (t + 2 < seq.n_tiles) {
    int k2, h2;
    seq.tile(t + 2, &k2, &h2);
    issue_tile(seq.kbase(t + 2), seq.stride(t + 2), k2, h2, lds0 + KF, la);
  }
  if (MORE) {
    int nk0, nhi;
    seq.tile(t + 1, &nk0, &nhi);
    issue_tile(seq.vbase(t + 1), seq.stride(t + 1), nk0, nhi, lds0 + VF, la);
    // one wave-uniform test per tile: does any of its keys need a mask for this wavefront?
    const bool anchor_tile = t + 1 < seq.n_a;
    const int mask_from = anchor_tile ? nhi : (wave_lo < nhi ? wave_lo : nhi);
    const bool need_mask = nk0 + TKEYS > mask_from;
    // The two wavefronts of a SIMD take turns at the higher issue priority, one
    // stage each.  With equal priorities the arbiter keeps favouring the same one,
    // which then reaches the tile barrier some 1100 cycles before its neighbour
    // (541 cycles of barrier wait per wavefront and tile on average); taking turns
    // brings both there together (218 cycles).
    if (la.upper) __builtin_amdgcn_s_setprio(1); else __builtin_amdgcn_s_setprio(0);
    stage<SAFE, true, true, true, KN, VC, false, true, KN + H, VC + H>(w, la, r.sA, r.sB, r.pB, r.pA,
                                                                       c, alpha, pre);
    if (la.upper) __builtin_amdgcn_s_setprio(0); else __builtin_amdgcn_s_setprio(1);
    if (SAFE) rescale(w, alpha);
    if (need_mask) mask_if_needed(r.sA, nk0, nhi, wave_lo, row_lim, la.j4, anchor_tile);
    stage<SAFE, true, true, true, KN + H, VC + H, true>(w, la, r.sB, r.sA, r.pA, r.pB, c, alpha, pre);
    if (SAFE) rescale(w, alpha);
    if (need_mask) mask_if_needed(r.sB, nk0 + 32, nhi, wave_lo, row_lim, la.j4, anchor_tile);
  } else {
    stage<SAFE, false, true, true, 0, VC>(w, la, r.sA, r.sB, r.pB, r.pA, c, alpha, pre);
    if (SAFE) rescale(w, alpha);
    stage<SAFE, false, false, true, 0, VC + H>(w, la, r.sB, r.sA, r.pA, r.pB, c, alpha, pre);
  }
}

// Walk a tile sequence once for the calling wavefront (all wavefronts of
// the workgroup call this with the same sequence).
//   row_lim     this lane's exclusive causal key bound per row block (0 = inactive row)
//   wave_lo     smallest row_lim among the wavefront's active rows: key tiles that
//               end at or below it need no causal mask
template <bool SAFE>
__device__ __forceinline__ void key_loop(WaveState& w, const LaneAddr& la, const TileSeq& seq,
                                         const int (&row_lim)[RB], int wave_lo, float c,
                                         unsigned lds0) {
  const int T = seq.n_tiles;
  constexpr int K0 = LDS_K0, K1 = LDS_K1, V0 = LDS_V0, V1 = LDS_V1, H = 32 * ROWB;
  LoopRegs r;
  float alpha[RB];
  PreFrag pre;
  int key0, hi;

  // Prologue: K tile 0, V tile 0 and K tile 1 in flight; scores of tile 0.
  seq.tile(0, &key0, &hi);
  issue_tile(seq.kbase(0), seq.stride(0), key0, hi, lds0 + K0, la);
  issue_tile(seq.vbase(0), seq.stride(0), key0, hi, lds0 + V0, la);
  if (T > 1) {
    int k1, h1;
    seq.tile(1, &k1, &h1);
    issue_tile(seq.kbase(1), seq.stride(1), k1, h1, lds0 + K1, la);
    wait_vmcnt_2tiles();
  } else {
    wait_vmcnt0();
  }
  __builtin_amdgcn_s_barrier();
  stage<SAFE, true, false, false, K0, 0>(w, la, r.sA, r.sA, r.pA, r.pA, c, alpha, pre);
  mask_if_needed(r.sA, key0, hi, wave_lo, row_lim, la.j4, seq.n_a > 0);
  stage<SAFE, true, false, false, K0 + H, 0>(w, la, r.sB, r.sA, r.pA, r.pA, c, alpha, pre);
  mask_if_needed(r.sB, key0 + 32, hi, wave_lo, row_lim, la.j4, seq.n_a > 0);
  // first unit: its row maximum becomes the reference (nothing to rescale yet)
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    raise_reference(w, rb, r.sA[rb], c);
    if (SAFE) w.l[rb] = softmax_unit(r.sA[rb], w.neg_mc[rb], r.pA[rb], c);
    else softmax_unit_p(r.sA[rb], w.neg_mc[rb], r.pA[rb], c);
  }

  // Tile t: V tile t is consumed while K tile t+1 produces the next scores.
  // The loop is unrolled by two so that every LDS buffer offset is an immediate
  // and the accumulators flow through straight-line code.
  int t = 0;
  for (; t + 2 < T; t += 2) {
    tile_step<SAFE, true, K1, V0, K0, V1>(w, la, seq, t, row_lim, wave_lo, c, lds0, r);
    tile_step<SAFE, true, K0, V1, K1, V0>(w, la, seq, t + 1, row_lim, wave_lo, c, lds0, r);
  }
  if (T - t == 2) {
    tile_step<SAFE, true, K1, V0, K0, V1>(w, la, seq, t, row_lim, wave_lo, c, lds0, r);
    tile_step<SAFE, false, K0, V1, K1, V0>(w, la, seq, t + 1, row_lim, wave_lo, c, lds0, r);
  } else {
    tile_step<SAFE, false, K1, V0, K0, V1>(w, la, seq, t, row_lim, wave_lo, c, lds0, r);
  }
  __builtin_amdgcn_s_setprio(0);
}

__device__ __forceinline__ void reset_state(WaveState& w) {
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) w.o[rb][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    w.m[rb] = -INFINITY;
    w.neg_mc[rb] = 0.f;
    w.l[rb] = 0.f;
    w.lacc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  w.lmax = 0.f;
}

// LDS addresses of the calling lane.
__device__ __forceinline__ LaneAddr lane_addr(unsigned lds0) {
  LaneAddr la;
  la.tid = threadIdx.x;
  const int lane = la.tid & 63;
  const int col = lane & 15;
  la.j4 = lane >> 4;
  // eight wavefronts on four SIMDs: wavefronts w and w + 4 share one
  la.upper = __builtin_amdgcn_readfirstlane((la.tid >> 8) & 1) != 0;
  // K operand: in MFMA step t, lane (col, j4) reads row col, chunk 4 j4 + t (any
  // assignment of d-chunks to (t, j4) works as long as Q uses the same one; this
  // one keeps the 16-byte reads of a wavefront free of LDS bank conflicts, the
  // transposed one, 4t + j4, does not)
#pragma unroll
  for (int t = 0; t < 4; ++t) la.k[t] = lds0 + col * ROWB + (((4 * la.j4 + t) ^ swz(col)) << 4);
  // V^T operand: source lane addresses row 4 j4 + col/4 (+16 for the second
  // read), columns 16 dt + 4 (lane % 4) .. +3
  const int rr = 4 * la.j4 + (col >> 2);
#pragma unroll
  for (int dt = 0; dt < 8; ++dt)
    la.v[dt] = lds0 + rr * ROWB + (((2 * dt + ((lane & 3) >> 1)) ^ swz(rr)) << 4) + 8 * (lane & 1);
  la.dma = ((la.tid & 15) ^ swz(la.tid >> 4)) << 4;
  return la;
}

// Attention of the workgroup's rows over a tile sequence: the fast loop, and the
// exact loop again if any wavefront's scores left the fast loop's safe range.
__device__ __forceinline__ void attend(WaveState& w, const TileSeq& seq, const int (&row_lim)[RB],
                                       int wave_lo, float c, unsigned lds0) {
  const LaneAddr la = lane_addr(lds0);
  if (seq.n_tiles == 0) return;
  // Consume the Q fragments here so that the compiler places its own wait for
  // their loads before the first DMA is in flight (and none inside the loops).
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int t = 0; t < 4; ++t) asm volatile("" : "+v"(w.q[rb][t]));
  {
    const __bf16 o = (la.tid & 15) == 0 ? (__bf16)1.0f : (__bf16)0.0f;
    w.ones = bf16x8{o, o, o, o, o, o, o, o};
  }
  key_loop<false>(w, la, seq, row_lim, wave_lo, c, lds0);
  // row 0 of the ones-row product sits in element 0 of the lanes with j4 == 0: the row's whole sum
  // (quad_sum over the row's four lanes then finds it once); sums that left the safe range show here
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    w.l[rb] = la.j4 == 0 ? w.lacc[rb][0] : 0.f;
    w.lmax = fmaxf(w.lmax, w.l[rb]);
  }

  // Did any row of any wavefront leave the safe range?  One LDS word per
  // wavefront; __syncthreads() (fence + barrier) orders the tile reads before the
  // flag writes, the writes before the reads, and the reads before any new DMA.
  __syncthreads();
  const bool bad = __builtin_amdgcn_ballot_w64(!(w.lmax < LSUM_LIMIT)) != 0;
  LDS_AS int* flags = (LDS_AS int*)(size_t)lds0;
  if ((la.tid & 63) == 0) flags[la.tid >> 6] = bad ? 1 : 0;
  __syncthreads();
  int any_bad = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) any_bad |= flags[i];
  __syncthreads();
  if (__builtin_expect(any_bad != 0, 0)) {
    reset_state(w);
    key_loop<true>(w, la, seq, row_lim, wave_lo, c, lds0);
  }
}

__device__ __forceinline__ void load_q(WaveState& w, int rb, const char* qrow, int j4) {
#pragma unroll
  for (int t = 0; t < 4; ++t) w.q[rb][t] = *(const bf16x8*)(qrow + (32 * j4 + 8 * t) * 2);
}

// Row block g of a workgroup (g = wave * RB + rb, WG_BLOCKS of them, 16 rows each)
// is head g % hpw of the workgroup's head group and token block g / hpw: the
// heads of a KV group come first, so that a wavefront's row blocks share their
// tokens (and their causal frontier) whenever the group has at least RB heads.

// ------------------------------------------------------------------ phase 1
// Work items are numbered (kv head fastest, then the rest; see launch_phase1_bf16)
// and dealt to eight queues, item v to queue v % 8 -- the XCD that workgroup v of
// a plain launch would run on, so that with Hkv a multiple of 8 an XCD's L2 serves
// one KV head.  The kernel is launched with one workgroup per CU; each takes the
// next item of its XCD's queue until that is empty, then of the other queues: the
// XCDs of one chip differ by a few per cent in clock under the power limit, and
// with a fixed share each the launch would last as long as the slowest needs.
// The eight counters belong to the launch (the caller's workspace, or a set of
// the library's own that no launch in flight holds); a one-workgroup kernel in
// front of the launch clears them.
__global__ void phase1_tickets_reset_kernel(unsigned int* tickets) {
  if (threadIdx.x < 8) tickets[threadIdx.x] = 0u;
}

// Next item for a workgroup whose own queue is `home`, or -1 when all are taken.
__device__ __forceinline__ int next_item(unsigned int* tickets, int home, unsigned n_items) {
  for (int k = 0; k < 8; ++k) {
    const unsigned q = (unsigned)(home + k) & 7u;
    const unsigned cnt = q < n_items ? (n_items - q + 7u) / 8u : 0u;   // items 8 t + q < n_items
    if (cnt == 0u) continue;
    const unsigned t = atomicAdd(&tickets[q], 1u);
    if (t < cnt) return (int)(8u * t + q);
  }
  return -1;
}

__device__ __forceinline__ void phase1_item(const Phase1Args& a, int hpw, int tpb, int n_hs, int id,
                                            char* lds) {
  const Geom& g = a.g;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int col = lane & 15, j4 = lane >> 4;
  const int tm = 16 * (WG_BLOCKS / hpw);         // tokens per workgroup

  // item decode: kv head fastest, then batch, head sub-group, tile within block
  // (late = heavy first), block (block 0, the lightest, last)
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
  int wg_last = row0 + tm < e ? row0 + tm : e;   // exclusive bound of the workgroup's tokens

  // K / V rows of this (batch, KV head): from the token-major inputs when the
  // call hands them over as they are (then this kernel also files them in the
  // cache), else from the head-major caches a preceding kernel has filled
  const bool from_input = a.Kin != nullptr;
  const int kv_stride = from_input ? g.Hkv * ROWB : ROWB;
  const char* Kb = from_input
      ? (const char*)a.Kin + ((size_t)beta * g.L * g.Hkv + kvh) * ROWB
      : (const char*)a.Kc + ((size_t)beta * g.Hkv + kvh) * (size_t)g.cap * ROWB;
  const char* Vb = from_input
      ? (const char*)a.Vin + ((size_t)beta * g.L * g.Hkv + kvh) * ROWB
      : (const char*)a.Vc + ((size_t)beta * g.Hkv + kvh) * (size_t)g.cap * ROWB;
  WaveState w;
  int head[RB], tok[RB], row_lim[RB];
  bool active[RB];
  int wave_lo = 0x7fffffff;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    int gb = wave * RB + rb;
    head[rb] = kvh * g.G + hs * hpw + gb % hpw;
    int tok0 = row0 + 16 * (gb / hpw);
    tok[rb] = tok0 + col;
    active[rb] = tok[rb] < e;
    int qtok = active[rb] ? tok[rb] : (tok0 < e ? tok0 : e - 1);
    load_q(w, rb, (const char*)a.Q + (((size_t)beta * g.L + qtok) * g.Hq + head[rb]) * ROWB, j4);
    // a row sees key k iff k < tok + 1; anchor keys always qualify (they precede
    // the block or sit in their own buffer)
    row_lim[rb] = active[rb] ? tok[rb] + 1 : 0;
    int lo = tok0 < e ? tok0 + 1 : 0;
    wave_lo = lo < wave_lo ? lo : wave_lo;
  }
  wave_lo = __builtin_amdgcn_readfirstlane(wave_lo);   // wave-uniform
  reset_state(w);

  // anchor rows (all visible: they precede the block or sit in their own
  // buffer), then the block's own rows up to the workgroup's last token
  TileSeq seq;
  int64_t a_lo, a_hi;
  const bool ext = anchor_range(g, a.anchor_mode, i, &a_lo, &a_hi);
  seq.a_lo = (int)a_lo;
  seq.a_hi = (int)a_hi;
  // external anchors: token-major, n_anchor * a rows per batch
  const size_t anchor_rows = (size_t)(a.anchor_mode == ANCHOR_PER_BLOCK ? n : 1) * g.a;
  seq.Ka = ext ? (const char*)a.Ka + ((size_t)beta * anchor_rows * g.Hkv + kvh) * ROWB : Kb;
  seq.Va = ext ? (const char*)a.Va + ((size_t)beta * anchor_rows * g.Hkv + kvh) * ROWB : Vb;
  seq.Kl = Kb;
  seq.Vl = Vb;
  seq.l_stride = kv_stride;
  seq.a_stride = ext ? g.Hkv * ROWB : kv_stride;
  seq.n_a = (seq.a_hi - seq.a_lo + TKEYS - 1) / TKEYS;
  seq.loc_lo = s;
  seq.loc_hi = wg_last;
  seq.n_tiles = seq.n_a + (wg_last - s + TKEYS - 1) / TKEYS;

  unsigned lds0 = (unsigned)(size_t)(LDS_AS char*)lds;
  attend(w, seq, row_lim, wave_lo, g.scale * LOG2E, lds0);

#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float l_tot = quad_sum(w.l[rb]);
    if (active[rb]) {
      float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
      char* orow = (char*)a.O + (((size_t)beta * g.L + tok[rb]) * g.Hq + head[rb]) * ROWB;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        bf16x4 v;
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = (__bf16)(w.o[rb][dt][k] * inv);
        *(bf16x4*)(orow + (16 * dt + 4 * j4) * 2) = v;
      }
      if (a.LSE && j4 == 0)
        a.LSE[((size_t)beta * g.Hq + head[rb]) * g.L + tok[rb]] =
            l_tot > 0.f ? (w.m[rb] * g.scale * LOG2E + __builtin_amdgcn_logf(l_tot)) * LN2 : -INFINITY;
    }
  }

  // Algorithm 1, "keep the block's K/V": the workgroup files the K and V rows of
  // its own tokens in the head-major caches (they were among the last tiles it
  // streamed, so these reads hit in L2).  One head sub-group per token range does it.
  if (from_input && hs == 0) {
    const int n_units = (wg_last - row0) * 16;            // 16-byte units per tensor
    char* kc = (char*)a.Kc + (((size_t)beta * g.Hkv + kvh) * (size_t)g.cap + row0) * ROWB;
    char* vc = (char*)a.Vc + (((size_t)beta * g.Hkv + kvh) * (size_t)g.cap + row0) * ROWB;
    // two units per thread and pass, all four loads before the stores: one round trip
    for (int u = tid; u < n_units; u += 2 * NT) {
      const int u2 = u + NT;
      const bool two = u2 < n_units;
      const size_t s1 = (size_t)(row0 + (u >> 4)) * kv_stride + (u & 15) * 16;
      const size_t s2 = two ? (size_t)(row0 + (u2 >> 4)) * kv_stride + (u2 & 15) * 16 : s1;
      const i32x4 k1 = *(const i32x4*)(Kb + s1), v1 = *(const i32x4*)(Vb + s1);
      const i32x4 k2 = *(const i32x4*)(Kb + s2), v2 = *(const i32x4*)(Vb + s2);
      *(i32x4*)(kc + (size_t)u * 16) = k1;
      *(i32x4*)(vc + (size_t)u * 16) = v1;
      if (two) {
        *(i32x4*)(kc + (size_t)u2 * 16) = k2;
        *(i32x4*)(vc + (size_t)u2 * 16) = v2;
      }
    }
  }
}

__global__ __launch_bounds__(NT, NW == 4 ? 2 : 1) void phase1_bf16_kernel(Phase1Args a, int hpw,
                                                                          int tpb, int n_hs,
                                                                          unsigned n_items) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  __shared__ int item;
  for (;;) {
    if (threadIdx.x == 0) item = next_item(a.tickets, blockIdx.x & 7, n_items);
    __syncthreads();
    const int id = item;
    __syncthreads();                 // everyone holds it before the next round overwrites it
    if (id < 0) return;              // every queue is empty: uniform over the workgroup
    phase1_item(a, hpw, tpb, n_hs, id, lds);
    __syncthreads();                 // the item's LDS reads are done before the next item's DMAs
  }
}

// ------------------------------------------------------------------ phase 2
// Local attention (Eq. 1) and log-sum-exp (log of Eq. 2) of a row tile over one
// split of the cache.  grid.x = ((batch * s_total + split) * n_hs + hs) * row_tiles + tile,
// grid.y = kv head.
__global__ __launch_bounds__(NT, NW == 4 ? 2 : 1) void phase2_rows_bf16_kernel(Phase2Args a, int hpw,
                                                                               int n_hs,
                                                                               int row_tiles) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const Geom& g = a.g;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int col = lane & 15, j4 = lane >> 4;
  const int tm = 16 * (WG_BLOCKS / hpw);

  int id = blockIdx.x;
  int tt = id % row_tiles; id /= row_tiles;
  int hs = id % n_hs; id /= n_hs;
  int sp = id % a.plan.s_total;
  int beta = id / a.plan.s_total;
  int kvh = blockIdx.y;

  int total = (int)visible_total(a);
  int64_t lo64, hi64;
  split_range(a.plan, g.L, g.b, total, sp, &lo64, &hi64);
  int lo = (int)lo64, hi = (int)hi64;

  const char* Kb = (const char*)a.Kc + ((size_t)beta * g.Hkv + kvh) * (size_t)g.cap * ROWB;
  const char* Vb = (const char*)a.Vc + ((size_t)beta * g.Hkv + kvh) * (size_t)g.cap * ROWB;
  WaveState w;
  int head[RB], jrow[RB], row_lim[RB];
  bool active[RB];
  int wave_lo = 0x7fffffff;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    int gb = wave * RB + rb;
    head[rb] = kvh * g.G + hs * hpw + gb % hpw;
    int j0 = tt * tm + 16 * (gb / hpw);
    jrow[rb] = j0 + col;
    active[rb] = jrow[rb] < a.q_len;
    int qj = active[rb] ? jrow[rb] : (j0 < a.q_len ? j0 : a.q_len - 1);
    load_q(w, rb, (const char*)a.Qq + (((size_t)beta * a.q_len + qj) * g.Hq + head[rb]) * ROWB, j4);
    row_lim[rb] = active[rb] ? (int)visible_limit(a, jrow[rb]) : 0;
    int l0 = j0 < a.q_len ? (int)visible_limit(a, j0) : 0;
    wave_lo = l0 < wave_lo ? l0 : wave_lo;
  }
  wave_lo = __builtin_amdgcn_readfirstlane(wave_lo);   // wave-uniform
  reset_state(w);

  TileSeq seq;
  seq.a_lo = 0; seq.a_hi = 0; seq.n_a = 0; seq.loc_lo = lo; seq.loc_hi = hi;
  seq.Ka = Kb; seq.Va = Vb; seq.Kl = Kb; seq.Vl = Vb;
  seq.a_stride = ROWB; seq.l_stride = ROWB;
  seq.n_tiles = hi > lo ? (hi - lo + TKEYS - 1) / TKEYS : 0;

  unsigned lds0 = (unsigned)(size_t)(LDS_AS char*)lds;
  attend(w, seq, row_lim, wave_lo, g.scale * LOG2E, lds0);

#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float l_tot = quad_sum(w.l[rb]);
    if (active[rb]) {
      float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
      size_t r = (((size_t)beta * a.plan.s_total + sp) * g.Hq + head[rb]) * a.q_len + jrow[rb];
      float* orow = a.O_sub + r * D;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) *(f32x4*)(orow + 16 * dt + 4 * j4) = w.o[rb][dt] * inv;
      if (j4 == 0)
        a.LSE_sub[r] = l_tot > 0.f ? (w.m[rb] * g.scale * LOG2E + __builtin_amdgcn_logf(l_tot)) * LN2
                                   : -INFINITY;
    }
  }
}

}  // namespace

// Heads of one KV group that share a workgroup of the row-tiled kernels: the
// largest of 8, 4, 2, 1 that divides G; the workgroup's 16-row blocks are split
// evenly among them.
int flash_heads_per_workgroup(int G) {
  for (int h = 8; h > 1; h >>= 1)
    if (h <= WG_BLOCKS && G % h == 0) return h;
  return 1;
}
int flash_tokens_per_workgroup(int G) { return 16 * (WG_BLOCKS / flash_heads_per_workgroup(G)); }

// The kernels' 64 KiB tile ring is dynamic LDS; the runtime wants to be told
// once per kernel and device that a launch may ask for that much.
enum { ATTR_PHASE1 = 0, ATTR_PHASE2_ROWS = 1 };
static hipError_t allow_tile_ring(int which, const void* kernel) {
  static std::atomic<bool> done[2][64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev >= 0 && dev < 64 && done[which][dev].load(std::memory_order_acquire)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 4 * TILEB);
  if (e == hipSuccess && dev >= 0 && dev < 64) done[which][dev].store(true, std::memory_order_release);
  return e;
}

hipError_t launch_phase1_bf16(const Phase1Args& a, hipStream_t st) {
  const Geom& g = a.g;
  int hpw = flash_heads_per_workgroup(g.G);
  int tm = flash_tokens_per_workgroup(g.G);
  int n_hs = g.G / hpw;
  int64_t n = (g.L + g.b - 1) / g.b;
  int64_t bmax = g.b < g.L ? g.b : g.L;
  int tpb = (int)((bmax + tm - 1) / tm);
  int64_t wgs = (int64_t)g.Hkv * g.B * n_hs * tpb * n;
  if (wgs > 0x7fffffff) return hipErrorInvalidValue;
  hipError_t e = allow_tile_ring(ATTR_PHASE1, (const void*)phase1_bf16_kernel);
  if (e != hipSuccess) return e;
  // one workgroup per CU (registers and LDS admit no more), never more than items
  int n_cu = a.n_cu;
  if (n_cu <= 0 || !a.tickets) return hipErrorInvalidValue;
  if (NW == 4) n_cu *= 2;
  const unsigned resident = (unsigned)(wgs < n_cu ? wgs : n_cu);
  if (resident == 0) return hipSuccess;
  phase1_tickets_reset_kernel<<<1, 64, 0, st>>>(a.tickets);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  phase1_bf16_kernel<<<dim3(resident), NT, 4 * TILEB, st>>>(a, hpw, tpb, n_hs, (unsigned)wgs);
  return hipGetLastError();
}

hipError_t launch_phase2_rows_bf16(const Phase2Args& a, hipStream_t st) {
  const Geom& g = a.g;
  int hpw = flash_heads_per_workgroup(g.G);
  int tm = flash_tokens_per_workgroup(g.G);
  int n_hs = g.G / hpw;
  int row_tiles = (a.q_len + tm - 1) / tm;
  int64_t gx = (int64_t)g.B * a.plan.s_total * n_hs * row_tiles;
  if (gx > 0x7fffffff || g.Hkv > 65535) return hipErrorInvalidValue;
  hipError_t e = allow_tile_ring(ATTR_PHASE2_ROWS, (const void*)phase2_rows_bf16_kernel);
  if (e != hipSuccess) return e;
  phase2_rows_bf16_kernel<<<dim3((unsigned)gx, (unsigned)g.Hkv), NT, 4 * TILEB, st>>>(a, hpw, n_hs,
                                                                                      row_tiles);
  return hipGetLastError();
}

}  // namespace star
