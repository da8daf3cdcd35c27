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
//   * Softmax runs in the log2 domain in fp32; the accumulator rescale is
//     skipped (wave-uniform branch) whenever no row maximum moved in the tile.
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

// 16-byte DMA global -> LDS: lane L's data lands at lds_base + 16 * L.
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(gptr), "s"(lds_base) : "memory");
}

__device__ __forceinline__ bf16x8 lds_read_b128(unsigned addr) {
  return *(LDS_AS bf16x8*)(addr);
}

// Transposing LDS read; see the V^T fragment description in attend().
__device__ __forceinline__ s16x4 lds_read_tr16(unsigned addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(addr));
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
  float m;            // running maximum of the raw logits (pair-uniform)
  float l;            // this lane's share of the running sum of 2^((s-m) c)
};

// Issue the DMA of one K tile and one V tile.  Thread `tid` moves the 16-byte
// unit (row it*16 + tid/16, slot tid%16) for it = 0..3; rows past `hi` re-read
// the last valid row (they are masked in the score tile).
__device__ __forceinline__ void issue_tile(const char* Kb, const char* Vb, int key0, int hi,
                                           unsigned ldsK, unsigned ldsV, int tid, int chunk_off) {
  int wave_base = __builtin_amdgcn_readfirstlane((tid & ~63) * 16);
  int r0 = key0 + (tid >> 4);
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    int key = r0 + it * 16;
    key = key < hi ? key : hi - 1;
    size_t off = (size_t)key * ROWB + chunk_off;
    dma16(Kb + off, ldsK + it * 4096 + wave_base);
    dma16(Vb + off, ldsV + it * 4096 + wave_base);
  }
}

// One 64-key tile for one wavefront.
//   key0        first key of the tile
//   lim         this lane's exclusive key bound (min of the row's causal bound
//               and the range end); only used when `masked`
//   masked      wave-uniform: some element of the tile may be invisible
template <int KOFF, int VOFF>
__device__ __forceinline__ void compute_tile(WaveState& w, const unsigned (&kaddr)[8],
                                             const unsigned (&vaddr)[4][2], int key0, int lim,
                                             bool masked, float c, int half) {
  f32x16 s[2];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
    for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      bf16x8 a = lds_read_b128(kaddr[t] + KOFF + kb * 32 * ROWB);
      s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, w.q[t], s[kb], 0, 0, 0);
    }
  }
  if (masked) {
    // element v of sub-tile kb is key key0 + 32kb + 8(v/4) + 4*half + v%4
    int x = lim - key0 - 4 * half;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        s[kb][v] = (32 * kb + 8 * (v / 4) + (v % 4)) < x ? s[kb][v] : -INFINITY;
  }
  float tmax = s[0][0];
#pragma unroll
  for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, s[0][v]);
#pragma unroll
  for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, s[1][v]);
  tmax = pair_max(tmax);
  float m_new = fmaxf(w.m, tmax);
  if (__builtin_amdgcn_ballot_w64(m_new > w.m) != 0) {      // some row maximum moved
    float mm = m_new == -INFINITY ? 0.f : m_new;
    float alpha = __builtin_amdgcn_exp2f((w.m - mm) * c);   // 0 while w.m == -inf
    w.l *= alpha;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) w.o[dt][v] *= alpha;
    w.m = m_new;
  }
  float neg_mc = (w.m == -INFINITY ? 0.f : w.m) * -c;
  bf16x8 p[2][2];
  float lsum = 0.f;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][v], c, neg_mc));
      lsum += e;
      p[kb][v / 8][v % 8] = (__bf16)e;
    }
  w.l += lsum;
  // O^T[32dt.., row] += V^T P^T.  For sub-tile kb and half-sub-tile cc the B
  // operand is p[kb][cc]: slot e of lane half `half` is key
  // 32kb + 16cc + 8(e/4) + 4*half + e%4, so the A operand needs, for d-row
  // lane%32, keys k0..k0+3 and k0+8..k0+11 with k0 = 32kb + 16cc + 4*half.
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int cc = 0; cc < 2; ++cc)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        s16x4 lo = lds_read_tr16(vaddr[dt][0] + VOFF + (32 * kb + 16 * cc) * ROWB);
        s16x4 hi = lds_read_tr16(vaddr[dt][1] + VOFF + (32 * kb + 16 * cc) * ROWB);
        bf16x8 a;
        bf16x4 lo_b = __builtin_bit_cast(bf16x4, lo), hi_b = __builtin_bit_cast(bf16x4, hi);
        a = __builtin_shufflevector(lo_b, hi_b, 0, 1, 2, 3, 4, 5, 6, 7);
        w.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p[kb][cc], w.o[dt], 0, 0, 0);
      }
}

// Walk a tile sequence for the calling wavefront.
//   row_lim     this lane's exclusive causal key bound (0 for an inactive row)
//   wave_lo/hi  min / max of row_lim over the wavefront's active rows
__device__ __forceinline__ void attend(WaveState& w, const TileSeq& seq, const char* Kb,
                                       const char* Vb, int row_lim, int wave_lo, int wave_hi,
                                       float c, unsigned lds0) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int half = lane >> 5;
  const int i32 = lane & 31;
  // K operand: lane (i32, half) reads row i32 (+32 kb), chunk 2t + half
  unsigned kaddr[8];
  {
    int x = half ^ swz(i32);
#pragma unroll
    for (int t = 0; t < 8; ++t) kaddr[t] = lds0 + i32 * ROWB + (((2 * t) ^ x) << 4);
  }
  // V^T operand: source lane addresses row 4*half + (lane%16)/4 (+8 for the
  // second read), columns 32dt + 16*((lane/16)%2) + 4*(lane%4) .. +3
  unsigned vaddr[4][2];
  {
    int q4 = (lane & 15) >> 2, gi = (lane >> 4) & 1;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        int r = 4 * half + q4 + 8 * u;
        int chunk = 4 * dt + 2 * gi + ((lane & 3) >> 1);
        vaddr[dt][u] = lds0 + r * ROWB + ((chunk ^ swz(r)) << 4) + 8 * (lane & 1);
      }
  }
  const int chunk_off = ((tid & 15) ^ swz(tid >> 4)) << 4;

  if (seq.n_tiles == 0) return;
  int key0, hi;
  seq.tile(0, &key0, &hi);
  issue_tile(Kb, Vb, key0, hi, lds0 + LDS_K0, lds0 + LDS_V0, tid, chunk_off);
  for (int idx = 0; idx < seq.n_tiles; idx += 2) {
    // ---- even tile: buffers 0
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    seq.tile(idx, &key0, &hi);
    if (idx + 1 < seq.n_tiles) {
      int k1, h1;
      seq.tile(idx + 1, &k1, &h1);
      issue_tile(Kb, Vb, k1, h1, lds0 + LDS_K1, lds0 + LDS_V1, tid, chunk_off);
    }
    if (key0 < wave_hi) {
      bool masked = key0 + TKEYS > wave_lo || key0 + TKEYS > hi;
      int lim = row_lim < hi ? row_lim : hi;
      compute_tile<LDS_K0, LDS_V0>(w, kaddr, vaddr, key0, lim, masked, c, half);
    }
    if (idx + 1 >= seq.n_tiles) break;
    // ---- odd tile: buffers 1
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    seq.tile(idx + 1, &key0, &hi);
    if (idx + 2 < seq.n_tiles) {
      int k1, h1;
      seq.tile(idx + 2, &k1, &h1);
      issue_tile(Kb, Vb, k1, h1, lds0 + LDS_K0, lds0 + LDS_V0, tid, chunk_off);
    }
    if (key0 < wave_hi) {
      bool masked = key0 + TKEYS > wave_lo || key0 + TKEYS > hi;
      int lim = row_lim < hi ? row_lim : hi;
      compute_tile<LDS_K1, LDS_V1>(w, kaddr, vaddr, key0, lim, masked, c, half);
    }
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
  w.l = 0.f;
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
  int wave_last = tok0 + 32 < e ? tok0 + 32 : e;

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
  int wave_hi = tok0 < e ? wave_last : 0;
  unsigned lds0 = (unsigned)(size_t)(LDS_AS char*)lds;
  attend(w, seq, Kb, Vb, row_lim, wave_lo, wave_hi, g.scale * LOG2E, lds0);

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
  int wave_last = j0 + 32 < a.q_len ? j0 + 32 : a.q_len;
  int wave_lo = j0 < a.q_len ? cl + j0 + 1 : 0;
  int wave_hi = j0 < a.q_len ? cl + wave_last : 0;
  unsigned lds0 = (unsigned)(size_t)(LDS_AS char*)lds;
  attend(w, seq, Kb, Vb, row_lim, wave_lo, wave_hi, g.scale * LOG2E, lds0);

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
