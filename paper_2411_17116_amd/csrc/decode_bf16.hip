// bf16 split-KV partial attention for decode-sized phase-2 calls (head_dim 128,
// G * q_len <= 16 rows per KV head): Eq. 1-2 evaluated per split of the cache,
// with Algorithm 2's "append, then attend" fused in.
//
// A decode step reads every cached K and V byte exactly once and does 4-8 flops
// per byte, so the kernel is built as an HBM stream:
//   * one wavefront per workgroup, one split (a set of keys of one KV head) per
//     workgroup, no barriers; without per-part outputs there is one split per
//     resident workgroup slot and split s is the comb of 32-key steps
//     s, s + S, s + 2S, ... so that at any moment the S wavefronts of a KV head
//     read one contiguous window of its cache (every memory channel busy, none
//     hot); with per-part outputs a split is a contiguous run inside one part;
//   * the wavefront DMAs 32-key steps of K and V (8 KiB each) straight into a
//     two-step LDS ring with global_load_lds_dwordx4 -- fully coalesced 1 KiB
//     bursts, no VGPRs held by data in flight -- and waits with partial vmcnt so
//     that one step (16 KiB) is in flight while one is consumed; 32 KiB of LDS
//     per workgroup lets four of them share a CU, one per SIMD (measured: four
//     wavefronts with one step ahead each stream 2 % faster than two with three
//     ahead, one wavefront per CU 15 % slower);
//   * all G query heads of the KV group (and up to 16/G new tokens) form the 16
//     columns of v_mfma_f32_16x16x32_bf16, so K and V are read once per KV head;
//     S^T = K Q^T leaves each lane with keys of one query column, and the
//     exponentiated tile is directly the B operand of O^T += V^T P^T, with V^T
//     fragments from the LDS transposing read;
//   * 16-byte chunks of a key row are rotated-XOR swizzled in LDS so both operand
//     reads are conflict-free;
//   * rows at or beyond cache_len are the new tokens: they are read from the
//     call's Kq/Vq and written to the cache by the workgroup whose split holds
//     them, so no separate append kernel runs before a decode step.
// Each workgroup writes its split's normalised output rows and their
// log-sum-exp; the merge kernel folds the splits (Eq. 3-4).
#include "star_internal.h"

namespace star {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int D = 128;
constexpr int ROWB = D * 2;
constexpr int STEP = 32;                 // keys per pipeline step
constexpr int STEPB = STEP * ROWB;       // 8 KiB of K (and of V) per step
#ifndef STAR_DECODE_RING
#define STAR_DECODE_RING 2
#endif
constexpr int RING = STAR_DECODE_RING;   // steps in the LDS ring
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

#define LDS_AS __attribute__((address_space(3)))

// chunk c of key row r sits in slot c ^ swz(r)
__device__ __forceinline__ int swz(int r) { return ((r << 1) & 15) | ((r >> 3) & 1); }

// 16-byte DMA global -> LDS (lane L lands at lds_base + 16 L), address = sbase + voff
__device__ __forceinline__ void dma16(const char* sbase, unsigned voff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(sbase), "s"(lds_base) : "memory");
}
// same with a full per-lane 64-bit address
__device__ __forceinline__ void dma16_flat(const char* ptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(ptr), "s"(lds_base) : "memory");
}

__device__ __forceinline__ float xor16(float x) {
  return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), 0x401F));
}
__device__ __forceinline__ float xor32_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor32_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

struct DecState {
  bf16x8 q[4];     // Q^T fragments: q[t] = Q[column lane%16][32*(lane/16) + 8t .. +7]
  f32x4 o[8];      // O^T: o[dt][v] = O[column][16dt + 4*(lane/16) + v]
  float m, l;
};

// Where a split's rows come from: cache rows below `cache_len`, the call's new
// tokens (token-major, `new_stride` bytes between tokens) from there on.
struct Source {
  const char* Kb;      // cache base of this (batch, kv head)
  const char* Vb;
  const char* Kn;      // new-token base of this (batch, kv head)
  const char* Vn;
  int cache_len;
  int new_stride;
};

// DMA one 32-key step of K and V into ring slot `slot`.  Instruction `it` moves
// rows 4it..4it+3; lane L moves (row 4it + L/16, slot L%16).  Rows at or past
// `hi` re-read the last valid row (they are masked in the score tile).
__device__ __forceinline__ void issue_step(const Source& src, int key0, int hi, unsigned lds_slot,
                                           int lane, const unsigned (&voff)[4]) {
  const unsigned ldsK = lds_slot, ldsV = lds_slot + STEPB;
  if (key0 + STEP <= hi && key0 + STEP <= src.cache_len) {   // whole step from the cache
    const char* kb = src.Kb + (size_t)key0 * ROWB;
    const char* vb = src.Vb + (size_t)key0 * ROWB;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      dma16(kb + (it >> 2) * 16 * ROWB, voff[it & 3], ldsK + it * 1024);
      dma16(vb + (it >> 2) * 16 * ROWB, voff[it & 3], ldsV + it * 1024);
    }
  } else {
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      int key = key0 + 4 * it + (lane >> 4);
      key = key < hi ? key : hi - 1;
      unsigned coff = voff[it & 3] & 255;
      size_t off = key < src.cache_len ? (size_t)key * ROWB
                                       : (size_t)(key - src.cache_len) * src.new_stride;
      const char* kp = (key < src.cache_len ? src.Kb : src.Kn) + off + coff;
      const char* vp = (key < src.cache_len ? src.Vb : src.Vn) + off + coff;
      dma16_flat(kp, ldsK + it * 1024);
      dma16_flat(vp, ldsV + it * 1024);
    }
  }
}

template <int SLOT>
__device__ __forceinline__ void compute_step(DecState& w, const unsigned (&kaddr)[4],
                                             const unsigned (&vaddr)[8], int key0, int lim,
                                             bool masked, float c, int j4) {
  constexpr int KOFF = SLOT * 2 * STEPB, VOFF = KOFF + STEPB;
  f32x4 s[2];
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
    s[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      bf16x8 a = *(LDS_AS bf16x8*)(size_t)(kaddr[t] + KOFF + kt * 16 * ROWB);
      s[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, w.q[t], s[kt], 0, 0, 0);
    }
  }
  if (masked) {
    int x = lim - key0 - 4 * j4;     // element (kt, v) is key key0 + 16kt + 4*j4 + v
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int v = 0; v < 4; ++v) s[kt][v] = (16 * kt + v) < x ? s[kt][v] : -INFINITY;
  }
  float tmax = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                     fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
  tmax = fmaxf(tmax, xor16(tmax));
  tmax = xor32_max(tmax);
  float m_new = fmaxf(w.m, tmax);
  if (__builtin_amdgcn_ballot_w64(m_new > w.m) != 0) {
    float mm = m_new == -INFINITY ? 0.f : m_new;
    float alpha = __builtin_amdgcn_exp2f((w.m - mm) * c);
    w.l *= alpha;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) w.o[dt] *= alpha;
    w.m = m_new;
  }
  float neg_mc = (w.m == -INFINITY ? 0.f : w.m) * -c;
  bf16x8 p;
  float lsum = 0.f;
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][v], c, neg_mc));
      lsum += e;
      p[4 * kt + v] = (__bf16)e;
    }
  w.l += lsum;
  // B operand slot e of lane group j4 is key 16(e/4) + 4*j4 + e%4; the A operand
  // (V^T, d-row lane%16) takes keys 4*j4..+3 and 16 + 4*j4..+3 from two
  // transposing reads.
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) {
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(size_t)(vaddr[dt] + VOFF));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(size_t)(vaddr[dt] + VOFF + 16 * ROWB));
    bf16x4 lo_b = __builtin_bit_cast(bf16x4, lo), hi_b = __builtin_bit_cast(bf16x4, hi);
    bf16x8 a = __builtin_shufflevector(lo_b, hi_b, 0, 1, 2, 3, 4, 5, 6, 7);
    w.o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, p, w.o[dt], 0, 0, 0);
  }
}

// Wait until at most `pending` of the most recently issued steps are in flight
// (16 DMA instructions per step).
__device__ __forceinline__ void wait_steps(int pending) {
  if (pending >= 3) asm volatile("s_waitcnt vmcnt(48)" ::: "memory");
  else if (pending == 2) asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
  else if (pending == 1) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// grid: x = split, y = kv head, z = batch; 64 threads
__global__ __launch_bounds__(64) void decode_bf16_kernel(Phase2Args a) {
  __shared__ __attribute__((aligned(1024))) char lds[RING * 2 * STEPB];
  const Geom& g = a.g;
  const int lane = threadIdx.x;
  const int qc = lane & 15, j4 = lane >> 4;
  const int sp = blockIdx.x, kvh = blockIdx.y, beta = blockIdx.z;
  const int R = g.G * a.q_len;                 // <= 16 live columns
  const int j = qc / g.G, head = kvh * g.G + qc % g.G;
  const bool live = qc < R;

  const int cache_len = (int)a.cache_len;
  const int total = (int)visible_total(a);
  // step `cur` of this split covers keys [base + cur * stride, +32) below hi
  int base, stride, nsteps, hi;
  if (a.plan.flat) {
    const int S = a.plan.s_total, T = (total + STEP - 1) / STEP;
    base = sp * STEP;
    stride = S * STEP;
    nsteps = sp < T ? (T - sp + S - 1) / S : 0;
    hi = total;
  } else {
    int64_t lo64, hi64;
    split_range(a.plan, g.L, g.b, total, sp, &lo64, &hi64);
    base = (int)lo64;
    stride = STEP;
    hi = (int)hi64;
    nsteps = hi > base ? (hi - base + STEP - 1) / STEP : 0;
  }
  size_t r = (((size_t)beta * a.plan.s_total + sp) * g.Hq + head) * a.q_len + j;
  if (nsteps == 0) {                           // empty split (short block, unused tail)
    if (live && j4 == 0) a.LSE_sub[r] = -INFINITY;
    return;
  }

  Source src;
  src.Kb = (const char*)a.Kc + ((size_t)beta * g.Hkv + kvh) * (size_t)g.cap * ROWB;
  src.Vb = (const char*)a.Vc + ((size_t)beta * g.Hkv + kvh) * (size_t)g.cap * ROWB;
  src.Kn = (const char*)a.Kn + ((size_t)beta * a.q_len * g.Hkv + kvh) * ROWB;
  src.Vn = (const char*)a.Vn + ((size_t)beta * a.q_len * g.Hkv + kvh) * ROWB;
  // without new-token tensors the caches already hold the appended rows
  const bool fused_append = a.Kn != nullptr;
  src.cache_len = fused_append ? cache_len : total;
  src.new_stride = g.Hkv * ROWB;

  // Algorithm 2, append: the new tokens whose rows fall into this split's steps
  // join the cache (16 lanes move one 256-byte row of K and of V).
  if (fused_append && hi > cache_len) {
    for (int key = cache_len + (lane >> 4); key < hi; key += 4) {
      const int rel = key - base;
      if (rel < 0 || (rel % stride) >= STEP) continue;      // another split's step
      size_t so = (size_t)(key - cache_len) * src.new_stride + (lane & 15) * 16;
      size_t dof = (size_t)key * ROWB + (lane & 15) * 16;
      *(i32x4*)(const_cast<char*>(src.Kb) + dof) = *(const i32x4*)(src.Kn + so);
      *(i32x4*)(const_cast<char*>(src.Vb) + dof) = *(const i32x4*)(src.Vn + so);
    }

    // the stores are complete before DMAs are counted
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }

  // The query loads are issued here and consumed after the first step's wait:
  // their latency overlaps the first DMAs instead of preceding them.
  DecState w;
  {
    const char* qrow = (const char*)a.Qq + (((size_t)beta * a.q_len + (live ? j : 0)) * g.Hq +
                                            (live ? head : kvh * g.G)) * ROWB;
#pragma unroll
    for (int t = 0; t < 4; ++t) w.q[t] = *(const bf16x8*)(qrow + (32 * j4 + 8 * t) * 2);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) w.o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    w.m = -INFINITY;
    w.l = 0.f;
  }

  const unsigned lds0 = (unsigned)(size_t)(LDS_AS char*)lds;
  // K operand: in MFMA step t, lane (i = lane%16, j4) reads row i, chunk 4 j4 + t
  // (Q uses the same assignment of d-chunks; the transposed one, 4t + j4, costs
  // LDS bank conflicts on these 16-byte reads)
  unsigned kaddr[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) kaddr[t] = lds0 + qc * ROWB + (((4 * j4 + t) ^ swz(qc)) << 4);
  // V^T operand: source lane addresses row 4*j4 + (lane%16)/4 (+16 for the second
  // read), columns 16dt + 4*(lane%4) .. +3
  unsigned vaddr[8];
  {
    int rr = 4 * j4 + (qc >> 2);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
      vaddr[dt] = lds0 + rr * ROWB + (((2 * dt + ((lane & 3) >> 1)) ^ swz(rr)) << 4) + 8 * (lane & 1);
  }
  // DMA lane offsets: row (4it + lane/16) of a 16-row group, swizzled chunk
  unsigned voff[4];
#pragma unroll
  for (int it = 0; it < 4; ++it)
    voff[it] = (4 * it + (lane >> 4)) * ROWB + (((lane & 15) ^ swz(4 * it + (lane >> 4))) << 4);

  const float c = g.scale * LOG2E;
  // keys below free_hi (what the call's first token sees) are visible to every
  // live column, so only steps reaching past it take the masking path
  const int row_lim = live ? (int)visible_limit(a, j) : 0;
  const int lim = row_lim < hi ? row_lim : hi;
  const int first_lim = (int)visible_limit(a, 0);
  const int free_hi = first_lim < hi ? first_lim : hi;

  // ring slot of step s is s % RING; AHEAD = RING - 1 steps are in flight while
  // one is consumed
  constexpr int AHEAD = RING - 1;
  static_assert(RING >= 2 && RING <= 4, "vmcnt holds at most 63 outstanding DMAs");
#pragma unroll
  for (int i = 0; i < AHEAD; ++i)
    if (i < nsteps) issue_step(src, base + i * stride, hi, lds0 + i * 2 * STEPB, lane, voff);
  for (int s = 0; s < nsteps; s += RING) {
#pragma unroll
    for (int u = 0; u < RING; ++u) {
      const int cur = s + u;
      if (cur >= nsteps) break;
      const int key0 = base + cur * stride;
      // the slot that held step cur-1 is free: every LDS read of it has returned
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (cur + AHEAD < nsteps)
        issue_step(src, key0 + AHEAD * stride, hi, lds0 + ((u + AHEAD) % RING) * 2 * STEPB, lane, voff);
      int later = nsteps - 1 - cur;
      wait_steps(later < AHEAD ? later : AHEAD);
      if (cur == 0) {
        // first use of the query: the loads were issued before every DMA, so the
        // wait above covers them; dead columns contribute zeros
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          asm volatile("" : "+v"(w.q[t]));
          if (!live) w.q[t] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
      }
      const bool masked = key0 + STEP > free_hi;
      if (u == 0) compute_step<0>(w, kaddr, vaddr, key0, lim, masked, c, j4);
      else if (u == 1) compute_step<1>(w, kaddr, vaddr, key0, lim, masked, c, j4);
      else if (u == 2) compute_step<2>(w, kaddr, vaddr, key0, lim, masked, c, j4);
      else compute_step<3>(w, kaddr, vaddr, key0, lim, masked, c, j4);
    }
  }

  float l_tot = w.l + xor16(w.l);
  l_tot = xor32_sum(l_tot);
  if (live) {
    float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    float* orow = a.O_sub + r * D;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) *(f32x4*)(orow + 16 * dt + 4 * j4) = w.o[dt] * inv;
    if (j4 == 0)
      a.LSE_sub[r] = l_tot > 0.f ? (w.m * c + __builtin_amdgcn_logf(l_tot)) * LN2 : -INFINITY;
  }
}

}  // namespace

hipError_t launch_phase2_decode_bf16(const Phase2Args& a, hipStream_t st) {
  const Geom& g = a.g;
  if (g.Hkv > 65535 || g.B > 65535) return hipErrorInvalidValue;
  decode_bf16_kernel<<<dim3((unsigned)a.plan.s_total, (unsigned)g.Hkv, (unsigned)g.B), 64, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace star
