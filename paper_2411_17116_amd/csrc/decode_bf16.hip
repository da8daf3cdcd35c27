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
//   * a batch of NS steps is loaded into registers with plain 16-byte loads and
//     then consumed in order -- K (8 KiB a step) straight in the layout the MFMA
//     wants: lane (i, j4) takes key i, bytes 64t + 16 j4 .. +15 of its row for
//     t = 0..3; V (8 KiB a step) as 1 KiB-contiguous bursts.  All waits are the
//     compiler's (straight-line code, static register indices); while one
//     wavefront computes, the other wavefronts of the CU keep the stream going;
//   * a cache too large to stay in the 256 MB last-level cache between steps is
//     read with non-temporal loads (every byte is used once: leaving it out of
//     the caches is worth 9-16 % of the step at 0.5-4 GB); a smaller one with
//     ordinary loads, so that the next step finds it there;
//   * all G query heads of the KV group (and up to 16/G new tokens) form the 16
//     columns of v_mfma_f32_16x16x32_bf16, so K and V are read once per KV head;
//     S^T = K Q^T leaves each lane with keys of one query column, and the
//     exponentiated tile is directly the B operand of O^T += V^T P^T; V goes
//     through a small LDS buffer (two 8 KiB halves used alternately) only to be
//     read back transposed, 16-byte chunks rotated-XOR swizzled so that writes
//     and transposing reads are conflict-free;
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
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

#define LDS_AS __attribute__((address_space(3)))

// chunk c of key row r sits in slot c ^ swz(r)
__device__ __forceinline__ int swz(int r) { return ((r << 1) & 15) | ((r >> 3) & 1); }

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
  bf16x8 q[4];     // Q^T fragments: q[t] = Q[column lane%16][32t + 8*(lane/16) .. +7]
  f32x4 o[8];      // O^T: o[dt][v] = O[column][16dt + 4*(lane/16) + v]
  float m, l;
};

// One 32-key step in registers.
struct StepRegs {
  i32x4 k[8];      // k[4kt + t]: key 16kt + lane%16, bytes 64t + 16*(lane/16) .. +15 (MFMA A operand)
  i32x4 v[8];      // v[it]: key 4it + lane/16, bytes 16*(lane%16) .. +15
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

// Load the step [key0, key0 + 32).  Rows at or past `hi` re-read the last valid
// row (they are masked in the score tile).
template <bool NT>
__device__ __forceinline__ void load_step(StepRegs& r, const Source& src, int key0, int hi, int lane) {
  const int col = lane & 15, j4 = lane >> 4;
  if (key0 + STEP <= hi && key0 + STEP <= src.cache_len) {   // whole step from the cache
    const char* kp = src.Kb + (size_t)key0 * ROWB + col * ROWB + j4 * 16;
    const char* vp = src.Vb + (size_t)key0 * ROWB + j4 * ROWB + col * 16;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const i32x4* ka = (const i32x4*)(kp + (it >> 2) * 16 * ROWB + (it & 3) * 64);
      const i32x4* va = (const i32x4*)(vp + it * 4 * ROWB);
      r.k[it] = NT ? __builtin_nontemporal_load(ka) : *ka;
      r.v[it] = NT ? __builtin_nontemporal_load(va) : *va;
    }
  } else {
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      int kk = key0 + 16 * (it >> 2) + col;
      kk = kk < hi ? kk : hi - 1;
      const char* kp = kk < src.cache_len ? src.Kb + (size_t)kk * ROWB
                                          : src.Kn + (size_t)(kk - src.cache_len) * src.new_stride;
      r.k[it] = *(const i32x4*)(kp + (it & 3) * 64 + j4 * 16);
      int vk = key0 + 4 * it + j4;
      vk = vk < hi ? vk : hi - 1;
      const char* vp = vk < src.cache_len ? src.Vb + (size_t)vk * ROWB
                                          : src.Vn + (size_t)(vk - src.cache_len) * src.new_stride;
      r.v[it] = *(const i32x4*)(vp + col * 16);
    }
  }
}

// VOFF (0 or STEPB) selects the LDS half this step's V goes through.
__device__ __forceinline__ void compute_step(const int VOFF, DecState& w, const StepRegs& r,
                                             const unsigned (&vw)[4], const unsigned (&vaddr)[8],
                                             int key0, int lim, bool masked, float c, int j4) {
  // V rows into LDS (row 4it + lane/16, swizzled chunk lane%16)
#pragma unroll
  for (int it = 0; it < 8; ++it)
    *(LDS_AS i32x4*)(size_t)(vw[it & 3] + VOFF + (it >> 2) * 16 * ROWB) = r.v[it];
  f32x4 s[2];
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
    s[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 4; ++t)
      s[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, r.k[4 * kt + t]),
                                                      w.q[t], s[kt], 0, 0, 0);
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

// grid: x = split, y = kv head, z = batch; 64 threads.  NS = steps per batch of
// loads, NT = non-temporal loads.
template <int NS, bool NT>
__global__ __launch_bounds__(64) void decode_bf16_kernel(Phase2Args a) {
  __shared__ __attribute__((aligned(1024))) char lds[2 * STEPB];
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
  }

  DecState w;
  {
    const char* qrow = (const char*)a.Qq + (((size_t)beta * a.q_len + (live ? j : 0)) * g.Hq +
                                            (live ? head : kvh * g.G)) * ROWB;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      bf16x8 v = *(const bf16x8*)(qrow + (32 * t + 8 * j4) * 2);
      if (!live) v = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};     // dead columns contribute zeros
      w.q[t] = v;
    }
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) w.o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    w.m = -INFINITY;
    w.l = 0.f;
  }

  const unsigned lds0 = (unsigned)(size_t)(LDS_AS char*)lds;
  // V rows into LDS: lane writes row 4it + lane/16, chunk lane%16 (swizzled)
  unsigned vw[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    int row = 4 * it + j4;
    vw[it] = lds0 + row * ROWB + ((qc ^ swz(row)) << 4);
  }
  // V^T operand: source lane addresses row 4*j4 + (lane%16)/4 (+16 for the second
  // read), columns 16dt + 4*(lane%4) .. +3
  unsigned vaddr[8];
  {
    int rr = 4 * j4 + (qc >> 2);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
      vaddr[dt] = lds0 + rr * ROWB + (((2 * dt + ((lane & 3) >> 1)) ^ swz(rr)) << 4) + 8 * (lane & 1);
  }

  const float c = g.scale * LOG2E;
  // keys below free_hi (what the call's first token sees) are visible to every
  // live column, so only steps reaching past it take the masking path
  const int row_lim = live ? (int)visible_limit(a, j) : 0;
  const int lim = row_lim < hi ? row_lim : hi;
  const int first_lim = (int)visible_limit(a, 0);
  const int free_hi = first_lim < hi ? first_lim : hi;

  // NS steps are loaded into registers at once and then consumed in order; the
  // other wavefronts of the CU stream while this one computes
  for (int s = 0; s < nsteps; s += NS) {
    StepRegs r[NS];
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      const int cur = s + u < nsteps ? s + u : nsteps - 1;     // past the end: re-read the last step
      load_step<NT>(r[u], src, base + cur * stride, hi, lane);
    }
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      if (s + u >= nsteps) break;
      const int key0 = base + (s + u) * stride;
      const bool masked = key0 + STEP > free_hi;
      compute_step((u & 1) * STEPB, w, r[u], vw, vaddr, key0, lim, masked, c, j4);
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
  const dim3 grid((unsigned)a.plan.s_total, (unsigned)g.Hkv, (unsigned)g.B);
  if (decode_cache_resident(g, visible_total(a))) decode_bf16_kernel<1, false><<<grid, 64, 0, st>>>(a);
  else decode_bf16_kernel<2, true><<<grid, 64, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace star
