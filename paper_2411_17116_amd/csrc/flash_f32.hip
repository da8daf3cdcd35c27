// fp32 path (head_dim 64 or 128): one thread owns one query row.
//
// The row's query and output accumulator live in registers, K/V tiles of the
// row tile's key ranges are staged through LDS and read as broadcasts, and the
// online softmax (running maximum + rescaled sum) runs per thread with no
// cross-lane traffic.  The same row routine serves phase 1 (Section 2.1: key
// ranges = anchor + own block up to the row) and the phase-2 partial attention
// of one split (Eq. 1-2: key range = the split, limited to the keys the token
// may see).  Arithmetic is fp32 throughout so the result stays within 1e-5 of
// an fp64 evaluation at the sizes this path is meant for.
#include "star_internal.h"

namespace star {

namespace {

constexpr int ROWS = 64;   // rows (threads) per workgroup
constexpr int TK = 32;     // keys per LDS tile
constexpr int CH = 8;      // keys per softmax update

typedef __attribute__((ext_vector_type(4))) float f32x4;

template <int D>
struct RowState {
  float q[D];
  float o[D];
  float m;   // running maximum of the log2-domain logits
  float l;   // running sum of 2^(logit - m)
};

// Attend the workgroup's rows to keys [lo, hi) of one KV head.  `limit` is this
// thread's exclusive key bound (a key is visible iff key < limit).
template <int D>
__device__ __forceinline__ void attend_range(RowState<D>& st, const float* __restrict__ Kb,
                                             const float* __restrict__ Vb, int64_t lo, int64_t hi,
                                             int64_t limit, float* Ks, float* Vs) {
  const int tid = threadIdx.x;
  for (int64_t k0 = lo; k0 < hi; k0 += TK) {
    __syncthreads();
    // cooperative tile load, 16 bytes per thread per step; rows past `hi` are
    // clamped to the last valid key (they are masked below)
    constexpr int VPR = D / 4;
    for (int v = tid; v < TK * VPR; v += ROWS) {
      int r = v / VPR, c = v - r * VPR;
      int64_t key = k0 + r < hi ? k0 + r : hi - 1;
      ((f32x4*)Ks)[v] = *(const f32x4*)(Kb + key * D + c * 4);
      ((f32x4*)Vs)[v] = *(const f32x4*)(Vb + key * D + c * 4);
    }
    __syncthreads();
    for (int c0 = 0; c0 < TK; c0 += CH) {
      if (k0 + c0 >= hi) break;
      // two partial sums per logit, added at the end: chains of d/2 terms keep the
      // rounding of a large logit (a planted pair reaches 25 in log2 units) down
      float s[CH], s2[CH];
#pragma unroll
      for (int kk = 0; kk < CH; ++kk) s[kk] = s2[kk] = 0.f;
#pragma unroll
      for (int dd = 0; dd < D; dd += 4) {
#pragma unroll
        for (int kk = 0; kk < CH; ++kk) {
          f32x4 kv = *(const f32x4*)(Ks + (c0 + kk) * D + dd);
          s[kk] = __builtin_fmaf(st.q[dd], kv[0], s[kk]);
          s2[kk] = __builtin_fmaf(st.q[dd + 1], kv[1], s2[kk]);
          s[kk] = __builtin_fmaf(st.q[dd + 2], kv[2], s[kk]);
          s2[kk] = __builtin_fmaf(st.q[dd + 3], kv[3], s2[kk]);
        }
      }
#pragma unroll
      for (int kk = 0; kk < CH; ++kk) s[kk] += s2[kk];
      float cmax = -INFINITY;
#pragma unroll
      for (int kk = 0; kk < CH; ++kk) {
        int64_t key = k0 + c0 + kk;
        bool vis = key < hi && key < limit;
        s[kk] = vis ? s[kk] : -INFINITY;
        cmax = fmaxf(cmax, s[kk]);
      }
      float m_new = fmaxf(st.m, cmax);
      if (m_new == -INFINITY) continue;            // nothing visible yet for this row
      float alpha = exp2f(st.m - m_new);           // 0 when st.m == -inf
      float p[CH];
      float psum = 0.f;
#pragma unroll
      for (int kk = 0; kk < CH; ++kk) {
        p[kk] = exp2f(s[kk] - m_new);              // 0 for masked keys
        psum += p[kk];
      }
      st.l = st.l * alpha + psum;
      st.m = m_new;
#pragma unroll
      for (int dd = 0; dd < D; dd += 4) {
        f32x4 acc = {st.o[dd] * alpha, st.o[dd + 1] * alpha, st.o[dd + 2] * alpha,
                     st.o[dd + 3] * alpha};
#pragma unroll
        for (int kk = 0; kk < CH; ++kk) {
          f32x4 vv = *(const f32x4*)(Vs + (c0 + kk) * D + dd);
          acc[0] = __builtin_fmaf(p[kk], vv[0], acc[0]);
          acc[1] = __builtin_fmaf(p[kk], vv[1], acc[1]);
          acc[2] = __builtin_fmaf(p[kk], vv[2], acc[2]);
          acc[3] = __builtin_fmaf(p[kk], vv[3], acc[3]);
        }
        st.o[dd] = acc[0]; st.o[dd + 1] = acc[1]; st.o[dd + 2] = acc[2]; st.o[dd + 3] = acc[3];
      }
    }
  }
}

template <int D>
__device__ __forceinline__ void load_row(RowState<D>& st, const float* q, bool active, float qk_scale) {
#pragma unroll
  for (int dd = 0; dd < D; dd += 4) {
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (active) v = *(const f32x4*)(q + dd);
    st.q[dd] = v[0] * qk_scale; st.q[dd + 1] = v[1] * qk_scale;
    st.q[dd + 2] = v[2] * qk_scale; st.q[dd + 3] = v[3] * qk_scale;
    st.o[dd] = st.o[dd + 1] = st.o[dd + 2] = st.o[dd + 3] = 0.f;
  }
  st.m = -INFINITY;
  st.l = 0.f;
}

template <int D>
__device__ __forceinline__ void store_row(const RowState<D>& st, float* o, float* lse) {
  float inv = st.l > 0.f ? 1.f / st.l : 0.f;
#pragma unroll
  for (int dd = 0; dd < D; dd += 4) {
    f32x4 v = {st.o[dd] * inv, st.o[dd + 1] * inv, st.o[dd + 2] * inv, st.o[dd + 3] * inv};
    *(f32x4*)(o + dd) = v;
  }
  if (lse) *lse = st.l > 0.f ? (st.m + log2f(st.l)) * 0.6931471805599453f : -INFINITY;
}

constexpr float LOG2E = 1.4426950408889634f;

// grid: x = block index * tiles_per_block + tile in block, y = query head, z = batch
template <int D>
__global__ __launch_bounds__(ROWS) void phase1_f32_kernel(Phase1Args a, int tiles_per_block) {
  __shared__ __attribute__((aligned(16))) float Ks[TK * D];
  __shared__ __attribute__((aligned(16))) float Vs[TK * D];
  const Geom& g = a.g;
  int i = blockIdx.x / tiles_per_block, t = blockIdx.x % tiles_per_block;
  int h = blockIdx.y, beta = blockIdx.z;
  int64_t s = (int64_t)i * g.b;
  int64_t e = s + g.b < g.L ? s + g.b : g.L;
  int64_t row0 = s + (int64_t)t * ROWS;
  if (row0 >= e) return;                              // tile beyond a short last block
  int64_t p = row0 + threadIdx.x;
  bool active = p < e;
  int kvh = h / g.G;
  const float* Kb = (const float*)a.Kc + ((int64_t)beta * g.Hkv + kvh) * g.cap * D;
  const float* Vb = (const float*)a.Vc + ((int64_t)beta * g.Hkv + kvh) * g.cap * D;
  RowState<D> st;
  load_row<D>(st, (const float*)a.Q + (((int64_t)beta * g.L + (active ? p : row0)) * g.Hq + h) * D,
              active, g.scale * LOG2E);
  int64_t limit = active ? p + 1 : 0;
  int64_t last = row0 + ROWS < e ? row0 + ROWS : e;   // exclusive bound of the tile's rows
  int64_t a_lo, a_hi;                                              // anchor: fully visible
  if (anchor_range(g, a.anchor_mode, i, &a_lo, &a_hi)) {
    const int64_t anchor_rows = (a.anchor_mode == ANCHOR_PER_BLOCK ? (g.L + g.b - 1) / g.b : 1) * g.a;
    const float* Kab = (const float*)a.Ka + ((int64_t)beta * g.Hkv + kvh) * anchor_rows * D;
    const float* Vab = (const float*)a.Va + ((int64_t)beta * g.Hkv + kvh) * anchor_rows * D;
    // rows of the anchor buffer are not positions: every one is visible
    attend_range<D>(st, Kab, Vab, a_lo, a_hi, active ? a_hi : 0, Ks, Vs);
  } else {
    attend_range<D>(st, Kb, Vb, a_lo, a_hi, limit, Ks, Vs);
  }
  attend_range<D>(st, Kb, Vb, s, last, limit, Ks, Vs);             // own block, causal
  if (active) {
    float* o = (float*)a.O + (((int64_t)beta * g.L + p) * g.Hq + h) * D;
    float* lse = a.LSE ? a.LSE + ((int64_t)beta * g.Hq + h) * g.L + p : nullptr;
    store_row<D>(st, o, lse);
  }
}

// grid: x = (batch * s_total + split) * row_tiles + row tile, y = query head
template <int D>
__global__ __launch_bounds__(ROWS) void phase2_f32_kernel(Phase2Args a, int row_tiles) {
  __shared__ __attribute__((aligned(16))) float Ks[TK * D];
  __shared__ __attribute__((aligned(16))) float Vs[TK * D];
  const Geom& g = a.g;
  int h = blockIdx.y;
  int bs = blockIdx.x / row_tiles;
  int beta = bs / a.plan.s_total, s = bs % a.plan.s_total;
  int j = (blockIdx.x % row_tiles) * ROWS + threadIdx.x;
  bool active = j < a.q_len;
  int64_t total = visible_total(a);
  int64_t lo, hi;
  split_range(a.plan, g.L, g.b, total, s, &lo, &hi);
  int kvh = h / g.G;
  const float* Kb = (const float*)a.Kc + ((int64_t)beta * g.Hkv + kvh) * g.cap * D;
  const float* Vb = (const float*)a.Vc + ((int64_t)beta * g.Hkv + kvh) * g.cap * D;
  RowState<D> st;
  load_row<D>(st, (const float*)a.Qq + (((int64_t)beta * a.q_len + (active ? j : 0)) * g.Hq + h) * D,
              active, g.scale * LOG2E);
  int64_t limit = active ? visible_limit(a, j) : 0;
  attend_range<D>(st, Kb, Vb, lo, hi, limit, Ks, Vs);
  if (active) {
    int64_t r = (((int64_t)beta * a.plan.s_total + s) * g.Hq + h) * a.q_len + j;
    store_row<D>(st, a.O_sub + r * D, a.LSE_sub + r);
  }
}

}  // namespace

hipError_t launch_phase1_f32(const Phase1Args& a, hipStream_t st) {
  const Geom& g = a.g;
  int64_t n = (g.L + g.b - 1) / g.b;
  int64_t bmax = g.b < g.L ? g.b : g.L;
  int tpb = (int)((bmax + ROWS - 1) / ROWS);
  if (n * tpb > 0x7fffffff) return hipErrorInvalidValue;
  dim3 grid((unsigned)(n * tpb), (unsigned)g.Hq, (unsigned)g.B);
  if (g.d == 64) phase1_f32_kernel<64><<<grid, ROWS, 0, st>>>(a, tpb);
  else phase1_f32_kernel<128><<<grid, ROWS, 0, st>>>(a, tpb);
  return hipGetLastError();
}

hipError_t launch_phase2_f32(const Phase2Args& a, hipStream_t st) {
  const Geom& g = a.g;
  int row_tiles = (a.q_len + ROWS - 1) / ROWS;
  if ((int64_t)g.B * a.plan.s_total * row_tiles > 0x7fffffff) return hipErrorInvalidValue;
  dim3 grid((unsigned)((int64_t)g.B * a.plan.s_total * row_tiles), (unsigned)g.Hq, 1);
  if (g.d == 64) phase2_f32_kernel<64><<<grid, ROWS, 0, st>>>(a, row_tiles);
  else phase2_f32_kernel<128><<<grid, ROWS, 0, st>>>(a, row_tiles);
  return hipGetLastError();
}

}  // namespace star
