// LSE merge (Eq. 3-4; Algorithm 2's running update): combines the per-split
// local attention outputs A_s and log-sum-exps lse_s of one query row into the
// global attention output,
//     lse = log sum_s exp(lse_s),   O = sum_s exp(lse_s - lse) A_s.
// Splits are first folded into their part (context block or tail) so that the
// per-part pair (A_m, lse_m) the paper's hosts would exchange can be written
// out; the parts are then folded in index order with the online-softmax update
//     lse' = logaddexp(lse, lse_m),  O' = exp(lse - lse') O + exp(lse_m - lse') A_m,
// which is what Eq. 3-4 evaluate to.  An empty split or part has lse = -inf and
// weight 0.  Under a flat split plan everything is one part.  The order of every
// fold is fixed, so results are deterministic.  The same kernel is the query
// host's aggregation of the pairs gathered from other hosts (Algorithm 2): the
// hosts' pairs are the splits of one part.  Besides the output in the storage
// dtype it can leave the merged pair itself, (A, lse) in fp32 -- what a host
// sends when its cache is one share of a larger one.
//
// merge_kernel: one workgroup per (batch, head, row): GROUPS groups of 32 lanes walk the
// splits of a part, each lane owning d/32 output elements and each group
// folding its splits with a running maximum (loads of INFL splits are in flight
// per group); the partial results are combined through LDS.  A decode step has
// few rows and 128 to 1024 splits per row (16 groups x 8 in flight: one to
// eight round trips); a query-encode call has thousands of rows and a few splits per
// part (8 groups x 4).  Traffic is s_total * (d + 1) floats per row
// -- negligible next to the cache.
//
// The fold over parts keeps a compensation term per accumulator (Kahan
// summation): a context cut into hundreds of small blocks is hundreds of
// sequential additions, and in fp32 their rounding errors would otherwise add up
// to the 1e-5 the fp32 path is held to.
#include "star_internal.h"

namespace star {

namespace {


// sum += x with the rounding error of the addition carried in `comp`
__device__ __forceinline__ void add_compensated(float& sum, float& comp, float x) {
  const float y = x - comp;
  const float t = sum + y;
  comp = (t - sum) - y;
  sum = t;
}

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f) {
  unsigned int u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

template <int D, int GROUPS, int INFL>
__global__ __launch_bounds__(32 * GROUPS) void merge_kernel(MergeArgs a) {
  constexpr int E = D / 32;                  // output elements per lane
  __shared__ float red_max[GROUPS];
  __shared__ float red_w[GROUPS];
  __shared__ float red_acc[GROUPS][D];
  const Geom& g = a.g;
  const int tid = threadIdx.x, grp = tid >> 5, li = tid & 31;
  int64_t row = blockIdx.x;                 // (beta, h, j), j fastest
  int j = (int)(row % a.q_len);
  int h = (int)((row / a.q_len) % g.Hq);
  int beta = (int)(row / ((int64_t)a.q_len * g.Hq));
  const SplitPlan& p = a.plan;
  const int64_t sub_stride = a.split_stride;                                 // rows between splits
  const int64_t base = (int64_t)beta * a.batch_stride + (int64_t)h * a.q_len + j;   // split 0
  const int n_parts = p.flat ? 1 : p.n_blocks + 1;

  float m_g = -INFINITY, l_g = 0.f, l_c = 0.f;
  float acc_g[E], acc_c[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc_g[e] = acc_c[e] = 0.f;

  for (int m = 0; m < n_parts; ++m) {
    int s_lo, s_hi;
    if (p.flat) { s_lo = 0; s_hi = p.s_total; }
    else if (m < p.n_blocks) { s_lo = m * p.spb; s_hi = s_lo + p.spb; }
    else { s_lo = p.n_blocks * p.spb; s_hi = p.s_total; }

    // Each group folds its splits (s_lo + grp, + GROUPS, ...) with a running maximum;
    // LSE and output loads of a split are independent of the fold, so several
    // splits are in flight at once.
    float pm = -INFINITY, wsum = 0.f;
    float acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.f;
    for (int s0 = s_lo + grp; s0 < s_hi; s0 += INFL * GROUPS) {
      float ls[INFL];
      float v[INFL][E];
#pragma unroll
      for (int u = 0; u < INFL; ++u) {
        int s = s0 + u * GROUPS;
        ls[u] = -INFINITY;
        if (s < s_hi) {
          ls[u] = a.LSE_sub[base + s * sub_stride];
          const float* src = a.O_sub + (base + s * sub_stride) * D + li * E;
#pragma unroll
          for (int e = 0; e < E; ++e) v[u][e] = src[e];
        }
      }
#pragma unroll
      for (int u = 0; u < INFL; ++u) {
        if (ls[u] == -INFINITY) continue;        // empty split: weight 0, output unset
        float m_new = fmaxf(pm, ls[u]);
        float sc_old = expf(pm - m_new);         // 0 for the first non-empty split
        float w = expf(ls[u] - m_new);
        wsum = wsum * sc_old + w;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = acc[e] * sc_old + w * v[u][e];
        pm = m_new;
      }
    }
    // combine the groups: bring every group to the common maximum
    __syncthreads();                         // previous part's reads of red_* are done
    if (li == 0) red_max[grp] = pm;
    __syncthreads();
    float pmax = red_max[0];
#pragma unroll
    for (int k = 1; k < GROUPS; ++k) pmax = fmaxf(pmax, red_max[k]);
    float adj = pm > -INFINITY ? expf(pm - pmax) : 0.f;
    if (li == 0) red_w[grp] = wsum * adj;
#pragma unroll
    for (int e = 0; e < E; ++e) red_acc[grp][li * E + e] = acc[e] * adj;
    __syncthreads();
    pm = pmax;

    if (grp == 0) {
      float wtot = 0.f;
#pragma unroll
      for (int k = 0; k < GROUPS; ++k) wtot += red_w[k];
      float A_m[E];
      float lse_m = -INFINITY;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        float t = 0.f;
#pragma unroll
        for (int k = 0; k < GROUPS; ++k) t += red_acc[k][li * E + e];
        A_m[e] = wtot > 0.f ? t / wtot : 0.f;
      }
      if (wtot > 0.f) lse_m = pm + logf(wtot);
      if (a.O_part) {
        int64_t pr = (((int64_t)beta * n_parts + m) * g.Hq + h) * a.q_len + j;
#pragma unroll
        for (int e = 0; e < E; ++e) a.O_part[pr * D + li * E + e] = A_m[e];
        if (li == 0) a.LSE_part[pr] = lse_m;
      }
      if (lse_m > -INFINITY) {
        float m_new = fmaxf(m_g, lse_m);
        float sc_old = expf(m_g - m_new);     // 0 on the first non-empty part
        float sc_new = expf(lse_m - m_new);
        if (sc_old != 1.f) {                  // the maximum moved: rescale sums and compensations
#pragma unroll
          for (int e = 0; e < E; ++e) { acc_g[e] *= sc_old; acc_c[e] *= sc_old; }
          l_g *= sc_old;
          l_c *= sc_old;
        }
#pragma unroll
        for (int e = 0; e < E; ++e) add_compensated(acc_g[e], acc_c[e], sc_new * A_m[e]);
        add_compensated(l_g, l_c, sc_new);
        m_g = m_new;
      }
    }
  }
  if (grp == 0) {
    int64_t orow = ((int64_t)beta * a.q_len + j) * g.Hq + h;
    int64_t arow = ((int64_t)beta * g.Hq + h) * a.q_len + j;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      float out = l_g > 0.f ? acc_g[e] / l_g : 0.f;
      if (a.A) a.A[arow * D + li * E + e] = out;
      if (!a.O) continue;
      if (a.out_bf16) ((unsigned short*)a.O)[orow * D + li * E + e] = f32_to_bf16_rne(out);
      else ((float*)a.O)[orow * D + li * E + e] = out;
    }
    if (a.LSE && li == 0) a.LSE[arow] = l_g > 0.f ? m_g + logf(l_g) : -INFINITY;
  }
}

// The same merge for calls with many rows and few splits per part (query
// encoding: thousands of rows, one to a few splits per context block; a handful
// of gathered host pairs): 32 lanes own a row, eight rows share a workgroup, and
// nothing crosses lanes -- no LDS, no barriers.  A part's splits are folded in
// index order with INFL loads in flight, the parts in index order after them.
template <int D, int INFL>
__global__ __launch_bounds__(256) void merge_rows_kernel(MergeArgs a, int64_t n_rows) {
  constexpr int E = D / 32;
  const Geom& g = a.g;
  const int li = threadIdx.x & 31;
  const int64_t row = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5);      // (beta, h, j), j fastest
  if (row >= n_rows) return;
  const int j = (int)(row % a.q_len);
  const int h = (int)((row / a.q_len) % g.Hq);
  const int beta = (int)(row / ((int64_t)a.q_len * g.Hq));
  const SplitPlan& p = a.plan;
  const int64_t base = (int64_t)beta * a.batch_stride + (int64_t)h * a.q_len + j;
  const int n_parts = p.flat ? 1 : p.n_blocks + 1;

  float m_g = -INFINITY, l_g = 0.f, l_c = 0.f;
  float acc_g[E], acc_c[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc_g[e] = acc_c[e] = 0.f;
  for (int m = 0; m < n_parts; ++m) {
    int s_lo, s_hi;
    if (p.flat) { s_lo = 0; s_hi = p.s_total; }
    else if (m < p.n_blocks) { s_lo = m * p.spb; s_hi = s_lo + p.spb; }
    else { s_lo = p.n_blocks * p.spb; s_hi = p.s_total; }
    float pm = -INFINITY, wsum = 0.f;
    float acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.f;
    for (int s0 = s_lo; s0 < s_hi; s0 += INFL) {
      float ls[INFL];
      float v[INFL][E];
#pragma unroll
      for (int u = 0; u < INFL; ++u) {
        const int s = s0 + u;
        ls[u] = -INFINITY;
        if (s < s_hi) {
          ls[u] = a.LSE_sub[base + s * a.split_stride];
          const float* src = a.O_sub + (base + s * a.split_stride) * D + li * E;
#pragma unroll
          for (int e = 0; e < E; ++e) v[u][e] = src[e];
        }
      }
#pragma unroll
      for (int u = 0; u < INFL; ++u) {
        if (ls[u] == -INFINITY) continue;        // empty split: weight 0, output unset
        float m_new = fmaxf(pm, ls[u]);
        float sc_old = expf(pm - m_new);         // 0 for the first non-empty split
        float w = expf(ls[u] - m_new);
        wsum = wsum * sc_old + w;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = acc[e] * sc_old + w * v[u][e];
        pm = m_new;
      }
    }
    float A_m[E];
#pragma unroll
    for (int e = 0; e < E; ++e) A_m[e] = wsum > 0.f ? acc[e] / wsum : 0.f;
    const float lse_m = wsum > 0.f ? pm + logf(wsum) : -INFINITY;
    if (a.O_part) {
      int64_t pr = (((int64_t)beta * n_parts + m) * g.Hq + h) * a.q_len + j;
#pragma unroll
      for (int e = 0; e < E; ++e) a.O_part[pr * D + li * E + e] = A_m[e];
      if (li == 0) a.LSE_part[pr] = lse_m;
    }
    if (lse_m > -INFINITY) {
      float m_new = fmaxf(m_g, lse_m);
      float sc_old = expf(m_g - m_new);          // 0 on the first non-empty part
      float sc_new = expf(lse_m - m_new);
      if (sc_old != 1.f) {                       // the maximum moved: rescale sums and compensations
#pragma unroll
        for (int e = 0; e < E; ++e) { acc_g[e] *= sc_old; acc_c[e] *= sc_old; }
        l_g *= sc_old;
        l_c *= sc_old;
      }
#pragma unroll
      for (int e = 0; e < E; ++e) add_compensated(acc_g[e], acc_c[e], sc_new * A_m[e]);
      add_compensated(l_g, l_c, sc_new);
      m_g = m_new;
    }
  }
  const int64_t orow = ((int64_t)beta * a.q_len + j) * g.Hq + h;
  const int64_t arow = ((int64_t)beta * g.Hq + h) * a.q_len + j;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    float out = l_g > 0.f ? acc_g[e] / l_g : 0.f;
    if (a.A) a.A[arow * D + li * E + e] = out;
    if (!a.O) continue;
    if (a.out_bf16) ((unsigned short*)a.O)[orow * D + li * E + e] = f32_to_bf16_rne(out);
    else ((float*)a.O)[orow * D + li * E + e] = out;
  }
  if (a.LSE && li == 0) a.LSE[arow] = l_g > 0.f ? m_g + logf(l_g) : -INFINITY;
}

}  // namespace

hipError_t launch_merge(const MergeArgs& a, hipStream_t st) {
  const int64_t rows = (int64_t)a.g.B * a.g.Hq * a.q_len;
  if (rows > 0x7fffffff) return hipErrorInvalidValue;
  const SplitPlan& p = a.plan;
  // splits the largest part is made of
  const int per_part = p.flat ? p.s_total : (p.spb > p.st ? p.spb : p.st);
  if (per_part <= 8 && rows >= 64) {
    // many rows, few splits each: a row per 32 lanes
    const unsigned wgs = (unsigned)((rows + 7) / 8);
    if (a.g.d == 64) merge_rows_kernel<64, 4><<<dim3(wgs), 256, 0, st>>>(a, rows);
    else merge_rows_kernel<128, 4><<<dim3(wgs), 256, 0, st>>>(a, rows);
  } else if (a.g.d == 64) {
    merge_kernel<64, 8, 4><<<dim3((unsigned)rows), 256, 0, st>>>(a);
  } else if (p.flat != 0 && p.s_total > 32) {
    // decode: few rows, many splits each
    merge_kernel<128, 16, 8><<<dim3((unsigned)rows), 512, 0, st>>>(a);
  } else {
    merge_kernel<128, 8, 4><<<dim3((unsigned)rows), 256, 0, st>>>(a);
  }
  return hipGetLastError();
}

}  // namespace star
