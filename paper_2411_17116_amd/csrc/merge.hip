// LSE merge (Eq. 3-4; Algorithm 2's running update): combines the per-split
// local attention outputs A_s and log-sum-exps lse_s of one query row into the
// global attention output,
//     lse = log sum_s exp(lse_s),   O = sum_s exp(lse_s - lse) A_s.
// Splits are first folded into their part (context block or tail) so that the
// per-part pair (A_m, lse_m) the paper's hosts would exchange can be written
// out; the parts are then folded in index order with the online-softmax update
//     lse' = logaddexp(lse, lse_m),  O' = exp(lse - lse') O + exp(lse_m - lse') A_m,
// which is what Eq. 3-4 evaluate to.  An empty split or part has lse = -inf and
// weight 0.  The order of the folds is fixed, so results are deterministic.
//
// One workgroup per (batch, head, row); thread t owns output element t.
// Traffic is s_total * (d + 1) floats per row -- negligible next to the cache.
#include "star_internal.h"

namespace star {

namespace {

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f) {
  unsigned int u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

__global__ void merge_kernel(MergeArgs a) {
  const Geom& g = a.g;
  const int d = g.d;
  int t = threadIdx.x;
  int64_t row = blockIdx.x;                 // (beta, h, j), j fastest
  int j = (int)(row % a.q_len);
  int h = (int)((row / a.q_len) % g.Hq);
  int beta = (int)(row / ((int64_t)a.q_len * g.Hq));
  const SplitPlan& p = a.plan;
  int64_t sub_stride = (int64_t)g.Hq * a.q_len;                       // rows between splits
  int64_t base = ((int64_t)beta * p.s_total * g.Hq + h) * a.q_len + j; // split 0
  int n_parts = p.n_blocks + 1;

  float m_g = -INFINITY, l_g = 0.f, acc_g = 0.f;
  for (int m = 0; m < n_parts; ++m) {
    int s_lo = m < p.n_blocks ? m * p.spb : p.n_blocks * p.spb;
    int s_hi = m < p.n_blocks ? s_lo + p.spb : p.s_total;
    float pm = -INFINITY;
    for (int s = s_lo; s < s_hi; ++s) pm = fmaxf(pm, a.LSE_sub[base + s * sub_stride]);
    float A_m = 0.f, lse_m = -INFINITY;
    if (pm > -INFINITY) {
      float wsum = 0.f, acc = 0.f;
      for (int s = s_lo; s < s_hi; ++s) {
        float ls = a.LSE_sub[base + s * sub_stride];
        if (ls == -INFINITY) continue;
        float w = expf(ls - pm);
        wsum += w;
        acc = __builtin_fmaf(w, a.O_sub[(base + s * sub_stride) * d + t], acc);
      }
      A_m = acc / wsum;
      lse_m = pm + logf(wsum);
    }
    if (a.O_part) {
      int64_t pr = (((int64_t)beta * n_parts + m) * g.Hq + h) * a.q_len + j;
      a.O_part[pr * d + t] = A_m;
      if (t == 0) a.LSE_part[pr] = lse_m;
    }
    if (lse_m > -INFINITY) {
      float m_new = fmaxf(m_g, lse_m);
      float sc_old = expf(m_g - m_new);     // 0 on the first non-empty part
      float sc_new = expf(lse_m - m_new);
      acc_g = acc_g * sc_old + sc_new * A_m;
      l_g = l_g * sc_old + sc_new;
      m_g = m_new;
    }
  }
  float out = l_g > 0.f ? acc_g / l_g : 0.f;
  int64_t orow = ((int64_t)beta * a.q_len + j) * g.Hq + h;
  if (a.out_bf16) ((unsigned short*)a.O)[orow * d + t] = f32_to_bf16_rne(out);
  else ((float*)a.O)[orow * d + t] = out;
}

}  // namespace

hipError_t launch_merge(const MergeArgs& a, hipStream_t st) {
  int64_t rows = (int64_t)a.g.B * a.g.Hq * a.q_len;
  merge_kernel<<<dim3((unsigned)rows), dim3((unsigned)a.g.d), 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace star
