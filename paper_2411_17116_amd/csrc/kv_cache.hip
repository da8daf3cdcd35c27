// KV-cache writer: Algorithm 1 keeps the K/V of every context block and drops
// the anchor copies, i.e. the cache holds each context token exactly once;
// Algorithm 2 appends the new tokens' K/V before they attend.  Both are the same
// layout change, token-major [B, T, Hkv, d] -> head-major [B, Hkv, cap, d], so a
// key tile of one KV head is one contiguous run of bytes for the attention
// kernels.  Pure HBM copy: 16 bytes per lane, reads fully contiguous, writes
// contiguous per (token, head) row.
#include "star_internal.h"

namespace star {

typedef __attribute__((ext_vector_type(4))) int i32x4;

__global__ __launch_bounds__(256) void cache_write_kernel(
    const i32x4* __restrict__ K, const i32x4* __restrict__ V,
    i32x4* __restrict__ Kc, i32x4* __restrict__ Vc,
    int64_t n_vec, int64_t n_tokens, int Hkv, int vpr, int64_t cap, int64_t dst_row) {
  const i32x4* src = blockIdx.y == 0 ? K : V;
  i32x4* dst = blockIdx.y == 0 ? Kc : Vc;
  if (src == nullptr) return;                 // this tensor is written elsewhere
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n_vec; v += stride) {
    int64_t row = v / vpr;            // (beta, t, g) flattened
    int c = (int)(v - row * vpr);
    int g = (int)(row % Hkv);
    int64_t bt = row / Hkv;
    int64_t t = bt % n_tokens;
    int64_t beta = bt / n_tokens;
    int64_t o = ((beta * Hkv + g) * cap + dst_row + t) * vpr + c;
    dst[o] = src[v];
  }
}

hipError_t launch_cache_write(const Geom& g, int dtype, const void* K, const void* V,
                              void* Kc, void* Vc, int64_t n_tokens, int64_t dst_row,
                              hipStream_t st) {
  int es = dtype == 0 ? 4 : 2;
  int vpr = g.d * es / 16;
  int64_t n_vec = (int64_t)g.B * n_tokens * g.Hkv * vpr;
  if (n_vec == 0) return hipSuccess;
  int64_t blocks = (n_vec + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  dim3 grid((unsigned)blocks, 2, 1);
  cache_write_kernel<<<grid, 256, 0, st>>>((const i32x4*)K, (const i32x4*)V, (i32x4*)Kc,
                                           (i32x4*)Vc, n_vec, n_tokens, g.Hkv, vpr, g.cap,
                                           dst_row);
  return hipGetLastError();
}

}  // namespace star
