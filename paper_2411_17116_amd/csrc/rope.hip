// Rotary position embedding for projections that arrive unrotated.
//
// Section 2.1 fixes the position every token carries (a context token keeps its
// index, the anchor keeps 0..a-1, a new token of phase 2 sits behind the cache),
// so the rotated key of an anchor token is the rotated key of that context token
// and one rotated K serves both roles.  The embedding itself is the one of the
// Llama family the paper evaluates: dimension i < d/2 pairs with i + d/2 and the
// pair is turned by pos * theta^(-2i/d).
//
// Two kernels, both pure HBM streams (16 bytes per access):
//   * rope_rotate_kernel      X [B, T, H, d] -> Y [B, T, H, d] (Y may be X),
//   * rope_cache_write_kernel K [B, T, Hkv, d] -> K cache [B, Hkv, cap, d]: the
//     layout change of the cache writer with the rotation applied on the way.
// A thread owns one (token, group of 16-byte chunk pairs): it evaluates the
// angles once -- in double precision, because pos * frequency reaches 1e6 rad
// and fp32 cannot hold its fractional turn -- and reuses the sines and cosines
// for every head of the token.
#include "star_internal.h"

namespace star {

namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

template <typename T> struct Chunk;
template <> struct Chunk<float> {
  static constexpr int N = 4;
  typedef f32x4 vec;
  static __device__ __forceinline__ void load(const void* p, float (&x)[4]) {
    f32x4 v = *(const f32x4*)p;
    x[0] = v[0]; x[1] = v[1]; x[2] = v[2]; x[3] = v[3];
  }
  static __device__ __forceinline__ void store(void* p, const float (&x)[4]) {
    *(f32x4*)p = f32x4{x[0], x[1], x[2], x[3]};
  }
};
template <> struct Chunk<__bf16> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void load(const void* p, float (&x)[8]) {
    bf16x8 v = *(const bf16x8*)p;
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = (float)v[e];
  }
  static __device__ __forceinline__ void store(void* p, const float (&x)[8]) {
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (__bf16)x[e];      // round to nearest even
    *(bf16x8*)p = v;
  }
};

// cos and sin of pos * theta^(-2i/d), i = i0 .. i0 + N - 1
template <int N>
__device__ __forceinline__ void angles(int64_t pos, int i0, int d, double log2_theta,
                                       float (&cs)[N], float (&sn)[N]) {
  const double TWO_PI = 6.283185307179586476925, INV_TWO_PI = 0.1591549430918953357689;
#pragma unroll
  for (int e = 0; e < N; ++e) {
    double inv_freq = exp2(-2.0 * (double)(i0 + e) / (double)d * log2_theta);
    double ang = (double)pos * inv_freq;
    double r = fma(-rint(ang * INV_TWO_PI), TWO_PI, ang);     // |r| <= pi
    double s, c;
    sincos(r, &s, &c);
    cs[e] = (float)c;
    sn[e] = (float)s;
  }
}

// Rows are [batch, token, head, d]; dst_row_stride / dst_head_stride describe
// where (batch, token, head) lands in the destination, in elements.
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(const T* X, T* Y, int64_t n_tokens,
                                                   int H, int d, int64_t pos0, double log2_theta,
                                                   int64_t dst_batch_stride, int64_t dst_token_stride,
                                                   int64_t dst_head_stride, int64_t n_threads) {
  constexpr int N = Chunk<T>::N;
  const int cpr = d / 2 / N;                       // chunk pairs per row
  int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= n_threads) return;
  int c = (int)(id % cpr);
  int64_t bt = id / cpr;
  int64_t t = bt % n_tokens, beta = bt / n_tokens;
  float cs[N], sn[N];
  angles<N>(pos0 + t, c * N, d, log2_theta, cs, sn);
  const T* src = X + (bt * H) * (int64_t)d + c * N;
  T* dst = Y + beta * dst_batch_stride + t * dst_token_stride + c * N;
  for (int h = 0; h < H; ++h) {
    float lo[N], hi[N], ylo[N], yhi[N];
    Chunk<T>::load(src + (int64_t)h * d, lo);
    Chunk<T>::load(src + (int64_t)h * d + d / 2, hi);
#pragma unroll
    for (int e = 0; e < N; ++e) {
      ylo[e] = lo[e] * cs[e] - hi[e] * sn[e];
      yhi[e] = hi[e] * cs[e] + lo[e] * sn[e];
    }
    Chunk<T>::store(dst + h * dst_head_stride, ylo);
    Chunk<T>::store(dst + h * dst_head_stride + d / 2, yhi);
  }
}

template <typename T>
hipError_t launch(const void* X, void* Y, int B, int64_t n_tokens, int H, int d, int64_t pos0,
                  double theta, int64_t sb, int64_t st_, int64_t sh, hipStream_t st) {
  int cpr = d / 2 / Chunk<T>::N;
  int64_t n_threads = (int64_t)B * n_tokens * cpr;
  if (n_threads == 0) return hipSuccess;
  int64_t blocks = (n_threads + 255) / 256;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  rope_kernel<T><<<dim3((unsigned)blocks), 256, 0, st>>>((const T*)X, (T*)Y, n_tokens, H, d, pos0,
                                                         log2(theta), sb, st_, sh, n_threads);
  return hipGetLastError();
}

}  // namespace

// X [B, n_tokens, H, d] -> Y, same layout (Y may alias X), token t at pos0 + t.
hipError_t launch_rope_rotate(int dtype, int B, int64_t n_tokens, int H, int d, int64_t pos0,
                              double theta, const void* X, void* Y, hipStream_t st) {
  int64_t sh = d, stk = (int64_t)H * d, sb = n_tokens * stk;
  return dtype == 0 ? launch<float>(X, Y, B, n_tokens, H, d, pos0, theta, sb, stk, sh, st)
                    : launch<__bf16>(X, Y, B, n_tokens, H, d, pos0, theta, sb, stk, sh, st);
}

// K [B, n_tokens, Hkv, d] -> rows [dst_row, dst_row + n_tokens) of the head-major
// cache [B, Hkv, cap, d], token t rotated at pos0 + t.
hipError_t launch_rope_cache_write(const Geom& g, int dtype, const void* K, void* Kc,
                                   int64_t n_tokens, int64_t dst_row, int64_t pos0, double theta,
                                   hipStream_t st) {
  int64_t sh = g.cap * g.d, stk = g.d, sb = (int64_t)g.Hkv * g.cap * g.d;
  size_t es = dtype == 0 ? 4 : 2;
  void* dst = (char*)Kc + (size_t)dst_row * g.d * es;
  return dtype == 0 ? launch<float>(K, dst, g.B, n_tokens, g.Hkv, g.d, pos0, theta, sb, stk, sh, st)
                    : launch<__bf16>(K, dst, g.B, n_tokens, g.Hkv, g.d, pos0, theta, sb, stk, sh, st);
}

}  // namespace star
