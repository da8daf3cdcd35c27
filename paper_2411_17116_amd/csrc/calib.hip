// Calibration kernels for the benchmark (libstarcalib.so; not part of the
// product library and never called by it): what this machine sustains for the
// two resources the hot path is priced against.
//   * star_calib_mfma: nothing but independent v_mfma_f32_16x16x32_bf16 on
//     register operands, two wavefronts per SIMD on every CU.  Run for a second
//     or so it shows the MFMA rate the chip holds at its power limit; the rate
//     depends on how much the operand bits toggle (constant operands run near
//     the nominal peak, random ones well below).
//   * star_calib_hbm_read: a grid-stride read of a buffer, 16 bytes per lane,
//     with ordinary or non-temporal loads: the ceiling for a kernel that streams
//     the KV cache once.
//   * star_calib_coexec: four wavefronts of a workgroup (one per SIMD) issue
//     MFMAs only, the other four (their SIMD neighbours) the VALU mix of an
//     attention softmax (9 multiply-adds and 4 exponentials per 8 MFMAs' worth of
//     scores); each wavefront reports its own cycle count.  Run with either group
//     alone and with both it shows how much of the two streams a SIMD executes at
//     the same time.
// All enqueue one kernel on the given stream; the caller times it (or reads the
// cycle counts).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int CALIB_WGS = 256;        // one workgroup per CU
constexpr int CALIB_THREADS = 512;    // 8 wavefronts: two per SIMD
constexpr int SEED_VECS = 4096;       // 64 KiB of operand bits

__global__ __launch_bounds__(CALIB_THREADS) void mfma_kernel(const u32x4* __restrict__ seed,
                                                             float* __restrict__ out, int iters) {
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = __builtin_bit_cast(bf16x8, seed[(threadIdx.x * 8 + i) % SEED_VECS]);
    b[i] = __builtin_bit_cast(bf16x8, seed[(threadIdx.x * 8 + i + SEED_VECS / 2) % SEED_VECS]);
  }
  f32x4 c[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) c[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      c[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[(i + 3) & 7], c[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += c[i][0] + c[i][1] + c[i][2] + c[i][3];
  out[blockIdx.x * CALIB_THREADS + threadIdx.x] = s;
}

template <bool NT>
__global__ __launch_bounds__(256) void read_kernel(const u32x4* __restrict__ src, size_t n_vec,
                                                   unsigned* __restrict__ out) {
  u32x4 acc = {0u, 0u, 0u, 0u};
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride)
    acc ^= NT ? __builtin_nontemporal_load(src + i) : src[i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}

constexpr int READ_WGS = 256 * 8;

// mode bit 0: wavefronts 0-3 run 8 independent MFMAs per iteration; bit 1:
// wavefronts 4-7 run 9 fused multiply-adds and 4 exponentials per iteration.
// cycles[8 * workgroup + wavefront] = shader clocks the wavefront's loop took.
__global__ __launch_bounds__(CALIB_THREADS) void coexec_kernel(float* __restrict__ out,
                                                               long long* __restrict__ cycles,
                                                               int iters, int mode, float seed) {
  const int wave = threadIdx.x >> 6;
  const long long t0 = clock64();
  float r = 0.f;
  if (wave < 4 && (mode & 1)) {
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a[i] = (__bf16)(seed + i + threadIdx.x);
      b[i] = (__bf16)(seed * i - threadIdx.x);
    }
    f32x4 c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 8; ++i) c[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) r += c[i][0] + c[i][1] + c[i][2] + c[i][3];
  } else if (wave >= 4 && (mode & 2)) {
    float x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = seed * (i + 1) + threadIdx.x * 1e-3f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int u = 0; u < 9; ++u) x[u & 7] = __builtin_fmaf(x[u & 7], 0.999f, 0.001f);
#pragma unroll
      for (int u = 0; u < 4; ++u) x[u] = __builtin_amdgcn_exp2f(x[u]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) r += x[i];
  }
  const long long t1 = clock64();
  out[blockIdx.x * CALIB_THREADS + threadIdx.x] = r;
  if ((threadIdx.x & 63) == 0) cycles[blockIdx.x * 8 + wave] = t1 - t0;
}

}  // namespace

extern "C" {

// Bytes of operand seed star_calib_mfma reads, and floats / words of output the
// two kernels write (device buffers the caller provides).
size_t star_calib_seed_bytes(void) { return (size_t)SEED_VECS * 16; }
size_t star_calib_out_words(void) {
  size_t a = (size_t)CALIB_WGS * CALIB_THREADS, b = (size_t)READ_WGS * 256;
  return a > b ? a : b;
}

// Flops one star_calib_mfma launch performs.
double star_calib_mfma_flops(int iters) {
  return (double)CALIB_WGS * (CALIB_THREADS / 64) * (double)iters * 8.0 * (2.0 * 16 * 16 * 32);
}

int star_calib_mfma(const void* seed, void* out, int iters, void* hip_stream) {
  if (!seed || !out || iters <= 0) return -1;
  mfma_kernel<<<CALIB_WGS, CALIB_THREADS, 0, (hipStream_t)hip_stream>>>((const u32x4*)seed,
                                                                        (float*)out, iters);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}

// nontemporal != 0: the loads carry the non-temporal hint (data used once).
// cycles: CALIB_WGS * 8 int64 (device).  mode: 1 = MFMA wavefronts only, 2 = VALU
// wavefronts only, 3 = both.
size_t star_calib_coexec_cycle_words(void) { return (size_t)CALIB_WGS * 8; }
int star_calib_coexec(void* out, void* cycles, int iters, int mode, void* hip_stream) {
  if (!out || !cycles || iters <= 0 || mode < 1 || mode > 3) return -1;
  coexec_kernel<<<CALIB_WGS, CALIB_THREADS, 0, (hipStream_t)hip_stream>>>(
      (float*)out, (long long*)cycles, iters, mode, 0.5f);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}

int star_calib_hbm_read(const void* src, size_t bytes, int nontemporal, void* out, void* hip_stream) {
  if (!src || !out || bytes < 16 || ((uintptr_t)src & 15u)) return -1;
  hipStream_t st = (hipStream_t)hip_stream;
  if (nontemporal) read_kernel<true><<<READ_WGS, 256, 0, st>>>((const u32x4*)src, bytes / 16, (unsigned*)out);
  else read_kernel<false><<<READ_WGS, 256, 0, st>>>((const u32x4*)src, bytes / 16, (unsigned*)out);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}

}  // extern "C"
