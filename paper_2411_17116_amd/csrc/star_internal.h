// Internal declarations shared by the translation units of libstarattn.
// Nothing here is part of the public ABI (see include/star_attn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace star {

// ---------------------------------------------------------------------------
// Phase-2 split plan: every part of the cache (one per context block, plus the
// tail) is cut into `splits of split_len keys`; a split never straddles a part
// boundary, so per-part results can be rebuilt from whole splits.
// Split index s in [0, n_blocks * spb) is context block s / spb, piece s % spb;
// indices from n_blocks * spb on are pieces of the tail.
// ---------------------------------------------------------------------------
//
// A "flat" plan ignores part boundaries: with S = s_total splits, split s is the
// comb of 32-key steps s, s + S, s + 2S, ... of everything the call may see
// (split_len only sizes S).  It is used by decode-sized calls that do not ask
// for per-part outputs, where equal splits (one per resident workgroup) that
// sweep the cache together matter more than part boundaries.
struct SplitPlan {
  int64_t split_len;   // keys per split (multiple of 32)
  int32_t spb;         // splits per context block
  int32_t st;          // splits for the tail [L, cache_capacity)
  int32_t n_blocks;    // n = ceil(L / b)
  int32_t s_total;     // n_blocks * spb + st  (flat: number of splits)
  int32_t decode;      // 1: streaming split-KV kernel, 0: row-tiled kernel
  int32_t flat;        // 1: splits ignore part boundaries
};

// Geometry every kernel needs.  Strides are in elements.
struct Geom {
  int32_t B, Hq, Hkv, G, d;
  int64_t L, b, a, cap;
  float scale;          // softmax scale (natural units)
};

// What prefixes a context block after the first (values of the public
// STAR_ATTN_ANCHOR_* constants).
enum AnchorMode {
  ANCHOR_FIRST = 0, ANCHOR_PREVIOUS = 1, ANCHOR_EXTERNAL = 2, ANCHOR_PER_BLOCK = 3,
  ANCHOR_ALL_BLOCKS = 4   // the call is a host's share: its first block is prefixed too
};

struct Phase1Args {
  Geom g;
  const void* Q;        // [B, L, Hq, d]
  void* O;              // [B, L, Hq, d]
  float* LSE;           // [B, Hq, L] or null
  const void* Kc;       // caches [B, Hkv, cap, d], already holding the context
  const void* Vc;
  int32_t anchor_mode;  // AnchorMode
  const void* Ka;       // ANCHOR_EXTERNAL / ALL_BLOCKS / PER_BLOCK: anchor keys / values of n_anchor
  const void* Va;       // = 1 / 1 / n anchors; head-major [B, Hkv, n_anchor * a, d] for the fp32
                        // kernel, token-major [B, n_anchor, a, Hkv, d] for the bf16 one
  const void* Kin;      // bf16 kernel: the token-major inputs [B, L, Hkv, d] to read keys /
  const void* Vin;      // values from (and to file in the caches); null: read the caches
  unsigned int* tickets;  // bf16 kernel: this launch's eight work-queue counters (device memory)
  int32_t n_cu;           // bf16 kernel: compute units of the device the call runs on
};

// Anchor key rows [*lo, *hi) of 0-based block i, and whether they index the
// external anchor buffers (true; rows counted over all of a batch's anchors) or
// the context keys (false).  Block 0 has none, unless the call's context is a
// host's share that starts after the global first block (ANCHOR_ALL_BLOCKS).
__host__ __device__ inline bool anchor_range(const Geom& g, int mode, int64_t i, int64_t* lo,
                                             int64_t* hi) {
  if (g.a == 0 || (i == 0 && mode != ANCHOR_ALL_BLOCKS)) { *lo = 0; *hi = 0; return false; }
  if (mode == ANCHOR_PREVIOUS) { *lo = i * g.b - g.a; *hi = i * g.b; return false; }
  if (mode == ANCHOR_PER_BLOCK) { *lo = i * g.a; *hi = (i + 1) * g.a; return true; }
  *lo = 0; *hi = g.a;
  return mode == ANCHOR_EXTERNAL || mode == ANCHOR_ALL_BLOCKS;
}

struct Phase2Args {
  Geom g;
  SplitPlan plan;
  int64_t cache_len;    // tokens cached before this call
  int32_t q_len;
  int32_t causal;       // 1: the new tokens are appended and token j sees rows [0, cache_len + j];
                        // 0: nothing is appended and every token sees rows [0, cache_len)
  const void* Qq;       // [B, q_len, Hq, d]
  const void* Kn;       // new tokens' K, V [B, q_len, Hkv, d]; null: the caches already
  const void* Vn;       // hold them (decode kernel: nothing to append, read the caches)
  void* Kc;             // caches; the new tokens are already appended unless the
  void* Vc;             // kernel appends them itself (decode path)
  float* O_sub;         // [B, s_total, Hq, q_len, d]   per-split local attention
  float* LSE_sub;       // [B, s_total, Hq, q_len]      per-split log-sum-exp
};

// Cache rows a phase-2 call may see in all, and new token j's exclusive bound.
__host__ __device__ inline int64_t visible_total(const Phase2Args& a) {
  return a.cache_len + (a.causal ? a.q_len : 0);
}
__host__ __device__ inline int64_t visible_limit(const Phase2Args& a, int j) {
  return a.causal ? a.cache_len + j + 1 : a.cache_len;
}

// Split s of (batch beta, head h, token j) is row
//   beta * batch_stride + s * split_stride + h * q_len + j
// of O_sub (d floats per row) and LSE_sub.
struct MergeArgs {
  Geom g;
  SplitPlan plan;
  int32_t q_len;
  int32_t out_bf16;
  const float* O_sub;
  const float* LSE_sub;
  int64_t batch_stride;
  int64_t split_stride;
  float* O_part;        // [B, n+1, Hq, q_len, d] or null
  float* LSE_part;      // [B, n+1, Hq, q_len] or null
  void* O;              // [B, q_len, Hq, d] in the storage dtype, or null
  float* A;             // the same result in fp32, [B, Hq, q_len, d] (Eq. 1 of everything
  float* LSE;           // merged), and its log-sum-exp [B, Hq, q_len]; each may be null
};

// The streaming decode kernel runs in two set-ups.  K and V of a call that fit
// the 256 MB last-level cache with room to spare are found there by the next
// decode step: ordinary loads, one step per batch, four single-wavefront
// workgroups per CU.  Larger ones are used once per step and gone before the
// next: non-temporal loads, two steps per batch (256 registers), three per CU.
__host__ __device__ inline bool decode_cache_resident(const Geom& g, int64_t total_keys) {
  return 2 * (int64_t)g.B * g.Hkv * total_keys * g.d * 2 <= ((int64_t)192 << 20);
}
inline int decode_workgroups_per_cu(bool resident) { return resident ? 4 : 3; }

// Key range [lo, hi) of split s of a plan that is not flat (hi clipped to what
// exists for this call).
__host__ __device__ inline void split_range(const SplitPlan& p, int64_t L, int64_t b,
                                            int64_t total_keys, int s, int64_t* lo, int64_t* hi) {
  int n_ctx = p.n_blocks * p.spb;
  if (s < n_ctx) {
    int64_t m = s / p.spb, piece = s % p.spb;
    int64_t blo = m * b, bhi = (m + 1) * b < L ? (m + 1) * b : L;
    int64_t x = blo + piece * p.split_len;
    int64_t y = x + p.split_len;
    *lo = x < bhi ? x : bhi;
    *hi = y < bhi ? y : bhi;
  } else {
    int64_t x = L + (int64_t)(s - n_ctx) * p.split_len;
    int64_t y = x + p.split_len;
    *lo = x < total_keys ? x : total_keys;
    *hi = y < total_keys ? y : total_keys;
  }
}

// Row tiling of the bf16 row-tiled kernels: heads of one KV group that share a
// workgroup, and tokens per workgroup (the split plan sizes its grids with them).
int flash_heads_per_workgroup(int G);
int flash_tokens_per_workgroup(int G);

// Compute units of the current device (cached per device; 0 if the runtime refuses).
int device_cu_count();

// Host-side launchers (each returns the hipError_t of its launch).
// K and / or V (a null source is skipped) into rows [dst_row, dst_row + n_tokens).
hipError_t launch_cache_write(const Geom& g, int dtype, const void* K, const void* V,
                              void* Kc, void* Vc, int64_t n_tokens, int64_t dst_row,
                              hipStream_t st);
hipError_t launch_rope_rotate(int dtype, int B, int64_t n_tokens, int H, int d, int64_t pos0,
                              double theta, const void* X, void* Y, hipStream_t st);
hipError_t launch_rope_cache_write(const Geom& g, int dtype, const void* K, void* Kc,
                                   int64_t n_tokens, int64_t dst_row, int64_t pos0, double theta,
                                   hipStream_t st);
hipError_t launch_phase1_f32(const Phase1Args& a, hipStream_t st);
hipError_t launch_phase2_f32(const Phase2Args& a, hipStream_t st);
hipError_t launch_phase1_bf16(const Phase1Args& a, hipStream_t st);
hipError_t launch_phase2_rows_bf16(const Phase2Args& a, hipStream_t st);
hipError_t launch_phase2_decode_bf16(const Phase2Args& a, hipStream_t st);
hipError_t launch_merge(const MergeArgs& a, hipStream_t st);

}  // namespace star
