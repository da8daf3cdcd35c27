/*
 * star_attn.h -- C ABI of the Star Attention hot path on one MI355X (gfx950).
 *
 * Star Attention (arXiv 2411.17116) runs long-context inference in two phases.
 * Phase 1 (Section 2.1, Algorithm 1, Figure 2) encodes the context with
 * block-local causal attention in which every block after the first is
 * prefixed by an anchor (the start of the first block); only the non-anchor
 * K/V is kept.  Phase 2 (Section 2.2, Eq. 1-4, Algorithm 2) lets query and
 * generated tokens attend to the whole cache: each cached part yields a local
 * attention output and the log of its softmax denominator, and the parts are
 * merged by rescaling with those log-sum-exp statistics.  star_attn_phase1 and
 * star_attn_phase2 treat the paper's context hosts as context blocks resident
 * on the one GPU; STAR_ATTN_ANCHOR_ALL_BLOCKS, star_attn_phase2_partial and
 * star_attn_merge are one host's share when the context is spread over several.
 *
 * Conventions
 *   - Every pointer is DEVICE memory owned by the caller unless it says "host".
 *     The library never allocates device memory, frees or keeps a pointer
 *     after a call returns.  The bf16 phase-1 kernel draws its row tiles from
 *     eight work-queue counters; they live in the call's workspace.  A caller
 *     that passes no workspace gets one of 64 sets in the library's static
 *     device memory instead (its only state): a set is handed out again only
 *     when the call that last used it has finished on the device, and a call
 *     that finds all 64 in flight -- or whose stream is being captured into a
 *     graph, where a set would be shared by every replay -- returns
 *     STAR_ATTN_ERR_BUSY without enqueueing anything.
 *   - Calls are asynchronous: work is enqueued on `hip_stream` (a hipStream_t
 *     passed as void*, NULL = the default stream) and the function returns
 *     without synchronising.  Calls on one stream run in order.
 *   - All tensors are contiguous, row-major, last index fastest.
 *   - dtype: STAR_ATTN_F32 (fp32 storage and arithmetic) or STAR_ATTN_BF16
 *     (bf16 storage, bf16 MFMA with fp32 accumulation and fp32 softmax).
 *     Partial outputs, LSE values and the workspace are always fp32.
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - All validation happens on the host before anything is enqueued: every
 *     error code but STAR_ATTN_ERR_LAUNCH_FAILED means no work was enqueued and
 *     no buffer was touched.  STAR_ATTN_ERR_LAUNCH_FAILED (the HIP runtime
 *     refused a kernel launch) may leave earlier kernels of the call on the
 *     stream, e.g. Q already rotated in place by a *_rope entry point.
 *   - Results are deterministic (no floating-point atomics).
 *   - Host threads: every entry point may be called from several threads at
 *     once (the per-device set-up and the hand-out of the static counter sets
 *     are behind a mutex); star_attn_phase2_static is the exception stated at
 *     its declaration, because its calls share one scratch buffer per GPU.
 */
#ifndef STAR_ATTN_H
#define STAR_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  STAR_ATTN_F32 = 0,
  STAR_ATTN_BF16 = 1
};

/* Status codes: 0 = success, negative = error. */
enum {
  STAR_ATTN_OK = 0,
  STAR_ATTN_ERR_INVALID_SHAPE = -1,        /* non-positive size, Hq % Hkv != 0, bad q_len/cache_len */
  STAR_ATTN_ERR_NULL_POINTER = -2,         /* a required pointer is NULL */
  STAR_ATTN_ERR_UNSUPPORTED_HEAD_DIM = -3, /* fp32: 64 or 128; bf16: 128 */
  STAR_ATTN_ERR_UNSUPPORTED_DTYPE = -4,
  STAR_ATTN_ERR_ANCHOR_GT_BLOCK = -5,      /* anchor outside [0, block] */
  STAR_ATTN_ERR_CACHE_OVERFLOW = -6,       /* ctx_len or cache_len + q_len exceeds cache_capacity */
  STAR_ATTN_ERR_WORKSPACE_TOO_SMALL = -7,
  STAR_ATTN_ERR_LAUNCH_FAILED = -8,        /* the HIP runtime refused a launch */
  STAR_ATTN_ERR_MISALIGNED = -9,           /* a tensor pointer is not 16-byte aligned */
  STAR_ATTN_ERR_INVALID_MODE = -10,        /* anchor_mode is none of STAR_ATTN_ANCHOR_* */
  STAR_ATTN_ERR_BUSY = -11                 /* bf16 phase 1 without a workspace: the library's own 64
                                              sets of work-queue counters all belong to launches
                                              still in flight, or the stream is being captured;
                                              pass a workspace (nothing was enqueued) */
};

/* What prefixes every context block after the first in phase 1. */
enum {
  STAR_ATTN_ANCHOR_FIRST = 0,     /* the method: the first a context tokens (Section 2.1) */
  STAR_ATTN_ANCHOR_PREVIOUS = 1,  /* ablation: the a tokens just before the block (Section 4.1) */
  STAR_ATTN_ANCHOR_EXTERNAL = 2,  /* ablation: anchor K/V handed in separately (Section 4.1) */
  STAR_ATTN_ANCHOR_PER_BLOCK = 3, /* ablation: a separately given anchor for every block, e.g. the
                                     first block encoded at position ids that follow the block */
  STAR_ATTN_ANCHOR_ALL_BLOCKS = 4 /* a context host's share (Algorithm 1): the call's context is a
                                     run of blocks that starts after the global first block, and
                                     the anchor handed in prefixes every one of them */
};

/* Problem shape; sizes in elements / tokens. */
typedef struct star_attn_shape {
  int32_t dtype;          /* STAR_ATTN_F32 or STAR_ATTN_BF16 */
  int32_t batch;          /* B  */
  int32_t n_q_heads;      /* Hq */
  int32_t n_kv_heads;     /* Hkv, divides Hq */
  int32_t head_dim;       /* d  */
  int32_t reserved;       /* set to 0 */
  int64_t ctx_len;        /* L: context tokens */
  int64_t block;          /* b >= 1: block size; n = ceil(L / b) blocks, the last may be short */
  int64_t anchor;         /* a in [0, b]: the first a context tokens prefix every block but the first */
  int64_t cache_capacity; /* rows per (batch, KV head) in the caches: >= L + every later append;
                             below 2^31 - 2^20 (as is block) */
  float   softmax_scale;  /* 0 selects 1/sqrt(d) (Eq. 1) */
  float   reserved2;      /* set to 0 */
} star_attn_shape;

/*
 * Bytes of device workspace star_attn_phase2 needs for calls with
 * q_len <= max_q_len (split-KV partial outputs and their log-sum-exps) on the
 * current device.  Returns 0 for an invalid shape.
 */
size_t star_attn_workspace_bytes(const star_attn_shape* shape, int64_t max_q_len);

/*
 * Phase 1: context encoding (Section 2.1; Algorithm 1; Figure 2).
 *
 * Context row p in block i = p / b (0-based) attends causally to
 *   keys [0, p]                      if i == 0,
 *   keys [0, a) and [i*b, p]         otherwise,
 * with logits scale * q.k and a softmax over exactly those keys.  Rows of the
 * anchor copies are not outputs and their K/V is never stored: the caches get
 * every context token exactly once.
 *
 *   Q        in   [B, L, Hq,  d]
 *   K, V     in   [B, L, Hkv, d]   (taken as post-RoPE; the anchor keeps its
 *                                   original positions, so one K serves both roles)
 *   O_ctx    out  [B, L, Hq, d]    same dtype as the inputs
 *   LSE_ctx  out  [B, Hq, L] fp32, natural log of each row's softmax
 *                 denominator of the scaled logits; may be NULL
 *   K_cache, V_cache  out  [B, Hkv, cache_capacity, d]; rows [0, L) are written,
 *                 the rest is left untouched
 *   workspace     bf16: at least star_attn_phase1_workspace_bytes(shape,
 *                 STAR_ATTN_ANCHOR_FIRST) bytes (256), 16-byte aligned; it holds the
 *                 launch's work-queue counters (cleared on the stream by the call,
 *                 contents are scratch afterwards), so calls with workspaces of their
 *                 own may overlap freely and may be captured into graphs.  NULL: the
 *                 library's own counters are used (see Conventions;
 *                 STAR_ATTN_ERR_BUSY when none is free).  fp32: unused.
 */
int star_attn_phase1(const star_attn_shape* shape,
                     const void* Q, const void* K, const void* V,
                     void* O_ctx, float* LSE_ctx,
                     void* K_cache, void* V_cache,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Phase 1 under the anchor variants of the ablation study (Section 4.1,
 * "Position and Content of Anchor Block"; Section 4.2 varies a).  Block 0 is
 * plain causal attention in every mode.  Context row p of block i >= 1 attends to
 *   STAR_ATTN_ANCHOR_FIRST     keys [0, a) and [i*b, p]   (== star_attn_phase1),
 *   STAR_ATTN_ANCHOR_PREVIOUS  keys [i*b - a, p]          (the previous block's
 *                              last a tokens serve as anchor),
 *   STAR_ATTN_ANCHOR_EXTERNAL  all a rows of K_anchor / V_anchor, then keys
 *                              [i*b, p] of K / V: the anchor's content, or the
 *                              position ids it was encoded with, differ from
 *                              the context's first tokens,
 *   STAR_ATTN_ANCHOR_PER_BLOCK all a rows of slice i of K_anchor / V_anchor, then
 *                              keys [i*b, p]: one anchor per block (position ids
 *                              "same as previous block" or sampled per block).
 *   STAR_ATTN_ANCHOR_ALL_BLOCKS  as EXTERNAL, and block 0 of the call is prefixed
 *                              as well: Algorithm 1 as it runs on a host that owns
 *                              blocks i0 .. i1-1 (i0 >= 1) of a longer context.  The
 *                              host passes its own tokens as Q / K / V (L = their
 *                              number), the first a tokens' K / V of the whole
 *                              context as the anchor, and keeps only its own
 *                              tokens' K / V, in its own caches.
 * a = 0 is "no anchor" in every mode.  The caches receive the context tokens
 * only, exactly as in star_attn_phase1.
 *
 *   K_anchor, V_anchor  in  [B, a, Hkv, d] (EXTERNAL, ALL_BLOCKS) or [B, n, a, Hkv, d] with
 *                 n = ceil(L / b) (PER_BLOCK; slice 0 is never read), dtype of the
 *                 inputs; read only in these modes with a > 0 (else may be NULL)
 *   workspace     at least star_attn_phase1_workspace_bytes(shape, mode) bytes,
 *                 256-byte aligned, scratch.  bf16: the work-queue counters, as in
 *                 star_attn_phase1 (NULL selects the library's own).  fp32:
 *                 a head-major copy of separately given anchors; unused and may be
 *                 NULL / 0 when that size is 0
 *   other arguments as in star_attn_phase1
 * Errors as in star_attn_phase1, plus STAR_ATTN_ERR_INVALID_MODE and
 * STAR_ATTN_ERR_WORKSPACE_TOO_SMALL.
 */
int star_attn_phase1_anchor(const star_attn_shape* shape, int anchor_mode,
                            const void* Q, const void* K, const void* V,
                            const void* K_anchor, const void* V_anchor,
                            void* O_ctx, float* LSE_ctx,
                            void* K_cache, void* V_cache,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* Workspace bytes of star_attn_phase1 / _anchor / _rope: 256 for bf16 (the launch's work-queue
 * counters), the anchor copies for separately given anchors in fp32, else 0; 0 for an invalid shape. */
size_t star_attn_phase1_workspace_bytes(const star_attn_shape* shape, int anchor_mode);

/*
 * Phase 2: query encoding or one decode step (Section 2.2; Eq. 1-4; Algorithm 2).
 *
 * The q_len new tokens' K/V are first appended at cache rows
 * [cache_len, cache_len + q_len); then new token j attends to cache rows
 * [0, cache_len + j] (all context keys, the earlier tail tokens, and itself).
 * The cache is processed as parts: part m < n is context block m
 * (rows [m*b, min((m+1)*b, L))), part n is the tail (rows [L, cache_len + j]).
 * Each part gives A_m (Eq. 1) and lse_m = log of Eq. 2; the result is
 * O = sum_m exp(lse_m - lse) A_m with lse = log sum_m exp(lse_m)  (Eq. 3-4).
 * Parts may be split further internally; what is exposed is per part.
 *
 *   cache_len  tokens already cached: L for the query call, then L + lq, ...
 *              (the caller advances it by q_len after each call); >= L
 *   Qq         in   [B, q_len, Hq,  d]
 *   Kq, Vq     in   [B, q_len, Hkv, d]
 *   K_cache, V_cache  in/out, layout as in phase 1
 *   O_part     out  [B, P, Hq, q_len, d] fp32, P = n + 1; may be NULL
 *   LSE_part   out  [B, P, Hq, q_len]    fp32 (-inf for an empty part); may be
 *              NULL; O_part and LSE_part must be both given or both NULL
 *   O          out  [B, q_len, Hq, d], dtype of the inputs
 *   workspace  at least star_attn_workspace_bytes(shape, q_len) bytes, 256-byte
 *              aligned; contents are scratch
 */
int star_attn_phase2(const star_attn_shape* shape,
                     int64_t cache_len, int64_t q_len,
                     const void* Qq, const void* Kq, const void* Vq,
                     void* K_cache, void* V_cache,
                     float* O_part, float* LSE_part,
                     void* O,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * star_attn_phase2 for callers that can neither allocate nor bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same computation, same kernels and the same bits as star_attn_phase2
 * without per-part outputs; the per-split pairs that call keeps in its workspace
 * go to a static device array of STAR_ATTN_STATIC_SCRATCH_BYTES inside the
 * library instead.  The call allocates and frees nothing (the array's device
 * address is looked up once per device, on the first call there).
 *
 *   - The scratch a call needs is star_attn_phase2_plan(...).workspace_bytes: at
 *     most 8.5 MB for any decode-sized call (G * q_len <= 16) on an MI355X, 0.2 to
 *     tens of MB for query encoding.  A call that needs more than
 *     STAR_ATTN_STATIC_SCRATCH_BYTES is refused with
 *     STAR_ATTN_ERR_WORKSPACE_TOO_SMALL before anything is enqueued.
 *   - Every call on a GPU shares that GPU's one array: calls on one stream run in
 *     order and are safe; calls that overlap on one GPU (two streams, two
 *     threads, two graphs replayed at once) race on it and give wrong results.
 *     Nothing in it has to start at zero and nothing in it survives a call.
 *   - Each GPU the process uses holds its own 16 MiB copy until the process ends.
 * Arguments and errors otherwise as in star_attn_phase2.
 */
#define STAR_ATTN_STATIC_SCRATCH_BYTES (16u << 20)

int star_attn_phase2_static(const star_attn_shape* shape,
                            int64_t cache_len, int64_t q_len,
                            const void* Qq, const void* Kq, const void* Vq,
                            void* K_cache, void* V_cache,
                            void* O, void* hip_stream);

/*
 * Phase 2 on one host of several (Section 2.2; Algorithm 2).
 *
 * When the cache is spread over hosts, the new tokens' queries go to every
 * host, each host returns the pair (A_h, log s_h) of Eq. 1-2 for its own cache,
 * and the query host combines the gathered pairs with Eq. 3-4.
 * star_attn_phase2_partial is one host's share of such a call and
 * star_attn_merge is the query host's aggregation; moving the pairs between
 * devices is the caller's business.  `shape` describes the HOST's share:
 * ctx_len = the context tokens its caches hold, cache_capacity = its caches' rows.
 *
 * star_attn_phase2_partial
 *   Kq, Vq     both NULL: a context host.  Nothing is appended and every new
 *              token attends to cache rows [0, cache_len), all visible.
 *              both given: the query host.  As in star_attn_phase2 they are
 *              appended at rows [cache_len, cache_len + q_len) and new token j
 *              attends to rows [0, cache_len + j].
 *   A          out  [B, Hq, q_len, d] fp32: local attention output (Eq. 1)
 *   LSE        out  [B, Hq, q_len] fp32: natural log of the softmax denominator
 *              of the scaled logits (log of Eq. 2)
 *   other arguments, workspace and errors as in star_attn_phase2
 *
 * star_attn_merge  (B, Hq, d and the dtype of O come from `shape`; its other
 *                   fields must be valid but are not used)
 *   n_parts    number of gathered pairs, >= 1
 *   A_parts    in   [n_parts, B, Hq, q_len, d] fp32 (one contiguous slab per host)
 *   LSE_parts  in   [n_parts, B, Hq, q_len] fp32; -inf marks a host that saw no
 *              key: its slab is not read and it contributes nothing
 *   O          out  [B, q_len, Hq, d] in the storage dtype; may be NULL if A is given
 *   A, LSE     out  the merged pair in fp32, layouts as above (for merging in
 *              stages); each may be NULL
 * Needs no workspace.  Pairs are folded in index order: deterministic.
 */
int star_attn_phase2_partial(const star_attn_shape* shape,
                             int64_t cache_len, int64_t q_len,
                             const void* Qq, const void* Kq, const void* Vq,
                             void* K_cache, void* V_cache,
                             float* A, float* LSE,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

int star_attn_merge(const star_attn_shape* shape, int64_t n_parts, int64_t q_len,
                    const float* A_parts, const float* LSE_parts,
                    void* O, float* A, float* LSE, void* hip_stream);

/*
 * Unrotated projections: rotary position embedding applied inside the calls.
 *
 * Section 2.1 fixes the position every token carries: context token t sits at
 * pos0 + t (the anchor therefore keeps positions pos0 .. pos0 + a - 1, and the
 * rotated key of an anchor token is the rotated key of that context token, so
 * one rotated K serves both roles); the j-th new token of a phase-2 call sits
 * at pos0 + cache_len + j.  The embedding is the one of the Llama family the
 * paper evaluates: dimension i < d/2 pairs with dimension i + d/2 and the pair
 * is turned by the angle pos * rope_theta^(-2i/d)
 *     y_i = x_i cos - x_(i+d/2) sin,   y_(i+d/2) = x_(i+d/2) cos + x_i sin.
 * Angles are evaluated in double precision; the rotation runs in fp32 and the
 * result is rounded once to the storage dtype.
 *
 * star_attn_phase1_rope / star_attn_phase2_rope are star_attn_phase1 /
 * star_attn_phase2 on unrotated Q and K:
 *   Q, Qq   in/out  rotated IN PLACE (on return they hold the rotated queries)
 *   K, Kq   in      unrotated; they are rotated on their way into K_cache, so
 *                   the cache holds rotated keys (what later calls attend to)
 *   rope_theta      base of the frequencies, > 1 (e.g. 10000, 500000)
 *   pos0            position of context token 0, >= 0
 * Every other argument, the outputs and the error codes are those of the plain
 * entry points; a rope_theta or pos0 out of range is STAR_ATTN_ERR_INVALID_SHAPE.
 *
 * star_attn_rope is the rotation alone: X [B, n_tokens, n_heads, d] -> Y (same
 * layout; Y may be X), token t at pos0 + t; B, d and dtype come from `shape`.
 * With it a caller can build the separately rotated anchor of the position-id
 * ablations (Section 4.1) for STAR_ATTN_ANCHOR_EXTERNAL.
 */
int star_attn_phase1_rope(const star_attn_shape* shape, double rope_theta, int64_t pos0,
                          void* Q, const void* K, const void* V,
                          void* O_ctx, float* LSE_ctx,
                          void* K_cache, void* V_cache,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

int star_attn_phase2_rope(const star_attn_shape* shape, double rope_theta, int64_t pos0,
                          int64_t cache_len, int64_t q_len,
                          void* Qq, const void* Kq, const void* Vq,
                          void* K_cache, void* V_cache,
                          float* O_part, float* LSE_part,
                          void* O,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

int star_attn_rope(const star_attn_shape* shape, int32_t n_heads, int64_t n_tokens, int64_t pos0,
                   double rope_theta, const void* X, void* Y, void* hip_stream);

/*
 * What a star_attn_phase2 call with these arguments would run (Section 2.2: how the
 * cache is cut into the pieces whose pairs (A, lse) of Eq. 1-2 are merged by Eq. 3-4).
 * For logs, benchmarks and tests that must know which kernel set-up they exercised.
 * `out` is HOST memory.  Returns a status code; nothing is enqueued.
 */
typedef struct star_attn_plan_info {
  int32_t decode;          /* 1: streaming split-KV kernel (G * q_len <= 16, bf16); 0: row-tiled kernel */
  int32_t flat;            /* 1: splits ignore part boundaries (only without per-part outputs) */
  int32_t n_splits;        /* splits per (batch, KV head) */
  int32_t non_temporal;    /* 1: the decode kernel reads the cache with non-temporal loads */
  int32_t steps_per_batch; /* decode kernel: 32-key steps loaded per batch (1 or 2); else 0 */
  int32_t reserved;
  int64_t split_len;       /* keys per split */
  int64_t workspace_bytes; /* bytes of workspace this very call uses */
} star_attn_plan_info;

int star_attn_phase2_plan(const star_attn_shape* shape, int64_t cache_len, int64_t q_len,
                          int want_parts, star_attn_plan_info* out);

/* Static, NUL-terminated description of a status code (host memory, never freed). */
const char* star_attn_status_string(int status);

/*
 * Name of the kernel path a shape would use ("f32-valu", "bf16-mfma"), for
 * logs and benchmarks; NULL for an unsupported shape.  Host memory, static.
 */
const char* star_attn_kernel_path(const star_attn_shape* shape);

#ifdef __cplusplus
}
#endif
#endif /* STAR_ATTN_H */
