// C-ABI entry points of libstarattn: argument validation, the phase-2 split
// plan, and kernel dispatch.  All checks run on the host before anything is
// enqueued; no exception or HIP error state leaves these functions.
#include "../../include/star_attn.h"
#include "star_internal.h"

#include <math.h>

#include <mutex>

namespace star {

// ---------------------------------------------------------------------------
// Per-device facts and the library's only state: static device memory that
// serves callers who hand in no workspace.
// ---------------------------------------------------------------------------
constexpr int MAX_DEVICES = 64;
constexpr int TICKET_SLOTS = 64;      // fallback sets of phase-1 work-queue counters

// Fallback work-queue counters of the bf16 phase-1 kernel (eight per launch),
// used only when star_attn_phase1* gets no workspace.  In host code the name is
// a stand-in: the device address comes from hipGetSymbolAddress, once per device
// (see device_state()).
static __device__ __align__(256) unsigned int phase1_ticket_slots[TICKET_SLOTS][8];

// Scratch of star_attn_phase2_static (per-split outputs and log-sum-exps), for
// callers that cannot bring a workspace.  Every GPU the library runs on holds
// its own copy until the process ends.  As above, host code uses the address
// hipGetSymbolAddress returns, never the name.
static __device__ __align__(256) unsigned char scratch[STAR_ATTN_STATIC_SCRATCH_BYTES];

struct DeviceState {
  bool ready = false;
  int n_cu = 0;
  unsigned int* tickets = nullptr;          // device address of phase1_ticket_slots on this device
  unsigned char* scratch_ptr = nullptr;     // device address of scratch on this device
  hipEvent_t slot_done[TICKET_SLOTS] = {};  // recorded behind the launch that last used a slot
  bool slot_used[TICKET_SLOTS] = {};
  bool slot_pending[TICKET_SLOTS] = {};     // taken by a call that has not recorded its event yet
  unsigned next_slot = 0;
};
static DeviceState g_dev[MAX_DEVICES];
static std::mutex g_dev_mu;

// State of the current device (looked up once per device), or null if the HIP
// runtime refuses.  Holds g_dev_mu only while it fills an entry.
static DeviceState* device_state() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
  DeviceState* d = &g_dev[dev];
  std::lock_guard<std::mutex> lock(g_dev_mu);
  if (d->ready) return d;
  if (hipDeviceGetAttribute(&d->n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      d->n_cu <= 0)
    return nullptr;
  if (hipGetSymbolAddress((void**)&d->tickets, HIP_SYMBOL(phase1_ticket_slots)) != hipSuccess ||
      hipGetSymbolAddress((void**)&d->scratch_ptr, HIP_SYMBOL(scratch)) != hipSuccess ||
      !d->tickets || !d->scratch_ptr)
    return nullptr;
  d->ready = true;
  return d;
}

// Compute units of the current device; the MI355X's 256 when no device can be
// asked (size queries still answer on a machine without a GPU).
int device_cu_count() {
  DeviceState* d = device_state();
  return d ? d->n_cu : 256;
}

// A free set of fallback counters of the current device: one whose last launch
// has finished.  -1 when all TICKET_SLOTS sets belong to launches still in flight.
static int acquire_ticket_slot(DeviceState* d) {
  std::lock_guard<std::mutex> lock(g_dev_mu);
  for (int k = 0; k < TICKET_SLOTS; ++k) {
    const int slot = (int)((d->next_slot + k) % TICKET_SLOTS);
    if (d->slot_pending[slot]) continue;       // another thread is between taking it and its launch
    if (d->slot_used[slot] && hipEventQuery(d->slot_done[slot]) != hipSuccess) {
      (void)hipGetLastError();          // hipErrorNotReady is an answer, not a failure
      continue;
    }
    if (!d->slot_done[slot] &&
        hipEventCreateWithFlags(&d->slot_done[slot], hipEventDisableTiming) != hipSuccess)
      return -1;
    d->slot_used[slot] = true;
    d->slot_pending[slot] = true;
    d->next_slot = (unsigned)(slot + 1);
    return slot;
  }
  return -1;
}

static int validate_shape(const star_attn_shape* s) {
  if (!s) return STAR_ATTN_ERR_NULL_POINTER;
  if (s->dtype != STAR_ATTN_F32 && s->dtype != STAR_ATTN_BF16) return STAR_ATTN_ERR_UNSUPPORTED_DTYPE;
  if (s->batch <= 0 || s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->head_dim <= 0 ||
      s->ctx_len <= 0 || s->block <= 0 || s->cache_capacity <= 0)
    return STAR_ATTN_ERR_INVALID_SHAPE;
  if (s->n_q_heads % s->n_kv_heads != 0) return STAR_ATTN_ERR_INVALID_SHAPE;
  if (s->n_q_heads > 65535 || s->batch > 65535) return STAR_ATTN_ERR_INVALID_SHAPE;
  // the kernels index tokens with 32-bit integers
  if (s->cache_capacity > (int64_t)0x7ff00000 || s->block > (int64_t)0x7ff00000)
    return STAR_ATTN_ERR_INVALID_SHAPE;
  if (s->dtype == STAR_ATTN_F32) {
    if (s->head_dim != 64 && s->head_dim != 128) return STAR_ATTN_ERR_UNSUPPORTED_HEAD_DIM;
  } else {
    if (s->head_dim != 128) return STAR_ATTN_ERR_UNSUPPORTED_HEAD_DIM;
  }
  if (s->anchor < 0 || s->anchor > s->block) return STAR_ATTN_ERR_ANCHOR_GT_BLOCK;
  if (s->cache_capacity < s->ctx_len) return STAR_ATTN_ERR_CACHE_OVERFLOW;
  if (!(s->softmax_scale >= 0.f) || isinf(s->softmax_scale)) return STAR_ATTN_ERR_INVALID_SHAPE;
  return STAR_ATTN_OK;
}

static Geom make_geom(const star_attn_shape* s) {
  Geom g;
  g.B = s->batch; g.Hq = s->n_q_heads; g.Hkv = s->n_kv_heads; g.G = g.Hq / g.Hkv; g.d = s->head_dim;
  g.L = s->ctx_len; g.b = s->block; g.a = s->anchor; g.cap = s->cache_capacity;
  g.scale = s->softmax_scale > 0.f ? s->softmax_scale : 1.0f / sqrtf((float)s->head_dim);
  return g;
}

static int64_t ceil_div(int64_t x, int64_t y) { return (x + y - 1) / y; }
static int64_t round_up(int64_t x, int64_t y) { return ceil_div(x, y) * y; }

// Workgroups of the decode kernel that are resident at once on the current
// device (256 CUs on an MI355X): one split each under a flat plan.
static int64_t decode_slots(const Geom& g, int64_t total) {
  return device_cu_count() * (int64_t)decode_workgroups_per_cu(decode_cache_resident(g, total));
}
static int64_t decode_slots_max() { return device_cu_count() * (int64_t)4; }

// Split plan for a phase-2 call with q_len new tokens that can see `total`
// cache rows.  Decode-sized calls (G * q_len rows fit one 16-column MFMA tile)
// stream the cache: without per-part outputs the keys of each (batch, KV head)
// are cut into equal splits, one per resident workgroup; with per-part outputs
// the splits respect block boundaries.  Larger calls are compute-bound and use
// as few splits as still fill the GPU.
static bool make_plan(const star_attn_shape* s, int64_t q_len, int64_t total, bool want_parts,
                      SplitPlan* p) {
  Geom g = make_geom(s);
  int64_t n = ceil_div(g.L, g.b);
  int64_t bmax = g.b < g.L ? g.b : g.L;
  int64_t tail_cap = g.cap - g.L;
  int64_t rows = (int64_t)g.G * q_len;
  p->decode = (s->dtype == STAR_ATTN_BF16 && rows <= 16) ? 1 : 0;
  p->flat = 0;
  p->n_blocks = (int32_t)n;
  if (n > (1 << 24)) return false;
  int64_t split_len;
  if (p->decode && !want_parts) {
    int64_t pairs = (int64_t)g.B * g.Hkv;
    int64_t slots = decode_slots(g, total);
    if (slots <= 0) return false;                  // no usable device
    int64_t s0 = slots / pairs > 1 ? slots / pairs : 1;
    split_len = round_up(ceil_div(total, s0), 32);
    if (split_len < 64) split_len = 64;
    p->flat = 1;
    p->split_len = split_len;
    p->spb = 0;
    p->st = 0;
    p->s_total = (int32_t)ceil_div(total, split_len);
    return true;
  }
  if (p->decode) {
    int64_t key_heads = g.cap * g.B * g.Hkv;
    int64_t want = ceil_div(key_heads, 2048);
    split_len = 256;
    while (split_len < want && split_len < 4096) split_len *= 2;
  } else {
    int64_t wgs;   // workgroups per split
    if (s->dtype == STAR_ATTN_F32) {
      wgs = (int64_t)g.B * g.Hq * ceil_div(q_len, 64);
    } else {
      wgs = (int64_t)g.B * g.Hkv * (g.G / flash_heads_per_workgroup(g.G)) *
            ceil_div(q_len, flash_tokens_per_workgroup(g.G));
    }
    // one thread walks a whole split in the fp32 kernel, so short calls are cut
    // much finer there (down to one 32-key LDS tile per split)
    const int64_t min_len = s->dtype == STAR_ATTN_F32 ? 32 : 256;
    const int64_t want_wgs = s->dtype == STAR_ATTN_F32 ? 4096 : 256;   // bf16: one workgroup per CU
    int64_t spb = ceil_div(want_wgs, wgs * n);
    int64_t spb_max = bmax / min_len > 1 ? bmax / min_len : 1;
    if (spb > spb_max) spb = spb_max;
    if (spb < 1) spb = 1;
    split_len = round_up(ceil_div(bmax, spb), s->dtype == STAR_ATTN_F32 ? 32 : 64);
  }
  int64_t spb = ceil_div(bmax, split_len);
  int64_t st = tail_cap > 0 ? ceil_div(tail_cap, split_len) : 1;
  int64_t s_total = n * spb + st;
  if (s_total > (1 << 24)) return false;
  p->split_len = split_len;
  p->spb = (int32_t)spb;
  p->st = (int32_t)st;
  p->s_total = (int32_t)s_total;
  return true;
}

static size_t plan_bytes(const star_attn_shape* s, const SplitPlan& p, int64_t q_len) {
  size_t rows = (size_t)s->batch * (size_t)p.s_total * (size_t)s->n_q_heads * (size_t)q_len;
  size_t bytes = rows * (size_t)(s->head_dim + 1) * sizeof(float);
  return (bytes + 255) & ~(size_t)255;
}

static bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

// Rotary embedding requested by the *_rope entry points (theta == 0: none).
struct Rope {
  double theta;
  int64_t pos0;
};

static int validate_rope(const star_attn_shape* s, double theta, int64_t pos0) {
  if (!(theta > 1.0) || isinf(theta) || pos0 < 0 || pos0 > ((int64_t)1 << 40))
    return STAR_ATTN_ERR_INVALID_SHAPE;
  (void)s;    // every supported head_dim is even
  return STAR_ATTN_OK;
}

// Bytes of one head-major copy of the external anchor (K or V), 256-byte padded.
static size_t anchor_copy_bytes(const star_attn_shape* s, int anchor_mode) {
  size_t es = s->dtype == STAR_ATTN_F32 ? 4 : 2;
  size_t anchors = anchor_mode == STAR_ATTN_ANCHOR_PER_BLOCK
                       ? (size_t)((s->ctx_len + s->block - 1) / s->block) : 1;
  size_t n = (size_t)s->batch * (size_t)s->n_kv_heads * anchors * (size_t)s->anchor *
             (size_t)s->head_dim * es;
  return (n + 255) & ~(size_t)255;
}

// Bytes the bf16 phase-1 kernel's eight work-queue counters take in a workspace.
constexpr size_t TICKET_BYTES = 256;

}  // namespace star

using namespace star;

extern "C" {

size_t star_attn_workspace_bytes(const star_attn_shape* shape, int64_t max_q_len) {
  if (validate_shape(shape) != STAR_ATTN_OK || max_q_len <= 0) return 0;
  // The plan depends on q_len only through the number of row tiles, so the
  // largest requirement is found at tile boundaries and at max_q_len itself.
  size_t best = 0;
  auto consider = [&](int64_t q) {
    if (q < 1 || q > max_q_len) return;
    for (int parts = 0; parts < 2; ++parts) {
      SplitPlan p;
      // the number of splits never exceeds what the full cache needs
      if (!make_plan(shape, q, shape->cache_capacity, parts != 0, &p)) continue;
      if (p.flat) {   // a shorter cache may need one split more than the full one; bound it
        int64_t pairs = (int64_t)shape->batch * shape->n_kv_heads;
        int64_t s0 = decode_slots_max() / pairs > 1 ? decode_slots_max() / pairs : 1;
        if (p.s_total < s0) p.s_total = (int32_t)s0;
      }
      size_t b = plan_bytes(shape, p, q);
      if (b > best) best = b;
    }
  };
  for (int64_t q = 1; q <= max_q_len && q <= 64; ++q) consider(q);
  for (int64_t q = 64; q <= max_q_len; q += 32) { consider(q); consider(q + 1); }
  consider(max_q_len);
  return best;
}

size_t star_attn_phase1_workspace_bytes(const star_attn_shape* shape, int anchor_mode) {
  if (validate_shape(shape) != STAR_ATTN_OK) return 0;
  if (shape->dtype == STAR_ATTN_BF16) return TICKET_BYTES;     // the launch's work-queue counters
  const bool given = anchor_mode == STAR_ATTN_ANCHOR_EXTERNAL ||
                     anchor_mode == STAR_ATTN_ANCHOR_PER_BLOCK ||
                     anchor_mode == STAR_ATTN_ANCHOR_ALL_BLOCKS;
  return given ? 2 * anchor_copy_bytes(shape, anchor_mode) : 0;
}

}  // extern "C"

// Phase 1 behind every public variant.  With `rope`, Q is rotated in place and K
// on its way into the cache.
static int phase1_impl(const star_attn_shape* shape, int anchor_mode, const Rope* rope, void* Q,
                       const void* K, const void* V, const void* K_anchor, const void* V_anchor,
                       void* O_ctx, float* LSE_ctx, void* K_cache, void* V_cache, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
  int rc = validate_shape(shape);
  if (rc != STAR_ATTN_OK) return rc;
  if (rope && (rc = validate_rope(shape, rope->theta, rope->pos0)) != STAR_ATTN_OK) return rc;
  if (anchor_mode != STAR_ATTN_ANCHOR_FIRST && anchor_mode != STAR_ATTN_ANCHOR_PREVIOUS &&
      anchor_mode != STAR_ATTN_ANCHOR_EXTERNAL && anchor_mode != STAR_ATTN_ANCHOR_PER_BLOCK &&
      anchor_mode != STAR_ATTN_ANCHOR_ALL_BLOCKS)
    return STAR_ATTN_ERR_INVALID_MODE;
  if (!Q || !K || !V || !O_ctx || !K_cache || !V_cache) return STAR_ATTN_ERR_NULL_POINTER;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O_ctx) ||
      misaligned(K_cache) || misaligned(V_cache) || ((uintptr_t)LSE_ctx & 3u))
    return STAR_ATTN_ERR_MISALIGNED;
  const bool ext = (anchor_mode == STAR_ATTN_ANCHOR_EXTERNAL ||
                    anchor_mode == STAR_ATTN_ANCHOR_PER_BLOCK ||
                    anchor_mode == STAR_ATTN_ANCHOR_ALL_BLOCKS) && shape->anchor > 0;
  // the fp32 kernel reads a head-major copy of the external anchor (workspace);
  // the bf16 kernel reads the caller's tensors directly
  const bool ext_copy = ext && shape->dtype == STAR_ATTN_F32;
  if (ext) {
    if (!K_anchor || !V_anchor) return STAR_ATTN_ERR_NULL_POINTER;
    if (misaligned(K_anchor) || misaligned(V_anchor)) return STAR_ATTN_ERR_MISALIGNED;
  }
  if (ext_copy) {
    if (!workspace) return STAR_ATTN_ERR_NULL_POINTER;
    if ((uintptr_t)workspace & 255u) return STAR_ATTN_ERR_MISALIGNED;
    if (workspace_bytes < 2 * anchor_copy_bytes(shape, anchor_mode))
      return STAR_ATTN_ERR_WORKSPACE_TOO_SMALL;
  }
  Geom g = make_geom(shape);
  hipStream_t st = (hipStream_t)hip_stream;
  // The bf16 kernel's workgroups draw their row tiles from eight counters: the
  // caller's workspace if there is one, else a free set of the library's own.
  DeviceState* ds = nullptr;
  unsigned int* tickets = nullptr;
  int slot = -1;
  if (shape->dtype == STAR_ATTN_BF16) {
    if (workspace) {
      if ((uintptr_t)workspace & 15u) return STAR_ATTN_ERR_MISALIGNED;
      if (workspace_bytes < TICKET_BYTES) return STAR_ATTN_ERR_WORKSPACE_TOO_SMALL;
    }
    if (!(ds = device_state())) return STAR_ATTN_ERR_LAUNCH_FAILED;
    if (workspace) {
      tickets = (unsigned int*)workspace;
    } else {
      // a captured launch would carry its set into every replay of the graph
      hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
      if (hipStreamIsCapturing(st, &cap) != hipSuccess) (void)hipGetLastError();
      if (cap != hipStreamCaptureStatusNone) return STAR_ATTN_ERR_BUSY;
      if ((slot = acquire_ticket_slot(ds)) < 0) return STAR_ATTN_ERR_BUSY;
      tickets = ds->tickets + 8 * slot;
    }
  }
  // On every way out: the set is free again once everything enqueued so far is
  // done.  A set whose event could not be recorded is never handed out again.
  struct SlotRelease {
    DeviceState* ds; int slot; hipStream_t st;
    ~SlotRelease() {
      if (slot < 0) return;
      if (hipEventRecord(ds->slot_done[slot], st) != hipSuccess) { (void)hipGetLastError(); return; }
      std::lock_guard<std::mutex> lock(g_dev_mu);
      ds->slot_pending[slot] = false;
    }
  } slot_release{ds, slot, st};
  // Algorithm 1: keep the K/V of every block once (anchor copies never exist here).
  // The bf16 attention kernel reads plain inputs where they are and files them in
  // the caches itself; rotated keys and the fp32 kernel go through the caches.
  const bool fused_cache_write = shape->dtype == STAR_ATTN_BF16 && !rope;
  if (fused_cache_write) {
    // nothing to launch here
  } else if (rope) {
    if (launch_rope_rotate(shape->dtype, g.B, g.L, g.Hq, g.d, rope->pos0, rope->theta, Q, Q, st) !=
            hipSuccess ||
        launch_rope_cache_write(g, shape->dtype, K, K_cache, g.L, 0, rope->pos0, rope->theta, st) !=
            hipSuccess ||
        launch_cache_write(g, shape->dtype, nullptr, V, K_cache, V_cache, g.L, 0, st) != hipSuccess)
      return STAR_ATTN_ERR_LAUNCH_FAILED;
  } else if (launch_cache_write(g, shape->dtype, K, V, K_cache, V_cache, g.L, 0, st) != hipSuccess) {
    return STAR_ATTN_ERR_LAUNCH_FAILED;
  }
  Phase1Args a;
  a.g = g; a.Q = Q; a.O = O_ctx; a.LSE = LSE_ctx; a.Kc = K_cache; a.Vc = V_cache;
  a.anchor_mode = anchor_mode; a.Ka = K_anchor; a.Va = V_anchor;
  a.Kin = fused_cache_write ? K : nullptr;
  a.Vin = fused_cache_write ? V : nullptr;
  a.tickets = tickets;
  a.n_cu = ds ? ds->n_cu : 0;
  if (ext_copy) {
    // the separately given anchors, head-major like the caches: [B, Hkv, n_anchor * a, d]
    // (the [B, n_anchor, a, Hkv, d] input is [B, n_anchor * a, Hkv, d] token-major)
    const int64_t rows = (anchor_mode == STAR_ATTN_ANCHOR_PER_BLOCK ? ceil_div(g.L, g.b) : 1) * g.a;
    Geom ga = g;
    ga.cap = rows;
    char* wk = (char*)workspace;
    char* wv = wk + anchor_copy_bytes(shape, anchor_mode);
    if (launch_cache_write(ga, shape->dtype, K_anchor, V_anchor, wk, wv, rows, 0, st) != hipSuccess)
      return STAR_ATTN_ERR_LAUNCH_FAILED;
    a.Ka = wk; a.Va = wv;
  }
  hipError_t e = shape->dtype == STAR_ATTN_F32 ? launch_phase1_f32(a, st) : launch_phase1_bf16(a, st);
  return e == hipSuccess ? STAR_ATTN_OK : STAR_ATTN_ERR_LAUNCH_FAILED;
}

extern "C" {

int star_attn_phase1_anchor(const star_attn_shape* shape, int anchor_mode, const void* Q,
                            const void* K, const void* V, const void* K_anchor,
                            const void* V_anchor, void* O_ctx, float* LSE_ctx, void* K_cache,
                            void* V_cache, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
  return phase1_impl(shape, anchor_mode, nullptr, const_cast<void*>(Q), K, V, K_anchor, V_anchor,
                     O_ctx, LSE_ctx, K_cache, V_cache, workspace, workspace_bytes, hip_stream);
}

int star_attn_phase1(const star_attn_shape* shape, const void* Q, const void* K, const void* V,
                     void* O_ctx, float* LSE_ctx, void* K_cache, void* V_cache,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
  return phase1_impl(shape, STAR_ATTN_ANCHOR_FIRST, nullptr, const_cast<void*>(Q), K, V, nullptr,
                     nullptr, O_ctx, LSE_ctx, K_cache, V_cache, workspace, workspace_bytes,
                     hip_stream);
}

int star_attn_phase1_rope(const star_attn_shape* shape, double rope_theta, int64_t pos0, void* Q,
                          const void* K, const void* V, void* O_ctx, float* LSE_ctx,
                          void* K_cache, void* V_cache, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  Rope rope = {rope_theta, pos0};
  return phase1_impl(shape, STAR_ATTN_ANCHOR_FIRST, &rope, Q, K, V, nullptr, nullptr, O_ctx,
                     LSE_ctx, K_cache, V_cache, workspace, workspace_bytes, hip_stream);
}

int star_attn_rope(const star_attn_shape* shape, int32_t n_heads, int64_t n_tokens, int64_t pos0,
                   double rope_theta, const void* X, void* Y, void* hip_stream) {
  int rc = validate_shape(shape);
  if (rc != STAR_ATTN_OK) return rc;
  if ((rc = validate_rope(shape, rope_theta, pos0)) != STAR_ATTN_OK) return rc;
  if (n_heads <= 0 || n_tokens <= 0) return STAR_ATTN_ERR_INVALID_SHAPE;
  if (!X || !Y) return STAR_ATTN_ERR_NULL_POINTER;
  if (misaligned(X) || misaligned(Y)) return STAR_ATTN_ERR_MISALIGNED;
  hipError_t e = launch_rope_rotate(shape->dtype, shape->batch, n_tokens, n_heads, shape->head_dim,
                                    pos0, rope_theta, X, Y, (hipStream_t)hip_stream);
  return e == hipSuccess ? STAR_ATTN_OK : STAR_ATTN_ERR_LAUNCH_FAILED;
}

}  // extern "C"

// Phase 2 behind every public variant.  With `rope`, Qq is rotated in place and
// Kq on its way into the cache (new token j sits at pos0 + cache_len + j).
// `pair` (a host's share of a call): the result is left as the fp32 pair
// (A, LSE) instead of O, and Kq == Vq == NULL means "append nothing, every new
// token sees cache rows [0, cache_len)".
static int phase2_impl(const star_attn_shape* shape, const Rope* rope, int64_t cache_len,
                       int64_t q_len, void* Qq, const void* Kq, const void* Vq, void* K_cache,
                       void* V_cache, float* O_part, float* LSE_part, void* O, bool pair, float* A,
                       float* LSE, void* workspace, size_t workspace_bytes, void* hip_stream,
                       bool static_scratch = false) {
  int rc = validate_shape(shape);
  if (rc != STAR_ATTN_OK) return rc;
  if (rope && (rc = validate_rope(shape, rope->theta, rope->pos0)) != STAR_ATTN_OK) return rc;
  if (q_len <= 0 || q_len > (1 << 20) || cache_len < shape->ctx_len) return STAR_ATTN_ERR_INVALID_SHAPE;
  const bool append = !(pair && !Kq && !Vq);
  const int64_t total = cache_len + (append ? q_len : 0);
  if (total > shape->cache_capacity) return STAR_ATTN_ERR_CACHE_OVERFLOW;
  if (static_scratch) workspace_bytes = STAR_ATTN_STATIC_SCRATCH_BYTES;
  if (!Qq || !K_cache || !V_cache || (!workspace && !static_scratch)) return STAR_ATTN_ERR_NULL_POINTER;
  if (append && (!Kq || !Vq)) return STAR_ATTN_ERR_NULL_POINTER;
  if (pair ? (!A || !LSE) : !O) return STAR_ATTN_ERR_NULL_POINTER;
  if ((O_part == nullptr) != (LSE_part == nullptr)) return STAR_ATTN_ERR_NULL_POINTER;
  if (misaligned(Qq) || misaligned(Kq) || misaligned(Vq) || misaligned(K_cache) ||
      misaligned(V_cache) || misaligned(O) || misaligned(O_part) || ((uintptr_t)LSE_part & 3u) ||
      misaligned(A) || ((uintptr_t)LSE & 3u) || ((uintptr_t)workspace & 255u))
    return STAR_ATTN_ERR_MISALIGNED;
  SplitPlan plan;
  if (!make_plan(shape, q_len, total, O_part != nullptr, &plan))
    return STAR_ATTN_ERR_INVALID_SHAPE;
  if (workspace_bytes < plan_bytes(shape, plan, q_len)) return STAR_ATTN_ERR_WORKSPACE_TOO_SMALL;
  Geom g = make_geom(shape);
  if ((int64_t)g.B * plan.s_total * ((q_len + 31) / 32) * g.Hq > (int64_t)0x7fffffff)
    return STAR_ATTN_ERR_INVALID_SHAPE;
  if (static_scratch) {
    // the current device's copy of the static array (its address was looked up
    // once, with that device current)
    DeviceState* ds = device_state();
    if (!ds) return STAR_ATTN_ERR_LAUNCH_FAILED;
    workspace = ds->scratch_ptr;
  }
  hipStream_t st = (hipStream_t)hip_stream;

  // Algorithm 2: the new tokens' K/V join the cache before they attend.  The
  // streaming decode kernel appends them itself (it reads the new rows from
  // Kq/Vq and writes them to the cache); the other paths use the cache writer.
  // Unrotated keys cannot take the fused route (the decode kernel moves rows with
  // DMAs): they are rotated into the cache first.
  const bool fused_append = append && shape->dtype == STAR_ATTN_BF16 && plan.decode && !rope;
  if (!append) {
    // a context host's share: the cache is read as it is
  } else if (rope) {
    const int64_t pos = rope->pos0 + cache_len;
    if (launch_rope_rotate(shape->dtype, g.B, q_len, g.Hq, g.d, pos, rope->theta, Qq, Qq, st) !=
            hipSuccess ||
        launch_rope_cache_write(g, shape->dtype, Kq, K_cache, q_len, cache_len, pos, rope->theta,
                                st) != hipSuccess ||
        launch_cache_write(g, shape->dtype, nullptr, Vq, K_cache, V_cache, q_len, cache_len, st) !=
            hipSuccess)
      return STAR_ATTN_ERR_LAUNCH_FAILED;
  } else if (!fused_append && launch_cache_write(g, shape->dtype, Kq, Vq, K_cache, V_cache, q_len,
                                                 cache_len, st) != hipSuccess) {
    return STAR_ATTN_ERR_LAUNCH_FAILED;
  }

  size_t rows = (size_t)g.B * plan.s_total * g.Hq * (size_t)q_len;
  Phase2Args a;
  a.g = g; a.plan = plan; a.cache_len = cache_len; a.q_len = (int32_t)q_len;
  a.causal = append ? 1 : 0;
  a.Qq = Qq; a.Kc = K_cache; a.Vc = V_cache;
  a.Kn = fused_append ? Kq : nullptr;
  a.Vn = fused_append ? Vq : nullptr;
  a.O_sub = (float*)workspace;
  a.LSE_sub = (float*)workspace + rows * g.d;
  hipError_t e;
  if (shape->dtype == STAR_ATTN_F32) e = launch_phase2_f32(a, st);
  else if (plan.decode) e = launch_phase2_decode_bf16(a, st);
  else e = launch_phase2_rows_bf16(a, st);
  if (e != hipSuccess) return STAR_ATTN_ERR_LAUNCH_FAILED;

  MergeArgs m;
  m.g = g; m.plan = plan; m.q_len = (int32_t)q_len; m.out_bf16 = shape->dtype == STAR_ATTN_BF16;
  m.O_sub = a.O_sub; m.LSE_sub = a.LSE_sub; m.O_part = O_part; m.LSE_part = LSE_part;
  m.batch_stride = (int64_t)plan.s_total * g.Hq * q_len;
  m.split_stride = (int64_t)g.Hq * q_len;
  m.O = pair ? nullptr : O;
  m.A = pair ? A : nullptr;
  m.LSE = pair ? LSE : nullptr;
  return launch_merge(m, st) == hipSuccess ? STAR_ATTN_OK : STAR_ATTN_ERR_LAUNCH_FAILED;
}

extern "C" {

int star_attn_phase2(const star_attn_shape* shape, int64_t cache_len, int64_t q_len,
                     const void* Qq, const void* Kq, const void* Vq,
                     void* K_cache, void* V_cache, float* O_part, float* LSE_part, void* O,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
  return phase2_impl(shape, nullptr, cache_len, q_len, const_cast<void*>(Qq), Kq, Vq, K_cache,
                     V_cache, O_part, LSE_part, O, false, nullptr, nullptr, workspace,
                     workspace_bytes, hip_stream);
}

int star_attn_phase2_static(const star_attn_shape* shape, int64_t cache_len, int64_t q_len,
                            const void* Qq, const void* Kq, const void* Vq, void* K_cache,
                            void* V_cache, void* O, void* hip_stream) {
  return phase2_impl(shape, nullptr, cache_len, q_len, const_cast<void*>(Qq), Kq, Vq, K_cache,
                     V_cache, nullptr, nullptr, O, false, nullptr, nullptr, nullptr, 0, hip_stream,
                     /*static_scratch=*/true);
}

int star_attn_phase2_partial(const star_attn_shape* shape, int64_t cache_len, int64_t q_len,
                             const void* Qq, const void* Kq, const void* Vq, void* K_cache,
                             void* V_cache, float* A, float* LSE, void* workspace,
                             size_t workspace_bytes, void* hip_stream) {
  if ((Kq == nullptr) != (Vq == nullptr)) return STAR_ATTN_ERR_NULL_POINTER;
  return phase2_impl(shape, nullptr, cache_len, q_len, const_cast<void*>(Qq), Kq, Vq, K_cache,
                     V_cache, nullptr, nullptr, nullptr, true, A, LSE, workspace, workspace_bytes,
                     hip_stream);
}

int star_attn_merge(const star_attn_shape* shape, int64_t n_parts, int64_t q_len,
                    const float* A_parts, const float* LSE_parts, void* O, float* A, float* LSE,
                    void* hip_stream) {
  int rc = validate_shape(shape);
  if (rc != STAR_ATTN_OK) return rc;
  if (n_parts <= 0 || n_parts > (1 << 20) || q_len <= 0 || q_len > (1 << 20))
    return STAR_ATTN_ERR_INVALID_SHAPE;
  if (!A_parts || !LSE_parts || (!O && !A)) return STAR_ATTN_ERR_NULL_POINTER;
  if (misaligned(A_parts) || ((uintptr_t)LSE_parts & 3u) || misaligned(O) || misaligned(A) ||
      ((uintptr_t)LSE & 3u))
    return STAR_ATTN_ERR_MISALIGNED;
  Geom g = make_geom(shape);
  const int64_t rows = (int64_t)g.B * g.Hq * q_len;
  if (rows > (int64_t)0x7fffffff || rows * n_parts > ((int64_t)1 << 40)) return STAR_ATTN_ERR_INVALID_SHAPE;
  MergeArgs m;
  m.g = g;
  m.plan = SplitPlan{0, 0, 0, 0, (int32_t)n_parts, 0, 1};    // one part made of n_parts splits
  m.q_len = (int32_t)q_len;
  m.out_bf16 = shape->dtype == STAR_ATTN_BF16;
  m.O_sub = A_parts; m.LSE_sub = LSE_parts;
  m.batch_stride = (int64_t)g.Hq * q_len;                    // [n_parts, B, Hq, q_len, d]
  m.split_stride = rows;
  m.O_part = nullptr; m.LSE_part = nullptr;
  m.O = O; m.A = A; m.LSE = LSE;
  return launch_merge(m, (hipStream_t)hip_stream) == hipSuccess ? STAR_ATTN_OK
                                                                : STAR_ATTN_ERR_LAUNCH_FAILED;
}

int star_attn_phase2_rope(const star_attn_shape* shape, double rope_theta, int64_t pos0,
                          int64_t cache_len, int64_t q_len, void* Qq, const void* Kq,
                          const void* Vq, void* K_cache, void* V_cache, float* O_part,
                          float* LSE_part, void* O, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  Rope rope = {rope_theta, pos0};
  return phase2_impl(shape, &rope, cache_len, q_len, Qq, Kq, Vq, K_cache, V_cache, O_part,
                     LSE_part, O, false, nullptr, nullptr, workspace, workspace_bytes, hip_stream);
}

const char* star_attn_status_string(int status) {
  switch (status) {
    case STAR_ATTN_OK: return "ok";
    case STAR_ATTN_ERR_INVALID_SHAPE: return "invalid shape";
    case STAR_ATTN_ERR_NULL_POINTER: return "required pointer is NULL";
    case STAR_ATTN_ERR_UNSUPPORTED_HEAD_DIM: return "unsupported head_dim";
    case STAR_ATTN_ERR_UNSUPPORTED_DTYPE: return "unsupported dtype";
    case STAR_ATTN_ERR_ANCHOR_GT_BLOCK: return "anchor outside [0, block]";
    case STAR_ATTN_ERR_CACHE_OVERFLOW: return "cache capacity exceeded";
    case STAR_ATTN_ERR_WORKSPACE_TOO_SMALL:
      return "workspace too small (star_attn_phase2_static: the call needs more than the static scratch)";
    case STAR_ATTN_ERR_LAUNCH_FAILED: return "kernel launch failed";
    case STAR_ATTN_ERR_MISALIGNED: return "pointer not sufficiently aligned";
    case STAR_ATTN_ERR_INVALID_MODE: return "unknown anchor mode";
    case STAR_ATTN_ERR_BUSY:
      return "no workspace given and the library's own work-queue counters are all in flight "
             "(or the stream is being captured)";
    default: return "unknown status";
  }
}

int star_attn_phase2_plan(const star_attn_shape* shape, int64_t cache_len, int64_t q_len,
                          int want_parts, star_attn_plan_info* out) {
  int rc = validate_shape(shape);
  if (rc != STAR_ATTN_OK) return rc;
  if (!out) return STAR_ATTN_ERR_NULL_POINTER;
  if (q_len <= 0 || q_len > (1 << 20) || cache_len < shape->ctx_len) return STAR_ATTN_ERR_INVALID_SHAPE;
  const int64_t total = cache_len + q_len;
  if (total > shape->cache_capacity) return STAR_ATTN_ERR_CACHE_OVERFLOW;
  SplitPlan plan;
  if (!make_plan(shape, q_len, total, want_parts != 0, &plan)) return STAR_ATTN_ERR_INVALID_SHAPE;
  const bool resident = decode_cache_resident(make_geom(shape), total);
  out->decode = plan.decode;
  out->flat = plan.flat;
  out->n_splits = plan.s_total;
  out->non_temporal = plan.decode && !resident ? 1 : 0;
  out->steps_per_batch = plan.decode ? (resident ? 1 : 2) : 0;
  out->reserved = 0;
  out->split_len = plan.split_len;
  out->workspace_bytes = (int64_t)plan_bytes(shape, plan, q_len);
  return STAR_ATTN_OK;
}

const char* star_attn_kernel_path(const star_attn_shape* shape) {
  if (validate_shape(shape) != STAR_ATTN_OK) return nullptr;
  return shape->dtype == STAR_ATTN_F32 ? "f32-valu" : "bf16-mfma";
}

}  // extern "C"
