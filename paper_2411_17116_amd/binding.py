"""ctypes binding of libstarattn.so (see include/star_attn.h for the contract)."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

F32 = 0
BF16 = 1
ANCHOR_FIRST = 0
ANCHOR_PREVIOUS = 1
ANCHOR_EXTERNAL = 2
ANCHOR_PER_BLOCK = 3
ANCHOR_ALL_BLOCKS = 4

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class StarAttnError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"star_attn: {what} (status {code})")
        self.code = code


class StarShape(ctypes.Structure):
    """Mirror of `star_attn_shape`."""
    _fields_ = [
        ("dtype", ctypes.c_int32), ("batch", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("ctx_len", ctypes.c_int64), ("block", ctypes.c_int64), ("anchor", ctypes.c_int64),
        ("cache_capacity", ctypes.c_int64),
        ("softmax_scale", ctypes.c_float), ("reserved2", ctypes.c_float),
    ]

    @classmethod
    def make(cls, dtype, batch, n_q_heads, n_kv_heads, head_dim, ctx_len, block, anchor,
             cache_capacity, softmax_scale=0.0) -> "StarShape":
        if isinstance(dtype, torch.dtype):
            dtype = {torch.float32: F32, torch.bfloat16: BF16}.get(dtype, -1)
        elif isinstance(dtype, str):
            dtype = {"fp32": F32, "bf16": BF16}.get(dtype, -1)
        return cls(int(dtype), int(batch), int(n_q_heads), int(n_kv_heads), int(head_dim), 0,
                   int(ctx_len), int(block), int(anchor), int(cache_capacity),
                   float(softmax_scale), 0.0)


class PlanInfo(ctypes.Structure):
    """Mirror of `star_attn_plan_info`."""
    _fields_ = [
        ("decode", ctypes.c_int32), ("flat", ctypes.c_int32), ("n_splits", ctypes.c_int32),
        ("non_temporal", ctypes.c_int32), ("steps_per_batch", ctypes.c_int32),
        ("reserved", ctypes.c_int32), ("split_len", ctypes.c_int64),
        ("workspace_bytes", ctypes.c_int64),
    ]


def lib_path() -> str:
    return os.path.join(_HERE, "libstarattn.so")


def load_library():
    """Load the built library; raises if it has not been built (no fallback)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} not found: build it with `python -m paper_2411_17116_amd.build`")
    lib = ctypes.CDLL(path)
    P = ctypes.POINTER(StarShape)
    vp, sz, i64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int64
    lib.star_attn_workspace_bytes.restype = sz
    lib.star_attn_workspace_bytes.argtypes = [P, i64]
    lib.star_attn_phase1.restype = ctypes.c_int
    lib.star_attn_phase1.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.star_attn_phase1_anchor.restype = ctypes.c_int
    lib.star_attn_phase1_anchor.argtypes = [P, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                            vp, sz, vp]
    lib.star_attn_phase1_workspace_bytes.restype = sz
    lib.star_attn_phase1_workspace_bytes.argtypes = [P, ctypes.c_int]
    dbl = ctypes.c_double
    lib.star_attn_phase1_rope.restype = ctypes.c_int
    lib.star_attn_phase1_rope.argtypes = [P, dbl, i64, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.star_attn_phase2_rope.restype = ctypes.c_int
    lib.star_attn_phase2_rope.argtypes = [P, dbl, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                          sz, vp]
    lib.star_attn_rope.restype = ctypes.c_int
    lib.star_attn_rope.argtypes = [P, ctypes.c_int32, i64, i64, dbl, vp, vp, vp]
    lib.star_attn_phase2.restype = ctypes.c_int
    lib.star_attn_phase2.argtypes = [P, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.star_attn_phase2_static.restype = ctypes.c_int
    lib.star_attn_phase2_static.argtypes = [P, i64, i64, vp, vp, vp, vp, vp, vp, vp]
    lib.star_attn_phase2_partial.restype = ctypes.c_int
    lib.star_attn_phase2_partial.argtypes = [P, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.star_attn_merge.restype = ctypes.c_int
    lib.star_attn_merge.argtypes = [P, i64, i64, vp, vp, vp, vp, vp, vp]
    lib.star_attn_status_string.restype = ctypes.c_char_p
    lib.star_attn_status_string.argtypes = [ctypes.c_int]
    lib.star_attn_phase2_plan.restype = ctypes.c_int
    lib.star_attn_phase2_plan.argtypes = [P, i64, i64, ctypes.c_int, ctypes.POINTER(PlanInfo)]
    lib.star_attn_kernel_path.restype = ctypes.c_char_p
    lib.star_attn_kernel_path.argtypes = [P]
    _LIB = lib
    return lib


def status_string(code: int) -> str:
    return load_library().star_attn_status_string(int(code)).decode()


def kernel_path(shape: StarShape) -> Optional[str]:
    r = load_library().star_attn_kernel_path(ctypes.byref(shape))
    return r.decode() if r else None


def phase2_plan(shape: StarShape, cache_len: int, q_len: int, want_parts: bool = False) -> PlanInfo:
    """star_attn_phase2_plan: what a phase-2 call with these arguments would run."""
    info = PlanInfo()
    _check(load_library().star_attn_phase2_plan(ctypes.byref(shape), int(cache_len), int(q_len),
                                                int(bool(want_parts)), ctypes.byref(info)))
    return info


def workspace_bytes(shape: StarShape, max_q_len: int) -> int:
    return int(load_library().star_attn_workspace_bytes(ctypes.byref(shape), int(max_q_len)))


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("star_attn tensors must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(rc: int):
    if rc != 0:
        raise StarAttnError(rc, status_string(rc))


def alloc_cache(shape: StarShape, device="cuda"):
    """Caller-owned K/V caches [B, Hkv, cache_capacity, d] in the shape's dtype."""
    dt = torch.float32 if shape.dtype == F32 else torch.bfloat16
    dims = (shape.batch, shape.n_kv_heads, shape.cache_capacity, shape.head_dim)
    return torch.zeros(dims, dtype=dt, device=device), torch.zeros(dims, dtype=dt, device=device)


def alloc_workspace(shape: StarShape, max_q_len: int, device="cuda") -> torch.Tensor:
    n = workspace_bytes(shape, max_q_len)
    if n == 0:
        raise StarAttnError(-1, "invalid shape for workspace query")
    return torch.empty(n, dtype=torch.uint8, device=device)


def phase1(shape: StarShape, Q, K, V, O_ctx, K_cache, V_cache, LSE_ctx=None,
           workspace=None, stream=None) -> None:
    """star_attn_phase1: context encoding; fills O_ctx, the caches and LSE_ctx."""
    ws_n = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load_library().star_attn_phase1(
        ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(O_ctx), _ptr(LSE_ctx),
        _ptr(K_cache), _ptr(V_cache), _ptr(workspace), ws_n, _stream(stream))
    _check(rc)


def phase1_workspace_bytes(shape: StarShape, anchor_mode: int) -> int:
    return int(load_library().star_attn_phase1_workspace_bytes(ctypes.byref(shape), int(anchor_mode)))


def phase1_anchor(shape: StarShape, anchor_mode: int, Q, K, V, O_ctx, K_cache, V_cache,
                  K_anchor=None, V_anchor=None, LSE_ctx=None, workspace=None, stream=None) -> None:
    """star_attn_phase1_anchor: phase 1 under an anchor variant of the ablation study."""
    ws_n = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load_library().star_attn_phase1_anchor(
        ctypes.byref(shape), int(anchor_mode), _ptr(Q), _ptr(K), _ptr(V), _ptr(K_anchor),
        _ptr(V_anchor), _ptr(O_ctx), _ptr(LSE_ctx), _ptr(K_cache), _ptr(V_cache),
        _ptr(workspace), ws_n, _stream(stream))
    _check(rc)


def phase1_rope(shape: StarShape, rope_theta: float, Q, K, V, O_ctx, K_cache, V_cache, pos0=0,
                LSE_ctx=None, workspace=None, stream=None) -> None:
    """star_attn_phase1_rope: phase 1 on unrotated Q (rotated in place) and K."""
    ws_n = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load_library().star_attn_phase1_rope(
        ctypes.byref(shape), float(rope_theta), int(pos0), _ptr(Q), _ptr(K), _ptr(V), _ptr(O_ctx),
        _ptr(LSE_ctx), _ptr(K_cache), _ptr(V_cache), _ptr(workspace), ws_n, _stream(stream))
    _check(rc)


def phase2_rope(shape: StarShape, rope_theta: float, cache_len: int, Qq, Kq, Vq, K_cache, V_cache,
                O, workspace, pos0=0, O_part=None, LSE_part=None, stream=None) -> None:
    """star_attn_phase2_rope: phase 2 on unrotated Qq (rotated in place) and Kq."""
    q_len = Qq.shape[1]
    ws_n = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load_library().star_attn_phase2_rope(
        ctypes.byref(shape), float(rope_theta), int(pos0), int(cache_len), int(q_len), _ptr(Qq),
        _ptr(Kq), _ptr(Vq), _ptr(K_cache), _ptr(V_cache), _ptr(O_part), _ptr(LSE_part), _ptr(O),
        _ptr(workspace), ws_n, _stream(stream))
    _check(rc)


def rope(shape: StarShape, X, Y, rope_theta: float, pos0=0, stream=None) -> None:
    """star_attn_rope: rotate X [B, T, H, d] into Y (may be X), token t at pos0 + t."""
    rc = load_library().star_attn_rope(ctypes.byref(shape), int(X.shape[2]), int(X.shape[1]),
                                       int(pos0), float(rope_theta), _ptr(X), _ptr(Y),
                                       _stream(stream))
    _check(rc)


def phase2(shape: StarShape, cache_len: int, Qq, Kq, Vq, K_cache, V_cache, O, workspace,
           O_part=None, LSE_part=None, stream=None) -> None:
    """star_attn_phase2: appends Kq/Vq at cache_len, then global attention of the
    q_len = Qq.shape[1] new tokens; fills O (and the per-part outputs if given)."""
    q_len = Qq.shape[1]
    ws_n = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load_library().star_attn_phase2(
        ctypes.byref(shape), int(cache_len), int(q_len), _ptr(Qq), _ptr(Kq), _ptr(Vq),
        _ptr(K_cache), _ptr(V_cache), _ptr(O_part), _ptr(LSE_part), _ptr(O),
        _ptr(workspace), ws_n, _stream(stream))
    _check(rc)


STATIC_SCRATCH_BYTES = 16 << 20


def phase2_static(shape: StarShape, cache_len: int, Qq, Kq, Vq, K_cache, V_cache, O,
                  stream=None) -> None:
    """star_attn_phase2_static: star_attn_phase2 with the library's static scratch
    in place of a workspace (allocates nothing; calls must not overlap on a GPU)."""
    q_len = Qq.shape[1]
    rc = load_library().star_attn_phase2_static(
        ctypes.byref(shape), int(cache_len), int(q_len), _ptr(Qq), _ptr(Kq), _ptr(Vq),
        _ptr(K_cache), _ptr(V_cache), _ptr(O), _stream(stream))
    _check(rc)


def phase2_partial(shape: StarShape, cache_len: int, Qq, K_cache, V_cache, A, LSE, workspace,
                   Kq=None, Vq=None, stream=None) -> None:
    """star_attn_phase2_partial: one host's pair (A, LSE) for the q_len = Qq.shape[1]
    new tokens; with Kq/Vq the query host's share (append, then attend causally)."""
    q_len = Qq.shape[1]
    ws_n = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load_library().star_attn_phase2_partial(
        ctypes.byref(shape), int(cache_len), int(q_len), _ptr(Qq), _ptr(Kq), _ptr(Vq),
        _ptr(K_cache), _ptr(V_cache), _ptr(A), _ptr(LSE), _ptr(workspace), ws_n, _stream(stream))
    _check(rc)


def merge(shape: StarShape, A_parts, LSE_parts, O=None, A=None, LSE=None, stream=None) -> None:
    """star_attn_merge: Eq. 3-4 over the n_parts = A_parts.shape[0] gathered pairs."""
    n_parts, q_len = A_parts.shape[0], A_parts.shape[3]
    rc = load_library().star_attn_merge(
        ctypes.byref(shape), int(n_parts), int(q_len), _ptr(A_parts), _ptr(LSE_parts), _ptr(O),
        _ptr(A), _ptr(LSE), _stream(stream))
    _check(rc)
