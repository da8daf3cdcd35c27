"""fp64 CPU oracle for the Star Attention operator.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module; the product path (the HIP library and its Python binding) never
does, and this module shares no code with it.

Everything is plain numpy in float64, written from the paper's definitions:

* Phase 1 (Section 2.1, Algorithm 1, Figure 2): the context is cut into
  n = ceil(L / b) blocks; block 1 is attended causally on its own; every later
  block is prefixed by the anchor (the first `a` tokens of block 1, a <= b) and
  attended causally inside [anchor; block].  Only rows of real context tokens
  are outputs, and the KV cache keeps every context token exactly once (the
  anchor copies are dropped).
* Phase 2 (Section 2.2, Equations 1-4, Algorithm 2): new tokens are appended to
  the cache and then attend to everything before them and to themselves.  The
  cache is viewed as parts (one per context block plus the tail of query and
  decoded tokens); each part yields a local attention output (Eq. 1) and the log
  of its softmax denominator (Eq. 2, stored as a logarithm as Algorithm 2 does);
  parts are merged with Eq. 3-4.

Readings taken where the paper leaves a choice:
  - attention inside an augmented block is causal (decoder model, Figure 2);
  - an anchor shorter than the block means the first `a` tokens of block 1;
    block 1 itself is always plain causal attention over all of its tokens;
  - a ragged last block (L not a multiple of b) is allowed (Algorithm 1 uses a
    ceiling);
  - query head h reads KV head h // (Hq / Hkv);
  - the exchanged statistic is the natural-log LSE of the *scaled* logits;
  - the sequential merge in Algorithm 2 is implemented as the update that is
    consistent with Eq. 3-4:  s_new = logaddexp(s_old, s_h),
    A_new = exp(s_old - s_new) A_old + exp(s_h - s_new) A_h  (the printed update
    reuses the already-updated s_global and exponentiates A_h, which cannot be
    meant);
  - an empty part has LSE = -inf and output 0 and contributes nothing.

Layouts: Q [B, T, Hq, d]; K, V [B, T, Hkv, d]; caches [B, Hkv, cap, d].
Inputs may be float32 (e.g. bf16 values widened exactly) or float64; all
arithmetic below is float64.
"""
from __future__ import annotations

import math
from typing import Iterable, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


def softmax_scale(d: int, scale: Optional[float] = None) -> float:
    """1/sqrt(d) unless given (Eq. 1)."""
    return 1.0 / math.sqrt(d) if not scale else float(scale)


# --------------------------------------------------------------------------
# Phase 1
# --------------------------------------------------------------------------

def num_blocks(L: int, b: int) -> int:
    """n = ceil(L / b)  (Algorithm 1, block split)."""
    return -(-L // b)


def visible_keys(p: int, L: int, b: int, a: int) -> np.ndarray:
    """Indices of the context keys that context row `p` attends to in phase 1
    (Section 2.1; Figure 2): rows of block 1 see tokens 0..p; rows of a later
    block see the anchor tokens 0..a-1 and their own block up to p."""
    if not (0 <= p < L):
        raise ValueError("row outside the context")
    if not (0 <= a <= b):
        raise ValueError("anchor must satisfy 0 <= a <= b")
    i = p // b                      # 0-based block index
    if i == 0:
        return np.arange(0, p + 1)
    s = i * b
    return np.concatenate([np.arange(0, a), np.arange(s, p + 1)])


def attend(q: np.ndarray, Kv: np.ndarray, Vv: np.ndarray, scale: float
           ) -> Tuple[np.ndarray, float]:
    """Softmax attention of one query vector over the given keys (Eq. 1) and
    the log of its denominator (Eq. 2).  Empty key set -> (0, -inf)."""
    q = np.asarray(q, F64)
    Kv = np.asarray(Kv, F64)
    Vv = np.asarray(Vv, F64)
    if Kv.shape[0] == 0:
        return np.zeros(Vv.shape[1], F64), -math.inf
    logits = scale * (Kv @ q)
    m = logits.max()
    w = np.exp(logits - m)
    s = w.sum()
    return (w @ Vv) / s, float(m + math.log(s))


def phase1_row(Q, K, V, beta: int, h: int, p: int, b: int, a: int,
               scale: Optional[float] = None) -> Tuple[np.ndarray, float]:
    """Phase-1 output row and LSE for batch `beta`, query head `h`, context
    position `p`."""
    B, L, Hq, d = Q.shape
    Hkv = K.shape[2]
    g = h // (Hq // Hkv)
    ks = visible_keys(p, L, b, a)
    return attend(Q[beta, p, h], K[beta, ks, g], V[beta, ks, g],
                  softmax_scale(d, scale))


def phase1_rows(Q, K, V, triples: Iterable[Tuple[int, int, int]], b: int, a: int,
                scale: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Phase-1 outputs for a list of (batch, head, row) triples.
    Returns (O [len, d], LSE [len])."""
    triples = list(triples)
    O = np.zeros((len(triples), V.shape[3]), F64)
    LSE = np.zeros(len(triples), F64)
    for t, (beta, h, p) in enumerate(triples):
        O[t], LSE[t] = phase1_row(Q, K, V, beta, h, p, b, a, scale)
    return O, LSE


def phase1_full(Q, K, V, b: int, a: int, scale: Optional[float] = None
                ) -> Tuple[np.ndarray, np.ndarray]:
    """Phase-1 output for every context row: O [B, L, Hq, d], LSE [B, Hq, L]."""
    B, L, Hq, d = Q.shape
    O = np.zeros((B, L, Hq, V.shape[3]), F64)
    LSE = np.zeros((B, Hq, L), F64)
    for beta in range(B):
        for h in range(Hq):
            for p in range(L):
                O[beta, p, h], LSE[beta, h, p] = phase1_row(Q, K, V, beta, h, p, b, a, scale)
    return O, LSE


# --------------------------------------------------------------------------
# Rotary position embedding (the position encoding of the Llama models the paper
# evaluates; Section 2.1 fixes which position each token carries: a context
# token keeps its index in the context, and the anchor keeps 0..a-1 -- so the
# rotated key of an anchor token IS the rotated key of that context token and
# one K tensor serves both roles.  Phase 2: the j-th new token of a call made
# with `cache_len` cached tokens sits at position cache_len + j.)
# --------------------------------------------------------------------------

def rope_rotate(X, positions, theta: float) -> np.ndarray:
    """Rotary embedding of X [..., T, H, d] at integer `positions` [T] with
    base `theta`, in the half-split pairing of the Llama family: dimension i
    (i < d/2) pairs with dimension i + d/2, and the pair is turned by the angle
    pos * theta^(-2i/d):
        y_i       = x_i cos - x_(i+d/2) sin
        y_(i+d/2) = x_(i+d/2) cos + x_i sin."""
    X = np.asarray(X, F64)
    d = X.shape[-1]
    if d % 2:
        raise ValueError("head_dim must be even")
    half = d // 2
    inv_freq = np.asarray([float(theta) ** (-2.0 * i / d) for i in range(half)], F64)
    ang = np.asarray(positions, F64)[:, None] * inv_freq[None, :]        # [T, d/2]
    cos = np.cos(ang)[:, None, :]                                        # [T, 1, d/2]
    sin = np.sin(ang)[:, None, :]
    lo, hi = X[..., :half], X[..., half:]
    return np.concatenate([lo * cos - hi * sin, hi * cos + lo * sin], axis=-1)


def phase1_rope_rows(Q, K, V, triples, b: int, a: int, theta: float, pos0: int = 0,
                     scale: Optional[float] = None, storage=None
                     ) -> Tuple[np.ndarray, np.ndarray]:
    """Phase 1 on projections that have not been rotated yet: context token t
    is rotated at position pos0 + t, then the method runs unchanged.  Only the
    rows the triples need are rotated (row by row, as `phase1_row` walks them).

    `storage`, if given, maps a float64 array to the values a storage format
    can hold (e.g. round to bf16): the operator hands the rotated queries back
    and keeps the rotated keys in its cache in that format, and attention is
    defined on what is stored."""
    triples = list(triples)
    B, L, Hq, d = Q.shape
    Hkv = K.shape[2]
    O = np.zeros((len(triples), V.shape[3]), F64)
    LSE = np.zeros(len(triples), F64)
    sc = softmax_scale(d, scale)
    for t, (beta, h, p) in enumerate(triples):
        g = h // (Hq // Hkv)
        ks = visible_keys(p, L, b, a)
        q = rope_rotate(np.asarray(Q[beta, p, h], F64)[None, None, :], [pos0 + p], theta)[0, 0]
        Kr = rope_rotate(np.asarray(K[beta, ks, g], F64)[:, None, :], pos0 + ks, theta)[:, 0]
        if storage is not None:
            q, Kr = storage(q), storage(Kr)
        O[t], LSE[t] = attend(q, Kr, V[beta, ks, g], sc)
    return O, LSE


def kv_cache_rope(K, V, capacity: int, theta: float, pos0: int = 0):
    """The cache phase 1 leaves behind when it is handed unrotated keys: every
    context token once, its key rotated at its own position (float64)."""
    B, L, Hkv, d = K.shape
    Kr = rope_rotate(np.asarray(K, F64), pos0 + np.arange(L), theta)     # [B, L, Hkv, d]
    return kv_cache(Kr, np.asarray(V, F64), capacity)


def phase2_rope_inputs(Qn, Kn, cache_len: int, theta: float, pos0: int = 0):
    """Rotate the unrotated projections of a phase-2 call: its j-th new token
    sits at position pos0 + cache_len + j.  Returns (Q, K) in float64, to be
    appended / attended exactly like already-rotated inputs."""
    q_len = Qn.shape[1]
    pos = pos0 + cache_len + np.arange(q_len)
    return rope_rotate(np.asarray(Qn, F64), pos, theta), rope_rotate(np.asarray(Kn, F64), pos, theta)


# Anchor variants of the ablation study (Section 4.1, "Position and Content of
# Anchor Block"; Section 4.2 for the anchor size).  Block 1 is plain causal
# attention in every variant; the variants differ in what prefixes a later block.
ANCHOR_FIRST = 0      # the method itself: first `a` tokens of block 1
ANCHOR_PREVIOUS = 1   # "previous block as anchor": the `a` tokens just before the block
ANCHOR_EXTERNAL = 2   # anchor keys/values given separately (other content, or the
                      # first block's content encoded at other position ids)
ANCHOR_PER_BLOCK = 3  # a separately given anchor for every block (position ids that
                      # follow the block, e.g. "same as previous block")


def anchor_key_rows(i: int, b: int, a: int, mode: int) -> np.ndarray:
    """Context positions that prefix 0-based block i >= 1 when the anchor is
    taken from the context itself."""
    if mode == ANCHOR_FIRST:
        return np.arange(0, a)
    if mode == ANCHOR_PREVIOUS:
        return np.arange(i * b - a, i * b)
    raise ValueError("anchor rows are context positions only for FIRST / PREVIOUS")


def phase1_row_variant(Q, K, V, beta: int, h: int, p: int, b: int, a: int, mode: int,
                       K_anchor=None, V_anchor=None, scale: Optional[float] = None
                       ) -> Tuple[np.ndarray, float]:
    """Phase-1 row under an anchor variant.  The row attends to the anchor's
    `a` keys (all visible) followed by its own block up to itself; for
    ANCHOR_EXTERNAL the anchor keys/values are K_anchor, V_anchor [B, a, Hkv, d];
    for ANCHOR_PER_BLOCK they are [B, n, a, Hkv, d] and 0-based block i uses slice i
    (slice 0 is never read: block 1 has no anchor)."""
    B, L, Hq, d = Q.shape
    Hkv = K.shape[2]
    g = h // (Hq // Hkv)
    if not (0 <= a <= b):
        raise ValueError("anchor must satisfy 0 <= a <= b")
    i = p // b
    s = i * b
    own = np.arange(s, p + 1)
    sc = softmax_scale(d, scale)
    if i == 0:
        return attend(Q[beta, p, h], K[beta, own, g], V[beta, own, g], sc)
    if mode == ANCHOR_PER_BLOCK:
        if K_anchor.shape[1] != num_blocks(L, b) or K_anchor.shape[2] != a:
            raise ValueError("per-block anchors must be [B, n, a, Hkv, d]")
        Kv = np.concatenate([np.asarray(K_anchor[beta, i, :, g], F64), np.asarray(K[beta, own, g], F64)])
        Vv = np.concatenate([np.asarray(V_anchor[beta, i, :, g], F64), np.asarray(V[beta, own, g], F64)])
        return attend(Q[beta, p, h], Kv, Vv, sc)
    if mode == ANCHOR_EXTERNAL:
        if K_anchor.shape[1] != a or V_anchor.shape[1] != a:
            raise ValueError("external anchor must hold exactly `a` tokens")
        Kv = np.concatenate([np.asarray(K_anchor[beta, :, g], F64), np.asarray(K[beta, own, g], F64)])
        Vv = np.concatenate([np.asarray(V_anchor[beta, :, g], F64), np.asarray(V[beta, own, g], F64)])
        return attend(Q[beta, p, h], Kv, Vv, sc)
    ks = np.concatenate([anchor_key_rows(i, b, a, mode), own])
    return attend(Q[beta, p, h], K[beta, ks, g], V[beta, ks, g], sc)


def phase1_full_variant(Q, K, V, b: int, a: int, mode: int, K_anchor=None, V_anchor=None,
                        scale: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Every context row under an anchor variant: O [B, L, Hq, d], LSE [B, Hq, L]."""
    B, L, Hq, d = Q.shape
    O = np.zeros((B, L, Hq, V.shape[3]), F64)
    LSE = np.zeros((B, Hq, L), F64)
    for beta in range(B):
        for h in range(Hq):
            for p in range(L):
                O[beta, p, h], LSE[beta, h, p] = phase1_row_variant(
                    Q, K, V, beta, h, p, b, a, mode, K_anchor, V_anchor, scale)
    return O, LSE


def kv_cache(K, V, capacity: int) -> Tuple[np.ndarray, np.ndarray]:
    """KV cache after phase 1 (Algorithm 1: anchor KV discarded, block KV
    appended): every context token once, in order, rows beyond L zero.
    Layout [B, Hkv, capacity, d], dtype of the input."""
    B, L, Hkv, d = K.shape
    if capacity < L:
        raise ValueError("cache capacity below context length")
    Kc = np.zeros((B, Hkv, capacity, d), K.dtype)
    Vc = np.zeros((B, Hkv, capacity, V.shape[3]), V.dtype)
    for beta in range(B):
        for g in range(Hkv):
            Kc[beta, g, :L] = K[beta, :, g]
            Vc[beta, g, :L] = V[beta, :, g]
    return Kc, Vc


# --------------------------------------------------------------------------
# Phase 2
# --------------------------------------------------------------------------

def cache_append(Kc, Vc, cache_len: int, Kn, Vn) -> int:
    """Append the new tokens' K, V ([B, q_len, Hkv, d]) at rows
    [cache_len, cache_len + q_len) of the caches, in place (Algorithm 2: the
    query host appends before it attends).  Returns the new length."""
    B, q_len, Hkv, d = Kn.shape
    if cache_len + q_len > Kc.shape[2]:
        raise ValueError("cache overflow")
    for beta in range(B):
        for g in range(Hkv):
            Kc[beta, g, cache_len:cache_len + q_len] = Kn[beta, :, g]
            Vc[beta, g, cache_len:cache_len + q_len] = Vn[beta, :, g]
    return cache_len + q_len


def part_ranges(L: int, b: int, cache_len: int, j: int) -> List[Tuple[int, int]]:
    """Key ranges [lo, hi) of the parts new token `j` (0-based within this
    call) attends to, given `cache_len` tokens were cached before the call:
    one part per context block, then the tail [L, cache_len + j] which ends at
    the token itself."""
    n = num_blocks(L, b)
    parts = [(m * b, min((m + 1) * b, L)) for m in range(n)]
    parts.append((L, cache_len + j + 1))
    return parts


def merge_closed_form(A: np.ndarray, lse: np.ndarray) -> Tuple[np.ndarray, float]:
    """Eq. 3-4 with s_h = exp(lse_h): A_global = sum_h (s_h / s_global) A_h.
    Evaluated with the largest lse subtracted so that nothing overflows.
    A [P, d], lse [P]."""
    A = np.asarray(A, F64)
    lse = np.asarray(lse, F64)
    m = lse.max()
    if m == -math.inf:
        return np.zeros(A.shape[1], F64), -math.inf
    s = np.exp(lse - m)                 # s_h / exp(m); exp(-inf) = 0
    s_global = s.sum()                  # Eq. 3 (scaled by exp(-m))
    out = np.zeros(A.shape[1], F64)
    for h in range(A.shape[0]):
        if s[h] > 0.0:
            out += (s[h] / s_global) * A[h]     # Eq. 4
    return out, float(m + math.log(s_global))


def merge_sequential(A: np.ndarray, lse: np.ndarray,
                     order: Optional[Sequence[int]] = None) -> Tuple[np.ndarray, float]:
    """Algorithm 2's running merge (online softmax), in the given part order:
    start from the first part; for each further part update the global LSE with
    logaddexp and rescale both outputs by exp(old - new) and exp(part - new)."""
    A = np.asarray(A, F64)
    lse = np.asarray(lse, F64)
    order = list(range(A.shape[0])) if order is None else list(order)
    s_glob = float(lse[order[0]])
    A_glob = np.array(A[order[0]], F64) if s_glob > -math.inf else np.zeros(A.shape[1], F64)
    for h in order[1:]:
        s_h = float(lse[h])
        if s_h == -math.inf:
            continue
        if s_glob == -math.inf:
            s_glob, A_glob = s_h, np.array(A[h], F64)
            continue
        s_new = s_glob + math.log1p(math.exp(s_h - s_glob)) if s_h <= s_glob \
            else s_h + math.log1p(math.exp(s_glob - s_h))
        A_glob = math.exp(s_glob - s_new) * A_glob + math.exp(s_h - s_new) * A[h]
        s_glob = s_new
    return A_glob, s_glob


def attend_block(Qm: np.ndarray, Kh: np.ndarray, Vh: np.ndarray, scale: float,
                 allowed: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 1-2 for several query rows at once: A = softmax(scale Qm Kh^T) Vh and
    lse = log of the row denominators.  `allowed` [rows, keys] (bool) removes
    key/row pairs; a row with no key left gives (0, -inf).
    Qm [r, d], Kh, Vh [k, d] -> A [r, d], lse [r]."""
    Qm = np.asarray(Qm, F64)
    r = Qm.shape[0]
    if Kh.shape[0] == 0:
        return np.zeros((r, Vh.shape[1]), F64), np.full(r, -math.inf, F64)
    S = scale * (Qm @ np.asarray(Kh, F64).T)
    if allowed is not None:
        S = np.where(allowed, S, -math.inf)
    m = S.max(axis=1)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    W = np.exp(S - m_safe[:, None])            # exp(-inf) = 0 for removed pairs
    s = W.sum(axis=1)
    empty = s == 0.0
    A = (W @ np.asarray(Vh, F64)) / np.where(empty, 1.0, s)[:, None]
    with np.errstate(divide="ignore"):
        lse = np.where(empty, -math.inf, m_safe + np.log(s))
    return A, lse


def phase2_rows(Qn, Kc, Vc, L: int, b: int, cache_len: int,
                heads: Optional[Sequence[int]] = None,
                rows: Optional[Sequence[int]] = None,
                scale: Optional[float] = None):
    """Phase-2 attention of the `q_len` new tokens whose K, V have already been
    appended at rows [cache_len, cache_len + q_len) of Kc, Vc.

    Qn [B, q_len, Hq, d]; Kc, Vc [B, Hkv, cap, d].  `heads` / `rows` select the
    query heads / new-token indices to compute (default: all).  Returns a dict
      heads, rows   what was computed (nh heads, nr rows),
      O_part    [B, P, nh, nr, d]   local attention per part (Eq. 1),
      LSE_part  [B, P, nh, nr]      log of Eq. 2 per part,
      O         [B, nr, nh, d]      global attention: ONE softmax over every key
                                    the token may see (the definition the merge
                                    must reproduce),
      LSE       [B, nh, nr]
    with P = n + 1: part m < n is context block m+1, part n is the tail
    [L, cache_len + j] of token j (earlier query/decoded tokens and itself)."""
    B, q_len, Hq, d = Qn.shape
    Hkv = Kc.shape[1]
    G = Hq // Hkv
    heads = list(range(Hq)) if heads is None else list(heads)
    rows = list(range(q_len)) if rows is None else list(rows)
    sc = softmax_scale(d, scale)
    n = num_blocks(L, b)
    P = n + 1
    nh, nr = len(heads), len(rows)
    dv = Vc.shape[3]
    O_part = np.zeros((B, P, nh, nr, dv), F64)
    LSE_part = np.full((B, P, nh, nr), -math.inf, F64)
    O = np.zeros((B, nr, nh, dv), F64)
    LSE = np.zeros((B, nh, nr), F64)
    total = cache_len + q_len
    jj = np.asarray(rows)
    key_pos = np.arange(total)
    # token j sees keys 0 .. cache_len + j (itself included)
    sees = key_pos[None, :] <= (cache_len + jj)[:, None]
    for beta in range(B):
        g_loaded = None
        for hi, h in enumerate(heads):
            g = h // G
            if g != g_loaded:           # keep one KV head in float64 at a time
                K64 = np.asarray(Kc[beta, g, :total], F64)
                V64 = np.asarray(Vc[beta, g, :total], F64)
                g_loaded = g
            Qm = np.asarray(Qn[beta, jj, h], F64)
            for m in range(n):
                lo, hi_ = m * b, min((m + 1) * b, L)
                O_part[beta, m, hi], LSE_part[beta, m, hi] = attend_block(
                    Qm, K64[lo:hi_], V64[lo:hi_], sc)
            O_part[beta, n, hi], LSE_part[beta, n, hi] = attend_block(
                Qm, K64[L:], V64[L:], sc, sees[:, L:])
            A, lse = attend_block(Qm, K64, V64, sc, sees)
            O[beta, :, hi] = A
            LSE[beta, hi] = lse
    return {"heads": heads, "rows": rows, "O_part": O_part, "LSE_part": LSE_part,
            "O": O, "LSE": LSE}


def phase2_merged(O_part: np.ndarray, LSE_part: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Apply Eq. 3-4 to every (batch, head, row) of a phase2_rows result.
    O_part [B, P, nh, q, d], LSE_part [B, P, nh, q] -> O [B, q, nh, d], LSE [B, nh, q]."""
    B, P, nh, q_len, d = O_part.shape
    O = np.zeros((B, q_len, nh, d), F64)
    LSE = np.zeros((B, nh, q_len), F64)
    for beta in range(B):
        for hi in range(nh):
            for j in range(q_len):
                O[beta, j, hi], LSE[beta, hi, j] = merge_closed_form(
                    O_part[beta, :, hi, j], LSE_part[beta, :, hi, j])
    return O, LSE
