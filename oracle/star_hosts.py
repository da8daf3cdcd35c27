"""fp64 CPU oracle for Star Attention as the paper states it: host by host.
TEST INFRASTRUCTURE ONLY (same rules as star_oracle: tests, the smoke check and
the benchmark's CPU-baseline leg only; no code shared with the HIP path).

star_oracle writes the operator down as one set of visible keys per row.  This
module writes down what each HOST does in Algorithms 1 and 2, literally:

* Phase 1 (Section 2.1, Algorithm 1).  A host that owns context block c_i
  (i > 1) builds the augmented block c'_i = [anchor; c_i] -- anchor = the first
  `a` tokens of c_1 -- runs ordinary causal attention over all |anchor| + |c_i|
  tokens of it, throws the anchor's output rows and the anchor's K/V away and
  keeps the block's.  The owner of c_1 runs causal attention over c_1 alone.
  A host may own several consecutive blocks; it treats each the same way.
* Phase 2 (Section 2.2, Algorithm 2).  The new tokens' queries go to every
  host.  Each host attends with them over its own cache and returns the local
  attention output A_h (Eq. 1) and the logarithm of its softmax denominator s_h
  (Eq. 2).  One host, the query host, first appends the new tokens' K/V to its
  cache, so that its part also holds the earlier new tokens and the token
  itself (causally).  The query host then gathers all (A_h, log s_h) and
  combines them with Eq. 3-4.

Nothing here calls star_oracle's visible-key rule; tests compare the two.
Layouts: Q [B, T, Hq, d]; K, V [B, T, Hkv, d]; caches [B, Hkv, cap, d];
per-host partials A [B, Hq, q_len, d], lse [B, Hq, q_len].
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


def block_runs(n_blocks: int, n_hosts: int) -> List[Tuple[int, int]]:
    """Consecutive runs [i0, i1) of 0-based block indices, one per host, as even
    as possible (earlier hosts take the larger runs).  With n_hosts == n_blocks
    every host owns one block, the paper's setting; a host may also own none."""
    if n_hosts < 1:
        raise ValueError("at least one host")
    base, extra = divmod(n_blocks, n_hosts)
    runs, i = [], 0
    for h in range(n_hosts):
        k = base + (1 if h < extra else 0)
        runs.append((i, i + k))
        i += k
    return runs


def causal_attention(Qs: np.ndarray, Ks: np.ndarray, Vs: np.ndarray, scale: float
                     ) -> Tuple[np.ndarray, np.ndarray]:
    """Textbook causal softmax attention of one head over one sequence:
    row t attends to rows 0..t.  Qs, Ks [T, d], Vs [T, dv] -> (O [T, dv], lse [T])."""
    Qs, Ks, Vs = (np.asarray(x, F64) for x in (Qs, Ks, Vs))
    T = Qs.shape[0]
    S = scale * (Qs @ Ks.T)
    S = np.where(np.tril(np.ones((T, T), bool)), S, -math.inf)
    m = S.max(axis=1)
    W = np.exp(S - m[:, None])
    s = W.sum(axis=1)
    return (W @ Vs) / s[:, None], m + np.log(s)


def host_phase1(Q, K, V, run: Tuple[int, int], b: int, a: int, scale: Optional[float] = None,
                return_anchor_rows: bool = False):
    """What the host owning blocks run = [i0, i1) does in phase 1 (Algorithm 1).

    Q, K, V are the WHOLE context's projections; the host reads its own blocks'
    tokens and the anchor tokens 0..a-1 (what it is sent).  Returns
      O    [B, T_h, Hq, d]  outputs of the host's own tokens, in order,
      LSE  [B, Hq, T_h],
      Kh, Vh [B, T_h, Hkv, d]  the K/V it keeps (anchor copies dropped),
    and with return_anchor_rows also the list (one entry per owned block after
    the global first) of the anchor rows' outputs [B, a, Hq, d] that the host
    computes and throws away."""
    B, L, Hq, d = Q.shape
    Hkv = K.shape[2]
    G = Hq // Hkv
    sc = 1.0 / math.sqrt(d) if not scale else float(scale)
    if not (0 <= a <= b):
        raise ValueError("anchor must satisfy 0 <= a <= b")
    i0, i1 = run
    lo, hi = min(i0 * b, L), min(i1 * b, L)
    T_h = hi - lo
    O = np.zeros((B, T_h, Hq, V.shape[3]), F64)
    LSE = np.zeros((B, Hq, T_h), F64)
    dropped = []
    for i in range(i0, i1):
        s, e = i * b, min((i + 1) * b, L)
        if s >= e:
            continue
        # the augmented block: anchor tokens first (none for the global first block)
        n_anc = 0 if i == 0 else a
        tok = np.concatenate([np.arange(0, n_anc), np.arange(s, e)])
        anc_out = np.zeros((B, n_anc, Hq, V.shape[3]), F64)
        for beta in range(B):
            for h in range(Hq):
                g = h // G
                o, lse = causal_attention(Q[beta, tok, h], K[beta, tok, g], V[beta, tok, g], sc)
                O[beta, s - lo:e - lo, h] = o[n_anc:]          # anchor rows are not outputs
                LSE[beta, h, s - lo:e - lo] = lse[n_anc:]
                anc_out[beta, :, h] = o[:n_anc]
        if i > 0:
            dropped.append(anc_out)
    Kh = np.array(K[:, lo:hi])                                   # the block's K/V only
    Vh = np.array(V[:, lo:hi])
    if return_anchor_rows:
        return O, LSE, Kh, Vh, dropped
    return O, LSE, Kh, Vh


def host_cache(Kh, Vh, capacity: int) -> Tuple[np.ndarray, np.ndarray]:
    """A host's KV cache [B, Hkv, capacity, d] holding its kept tokens in order."""
    B, T, Hkv, d = Kh.shape
    if capacity < T:
        raise ValueError("cache capacity below the host's tokens")
    Kc = np.zeros((B, Hkv, capacity, d), Kh.dtype)
    Vc = np.zeros((B, Hkv, capacity, Vh.shape[3]), Vh.dtype)
    Kc[:, :, :T] = np.transpose(Kh, (0, 2, 1, 3))
    Vc[:, :, :T] = np.transpose(Vh, (0, 2, 1, 3))
    return Kc, Vc


def host_phase2(Qn, Kc, Vc, cache_len: int, Kn=None, Vn=None, scale: Optional[float] = None
                ) -> Tuple[np.ndarray, np.ndarray]:
    """One host's share of a phase-2 call (Algorithm 2): local attention of the
    q_len new tokens over the host's cache, (A_h, log s_h) of Eq. 1-2.

    A context host (Kn, Vn None) attends to its cache rows [0, cache_len), all of
    them visible to every new token.  The query host (Kn, Vn given) first appends
    the new tokens' K/V at rows [cache_len, cache_len + q_len) of ITS caches, in
    place, and new token j then sees rows [0, cache_len + j].
    Returns A [B, Hq, q_len, d], lse [B, Hq, q_len]; no visible row -> (0, -inf)."""
    B, q_len, Hq, d = Qn.shape
    Hkv = Kc.shape[1]
    G = Hq // Hkv
    sc = 1.0 / math.sqrt(d) if not scale else float(scale)
    if Kn is not None:
        if cache_len + q_len > Kc.shape[2]:
            raise ValueError("cache overflow")
        Kc[:, :, cache_len:cache_len + q_len] = np.transpose(Kn, (0, 2, 1, 3))
        Vc[:, :, cache_len:cache_len + q_len] = np.transpose(Vn, (0, 2, 1, 3))
    A = np.zeros((B, Hq, q_len, Vc.shape[3]), F64)
    lse = np.full((B, Hq, q_len), -math.inf, F64)
    for beta in range(B):
        for h in range(Hq):
            g = h // G
            for j in range(q_len):
                n_vis = cache_len + j + 1 if Kn is not None else cache_len
                if n_vis == 0:
                    continue
                Kv = np.asarray(Kc[beta, g, :n_vis], F64)
                Vv = np.asarray(Vc[beta, g, :n_vis], F64)
                logits = sc * (Kv @ np.asarray(Qn[beta, j, h], F64))
                m = logits.max()
                w = np.exp(logits - m)
                s = w.sum()                                   # Eq. 2 (times exp(-m))
                A[beta, h, j] = (w @ Vv) / s                  # Eq. 1
                lse[beta, h, j] = m + math.log(s)
    return A, lse


def gather_merge(A_hosts: Sequence[np.ndarray], lse_hosts: Sequence[np.ndarray]
                 ) -> Tuple[np.ndarray, np.ndarray]:
    """The query host's aggregation (Eq. 3-4): s_global = sum_h s_h and
    A_global = sum_h (s_h / s_global) A_h, with s_h = exp(lse_h) evaluated
    relative to the largest lse.  A_hosts[h] [B, Hq, q_len, d], lse_hosts[h]
    [B, Hq, q_len] -> O [B, q_len, Hq, d], LSE [B, Hq, q_len]."""
    A = np.stack([np.asarray(x, F64) for x in A_hosts])          # [H, B, Hq, q, d]
    lse = np.stack([np.asarray(x, F64) for x in lse_hosts])      # [H, B, Hq, q]
    m = lse.max(axis=0)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    s = np.exp(lse - m_safe[None])                               # s_h / exp(m); 0 for empty hosts
    s_global = s.sum(axis=0)                                     # Eq. 3
    nothing = s_global == 0.0
    wgt = s / np.where(nothing, 1.0, s_global)[None]             # s_h / s_global
    O = (wgt[..., None] * A).sum(axis=0)                         # Eq. 4
    with np.errstate(divide="ignore"):
        LSE = np.where(nothing, -math.inf, m_safe + np.log(s_global))
    return np.transpose(O, (0, 2, 1, 3)), LSE


def run_cluster(Q, K, V, b: int, a: int, n_hosts: int, calls, capacity_tail: int,
                query_host: Optional[int] = None, scale: Optional[float] = None):
    """Both phases on `n_hosts` simulated hosts.  `calls` is a list of
    (Qn, Kn, Vn) phase-2 calls made one after the other (query, then decode
    steps).  Returns (O_ctx [B, L, Hq, d], LSE_ctx [B, Hq, L], [O of each call],
    [LSE of each call], per-host caches, per-host cache lengths)."""
    B, L, Hq, d = Q.shape
    n = -(-L // b)
    runs = block_runs(n, n_hosts)
    qh = n_hosts - 1 if query_host is None else query_host
    O_ctx = np.zeros((B, L, Hq, V.shape[3]), F64)
    LSE_ctx = np.zeros((B, Hq, L), F64)
    caches, lens = [], []
    for h, run in enumerate(runs):
        O, LSE, Kh, Vh = host_phase1(Q, K, V, run, b, a, scale)
        lo = min(run[0] * b, L)
        O_ctx[:, lo:lo + O.shape[1]] = O
        LSE_ctx[:, :, lo:lo + O.shape[1]] = LSE
        caches.append(host_cache(Kh, Vh, Kh.shape[1] + (capacity_tail if h == qh else 0)))
        lens.append(Kh.shape[1])
    outs, lses = [], []
    for Qn, Kn, Vn in calls:
        A_h, l_h = [], []
        for h in range(n_hosts):
            Kc, Vc = caches[h]
            if h == qh:
                A, l = host_phase2(Qn, Kc, Vc, lens[h], Kn, Vn, scale)
            else:
                A, l = host_phase2(Qn, Kc, Vc, lens[h], None, None, scale)
            A_h.append(A)
            l_h.append(l)
        lens[qh] += Qn.shape[1]
        O, LSE = gather_merge(A_h, l_h)
        outs.append(O)
        lses.append(LSE)
    return O_ctx, LSE_ctx, outs, lses, caches, lens
