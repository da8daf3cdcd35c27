"""Brute-force checker for the oracle.  TEST INFRASTRUCTURE ONLY (tiny inputs).

Written separately from the row-wise oracle and deliberately different in
shape: it materialises the whole token-level mask that Figure 2 draws at block
level and evaluates a dense masked softmax, so that a wrong index, a dropped
term or a transposed operand in the oracle shows up as a disagreement.
Nothing here imports the oracle or the HIP path.
"""
from __future__ import annotations

import math

import numpy as np


def phase1_mask(L: int, b: int, a: int) -> np.ndarray:
    """mask[p, k] = True iff context row p may attend to context key k in
    phase 1.  Built block by block from the picture in Figure 2: block 1 is a
    lower triangle; block i > 1 is [all `a` anchor columns | lower triangle on
    its own columns]; everything else is empty."""
    mask = np.zeros((L, L), dtype=bool)
    n = -(-L // b)
    for i in range(n):
        s, e = i * b, min((i + 1) * b, L)
        for p in range(s, e):
            for k in range(s, p + 1):
                mask[p, k] = True
            if i > 0:
                for k in range(a):
                    mask[p, k] = True
    return mask


def previous_anchor_mask(L: int, b: int, a: int) -> np.ndarray:
    """Token-level mask of the "previous block as anchor" ablation (Section 4.1):
    block 1 is a lower triangle; a later block sees the `a` columns just left of
    its own columns, all of them, and a lower triangle on its own columns."""
    mask = np.zeros((L, L), dtype=bool)
    n = -(-L // b)
    for i in range(n):
        s, e = i * b, min((i + 1) * b, L)
        for p in range(s, e):
            for k in range(s, p + 1):
                mask[p, k] = True
            if i > 0:
                for k in range(s - a, s):
                    mask[p, k] = True
    return mask


def external_anchor_dense(Q, K, V, Ka, Va, b: int, scale=None):
    """Phase 1 with separately given anchor keys/values, by brute force: for
    every block after the first, lay out the sequence [anchor; block] as Figure 2
    draws it, run dense causal-within-[anchor; block] attention with an explicit
    mask, and keep the rows of the block.  Ka, Va [B, a, Hkv, d], or
    [B, n, a, Hkv, d] for one anchor per block (block i uses slice i).
    Returns O [B, L, Hq, d], LSE [B, Hq, L]."""
    B, L, Hq, d = Q.shape
    Hkv = K.shape[2]
    G = Hq // Hkv
    per_block = Ka.ndim == 5
    a = Ka.shape[2] if per_block else Ka.shape[1]
    sc = 1.0 / math.sqrt(d) if scale is None else scale
    n = -(-L // b)
    O = np.zeros((B, L, Hq, d))
    LSE = np.zeros((B, Hq, L))
    for beta in range(B):
        for h in range(Hq):
            g = h // G
            for i in range(n):
                s, e = i * b, min((i + 1) * b, L)
                rows = e - s
                pre = 0 if i == 0 else a
                ka = Ka[beta, i, :, g] if per_block else Ka[beta, :, g]
                va = Va[beta, i, :, g] if per_block else Va[beta, :, g]
                kk = K[beta, s:e, g] if i == 0 else np.concatenate([ka, K[beta, s:e, g]])
                vv = V[beta, s:e, g] if i == 0 else np.concatenate([va, V[beta, s:e, g]])
                mask = np.zeros((rows, pre + rows), dtype=bool)
                for r in range(rows):
                    mask[r, :pre + r + 1] = True
                o, l = dense_masked_attention(Q[beta, s:e, h], kk, vv, mask, sc)
                O[beta, s:e, h] = o
                LSE[beta, h, s:e] = l
    return O, LSE


def dense_masked_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray,
                           mask: np.ndarray, scale: float):
    """softmax(mask(scale * q k^T)) v for one head.  q [Tq, d], k, v [Tk, d],
    mask [Tq, Tk].  Returns (out [Tq, d], lse [Tq])."""
    q = q.astype(np.float64)
    k = k.astype(np.float64)
    v = v.astype(np.float64)
    Tq, Tk = mask.shape
    out = np.zeros((Tq, v.shape[1]))
    lse = np.zeros(Tq)
    for p in range(Tq):
        logits = []
        idx = []
        for j in range(Tk):
            if mask[p, j]:
                logits.append(scale * float(np.dot(q[p], k[j])))
                idx.append(j)
        top = max(logits)
        den = sum(math.exp(x - top) for x in logits)
        acc = np.zeros(v.shape[1])
        for x, j in zip(logits, idx):
            acc += (math.exp(x - top) / den) * v[j]
        out[p] = acc
        lse[p] = top + math.log(den)
    return out, lse


def phase1_dense(Q, K, V, b: int, a: int, scale=None):
    """Phase 1 for every (batch, head): O [B, L, Hq, d], LSE [B, Hq, L]."""
    B, L, Hq, d = Q.shape
    Hkv = K.shape[2]
    G = Hq // Hkv
    sc = 1.0 / math.sqrt(d) if scale is None else scale
    mask = phase1_mask(L, b, a)
    O = np.zeros((B, L, Hq, d))
    LSE = np.zeros((B, Hq, L))
    for beta in range(B):
        for h in range(Hq):
            o, l = dense_masked_attention(Q[beta, :, h], K[beta, :, h // G],
                                          V[beta, :, h // G], mask, sc)
            O[beta, :, h] = o
            LSE[beta, h] = l
    return O, LSE


def phase2_dense(Qn, K_all, V_all, n_before: int, scale=None):
    """Global attention of new tokens by brute force: K_all, V_all
    [B, n_before + q_len, Hkv, d] hold every earlier token (context, then tail)
    followed by the new tokens themselves; new token j sees keys
    0 .. n_before + j.  Returns (O [B, q_len, Hq, d], LSE [B, Hq, q_len])."""
    B, q_len, Hq, d = Qn.shape
    Hkv = K_all.shape[2]
    G = Hq // Hkv
    sc = 1.0 / math.sqrt(d) if scale is None else scale
    Tk = n_before + q_len
    mask = np.zeros((q_len, Tk), dtype=bool)
    for j in range(q_len):
        mask[j, :n_before + j + 1] = True
    O = np.zeros((B, q_len, Hq, d))
    LSE = np.zeros((B, Hq, q_len))
    for beta in range(B):
        for h in range(Hq):
            o, l = dense_masked_attention(Qn[beta, :, h], K_all[beta, :Tk, h // G],
                                          V_all[beta, :Tk, h // G], mask, sc)
            O[beta, :, h] = o
            LSE[beta, h] = l
    return O, LSE
