"""Pins for the fp64 oracle: every check below compares the oracle with
something other than itself -- a separately written brute force, a library
attention routine, a closed form, an invariant, or the block pattern the paper
draws in Figure 2.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import brute_force as bf
from oracle import star_oracle as so

RNG = np.random.default_rng(20241117)
TOL = 1e-11


def rand_qkv(B, L, Hq, Hkv, d, scale=1.0, rng=RNG):
    Q = rng.standard_normal((B, L, Hq, d)) * scale
    K = rng.standard_normal((B, L, Hkv, d))
    V = rng.standard_normal((B, L, Hkv, d))
    return Q, K, V


def sdpa_causal(q, k, v, scale=None):
    """Library causal attention (torch CPU, float64) for one head: [T, d]."""
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(x)).double()[None, None]
                  for x in (q, k, v))
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True,
                                                           scale=scale)
    return out[0, 0].numpy()


SHAPES = [
    # B, L, Hq, Hkv, d, b, a
    (1, 23, 1, 1, 8, 8, 8),      # ragged last block, a == b
    (2, 24, 4, 2, 4, 8, 3),      # GQA, anchor shorter than block
    (1, 20, 2, 1, 8, 5, 0),      # no anchor
    (1, 17, 3, 1, 16, 6, 6),     # G = 3, ragged
    (1, 9, 2, 2, 4, 16, 16),     # single block (b > L)
    (1, 12, 1, 1, 4, 1, 1),      # blocks of one token
]


@pytest.mark.parametrize("B,L,Hq,Hkv,d,b,a", SHAPES)
def test_I0_phase1_matches_brute_force(B, L, Hq, Hkv, d, b, a):
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d, scale=2.0)
    O, LSE = so.phase1_full(Q, K, V, b, a)
    Ob, LSEb = bf.phase1_dense(Q, K, V, b, a)
    assert np.abs(O - Ob).max() < TOL
    assert np.abs(LSE - LSEb).max() < TOL


def test_I1_block_not_smaller_than_context_is_full_causal():
    B, L, Hq, Hkv, d = 1, 40, 4, 2, 8
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d, scale=1.7)
    for b in (40, 64):
        O, _ = so.phase1_full(Q, K, V, b, b)
        for h in range(Hq):
            ref = sdpa_causal(Q[0, :, h], K[0, :, h // 2], V[0, :, h // 2])
            assert np.abs(O[0, :, h] - ref).max() < TOL


def test_I2_first_block_is_plain_causal_whatever_the_anchor():
    B, L, Hq, Hkv, d, b = 1, 50, 2, 1, 8, 16
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    for a in (0, 5, 16):
        O, _ = so.phase1_full(Q, K, V, b, a)
        for h in range(Hq):
            ref = sdpa_causal(Q[0, :b, h], K[0, :b, 0], V[0, :b, 0])
            assert np.abs(O[0, :b, h] - ref).max() < TOL


def test_I2b_two_blocks_full_anchor_is_full_causal():
    B, L, Hq, Hkv, d, b = 1, 32, 2, 2, 8, 16
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    O, _ = so.phase1_full(Q, K, V, b, b)
    for h in range(Hq):
        ref = sdpa_causal(Q[0, :, h], K[0, :, h], V[0, :, h])
        assert np.abs(O[0, :, h] - ref).max() < TOL


@pytest.mark.parametrize("L,b,a", [(37, 10, 10), (37, 10, 4), (48, 16, 16)])
def test_I4_later_blocks_equal_library_attention_on_anchor_plus_block(L, b, a):
    B, Hq, Hkv, d = 1, 2, 1, 8
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d, scale=1.5)
    O, _ = so.phase1_full(Q, K, V, b, a)
    for i in range(1, -(-L // b)):
        s, e = i * b, min((i + 1) * b, L)
        for h in range(Hq):
            qa = np.concatenate([Q[0, :a, h], Q[0, s:e, h]])
            ka = np.concatenate([K[0, :a, 0], K[0, s:e, 0]])
            va = np.concatenate([V[0, :a, 0], V[0, s:e, 0]])
            ref = sdpa_causal(qa, ka, va)[a:]
            assert np.abs(O[0, s:e, h] - ref).max() < TOL


def test_fig2_block_pattern():
    """Reduce the oracle's token-level key sets to block level and compare with
    the pattern printed in Figure 2 (5 context blocks + the query)."""
    path = os.path.join(os.path.dirname(__file__), "golden", "fig2_block_pattern.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    want = np.array([[int(x) for x in r[1:]] for r in rows])
    n, b, lq = 5, 4, 3
    L = n * b
    got = np.zeros((n + 1, n + 1), dtype=int)
    for p in range(L):
        ks = so.visible_keys(p, L, b, b)
        # a black cell means the whole (causal part of the) block is visible
        for j in range(n):
            seen = np.intersect1d(ks, np.arange(j * b, (j + 1) * b)).size
            if seen:
                got[p // b, j] = 1
                full = b if j != p // b else (p - j * b + 1)
                assert seen == full
    for j in range(lq):
        parts = so.part_ranges(L, b, L, j)
        assert parts[:n] == [(m * b, (m + 1) * b) for m in range(n)]
        assert parts[n] == (L, L + j + 1)
        got[n, :] = 1
    assert (got == want).all()


def test_I6_one_hot_values_read_back_probabilities():
    B, L, Hq, Hkv, d, b, a = 1, 30, 2, 1, 8, 8, 5
    Q, K, _ = rand_qkv(B, L, Hq, Hkv, d)
    V = np.eye(L)[None, :, None, :]              # V[k] = e_k, value dim L
    O, _ = so.phase1_full(Q, K, V, b, a)
    mask = bf.phase1_mask(L, b, a)
    for h in range(Hq):
        P = O[0, :, h]                            # [row, key] probabilities
        assert (P[~mask] == 0.0).all()
        assert (P[mask] > 0.0).all()
        assert np.abs(P.sum(axis=1) - 1.0).max() < 1e-13
    # number of visible keys: p+1 in block 1, a + (p - s + 1) afterwards
    for p in range(L):
        cnt = p + 1 if p < b else a + (p - (p // b) * b + 1)
        assert mask[p].sum() == cnt == so.visible_keys(p, L, b, a).size


def test_closed_form_zero_queries_give_means_and_log_counts():
    B, L, Hq, Hkv, d, b, a = 1, 26, 1, 1, 4, 8, 6
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    Q[:] = 0.0
    O, LSE = so.phase1_full(Q, K, V, b, a)
    for p in range(L):
        ks = list(range(p + 1)) if p < b else list(range(a)) + list(range((p // b) * b, p + 1))
        assert np.abs(O[0, p, 0] - V[0, ks, 0].mean(axis=0)).max() < 1e-13
        assert abs(LSE[0, 0, p] - math.log(len(ks))) < 1e-13


def test_I7_constant_values_and_partition_of_unity():
    B, L, Hq, Hkv, d, b = 1, 21, 2, 1, 8, 8
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    v = RNG.standard_normal(d)
    V[:] = v
    O, _ = so.phase1_full(Q, K, V, b, b)
    assert np.abs(O - v).max() < 1e-13
    Kc, Vc = so.kv_cache(K, V, L + 4)
    Qn, Kn, Vn = rand_qkv(B, 4, Hq, Hkv, d)
    Vn[:] = v
    so.cache_append(Kc, Vc, L, Kn, Vn)
    r = so.phase2_rows(Qn, Kc, Vc, L, b, L)
    assert np.abs(r["O"] - v).max() < 1e-13
    w = np.exp(r["LSE_part"] - r["LSE"][:, None])      # [B, P, nh, q]
    assert np.abs(w.sum(axis=1) - 1.0).max() < 1e-13


def test_I8_shifting_all_keys_moves_only_the_lse():
    B, L, Hq, Hkv, d, b, a = 1, 28, 2, 1, 8, 8, 8
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    u = 40.0 * RNG.standard_normal(d)                   # large: exercises stability
    O0, L0 = so.phase1_full(Q, K, V, b, a)
    O1, L1 = so.phase1_full(Q, K + u, V, b, a)
    assert np.abs(O0 - O1).max() < 1e-9
    shift = (Q[0] @ u) / math.sqrt(d)                    # [L, Hq]
    assert np.abs((L1[0] - L0[0]) - shift.T).max() < 1e-9
    Kc, Vc = so.kv_cache(K, V, L + 3)
    Kc1, Vc1 = so.kv_cache(K + u, V, L + 3)
    Qn, Kn, Vn = rand_qkv(B, 3, Hq, Hkv, d)
    so.cache_append(Kc, Vc, L, Kn, Vn)
    so.cache_append(Kc1, Vc1, L, Kn + u, Vn)
    r0 = so.phase2_rows(Qn, Kc, Vc, L, b, L)
    r1 = so.phase2_rows(Qn, Kc1, Vc1, L, b, L)
    assert np.abs(r0["O"] - r1["O"]).max() < 1e-9
    assert np.abs(r0["O_part"] - r1["O_part"]).max() < 1e-9
    shift_n = (Qn[0] @ u) / math.sqrt(d)                 # [q, Hq]
    assert np.abs((r1["LSE"][0] - r0["LSE"][0]) - shift_n.T).max() < 1e-9
    assert np.abs((r1["LSE_part"][0] - r0["LSE_part"][0]) - shift_n.T[None]).max() < 1e-9


def test_I9_other_blocks_cannot_leak_into_a_block():
    B, L, Hq, Hkv, d, b, a = 1, 40, 1, 1, 8, 8, 8
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    O0, _ = so.phase1_full(Q, K, V, b, a)
    for i in range(1, 5):
        K2, V2 = K.copy(), V.copy()
        for j in range(1, 5):
            if j != i:
                K2[:, j * b:(j + 1) * b] = np.nan
                V2[:, j * b:(j + 1) * b] = np.nan
        O1, _ = so.phase1_full(Q, K2, V2, b, a)
        assert np.array_equal(O0[:, i * b:(i + 1) * b], O1[:, i * b:(i + 1) * b])


def test_cache_holds_every_context_token_once():
    B, L, Hq, Hkv, d = 2, 19, 4, 2, 4
    _, K, V = rand_qkv(B, L, Hq, Hkv, d)
    Kc, Vc = so.kv_cache(K, V, L + 5)
    assert Kc.shape == (B, Hkv, L + 5, d)
    for beta in range(B):
        for g in range(Hkv):
            assert np.array_equal(Kc[beta, g, :L], K[beta, :, g])
            assert np.array_equal(Vc[beta, g, :L], V[beta, :, g])
    assert (Kc[:, :, L:] == 0).all() and (Vc[:, :, L:] == 0).all()
    with pytest.raises(ValueError):
        so.kv_cache(K, V, L - 1)


# ------------------------------------------------------------------ phase 2

def _phase2_setup(L, b, lq, nd, B=1, Hq=4, Hkv=2, d=8, qscale=2.0):
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    Kc, Vc = so.kv_cache(K, V, L + lq + nd)
    Qq, Kq, Vq = rand_qkv(B, lq, Hq, Hkv, d, scale=qscale)
    Qd, Kd, Vd = rand_qkv(B, nd, Hq, Hkv, d, scale=qscale)
    return (K, V, Kc, Vc, Qq, Kq, Vq, Qd, Kd, Vd)


@pytest.mark.parametrize("L,b", [(24, 8), (29, 8), (16, 32)])
def test_I5_phase2_equals_last_rows_of_causal_attention(L, b):
    lq, nd, Hq, Hkv = 5, 3, 4, 2
    K, V, Kc, Vc, Qq, Kq, Vq, Qd, Kd, Vd = _phase2_setup(L, b, lq, nd)
    # the oracle, call by call
    outs = []
    cache_len = L
    so.cache_append(Kc, Vc, cache_len, Kq, Vq)
    r = so.phase2_rows(Qq, Kc, Vc, L, b, cache_len)
    outs.append(r["O"]); cache_len += lq
    Om, _ = so.phase2_merged(r["O_part"], r["LSE_part"])
    assert np.abs(Om - r["O"]).max() < TOL
    for t in range(nd):
        so.cache_append(Kc, Vc, cache_len, Kd[:, t:t + 1], Vd[:, t:t + 1])
        r = so.phase2_rows(Qd[:, t:t + 1], Kc, Vc, L, b, cache_len)
        outs.append(r["O"]); cache_len += 1
        Om, _ = so.phase2_merged(r["O_part"], r["LSE_part"])
        assert np.abs(Om - r["O"]).max() < TOL
    O = np.concatenate(outs, axis=1)                      # [B, lq+nd, Hq, d]
    # library: causal attention over [context; query; decode], last rows
    Kall = np.concatenate([K, Kq, Kd], axis=1)
    Vall = np.concatenate([V, Vq, Vd], axis=1)
    Qall = np.concatenate([np.zeros((1, L, Hq, Qq.shape[3])), Qq, Qd], axis=1)
    for h in range(Hq):
        ref = sdpa_causal(Qall[0, :, h], Kall[0, :, h // 2], Vall[0, :, h // 2])[L:]
        assert np.abs(O[0, :, h] - ref).max() < TOL
    # separately written brute force, query-encode call
    Ob, LSEb = bf.phase2_dense(Qq, np.concatenate([K, Kq], 1), np.concatenate([V, Vq], 1), L)
    assert np.abs(outs[0] - Ob).max() < TOL


def test_I3_merge_is_order_and_partition_independent():
    L, lq = 24, 3
    K, V, Kc, Vc, Qq, Kq, Vq, *_ = _phase2_setup(L, 4, lq, 0)
    so.cache_append(Kc, Vc, L, Kq, Vq)
    base = None
    for b in (4, 6, 8, 24, 100):
        r = so.phase2_rows(Qq, Kc, Vc, L, b, L)
        Om, Lm = so.phase2_merged(r["O_part"], r["LSE_part"])
        if base is None:
            base = (r["O"], r["LSE"])
        assert np.abs(Om - base[0]).max() < TOL and np.abs(Lm - base[1]).max() < TOL
        assert np.abs(r["O"] - base[0]).max() < TOL
    # every permutation of the parts, sequential merge (Algorithm 2) vs Eq. 3-4
    r = so.phase2_rows(Qq, Kc, Vc, L, 6, L)            # 4 blocks + tail = 5 parts
    A = r["O_part"][0, :, 1, 2]
    lse = r["LSE_part"][0, :, 1, 2]
    want, want_lse = so.merge_closed_form(A, lse)
    assert np.abs(want - r["O"][0, 2, 1]).max() < TOL
    for perm in itertools.permutations(range(A.shape[0])):
        got, got_lse = so.merge_sequential(A, lse, perm)
        assert np.abs(got - want).max() < TOL and abs(got_lse - want_lse) < TOL


def test_merge_against_plain_sums_of_exponentials():
    """Eq. 3-4 typed out with s_h = exp(lse_h) directly (small magnitudes, so no
    stabilisation is needed) -- pins the stabilised merge and the corrected
    sequential update."""
    P, d = 6, 5
    A = RNG.standard_normal((P, d))
    lse = RNG.standard_normal(P) * 2.0
    s = np.exp(lse)
    want = (s[:, None] * A).sum(axis=0) / s.sum()
    for fn in (so.merge_closed_form, so.merge_sequential):
        got, got_lse = fn(A, lse)
        assert np.abs(got - want).max() < 1e-13
        assert abs(got_lse - math.log(s.sum())) < 1e-13
    # huge offsets must not overflow, and the result must not move
    for fn in (so.merge_closed_form, so.merge_sequential):
        got, got_lse = fn(A, lse + 5000.0)
        assert np.abs(got - want).max() < 1e-12
        assert abs(got_lse - 5000.0 - math.log(s.sum())) < 1e-9


def test_empty_parts_contribute_nothing():
    A = RNG.standard_normal((4, 3))
    lse = np.array([0.3, -math.inf, 1.1, -math.inf])
    A[1] = 123.0                                       # must be ignored
    want, want_lse = so.merge_closed_form(A[[0, 2]], lse[[0, 2]])
    for order in ([0, 1, 2, 3], [1, 3, 0, 2], [3, 2, 1, 0]):
        got, got_lse = so.merge_sequential(A, lse, order)
        assert np.abs(got - want).max() < 1e-13 and abs(got_lse - want_lse) < 1e-13
    got, got_lse = so.merge_closed_form(A, lse)
    assert np.abs(got - want).max() < 1e-13 and abs(got_lse - want_lse) < 1e-13
    z, zl = so.merge_closed_form(A, np.full(4, -math.inf))
    assert (z == 0).all() and zl == -math.inf
    o, l = so.attend(np.ones(3), np.zeros((0, 3)), np.zeros((0, 3)), 1.0)
    assert (o == 0).all() and l == -math.inf


def test_decode_token_attends_to_itself_and_all_before():
    """With one-hot values the decode output is the probability vector: token t
    must put mass on exactly L + lq + t + 1 keys (Algorithm 2: append, then
    attend)."""
    L, b, lq, nd, d = 10, 4, 3, 2, 4
    total = L + lq + nd
    Q, K, _ = rand_qkv(1, L, 1, 1, d)
    V = np.eye(total)[None, :L, None, :]
    Kc, Vc = so.kv_cache(K, V, total)
    Qn, Kn, _ = rand_qkv(1, lq + nd, 1, 1, d)
    Vn = np.eye(total)[None, L:, None, :]
    cache_len = L
    so.cache_append(Kc, Vc, cache_len, Kn[:, :lq], Vn[:, :lq])
    r = so.phase2_rows(Qn[:, :lq], Kc, Vc, L, b, cache_len)
    for j in range(lq):
        assert (r["O"][0, j, 0] > 0).sum() == L + j + 1
        assert (r["O"][0, j, 0, L + j + 1:] == 0).all()
    cache_len += lq
    for t in range(nd):
        so.cache_append(Kc, Vc, cache_len, Kn[:, lq + t:lq + t + 1], Vn[:, lq + t:lq + t + 1])
        r = so.phase2_rows(Qn[:, lq + t:lq + t + 1], Kc, Vc, L, b, cache_len)
        assert (r["O"][0, 0, 0] > 0).sum() == L + lq + t + 1
        cache_len += 1


# ------------------------------------------------- the pins must have teeth

def test_planted_mistakes_are_caught(monkeypatch):
    """Plant typical mistakes in the oracle (on the CPU) and check that the
    pins above would notice each one."""
    B, L, Hq, Hkv, d, b, a = 1, 23, 2, 1, 8, 8, 5
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d, scale=2.0)
    Ob, _ = bf.phase1_dense(Q, K, V, b, a)
    good = so.visible_keys

    def no_self(p, L_, b_, a_):
        ks = good(p, L_, b_, a_)
        return ks[ks != p] if ks.size > 1 else ks

    def whole_first_block_as_anchor(p, L_, b_, a_):
        return good(p, L_, b_, b_)

    def anchor_in_block_one_only(p, L_, b_, a_):
        return np.arange(max(0, (p // b_) * b_), p + 1)

    for wrong in (no_self, whole_first_block_as_anchor, anchor_in_block_one_only):
        monkeypatch.setattr(so, "visible_keys", wrong)
        O, _ = so.phase1_full(Q, K, V, b, a)
        assert np.abs(O - Ob).max() > 1e-6
    monkeypatch.setattr(so, "visible_keys", good)

    # the merge update as printed in Algorithm 2 (reusing the updated LSE and
    # exponentiating the output) disagrees with Eq. 3-4
    A = RNG.standard_normal((3, 4)); lse = np.array([0.2, -0.7, 1.3])
    want, _ = so.merge_closed_form(A, lse)
    s_g, A_g = lse[0], A[0].copy()
    for h in (1, 2):
        s_g = s_g + math.log1p(math.exp(lse[h] - s_g))
        A_g = math.exp(lse[h] - s_g) * A_g + np.exp(A[h] - s_g) * A[h]
    assert np.abs(A_g - want).max() > 1e-3
