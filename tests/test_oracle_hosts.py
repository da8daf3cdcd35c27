"""Pins for the host-by-host oracle (Algorithms 1 and 2 as each host runs
them).  It is checked against things written separately from it: the row-wise
oracle's visible-key rule, the brute-force token mask, a library causal
attention on the concatenated sequence, and closed forms of the merge.  In the
other direction these are also pins of the row-wise oracle: two formulations of
the method, written apart, must agree.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import brute_force as bf
from oracle import star_hosts as sh
from oracle import star_oracle as so

RNG = np.random.default_rng(2411)
TOL = 1e-11

SHAPES = [
    # B, L, Hq, Hkv, d, b, a
    (1, 24, 1, 1, 8, 6, 6),
    (2, 23, 4, 2, 4, 8, 3),
    (1, 20, 2, 1, 8, 5, 0),
    (1, 9, 2, 2, 4, 16, 16),
    (1, 13, 3, 1, 4, 2, 1),
]


def rand_qkv(B, L, Hq, Hkv, d):
    return (RNG.standard_normal((B, L, Hq, d)) * 2.0, RNG.standard_normal((B, L, Hkv, d)),
            RNG.standard_normal((B, L, Hkv, d)))


def test_block_runs_cover_every_block_once():
    for n in (1, 2, 5, 8, 13):
        for H in (1, 2, 3, 8, 16):
            runs = sh.block_runs(n, H)
            assert len(runs) == H
            assert runs[0][0] == 0 and runs[-1][1] == n
            assert all(r0[1] == r1[0] for r0, r1 in zip(runs, runs[1:]))
            sizes = [i1 - i0 for i0, i1 in runs]
            assert max(sizes) - min(sizes) <= 1


def test_causal_attention_is_the_library_routine():
    T, d = 11, 8
    q, k, v = (RNG.standard_normal((T, d)) for _ in range(3))
    o, lse = sh.causal_attention(q, k, v, 0.3)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, None], torch.from_numpy(k)[None, None],
        torch.from_numpy(v)[None, None], is_causal=True, scale=0.3)[0, 0].numpy()
    assert np.abs(o - ref).max() < 1e-12
    # lse of row t is the log of sum_{k <= t} exp(scale q.k), typed out
    for t in range(T):
        assert abs(lse[t] - math.log(sum(math.exp(0.3 * float(q[t] @ k[u])) for u in range(t + 1)))) < 1e-12


@pytest.mark.parametrize("B,L,Hq,Hkv,d,b,a", SHAPES)
@pytest.mark.parametrize("n_hosts", [1, 2, 3, 7])
def test_host_phase1_is_the_row_rule_and_the_token_mask(B, L, Hq, Hkv, d, b, a, n_hosts):
    """Every host's outputs, put side by side, are phase 1 of the row-wise oracle
    and of the brute-force token mask, however the blocks are dealt to hosts."""
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    O_ref, LSE_ref = so.phase1_full(Q, K, V, b, a)
    mask = bf.phase1_mask(L, b, a)
    n = so.num_blocks(L, b)
    kept_k = []
    for run in sh.block_runs(n, n_hosts):
        O, LSE, Kh, Vh = sh.host_phase1(Q, K, V, run, b, a)
        lo = min(run[0] * b, L)
        hi = lo + O.shape[1]
        assert np.abs(O - O_ref[:, lo:hi]).max(initial=0.0) < TOL
        assert np.abs(LSE - LSE_ref[:, :, lo:hi]).max(initial=0.0) < TOL
        kept_k.append(Kh)
        assert np.array_equal(Vh, V[:, lo:hi])
    # the hosts' kept K, concatenated, hold every context token exactly once
    assert np.array_equal(np.concatenate(kept_k, axis=1), K)
    G = Hq // Hkv
    for beta in range(B):
        for h in range(Hq):
            o, l = bf.dense_masked_attention(Q[beta, :, h], K[beta, :, h // G], V[beta, :, h // G],
                                             mask, 1.0 / np.sqrt(d))
            assert np.abs(O_ref[beta, :, h] - o).max() < TOL


def test_discarded_anchor_rows_repeat_the_first_block():
    """Inside an augmented block the anchor rows see anchor keys only, so what a
    host computes for them and throws away equals the first block's first `a`
    output rows: dropping them loses nothing."""
    B, L, Hq, Hkv, d, b, a = 1, 22, 2, 1, 8, 6, 4
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    first, _, _, _ = sh.host_phase1(Q, K, V, (0, 1), b, a)
    _, _, _, _, dropped = sh.host_phase1(Q, K, V, (1, 4), b, a, return_anchor_rows=True)
    assert len(dropped) == 3
    for anc in dropped:
        assert np.abs(anc - first[:, :a]).max() < TOL


@pytest.mark.parametrize("B,L,Hq,Hkv,d,b,a", SHAPES)
@pytest.mark.parametrize("n_hosts,query_host", [(1, 0), (2, 1), (3, 0), (4, 2), (9, 8)])
def test_cluster_phase2_is_one_softmax_over_everything(B, L, Hq, Hkv, d, b, a, n_hosts, query_host):
    """Gathering (A_h, lse_h) from any number of hosts, with any of them as the
    query host, gives the global attention of the row-wise oracle: one softmax
    over [context; earlier new tokens; self].  Hosts that own no block (more
    hosts than blocks) contribute nothing."""
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    calls = [tuple(RNG.standard_normal((B, ql, H, d)) for H in (Hq, Hkv, Hkv)) for ql in (3, 1, 2)]
    O_ctx, LSE_ctx, outs, lses, caches, lens = sh.run_cluster(
        Q, K, V, b, a, n_hosts, calls, capacity_tail=6, query_host=query_host)
    O_ref, LSE_ref = so.phase1_full(Q, K, V, b, a)
    assert np.abs(O_ctx - O_ref).max() < TOL and np.abs(LSE_ctx - LSE_ref).max() < TOL
    Kc, Vc = so.kv_cache(K, V, L + 6)
    cache_len = L
    for (Qn, Kn, Vn), O, LSE in zip(calls, outs, lses):
        so.cache_append(Kc, Vc, cache_len, Kn, Vn)
        ref = so.phase2_rows(Qn, Kc, Vc, L, b, cache_len)
        assert np.abs(O - ref["O"]).max() < TOL
        assert np.abs(LSE - ref["LSE"]).max() < TOL
        cache_len += Qn.shape[1]
    assert sum(lens) == cache_len


def test_cluster_phase2_is_plain_causal_attention_on_the_whole_sequence():
    """The new tokens' outputs are the last rows of library causal attention over
    [context; new tokens] (Section 2.2: global attention), whatever b and the
    number of hosts."""
    B, L, Hq, Hkv, d, b, a, ql = 1, 19, 2, 1, 8, 4, 4, 5
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    Qn, Kn, Vn = (RNG.standard_normal((B, ql, H, d)) for H in (Hq, Hkv, Hkv))
    _, _, outs, _, _, _ = sh.run_cluster(Q, K, V, b, a, 5, [(Qn, Kn, Vn)], capacity_tail=ql)
    for h in range(Hq):
        q = torch.from_numpy(np.concatenate([Q[0, :, h], Qn[0, :, h]]))[None, None]
        k = torch.from_numpy(np.concatenate([K[0, :, 0], Kn[0, :, 0]]))[None, None]
        v = torch.from_numpy(np.concatenate([V[0, :, 0], Vn[0, :, 0]]))[None, None]
        ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)[0, 0].numpy()
        assert np.abs(outs[0][0, :, h] - ref[L:]).max() < 1e-11


def test_merge_weights_closed_form():
    """Zero query: every key weighs the same, so a host with k_h keys has
    s_h = k_h, lse_h = log k_h, A_h = the mean of its values, and Eq. 3-4 give
    weights k_h / sum k and the mean over all values."""
    d = 4
    sizes = [3, 1, 6]
    Qn = np.zeros((1, 1, 1, d))
    A_h, l_h, allv = [], [], []
    for k in sizes:
        Kc = RNG.standard_normal((1, 1, k, d))
        Vc = RNG.standard_normal((1, 1, k, d))
        A, l = sh.host_phase2(Qn, Kc, Vc, k)
        assert abs(l[0, 0, 0] - math.log(k)) < 1e-13
        assert np.abs(A[0, 0, 0] - Vc[0, 0].mean(axis=0)).max() < 1e-13
        A_h.append(A)
        l_h.append(l)
        allv.append(Vc[0, 0])
    O, LSE = sh.gather_merge(A_h, l_h)
    assert np.abs(O[0, 0, 0] - np.concatenate(allv).mean(axis=0)).max() < 1e-13
    assert abs(LSE[0, 0, 0] - math.log(sum(sizes))) < 1e-13


def test_gather_merge_agrees_with_both_merges_of_the_row_oracle():
    H, B, Hq, ql, d = 5, 2, 3, 4, 8
    A = RNG.standard_normal((H, B, Hq, ql, d))
    lse = RNG.standard_normal((H, B, Hq, ql)) * 10.0
    lse[1] = -math.inf                                   # a host with an empty cache
    O, LSE = sh.gather_merge(list(A), list(lse))
    for beta in range(B):
        for h in range(Hq):
            for j in range(ql):
                o1, l1 = so.merge_closed_form(A[:, beta, h, j], lse[:, beta, h, j])
                o2, l2 = so.merge_sequential(A[:, beta, h, j], lse[:, beta, h, j], [3, 1, 0, 4, 2])
                assert np.abs(O[beta, j, h] - o1).max() < 1e-12 and abs(LSE[beta, h, j] - l1) < 1e-12
                assert np.abs(O[beta, j, h] - o2).max() < 1e-12 and abs(LSE[beta, h, j] - l2) < 1e-12


def test_context_host_with_an_empty_cache_gives_minus_infinity():
    Qn = RNG.standard_normal((1, 2, 2, 4))
    A, lse = sh.host_phase2(Qn, np.zeros((1, 1, 0, 4)), np.zeros((1, 1, 0, 4)), 0)
    assert np.all(A == 0.0) and np.all(lse == -math.inf)
    O, LSE = sh.gather_merge([A, A], [lse, lse])
    assert np.all(O == 0.0) and np.all(LSE == -math.inf)


def test_planted_mistakes_are_caught():
    """A host that kept the anchor's K/V, or a query host that let a new token
    see later new tokens, must break the agreement with the row-wise oracle."""
    B, L, Hq, Hkv, d, b, a = 1, 16, 1, 1, 4, 4, 4
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    Qn, Kn, Vn = (RNG.standard_normal((B, 3, 1, d)) for _ in range(3))
    Kc, Vc = so.kv_cache(K, V, L + 3)
    so.cache_append(Kc, Vc, L, Kn, Vn)
    ref = so.phase2_rows(Qn, Kc, Vc, L, b, L)
    # mistake 1: the second host's cache also holds the anchor copy
    _, _, Kh, Vh = sh.host_phase1(Q, K, V, (1, 4), b, a)
    Kbad = np.concatenate([K[:, :a], Kh], axis=1)
    Vbad = np.concatenate([V[:, :a], Vh], axis=1)
    _, _, K0, V0 = sh.host_phase1(Q, K, V, (0, 1), b, a)
    c0 = sh.host_cache(K0, V0, K0.shape[1] + 3)
    A0, l0 = sh.host_phase2(Qn, c0[0], c0[1], K0.shape[1], Kn, Vn)
    cb = sh.host_cache(Kbad, Vbad, Kbad.shape[1])
    Ab, lb = sh.host_phase2(Qn, cb[0], cb[1], Kbad.shape[1])
    O, _ = sh.gather_merge([A0, Ab], [l0, lb])
    assert np.abs(O - ref["O"]).max() > 1e-6
    # mistake 2: no causal mask among the new tokens (treated like a context host
    # whose cache already holds all of them)
    cg = sh.host_cache(Kh, Vh, Kh.shape[1])
    Ag, lg = sh.host_phase2(Qn, cg[0], cg[1], Kh.shape[1])
    c0 = sh.host_cache(K0, V0, K0.shape[1] + 3)
    c0[0][:, :, K0.shape[1]:] = np.transpose(Kn, (0, 2, 1, 3))
    c0[1][:, :, K0.shape[1]:] = np.transpose(Vn, (0, 2, 1, 3))
    A1, l1 = sh.host_phase2(Qn, c0[0], c0[1], K0.shape[1] + 3)
    O, _ = sh.gather_merge([A1, Ag], [l1, lg])
    assert np.abs(O[:, :-1] - ref["O"][:, :-1]).max() > 1e-6      # every token but the last is wrong
    assert np.abs(O[:, -1] - ref["O"][:, -1]).max() < TOL         # the last one sees everything anyway
