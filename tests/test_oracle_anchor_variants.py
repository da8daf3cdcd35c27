"""Pins for the oracle's anchor variants (ablation study, Section 4.1 / 4.2):
the previous block as anchor, and anchor keys/values given separately.  Each
check compares the oracle with a separately written brute force, a library
attention routine, or a case in which the variant must reduce to the method
itself.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import brute_force as bf
from oracle import star_oracle as so

RNG = np.random.default_rng(411)
TOL = 1e-11

SHAPES = [
    # B, L, Hq, Hkv, d, b, a
    (1, 23, 1, 1, 8, 8, 8),
    (2, 24, 4, 2, 4, 8, 3),
    (1, 20, 2, 1, 8, 5, 0),
    (1, 17, 3, 1, 16, 6, 6),
    (1, 9, 2, 2, 4, 16, 16),
    (1, 12, 1, 1, 4, 1, 1),
]


def rand_qkv(B, L, Hq, Hkv, d):
    return (RNG.standard_normal((B, L, Hq, d)) * 2.0, RNG.standard_normal((B, L, Hkv, d)),
            RNG.standard_normal((B, L, Hkv, d)))


@pytest.mark.parametrize("B,L,Hq,Hkv,d,b,a", SHAPES)
def test_previous_anchor_matches_brute_force_mask(B, L, Hq, Hkv, d, b, a):
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    O, LSE = so.phase1_full_variant(Q, K, V, b, a, so.ANCHOR_PREVIOUS)
    mask = bf.previous_anchor_mask(L, b, a)
    G = Hq // Hkv
    for beta in range(B):
        for h in range(Hq):
            o, l = bf.dense_masked_attention(Q[beta, :, h], K[beta, :, h // G], V[beta, :, h // G],
                                             mask, 1.0 / np.sqrt(d))
            assert np.abs(O[beta, :, h] - o).max() < TOL
            assert np.abs(LSE[beta, h] - l).max() < TOL


@pytest.mark.parametrize("B,L,Hq,Hkv,d,b,a", SHAPES)
def test_external_anchor_matches_brute_force(B, L, Hq, Hkv, d, b, a):
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    Ka = RNG.standard_normal((B, a, Hkv, d))
    Va = RNG.standard_normal((B, a, Hkv, d))
    O, LSE = so.phase1_full_variant(Q, K, V, b, a, so.ANCHOR_EXTERNAL, Ka, Va)
    Ob, LSEb = bf.external_anchor_dense(Q, K, V, Ka, Va, b)
    assert np.abs(O - Ob).max() < TOL
    assert np.abs(LSE - LSEb).max() < TOL


@pytest.mark.parametrize("B,L,Hq,Hkv,d,b,a", SHAPES)
def test_external_anchor_with_the_first_tokens_is_the_method_itself(B, L, Hq, Hkv, d, b, a):
    """Handing the first `a` context tokens in as the external anchor must give
    phase 1 of the method (checked against the brute force of the method)."""
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    a_eff = min(a, L)
    O, LSE = so.phase1_full_variant(Q, K, V, b, a_eff, so.ANCHOR_EXTERNAL,
                                    K[:, :a_eff].copy(), V[:, :a_eff].copy())
    Ob, LSEb = bf.phase1_dense(Q, K, V, b, a_eff)
    assert np.abs(O - Ob).max() < TOL
    assert np.abs(LSE - LSEb).max() < TOL


def test_variant_entry_with_first_mode_is_the_method_itself():
    Q, K, V = rand_qkv(1, 30, 2, 1, 8)
    O, LSE = so.phase1_full_variant(Q, K, V, 7, 5, so.ANCHOR_FIRST)
    Ob, LSEb = bf.phase1_dense(Q, K, V, 7, 5)
    assert np.abs(O - Ob).max() < TOL and np.abs(LSE - LSEb).max() < TOL


def test_previous_block_anchor_is_library_sliding_window_attention():
    """With a = b, rows of block i >= 2 are the last rows of library causal
    attention over the two consecutive blocks [c_(i-1); c_i]."""
    B, L, Hq, Hkv, d, b = 1, 50, 2, 1, 8, 12
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    O, _ = so.phase1_full_variant(Q, K, V, b, b, so.ANCHOR_PREVIOUS)
    for i in range(1, -(-L // b)):
        s, e = i * b, min((i + 1) * b, L)
        for h in range(Hq):
            q = np.concatenate([np.zeros((b, d)), Q[0, s:e, h]])
            tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(x)).double()[None, None]
                          for x in (q, K[0, s - b:e, 0], V[0, s - b:e, 0]))
            ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
            assert np.abs(O[0, s:e, h] - ref[0, 0, b:].numpy()).max() < 1e-10


def test_previous_anchor_with_two_full_blocks_is_full_causal_attention():
    B, L, Hq, Hkv, d, b = 1, 16, 2, 2, 4, 8
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    O, LSE = so.phase1_full_variant(Q, K, V, b, b, so.ANCHOR_PREVIOUS)
    Ob, LSEb = bf.phase1_dense(Q, K, V, L, L)          # one block = full causal
    assert np.abs(O - Ob).max() < TOL and np.abs(LSE - LSEb).max() < TOL


def test_previous_anchor_reads_nothing_outside_its_window():
    """Garbage in every block other than the row's own and the anchor window
    just before it must not change the row."""
    B, L, Hq, Hkv, d, b, a = 1, 40, 1, 1, 4, 10, 4
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    O, _ = so.phase1_full_variant(Q, K, V, b, a, so.ANCHOR_PREVIOUS)
    i = 2
    s, e = i * b, (i + 1) * b
    K2, V2 = K.copy(), V.copy()
    K2[:, :s - a] = np.nan; V2[:, :s - a] = np.nan
    K2[:, e:] = np.nan; V2[:, e:] = np.nan
    for p in range(s, e):
        o, _ = so.phase1_row_variant(Q, K2, V2, 0, 0, p, b, a, so.ANCHOR_PREVIOUS)
        assert np.array_equal(o, O[0, p, 0])


def test_a_shifted_anchor_window_is_caught():
    """A plausible mistake -- the window [s - a - 1, s - 1) instead of [s - a, s)
    -- disagrees with the brute-force mask."""
    B, L, Hq, Hkv, d, b, a = 1, 24, 1, 1, 4, 8, 3
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    mask = bf.previous_anchor_mask(L, b, a)
    o_ref, _ = bf.dense_masked_attention(Q[0, :, 0], K[0, :, 0], V[0, :, 0], mask, 0.5)
    p = 2 * b + 1
    ks = np.concatenate([np.arange(2 * b - a - 1, 2 * b - 1), np.arange(2 * b, p + 1)])
    o_bad, _ = so.attend(Q[0, p, 0], K[0, ks, 0], V[0, ks, 0], 0.5)
    assert np.abs(o_bad - o_ref[p]).max() > 1e-6


@pytest.mark.parametrize("B,L,Hq,Hkv,d,b,a", SHAPES)
def test_per_block_anchors_match_brute_force(B, L, Hq, Hkv, d, b, a):
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    n = -(-L // b)
    Ka = RNG.standard_normal((B, n, a, Hkv, d))
    Va = RNG.standard_normal((B, n, a, Hkv, d))
    O, LSE = so.phase1_full_variant(Q, K, V, b, a, so.ANCHOR_PER_BLOCK, Ka, Va)
    Ob, LSEb = bf.external_anchor_dense(Q, K, V, Ka, Va, b)
    assert np.abs(O - Ob).max() < TOL
    assert np.abs(LSE - LSEb).max() < TOL


def test_per_block_anchors_that_are_all_alike_are_one_external_anchor():
    B, L, Hq, Hkv, d, b, a = 1, 26, 2, 1, 8, 7, 4
    Q, K, V = rand_qkv(B, L, Hq, Hkv, d)
    Ka = RNG.standard_normal((B, a, Hkv, d))
    Va = RNG.standard_normal((B, a, Hkv, d))
    n = -(-L // b)
    O1, L1 = so.phase1_full_variant(Q, K, V, b, a, so.ANCHOR_EXTERNAL, Ka, Va)
    O2, L2 = so.phase1_full_variant(Q, K, V, b, a, so.ANCHOR_PER_BLOCK,
                                    np.repeat(Ka[:, None], n, axis=1), np.repeat(Va[:, None], n, axis=1))
    assert np.array_equal(O1, O2) and np.array_equal(L1, L2)


def test_position_id_ablation_composes_from_rotation_and_per_block_anchors():
    """Section 4.1, "position IDs same as previous block": the anchor keeps the
    first block's content but is encoded at the positions just before each
    block.  Composed here from the rotation and per-block anchors, and checked
    against a brute force that lays out [anchor at those positions; block]
    explicitly.  With rotary embeddings logits depend on position differences
    only, so this anchor is the first block seen from a = b tokens away."""
    B, L, Hq, Hkv, d, b, theta = 1, 24, 2, 1, 8, 8, 10000.0
    a = b
    Qp, Kp, V = rand_qkv(B, L, Hq, Hkv, d)            # unrotated projections
    pos = np.arange(L)
    Q = so.rope_rotate(Qp, pos, theta)
    K = so.rope_rotate(Kp, pos, theta)
    n = L // b
    Ka = np.zeros((B, n, a, Hkv, d))
    Va = np.zeros((B, n, a, Hkv, d))
    for i in range(1, n):
        Ka[:, i] = so.rope_rotate(Kp[:, :a], i * b - a + np.arange(a), theta)   # ids of the previous block
        Va[:, i] = V[:, :a]
    O, LSE = so.phase1_full_variant(Q, K, V, b, a, so.ANCHOR_PER_BLOCK, Ka, Va)
    # brute force: block i attends [first block's tokens at positions s-a..s-1 ; its own tokens]
    for i in range(1, n):
        s = i * b
        for h in range(Hq):
            kk = np.concatenate([Ka[0, i, :, 0], K[0, s:s + b, 0]])
            vv = np.concatenate([V[0, :a, 0], V[0, s:s + b, 0]])
            mask = np.zeros((b, a + b), dtype=bool)
            for r in range(b):
                mask[r, :a + r + 1] = True
            o, l = bf.dense_masked_attention(Q[0, s:s + b, h], kk, vv, mask, 1.0 / np.sqrt(d))
            assert np.abs(O[0, s:s + b, h] - o).max() < 1e-10
            assert np.abs(LSE[0, h, s:s + b] - l).max() < 1e-10
    # ... and it differs from the method itself (ids 0..a-1), so the test is not vacuous
    O0, _ = so.phase1_full_variant(Q, K, V, b, a, so.ANCHOR_FIRST)
    assert np.abs(O0[0, b:] - O[0, b:]).max() > 1e-3
