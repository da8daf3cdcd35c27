"""Pins for the oracle's rotary position embedding: a complex-number
formulation evaluated by numpy's complex routines, the property that makes the
embedding "relative" (logits depend on position differences only), and exact
special cases.  CPU only."""
import numpy as np
import pytest

from oracle import brute_force as bf
from oracle import star_oracle as so

RNG = np.random.default_rng(2104_09864)


def rope_complex(X, positions, theta):
    """x_i + i x_(i+d/2), multiplied by exp(i pos theta^(-2i/d)) with numpy's
    complex arithmetic."""
    d = X.shape[-1]
    half = d // 2
    z = X[..., :half] + 1j * X[..., half:]
    w = np.exp(1j * np.outer(np.asarray(positions, np.float64),
                             np.power(float(theta), -np.arange(half) * 2.0 / d)))
    y = z * w[:, None, :]
    return np.concatenate([y.real, y.imag], axis=-1)


@pytest.mark.parametrize("d,theta", [(8, 10000.0), (64, 10000.0), (128, 500000.0)])
def test_rotation_equals_complex_multiplication(d, theta):
    X = RNG.standard_normal((2, 37, 3, d))
    pos = RNG.integers(0, 200000, size=37)
    got = so.rope_rotate(X, pos, theta)
    assert np.abs(got - rope_complex(X, pos, theta)).max() < 1e-9


def test_position_zero_is_the_identity_and_norms_are_kept():
    X = RNG.standard_normal((1, 5, 2, 16))
    assert np.array_equal(so.rope_rotate(X, np.zeros(5, int), 10000.0), X)
    Y = so.rope_rotate(X, [3, 1000, 77, 123456, 9], 10000.0)
    assert np.abs(np.linalg.norm(Y, axis=-1) - np.linalg.norm(X, axis=-1)).max() < 1e-12
    # pairwise norms too: each (i, i + d/2) pair is turned, nothing else mixes
    assert np.abs((Y[..., :8] ** 2 + Y[..., 8:] ** 2) - (X[..., :8] ** 2 + X[..., 8:] ** 2)).max() < 1e-12


def test_two_dimensional_head_is_a_plane_rotation():
    x = np.array([[[[1.0, 0.0]]]])
    y = so.rope_rotate(x, [1], 10000.0)          # d = 2: one pair, frequency theta^0 = 1
    assert np.abs(y[0, 0, 0] - [np.cos(1.0), np.sin(1.0)]).max() < 1e-15
    y = so.rope_rotate(np.array([[[[0.0, 1.0]]]]), [2], 10000.0)
    assert np.abs(y[0, 0, 0] - [-np.sin(2.0), np.cos(2.0)]).max() < 1e-15


def test_logits_depend_on_position_differences_only():
    d = 32
    q = RNG.standard_normal((1, 1, 1, d))
    k = RNG.standard_normal((1, 1, 1, d))
    def logit(pq, pk):
        return float(so.rope_rotate(q, [pq], 1e4)[0, 0, 0] @ so.rope_rotate(k, [pk], 1e4)[0, 0, 0])
    base = logit(1000, 993)
    for shift in (1, 17, 50000):
        assert abs(logit(1000 + shift, 993 + shift) - base) < 1e-8
    assert abs(logit(1000, 994) - base) > 1e-3     # ... and do depend on the difference


def test_phase1_with_rotation_matches_brute_force_on_rotated_tensors():
    B, L, Hq, Hkv, d, b, a, theta = 1, 22, 4, 2, 8, 6, 4, 10000.0
    Q = RNG.standard_normal((B, L, Hq, d)) * 2
    K = RNG.standard_normal((B, L, Hkv, d))
    V = RNG.standard_normal((B, L, Hkv, d))
    triples = [(0, h, p) for h in range(Hq) for p in range(L)]
    O, LSE = so.phase1_rope_rows(Q, K, V, triples, b, a, theta, pos0=5)
    Qr = rope_complex(Q, 5 + np.arange(L), theta)
    Kr = rope_complex(K, 5 + np.arange(L), theta)
    Ob, LSEb = bf.phase1_dense(Qr, Kr, V, b, a)
    for t, (beta, h, p) in enumerate(triples):
        assert np.abs(O[t] - Ob[beta, p, h]).max() < 1e-10
        assert abs(LSE[t] - LSEb[beta, h, p]) < 1e-10


def test_shifting_every_position_leaves_a_single_block_unchanged():
    """One block = full causal attention, where only position differences enter:
    pos0 must not matter.  (With several blocks it does not matter either, since
    the anchor moves with the context; checked on the second block.)"""
    B, L, Hq, Hkv, d = 1, 20, 2, 1, 16
    Q = RNG.standard_normal((B, L, Hq, d))
    K = RNG.standard_normal((B, L, Hkv, d))
    V = RNG.standard_normal((B, L, Hkv, d))
    triples = [(0, h, p) for h in range(Hq) for p in range(L)]
    for b, a in ((32, 32), (8, 8)):
        O0, L0 = so.phase1_rope_rows(Q, K, V, triples, b, a, 1e4, pos0=0)
        O1, L1 = so.phase1_rope_rows(Q, K, V, triples, b, a, 1e4, pos0=4321)
        assert np.abs(O0 - O1).max() < 1e-9 and np.abs(L0 - L1).max() < 1e-9


def test_cache_holds_rotated_keys_and_plain_values():
    B, L, Hkv, d = 2, 9, 2, 8
    K = RNG.standard_normal((B, L, Hkv, d))
    V = RNG.standard_normal((B, L, Hkv, d))
    Kc, Vc = so.kv_cache_rope(K, V, 12, 1e4, pos0=3)
    Kr = rope_complex(K, 3 + np.arange(L), 1e4)
    for beta in range(B):
        for g in range(Hkv):
            assert np.abs(Kc[beta, g, :L] - Kr[beta, :, g]).max() < 1e-12
            assert np.array_equal(Vc[beta, g, :L], V[beta, :, g])
    assert not Kc[:, :, L:].any() and not Vc[:, :, L:].any()


def test_a_wrong_pairing_is_caught():
    """Pairing neighbours (2i, 2i+1) instead of (i, i + d/2) -- the other common
    convention -- must disagree with the oracle."""
    d = 8
    X = RNG.standard_normal((1, 3, 1, d))
    pos = [1, 2, 3]
    inv = np.power(1e4, -np.arange(d // 2) * 2.0 / d)
    ang = np.outer(pos, inv)
    Y = np.empty_like(X)
    Y[..., 0::2] = X[..., 0::2] * np.cos(ang)[:, None, :] - X[..., 1::2] * np.sin(ang)[:, None, :]
    Y[..., 1::2] = X[..., 1::2] * np.cos(ang)[:, None, :] + X[..., 0::2] * np.sin(ang)[:, None, :]
    assert np.abs(Y - so.rope_rotate(X, pos, 1e4)).max() > 1e-2


def test_phase2_inputs_sit_behind_the_cache():
    Qn = RNG.standard_normal((1, 3, 2, 8))
    Kn = RNG.standard_normal((1, 3, 1, 8))
    Qr, Kr = so.phase2_rope_inputs(Qn, Kn, cache_len=40, theta=1e4, pos0=2)
    assert np.abs(Qr - rope_complex(Qn, [42, 43, 44], 1e4)).max() < 1e-12
    assert np.abs(Kr - rope_complex(Kn, [42, 43, 44], 1e4)).max() < 1e-12
