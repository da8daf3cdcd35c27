"""Seeded random small shapes through the whole hot path, every row against the
oracle: odd sizes, tiny blocks, anchors of every size, contexts shorter than a
key tile, head counts that exercise every GQA packing."""
import numpy as np
import pytest

import workloads
from tests import parity_harness as ph

pytestmark = pytest.mark.gpu


def _cases(dtype, n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for k in range(n):
        Hkv = int(rng.choice([1, 2, 3]))
        G = int(rng.choice([1, 2, 3, 4, 8])) if dtype == "bf16" else int(rng.choice([1, 2, 4]))
        L = int(rng.choice([1, 7, 33, 64, 65, 200, 513, 1100, 2300]))
        b = int(rng.choice([1, 5, 16, 63, 64, 100, 256, 700, 4096]))
        a = int(rng.integers(0, b + 1)) if rng.random() < 0.7 else int(rng.choice([0, b]))
        lq = int(rng.choice([1, 2, 3, 15, 16, 17, 33, 70]))
        nd = int(rng.choice([0, 1, 3]))
        B = int(rng.choice([1, 2]))
        d = 128 if dtype == "bf16" else int(rng.choice([64, 128]))
        out.append(pytest.param(B, Hkv * G, Hkv, d, L, b, a, lq, nd, 1000 * seed + k,
                                id=f"{dtype}-B{B}-H{Hkv * G}/{Hkv}-d{d}-L{L}-b{b}-a{a}-lq{lq}-nd{nd}"))
    return out


@pytest.mark.parametrize("B,Hq,Hkv,d,L,b,a,lq,nd,seed", _cases("bf16", 14, 7))
def test_random_bf16_shapes(B, Hq, Hkv, d, L, b, a, lq, nd, seed):
    cfg = workloads.StarConfig("fuzz", "bf16", B, Hq, Hkv, d, L, b, a, lq, nd, seed=seed, n_planted=2)
    rep = ph.run_parity(cfg, all_rows=True)
    print(f"\n[{cfg}] {rep.detail}", flush=True)
    assert rep.ok, rep.detail


@pytest.mark.parametrize("B,Hq,Hkv,d,L,b,a,lq,nd,seed", _cases("fp32", 8, 11))
def test_random_fp32_shapes(B, Hq, Hkv, d, L, b, a, lq, nd, seed):
    cfg = workloads.StarConfig("fuzz", "fp32", B, Hq, Hkv, d, L, b, a, lq, nd, seed=seed, n_planted=2)
    rep = ph.run_parity(cfg, all_rows=True)
    print(f"\n[{cfg}] {rep.detail}", flush=True)
    assert rep.ok, rep.detail
