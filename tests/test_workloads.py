"""The seeded workload generator: shapes, determinism, and that planted pairs do
what the recipe says (checked with the oracle on a small configuration)."""
import math

import numpy as np
import torch

import workloads
from oracle import star_oracle as so


def test_config_table_matches_the_five_benchmark_shapes():
    c = workloads.CONFIGS
    assert (c["C1"].dtype, c["C1"].L, c["C1"].b, c["C1"].a, c["C1"].d) == ("fp32", 1024, 256, 256, 64)
    assert (c["C2"].Hq, c["C2"].Hkv, c["C2"].L, c["C2"].b, c["C2"].lq, c["C2"].nd) == (32, 8, 32768, 4096, 128, 64)
    assert (c["C3"].L, c["C3"].b, c["C3"].a, c["C3"].lq, c["C3"].nd) == (131072, 16384, 16384, 256, 128)
    assert (c["C4"].L, c["C4"].b, c["C4"].n_blocks, c["C4"].q_scale) == (1048576, 32768, 32, 1.5)
    assert (c["C5"].B, c["C5"].Hq, c["C5"].Hkv, c["C5"].b, c["C5"].a) == (4, 64, 8, 8192, 2048)
    for cfg in c.values():
        assert cfg.cache_capacity == cfg.L + cfg.lq + cfg.nd


def test_inputs_are_seeded_and_shaped():
    cfg = workloads.StarConfig("t", "bf16", 2, 4, 2, 128, 96, 32, 16, 5, 3, seed=5, n_planted=4)
    a = workloads.make_inputs(cfg, "cpu")
    b = workloads.make_inputs(cfg, "cpu")
    for name in ("Q", "K", "V", "Qq", "Kq", "Vq", "Qd", "Kd", "Vd"):
        x, y = getattr(a, name), getattr(b, name)
        assert x.dtype == torch.bfloat16 and torch.equal(x, y)
    assert a.Q.shape == (2, 96, 4, 128) and a.K.shape == (2, 96, 2, 128)
    assert a.Qq.shape == (2, 5, 4, 128) and a.Kd.shape == (2, 3, 2, 128)
    assert a.planted_ctx == b.planted_ctx and len(a.planted_ctx) == 2 * 4 * 4


def test_planted_rows_are_peaky_where_visible_and_inert_where_hidden():
    cfg = workloads.StarConfig("t", "fp32", 1, 2, 1, 64, 256, 64, 32, 6, 2, seed=9, n_planted=8)
    inp = workloads.make_inputs(cfg, "cpu")
    Q, K, V = (x.numpy() for x in (inp.Q, inp.K, inp.V))
    seen = hidden = 0
    for (beta, h, r, k) in inp.planted_ctx:
        ks = so.visible_keys(r, cfg.L, cfg.b, cfg.a)
        assert np.allclose(Q[beta, r, h], cfg.gamma * K[beta, k, 0], atol=1e-6)
        logits = (K[beta, ks, 0].astype(np.float64) @ Q[beta, r, h]) / math.sqrt(cfg.d)
        p = np.exp(logits - logits.max()); p /= p.sum()
        if k in ks:
            seen += 1
            assert p[list(ks).index(k)] > 0.5            # the needle takes most of the mass
        else:
            hidden += 1
            assert p.max() < 0.5                          # phase 1 cannot see it
    assert seen > 0 and hidden > 0
    # query/decode rows: the first pair of every head points into the tail
    tails = [k for (_, _, _, k) in inp.planted_q if k >= cfg.L]
    assert len(tails) == cfg.B * cfg.Hq


def test_parity_samples_cover_block_and_tile_edges():
    cfg = workloads.CONFIGS["C3"]
    tr = workloads.phase1_sample(cfg, [], n_random=32)
    rows = {r for (_, _, r) in tr}
    for i in range(cfg.n_blocks):
        s = i * cfg.b
        assert {s, s + cfg.b - 1, s + 127, s + 128} <= rows
    assert all(0 <= b < cfg.B and 0 <= h < cfg.Hq and 0 <= r < cfg.L for b, h, r in tr)
    hs = workloads.phase2_heads(cfg)
    assert 0 in hs and cfg.G - 1 in hs and cfg.Hq - 1 in hs
