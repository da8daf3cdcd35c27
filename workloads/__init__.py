"""Seeded synthetic workloads for the Star Attention hot path.

This module only *produces inputs*: shapes, random tensors, planted
query/key pairs and the list of rows a parity test looks at.  It contains none
of the method's arithmetic (no softmax, no masking rule, no merge) and is the
only code the CPU oracle's tests and the HIP path's tests have in common.

The five configurations are the attention shapes the paper evaluates
(Llama-3.1-8B / 70B, block = sequence/4 or a fixed 32K block for 1M tokens,
a reduced anchor for the anchor-size study; Section 3.1, Section 4.2 and the
block-size / anchor-size figures).  The paper measures on RULER-style
retrieval tasks; the "planted pairs" below stand in for them: a few query rows
are made to point at one far-away key so that the softmax is peaky, as it is
for a needle-in-a-haystack prompt.  No benchmark item is reproduced.

Tensor layouts (all contiguous):
    Q  [B, L, Hq, d]     K, V  [B, L, Hkv, d]          context (phase 1)
    Qq [B, lq, Hq, d]    Kq, Vq [B, lq, Hkv, d]        query tokens (phase 2)
    Qd [B, nd, Hq, d]    Kd, Vd [B, nd, Hkv, d]        decode-step tokens
Values are generated in fp32, rounded once to the configuration's dtype and
then handed to both sides unchanged.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class StarConfig:
    name: str
    dtype: str          # "fp32" | "bf16"
    B: int
    Hq: int
    Hkv: int
    d: int
    L: int              # context tokens
    b: int              # block size
    a: int              # anchor size (0 <= a <= b)
    lq: int             # query tokens
    nd: int             # decode steps
    seed: int
    q_scale: float = 1.0    # multiplies every Q-type tensor
    n_planted: int = 0      # planted (query row, key) pairs per (batch, head)
    gamma: float = 1.5      # planted row := gamma * key

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def n_blocks(self) -> int:
        return -(-self.L // self.b)

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    @property
    def elem_size(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    @property
    def cache_capacity(self) -> int:
        return self.L + self.lq + self.nd

    def scaled(self, **kw) -> "StarConfig":
        return replace(self, **kw)


CONFIGS: Dict[str, StarConfig] = {
    "C1": StarConfig("C1", "fp32", 1, 1, 1, 64, 1024, 256, 256, 32, 8, seed=1235),
    "C2": StarConfig("C2", "bf16", 1, 32, 8, 128, 32768, 4096, 4096, 128, 64,
                     seed=1236, n_planted=16),
    "C3": StarConfig("C3", "bf16", 1, 32, 8, 128, 131072, 16384, 16384, 256, 128,
                     seed=1237, n_planted=16),
    "C4": StarConfig("C4", "bf16", 1, 32, 8, 128, 1048576, 32768, 32768, 64, 32,
                     seed=1238, q_scale=1.5),
    "C5": StarConfig("C5", "bf16", 4, 64, 8, 128, 131072, 8192, 2048, 128, 64,
                     seed=1239, n_planted=16),
}


@dataclass
class StarInputs:
    cfg: StarConfig
    Q: torch.Tensor
    K: torch.Tensor
    V: torch.Tensor
    Qq: torch.Tensor
    Kq: torch.Tensor
    Vq: torch.Tensor
    Qd: torch.Tensor
    Kd: torch.Tensor
    Vd: torch.Tensor
    # planted pairs: (batch, head, row, key); for phase 2 `row` indexes the
    # concatenation [query tokens; decode tokens] and `key` the concatenation
    # [context; query tokens; decode tokens].
    planted_ctx: List[Tuple[int, int, int, int]] = field(default_factory=list)
    planted_q: List[Tuple[int, int, int, int]] = field(default_factory=list)


def _randn(shape, gen, device, dtype, scale=1.0, chunk_rows=1 << 16):
    """Seeded N(0, scale^2) tensor of `shape` = [B, T, H, d], drawn in fp32 in
    fixed-size chunks along T (so memory stays bounded) and rounded to `dtype`."""
    B, T, H, d = shape
    out = torch.empty(shape, dtype=dtype, device=device)
    for beta in range(B):
        for t0 in range(0, T, chunk_rows):
            t1 = min(T, t0 + chunk_rows)
            x = torch.randn((t1 - t0, H, d), generator=gen, device=device,
                            dtype=torch.float32)
            if scale != 1.0:
                x.mul_(scale)
            out[beta, t0:t1] = x.to(dtype)
    return out


def _plant_context(cfg: StarConfig, rng: np.random.Generator):
    """Choose (batch, head, row, key) pairs for the context tensor.  Of each
    head's pairs, 3/8 point into the anchor from a later block, 3/8 into the
    row's own block at or before the row, and 1/4 into a block the row cannot
    see in phase 1 (between the anchor and its own block) when one exists."""
    pairs = []
    n, b, a, L = cfg.n_blocks, cfg.b, cfg.a, cfg.L
    if cfg.n_planted == 0:
        return pairs
    n_anchor = (cfg.n_planted * 3) // 8
    n_hidden = cfg.n_planted // 4
    for beta in range(cfg.B):
        for h in range(cfg.Hq):
            rows = set()
            for t in range(cfg.n_planted):
                for _ in range(64):
                    i = int(rng.integers(1, n)) if n > 1 else 0
                    s, e = i * b, min((i + 1) * b, L)
                    r = int(rng.integers(s, e))
                    if r not in rows:
                        break
                rows.add(r)
                kind = "anchor" if t < n_anchor else (
                    "hidden" if t < n_anchor + n_hidden else "own")
                if kind == "anchor" and (i == 0 or a == 0):
                    kind = "own"
                if kind == "hidden" and not (i >= 1 and s > a):
                    kind = "own"
                if kind == "anchor":
                    k = int(rng.integers(0, a))
                elif kind == "hidden":
                    k = int(rng.integers(a, s))
                else:
                    k = int(rng.integers(s, r + 1))
                pairs.append((beta, h, r, k))
    return pairs


def _plant_query(cfg: StarConfig, rng: np.random.Generator):
    """Pairs for the query + decode rows: keys spread over distinct context
    blocks, plus one per head that points into the tail (an earlier query or
    decode token)."""
    pairs = []
    T = cfg.lq + cfg.nd
    if cfg.n_planted == 0 or T == 0:
        return pairs
    n = cfg.n_blocks
    cnt = min(cfg.n_planted, T)
    for beta in range(cfg.B):
        for h in range(cfg.Hq):
            rows = rng.choice(T, size=cnt, replace=False)
            for t, j in enumerate(int(x) for x in rows):
                if t == 0:
                    k = cfg.L + int(rng.integers(0, j + 1))
                else:
                    blk = (t - 1) % n
                    s, e = blk * cfg.b, min((blk + 1) * cfg.b, cfg.L)
                    k = int(rng.integers(s, e))
                pairs.append((beta, h, j, k))
    return pairs


def make_inputs(cfg: StarConfig, device: str | torch.device = "cpu") -> StarInputs:
    """Draw every tensor of one configuration from `cfg.seed` on `device`.

    The generator is torch's seeded generator for that device; the values a
    test compares are always the ones this call returned (the oracle receives
    host copies of the very same rounded tensors)."""
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed)
    dt = cfg.torch_dtype
    B, Hq, Hkv, d = cfg.B, cfg.Hq, cfg.Hkv, cfg.d
    qs = cfg.q_scale
    Q = _randn((B, cfg.L, Hq, d), gen, device, dt, qs)
    K = _randn((B, cfg.L, Hkv, d), gen, device, dt)
    V = _randn((B, cfg.L, Hkv, d), gen, device, dt)
    Qq = _randn((B, cfg.lq, Hq, d), gen, device, dt, qs)
    Kq = _randn((B, cfg.lq, Hkv, d), gen, device, dt)
    Vq = _randn((B, cfg.lq, Hkv, d), gen, device, dt)
    Qd = _randn((B, cfg.nd, Hq, d), gen, device, dt, qs)
    Kd = _randn((B, cfg.nd, Hkv, d), gen, device, dt)
    Vd = _randn((B, cfg.nd, Hkv, d), gen, device, dt)

    rng = np.random.default_rng(cfg.seed)
    planted_ctx = _plant_context(cfg, rng)
    planted_q = _plant_query(cfg, rng)
    G = cfg.G

    if planted_ctx:
        idx = torch.tensor(planted_ctx, dtype=torch.long, device=device)
        bi, hi, ri, ki = idx.unbind(1)
        Q[bi, ri, hi] = (cfg.gamma * K[bi, ki, hi // G].float()).to(dt)
    if planted_q:
        Kall = torch.cat([Kq, Kd], dim=1)            # tail keys, index key - L
        for (beta, h, j, k) in planted_q:
            src = K[beta, k, h // G] if k < cfg.L else Kall[beta, k - cfg.L, h // G]
            row = (cfg.gamma * src.float()).to(dt)
            if j < cfg.lq:
                Qq[beta, j, h] = row
            else:
                Qd[beta, j - cfg.lq, h] = row
    return StarInputs(cfg, Q, K, V, Qq, Kq, Vq, Qd, Kd, Vd, planted_ctx, planted_q)


def phase1_sample(cfg: StarConfig, planted_ctx, n_random: int = 256,
                  tile: int = 128, max_planted: int = 128,
                  heads_structural: int = 4) -> List[Tuple[int, int, int]]:
    """Seeded list of (batch, head, row) triples a phase-1 parity test checks:
    first/last row of every block, rows around the anchor boundary offset
    inside each block, rows around `tile`-row edges, planted rows and random
    rows.  Heads for the structural rows cycle through the KV groups (both
    ends of a group)."""
    rng = np.random.default_rng(cfg.seed + 77)
    G = cfg.G
    heads = sorted({0, G - 1, cfg.Hq - G, cfg.Hq - 1, (cfg.Hq // 2) | 0})
    heads = heads[:max(1, heads_structural)] if len(heads) > heads_structural else heads
    rows = set()
    for i in range(cfg.n_blocks):
        s, e = i * cfg.b, min((i + 1) * cfg.b, cfg.L)
        cand = [s, s + 1, e - 1, e - 2, s + cfg.a - 1, s + cfg.a, s + cfg.a + 1,
                s + tile - 1, s + tile, s + tile + 1, e - tile, e - tile - 1]
        for r in cand:
            if s <= r < e:
                rows.add(r)
    out = set()
    for k, r in enumerate(sorted(rows)):
        out.add((int(rng.integers(0, cfg.B)), heads[k % len(heads)], r))
    if planted_ctx:
        sel = rng.choice(len(planted_ctx), size=min(max_planted, len(planted_ctx)),
                         replace=False)
        for t in sel:
            beta, h, r, _ = planted_ctx[int(t)]
            out.add((beta, h, r))
    for _ in range(n_random):
        out.add((int(rng.integers(0, cfg.B)), int(rng.integers(0, cfg.Hq)),
                 int(rng.integers(0, cfg.L))))
    return sorted(out)


def phase2_heads(cfg: StarConfig, n_extra: int = 2) -> List[int]:
    """Query heads a phase-2 parity test checks on every row: both ends of the
    first KV group, the last head, plus a few seeded ones."""
    rng = np.random.default_rng(cfg.seed + 99)
    heads = {0, cfg.G - 1, cfg.Hq - 1}
    for _ in range(n_extra):
        heads.add(int(rng.integers(0, cfg.Hq)))
    return sorted(heads)
