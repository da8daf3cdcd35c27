"""GPU parity of the entry points that take unrotated projections
(star_attn_rope, star_attn_phase1_rope, star_attn_phase2_rope) against the fp64
oracle, through the C-ABI."""
import numpy as np
import pytest
import torch

import paper_2411_17116_amd as sa
import workloads
from oracle import star_oracle as so
from tests import parity_harness as ph

pytestmark = pytest.mark.gpu


def _storage_close(got: torch.Tensor, want64: np.ndarray, dtype: str):
    """Rotated values as stored: fp32 within 2e-6 relative to the row scale;
    bf16 within one rounding step of the exact value (2^-8 relative, with slack
    for values that sit on a rounding boundary, plus the fp32 arithmetic error of
    the rotation, which dominates where a pair cancels to almost nothing)."""
    g = got.float().cpu().numpy().astype(np.float64)
    err = np.abs(g - want64)
    if dtype == "fp32":
        return float((err / (1.0 + np.abs(want64))).max()) <= 2e-6
    return bool((err <= 2.0 ** -7 * np.abs(want64) + 2e-6).all())


@pytest.mark.parametrize("dtype,d", [("fp32", 64), ("fp32", 128), ("bf16", 128)])
@pytest.mark.parametrize("pos0,theta", [(0, 10000.0), (1_000_000, 500000.0)])
def test_rotation_alone(dtype, d, pos0, theta):
    B, T, H = 2, 300, 3
    tdt = torch.float32 if dtype == "fp32" else torch.bfloat16
    gen = torch.Generator().manual_seed(d + pos0 % 97)
    X = torch.randn((B, T, H, d), generator=gen).to(tdt).cuda()
    shape = sa.StarShape.make(dtype, B, H, H, d, T, T, T, T)
    want = so.rope_rotate(X.float().cpu().numpy(), pos0 + np.arange(T), theta)
    Y = torch.empty_like(X)
    print(f"rope {dtype} d={d} pos0={pos0}", flush=True)
    sa.rope(shape, X, Y, theta, pos0=pos0)
    torch.cuda.synchronize()
    assert _storage_close(Y, want, dtype)
    X2 = X.clone()
    sa.rope(shape, X2, X2, theta, pos0=pos0)               # in place
    torch.cuda.synchronize()
    assert torch.equal(X2, Y)


def _stored(dtype):
    """The storage rounding of the operator's rotated tensors (it hands rotated Q
    back and keeps rotated K in the cache in the configuration's dtype; attention
    is defined on what is stored)."""
    if dtype == "fp32":
        return lambda x: np.asarray(x, np.float32).astype(np.float64)
    return lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(torch.bfloat16).double().numpy()


def _rope_path(cfg, theta, pos0, triples=None, heads=None, decode_steps=None):
    """Whole hot path on unrotated inputs against the oracle."""
    stored = _stored(cfg.dtype)
    inp = workloads.make_inputs(cfg, "cuda")
    run = ph.HipRun(cfg, inp, "cuda")
    tol = ph.TOL[cfg.dtype]
    # the oracle's view: rotate the stored (pre-rotation) values in float64
    Q0 = inp.Q.clone()
    print(f"[{cfg.name}] phase1_rope L={cfg.L} b={cfg.b} a={cfg.a} theta={theta} pos0={pos0}", flush=True)
    sa.phase1_rope(run.shape, theta, inp.Q, inp.K, inp.V, run.O_ctx, run.Kc, run.Vc, pos0=pos0,
                   LSE_ctx=run.LSE_ctx)
    torch.cuda.synchronize()
    if triples is None:
        triples = [(beta, h, p) for beta in range(cfg.B) for h in range(cfg.Hq) for p in range(cfg.L)]
    O_ref, L_ref = so.phase1_rope_rows(ph.LazyTensor(Q0), ph.LazyTensor(inp.K), ph.LazyTensor(inp.V),
                                       triples, cfg.b, cfg.a, theta, pos0=pos0, storage=stored)
    idx = torch.tensor(triples, dtype=torch.long, device="cuda")
    bi, hi, ri = idx.unbind(1)
    eo = np.abs(run.O_ctx[bi, ri, hi].float().cpu().numpy() - O_ref).max()
    el = np.abs(run.LSE_ctx[bi, hi, ri].cpu().numpy() - L_ref).max()
    print(f"   phase 1: max|dO|={eo:.3g} max|dLSE|={el:.3g}", flush=True)
    assert eo <= tol["o"] and el <= tol["lse"]
    # For the record (not asserted): the same rows against the oracle WITHOUT the
    # storage rounding of the rotated q and k, i.e. attention on the exact fp64
    # rotation.  The difference to the figures above is what rounding the rotated
    # tensors to the storage dtype costs -- input quantisation, not compute error.
    sub = triples if len(triples) <= 4096 else triples[:: len(triples) // 4096 + 1]
    O_u, L_u = so.phase1_rope_rows(ph.LazyTensor(Q0), ph.LazyTensor(inp.K), ph.LazyTensor(inp.V),
                                   sub, cfg.b, cfg.a, theta, pos0=pos0, storage=None)
    si = torch.tensor(sub, dtype=torch.long, device="cuda")
    sb, sh, sr = si.unbind(1)
    eo_u = np.abs(run.O_ctx[sb, sr, sh].float().cpu().numpy() - O_u).max()
    el_u = np.abs(run.LSE_ctx[sb, sh, sr].cpu().numpy() - L_u).max()
    print(f"   phase 1 against the unrounded fp64 rotation ({len(sub)} rows, not asserted): "
          f"max|dO|={eo_u:.3g} max|dLSE|={el_u:.3g}", flush=True)
    # Q was rotated in place; the cache holds rotated K and plain V (sampled heads)
    rows = sorted({p for _, _, p in triples})[:64]
    pos = pos0 + np.asarray(rows)
    for beta, g in [(0, 0), (cfg.B - 1, cfg.Hkv - 1)]:
        wantK = so.rope_rotate(inp.K[beta, rows, g].float().cpu().numpy()[:, None, :], pos, theta)[:, 0]
        assert _storage_close(run.Kc[beta, g, rows], wantK, cfg.dtype)
        assert torch.equal(run.Vc[beta, g, :cfg.L], inp.V[beta, :, g])
    wantQ = so.rope_rotate(Q0[0, rows].float().cpu().numpy(), pos, theta)
    assert _storage_close(inp.Q[0, rows], wantQ, cfg.dtype)

    # phase 2: the oracle rotates every appended tensor at its own positions and
    # then runs its ordinary definition on the rotated values
    heads = list(range(cfg.Hq)) if heads is None else heads
    def rot(t, start):
        n = t.shape[1]
        return torch.from_numpy(stored(so.rope_rotate(t.float().cpu().numpy(),
                                                      pos0 + start + np.arange(n), theta))).float()

    class RotatedContext:
        """Context keys rotated on demand (large contexts are not rotated whole)."""
        def __init__(self, K):
            self.K = K
            self.shape = K.shape
        def head(self, beta, g):
            return rot(self.K[beta:beta + 1, :, g:g + 1], 0)[0, :, 0]

    Qq0, Qd0 = inp.Qq.clone(), inp.Qd.clone()
    print("   phase 2: query call", flush=True)
    cl = run.cache_len
    O = torch.empty_like(inp.Qq)
    P = cfg.n_blocks + 1
    Op = torch.empty((cfg.B, P, cfg.Hq, cfg.lq, cfg.d), dtype=torch.float32, device="cuda")
    Lp = torch.empty((cfg.B, P, cfg.Hq, cfg.lq), dtype=torch.float32, device="cuda")
    sa.phase2_rope(run.shape, theta, cl, inp.Qq, inp.Kq, inp.Vq, run.Kc, run.Vc, O, run.ws, pos0=pos0,
                   O_part=Op, LSE_part=Lp)
    torch.cuda.synchronize()
    Kq_r, Kd_r = rot(inp.Kq, cfg.L), rot(inp.Kd, cfg.L + cfg.lq)
    Qq_r, Qd_r = rot(Qq0, cfg.L), rot(Qd0, cfg.L + cfg.lq)

    class Cache:
        """[B, Hkv, rows, d] view of rotated context + rotated appended keys."""
        def __init__(self, parts_fn, rows):
            self.parts_fn = parts_fn
            self.shape = (cfg.B, cfg.Hkv, rows, cfg.d)
        def __getitem__(self, idx):
            beta, g, sl = idx
            return self.parts_fn(beta, g)[sl].numpy()

    ctx = RotatedContext(inp.K)
    memo = {}
    def kparts(beta, g):
        if (beta, g) not in memo:
            memo.clear()
            memo[(beta, g)] = torch.cat([ctx.head(beta, g), Kq_r[beta, :, g], Kd_r[beta, :, g]], dim=0)
        return memo[(beta, g)]
    def vparts(beta, g):
        return torch.cat([inp.V[beta, :, g], inp.Vq[beta, :, g], inp.Vd[beta, :, g]], dim=0).float().cpu()
    total_rows = cfg.L + cfg.lq + cfg.nd
    Kc_o, Vc_o = Cache(kparts, total_rows), Cache(vparts, total_rows)

    ref = so.phase2_rows(Qq_r.numpy(), Kc_o, Vc_o, cfg.L, cfg.b, cl, heads=heads)
    hs = torch.tensor(heads, device="cuda")
    eo = np.abs(O[:, :, hs].float().cpu().numpy() - ref["O"]).max()
    exists = ~np.isneginf(ref["LSE_part"])
    ep = np.abs(Op[:, :, hs].cpu().numpy()[exists] - ref["O_part"][exists]).max()
    elp = np.abs(Lp[:, :, hs].cpu().numpy()[exists] - ref["LSE_part"][exists]).max()
    print(f"   query: max|dO|={eo:.3g} max|dO_part|={ep:.3g} max|dLSE_part|={elp:.3g}", flush=True)
    assert eo <= tol["o"] and ep <= tol["o"] and elp <= tol["lse"]
    run.cache_len += cfg.lq

    steps = list(range(cfg.nd)) if decode_steps is None else decode_steps
    outs = []
    for t in range(cfg.nd):
        O1 = torch.empty_like(inp.Qd[:, :1])
        q1 = inp.Qd[:, t:t + 1].contiguous()
        sa.phase2_rope(run.shape, theta, run.cache_len, q1, inp.Kd[:, t:t + 1].contiguous(),
                       inp.Vd[:, t:t + 1].contiguous(), run.Kc, run.Vc, O1, run.ws, pos0=pos0)
        run.cache_len += 1
        outs.append(O1)
    torch.cuda.synchronize()
    O_dec = torch.cat(outs, dim=1)
    ref = so.phase2_rows(Qd_r.numpy(), Kc_o, Vc_o, cfg.L, cfg.b, cfg.L + cfg.lq, heads=heads, rows=steps)
    got = O_dec[:, torch.tensor(steps, device="cuda")][:, :, hs].float().cpu().numpy()
    eo = np.abs(got - ref["O"]).max()
    print(f"   decode steps {steps}: max|dO|={eo:.3g}", flush=True)
    assert eo <= tol["o"]
    # appended keys are rotated in the cache, values are plain
    tail = slice(cfg.L, cfg.L + cfg.lq + cfg.nd)
    wantK = torch.cat([Kq_r[0, :, 0], Kd_r[0, :, 0]], dim=0).numpy().astype(np.float64)
    assert _storage_close(run.Kc[0, 0, tail], wantK, cfg.dtype)
    assert torch.equal(run.Vc[0, 0, tail], torch.cat([inp.Vq[0, :, 0], inp.Vd[0, :, 0]], dim=0))


@pytest.mark.parametrize("L,b,a,pos0", [(1000, 256, 256, 0), (777, 200, 37, 123456)])
def test_fp32_unrotated_inputs_every_row(L, b, a, pos0):
    cfg = workloads.StarConfig("f32rope", "fp32", 2, 4, 2, 64, L, b, a, 9, 3, seed=L)
    _rope_path(cfg, 10000.0, pos0)


@pytest.mark.parametrize("Hq,Hkv,L,b,a,lq,nd,pos0", [
    (4, 1, 2048, 512, 512, 40, 3, 0),
    (8, 2, 1500, 400, 100, 130, 2, 900_000),
    (2, 2, 1024, 256, 0, 3, 4, 7),          # q_len 3: decode-sized call with several new tokens
])
def test_bf16_unrotated_inputs_every_row(Hq, Hkv, L, b, a, lq, nd, pos0):
    cfg = workloads.StarConfig("bf16rope", "bf16", 2, Hq, Hkv, 128, L, b, a, lq, nd,
                               seed=Hq + L, n_planted=4)
    _rope_path(cfg, 500000.0, pos0)


def test_config2_shape_unrotated_inputs_sampled():
    cfg = workloads.CONFIGS["C2"]
    inp = workloads.make_inputs(cfg, "cuda")
    triples = workloads.phase1_sample(cfg, inp.planted_ctx, n_random=64)
    del inp
    _rope_path(cfg, 500000.0, 0, triples=triples, heads=[0, 3, 31], decode_steps=[0, cfg.nd - 1])
