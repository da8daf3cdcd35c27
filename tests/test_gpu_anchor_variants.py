"""GPU parity of star_attn_phase1_anchor (anchor variants of the ablation study,
Section 4.1 / 4.2) against the fp64 oracle, through the C-ABI."""
import numpy as np
import pytest
import torch

import paper_2411_17116_amd as sa
from tests import parity_harness as ph
import workloads
from oracle import star_oracle as so

pytestmark = pytest.mark.gpu


def _run_variant(cfg, mode, triples=None, seed=5):
    inp = workloads.make_inputs(cfg, "cuda")
    run = ph.HipRun(cfg, inp, "cuda")
    dt = inp.K.dtype
    Ka = Va = ws = None
    if mode in (sa.ANCHOR_EXTERNAL, sa.ANCHOR_PER_BLOCK):
        gen = torch.Generator(device="cpu").manual_seed(seed)
        dims = (cfg.B, cfg.a, cfg.Hkv, cfg.d) if mode == sa.ANCHOR_EXTERNAL else \
            (cfg.B, cfg.n_blocks, cfg.a, cfg.Hkv, cfg.d)
        Ka = torch.randn(dims, generator=gen).to(dt).cuda()
        Va = torch.randn(dims, generator=gen).to(dt).cuda()
        n = sa.phase1_workspace_bytes(run.shape, mode)
        ws = torch.empty(max(n, 256), dtype=torch.uint8, device="cuda")
    print(f"[{cfg.name}] mode={mode} L={cfg.L} b={cfg.b} a={cfg.a} Hq={cfg.Hq} Hkv={cfg.Hkv}", flush=True)
    sa.phase1_anchor(run.shape, mode, inp.Q, inp.K, inp.V, run.O_ctx, run.Kc, run.Vc,
                     K_anchor=Ka, V_anchor=Va, LSE_ctx=run.LSE_ctx, workspace=ws)
    torch.cuda.synchronize()
    if triples is None:
        triples = [(beta, h, p) for beta in range(cfg.B) for h in range(cfg.Hq) for p in range(cfg.L)]
    Qv, Kv, Vv = ph.LazyTensor(inp.Q), ph.LazyTensor(inp.K), ph.LazyTensor(inp.V)
    Kav = ph.LazyTensor(Ka) if Ka is not None else None
    Vav = ph.LazyTensor(Va) if Va is not None else None
    O_ref = np.zeros((len(triples), cfg.d))
    L_ref = np.zeros(len(triples))
    for t, (beta, h, p) in enumerate(triples):
        O_ref[t], L_ref[t] = so.phase1_row_variant(Qv, Kv, Vv, beta, h, p, cfg.b, cfg.a, mode, Kav, Vav)
    idx = torch.tensor(triples, dtype=torch.long, device="cuda")
    bi, hi, ri = idx.unbind(1)
    O_got = run.O_ctx[bi, ri, hi].float().cpu().numpy()
    L_got = run.LSE_ctx[bi, hi, ri].cpu().numpy()
    tol = ph.TOL[cfg.dtype]
    eo, el = np.abs(O_got - O_ref).max(), np.abs(L_got - L_ref).max()
    print(f"   max|dO|={eo:.3g} max|dLSE|={el:.3g}", flush=True)
    assert eo <= tol["o"] and el <= tol["lse"]
    # the caches hold the context only, whatever served as anchor
    for beta in range(cfg.B):
        for g in range(cfg.Hkv):
            assert torch.equal(run.Kc[beta, g, :cfg.L], inp.K[beta, :, g])
            assert torch.equal(run.Vc[beta, g, :cfg.L], inp.V[beta, :, g])
    return run, inp


MODES = [sa.ANCHOR_PREVIOUS, sa.ANCHOR_EXTERNAL, sa.ANCHOR_PER_BLOCK]


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("L,b,a", [(1000, 256, 256), (777, 200, 37), (300, 512, 512), (640, 128, 0)])
def test_fp32_anchor_variants_every_row(mode, L, b, a):
    cfg = workloads.StarConfig("f32var", "fp32", 2, 4, 2, 64, L, b, a, 4, 1, seed=L + a + mode)
    _run_variant(cfg, mode)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("Hq,Hkv,L,b,a", [
    (4, 1, 2048, 512, 512),     # aligned everything
    (8, 1, 1500, 400, 100),     # anchor window starts and ends inside key tiles
    (2, 2, 1024, 256, 33),      # one head per workgroup, tiny ragged anchor
    (4, 2, 900, 300, 0),        # no anchor
])
def test_bf16_anchor_variants_every_row(mode, Hq, Hkv, L, b, a):
    cfg = workloads.StarConfig("bf16var", "bf16", 2, Hq, Hkv, 128, L, b, a, 4, 1,
                               seed=Hq * 100 + L + mode, n_planted=4)
    _run_variant(cfg, mode)


def test_first_mode_of_the_variant_entry_equals_phase1():
    cfg = workloads.StarConfig("bf16first", "bf16", 1, 8, 2, 128, 2048, 512, 200, 4, 1, seed=12)
    inp = workloads.make_inputs(cfg, "cuda")
    r1, r2 = ph.HipRun(cfg, inp, "cuda"), ph.HipRun(cfg, inp, "cuda")
    r1.phase1()
    sa.phase1_anchor(r2.shape, sa.ANCHOR_FIRST, inp.Q, inp.K, inp.V, r2.O_ctx, r2.Kc, r2.Vc,
                     LSE_ctx=r2.LSE_ctx)
    torch.cuda.synchronize()
    assert torch.equal(r1.O_ctx, r2.O_ctx) and torch.equal(r1.LSE_ctx, r2.LSE_ctx)


def test_external_anchor_with_the_first_tokens_equals_phase1():
    cfg = workloads.StarConfig("bf16ext", "bf16", 1, 8, 2, 128, 2048, 512, 200, 4, 1, seed=13)
    inp = workloads.make_inputs(cfg, "cuda")
    r1, r2 = ph.HipRun(cfg, inp, "cuda"), ph.HipRun(cfg, inp, "cuda")
    r1.phase1()
    ws = torch.empty(max(sa.phase1_workspace_bytes(r2.shape, sa.ANCHOR_EXTERNAL), 256), dtype=torch.uint8,
                     device="cuda")
    sa.phase1_anchor(r2.shape, sa.ANCHOR_EXTERNAL, inp.Q, inp.K, inp.V, r2.O_ctx, r2.Kc, r2.Vc,
                     K_anchor=inp.K[:, :cfg.a].contiguous(), V_anchor=inp.V[:, :cfg.a].contiguous(),
                     LSE_ctx=r2.LSE_ctx, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(r1.O_ctx, r2.O_ctx) and torch.equal(r1.LSE_ctx, r2.LSE_ctx)


@pytest.mark.parametrize("mode", MODES)
def test_config3_shape_anchor_variants_sampled(mode):
    """The 8B / 128K shape under both variants, on the sampled rows of the main
    parity test (every block edge, anchor edge, tile edge and planted row)."""
    cfg = workloads.CONFIGS["C3"]
    inp = workloads.make_inputs(cfg, "cuda")
    triples = workloads.phase1_sample(cfg, inp.planted_ctx, n_random=96)
    del inp
    _run_variant(cfg, mode, triples=triples)


def test_position_id_ablation_end_to_end():
    """Section 4.1, "position IDs same as previous block", on the GPU path: the
    projections arrive unrotated; star_attn_rope rotates Q and K at their own
    positions and builds, for every block, the first block's keys rotated at the
    positions just before that block; star_attn_phase1_anchor (PER_BLOCK) then
    attends.  The oracle composes the same steps in fp64 (with the storage
    rounding of the rotated tensors)."""
    from tests.test_gpu_rope import _stored
    theta = 500000.0
    cfg = workloads.StarConfig("posids", "bf16", 1, 8, 2, 128, 2048, 512, 512, 4, 1, seed=41,
                               n_planted=4)
    inp = workloads.make_inputs(cfg, "cuda")
    run = ph.HipRun(cfg, inp, "cuda")
    stored = _stored(cfg.dtype)
    n, a, b = cfg.n_blocks, cfg.a, cfg.b
    Qp, Kp = inp.Q.clone(), inp.K.clone()
    sa.rope(run.shape, inp.Q, inp.Q, theta)
    sa.rope(run.shape, inp.K, inp.K, theta)
    Ka = torch.zeros((cfg.B, n, a, cfg.Hkv, cfg.d), dtype=inp.K.dtype, device="cuda")
    Va = torch.zeros_like(Ka)
    first = Kp[:, :a].contiguous()
    ashape = sa.StarShape.make(cfg.dtype, cfg.B, cfg.Hq, cfg.Hkv, cfg.d, a, a, a, a)
    for i in range(1, n):
        out = torch.empty_like(first)
        sa.rope(ashape, first, out, theta, pos0=i * b - a)
        Ka[:, i] = out
        Va[:, i] = inp.V[:, :a]
    sa.phase1_anchor(run.shape, sa.ANCHOR_PER_BLOCK, inp.Q, inp.K, inp.V, run.O_ctx, run.Kc, run.Vc,
                     K_anchor=Ka, V_anchor=Va, LSE_ctx=run.LSE_ctx)
    torch.cuda.synchronize()
    # oracle: same composition
    Qp64, Kp64 = Qp.float().cpu().numpy(), Kp.float().cpu().numpy()
    V64 = inp.V.float().cpu().numpy()
    pos = np.arange(cfg.L)
    Qr = stored(so.rope_rotate(Qp64, pos, theta))
    Kr = stored(so.rope_rotate(Kp64, pos, theta))
    Ka_o = np.zeros((cfg.B, n, a, cfg.Hkv, cfg.d))
    Va_o = np.zeros_like(Ka_o)
    for i in range(1, n):
        Ka_o[:, i] = stored(so.rope_rotate(Kp64[:, :a], i * b - a + np.arange(a), theta))
        Va_o[:, i] = V64[:, :a]
    triples = [(0, h, p) for h in (0, 3, 7) for p in list(range(0, cfg.L, 37)) + [b - 1, b, b + 1, cfg.L - 1]]
    eo = el = 0.0
    for beta, h, p in triples:
        o, l = so.phase1_row_variant(Qr, Kr, V64, beta, h, p, b, a, so.ANCHOR_PER_BLOCK, Ka_o, Va_o)
        eo = max(eo, float(np.abs(run.O_ctx[beta, p, h].float().cpu().numpy() - o).max()))
        el = max(el, abs(float(run.LSE_ctx[beta, h, p]) - l))
    print(f"   position-id ablation: max|dO|={eo:.3g} max|dLSE|={el:.3g}", flush=True)
    assert eo <= ph.TOL["bf16"]["o"] and el <= ph.TOL["bf16"]["lse"]
