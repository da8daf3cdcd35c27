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
    if mode == sa.ANCHOR_EXTERNAL:
        gen = torch.Generator(device="cpu").manual_seed(seed)
        Ka = torch.randn((cfg.B, cfg.a, cfg.Hkv, cfg.d), generator=gen).to(dt).cuda()
        Va = torch.randn((cfg.B, cfg.a, cfg.Hkv, cfg.d), generator=gen).to(dt).cuda()
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


MODES = [sa.ANCHOR_PREVIOUS, sa.ANCHOR_EXTERNAL]


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
