"""star_attn_phase2_static -- the entry point for callers that cannot allocate
-- against star_attn_phase2 on the same inputs, through the C ABI: two calls in
a row, the second smaller than the first (it must not see anything the first
left in the static scratch), then a decode loop; and the size limit."""
import ctypes

import pytest
import torch

import paper_2411_17116_amd as sa
import workloads
from tests import parity_harness as ph

pytestmark = pytest.mark.gpu


def _pair(cfg):
    inp = workloads.make_inputs(cfg, "cuda")
    a, b = ph.HipRun(cfg, inp, "cuda"), ph.HipRun(cfg, inp, "cuda")
    a.phase1()
    b.phase1()
    torch.cuda.synchronize()
    return inp, a, b


def test_static_scratch_entry_matches_the_workspace_entry():
    cfg = workloads.StarConfig("noalloc", "bf16", 2, 8, 2, 128, 6000, 1500, 700, 72, 5, seed=41,
                               n_planted=4)
    inp, ws_run, st_run = _pair(cfg)
    tol = ph.TOL["bf16"]["o"]

    def both(Qn, Kn, Vn, cache_len):
        O_ws, O_st = torch.empty_like(Qn), torch.full_like(Qn, 7.0)
        sa.phase2(ws_run.shape, cache_len, Qn, Kn, Vn, ws_run.Kc, ws_run.Vc, O_ws, ws_run.ws)
        sa.phase2_static(st_run.shape, cache_len, Qn, Kn, Vn, st_run.Kc, st_run.Vc, O_st)
        torch.cuda.synchronize()
        err = (O_ws.float() - O_st.float()).abs().max().item()
        return O_ws, O_st, err

    # call 1: query encoding, 72 tokens (row-tiled kernel, 9.6 MB of partials)
    print("call 1: 72 query tokens", flush=True)
    need = sa.phase2_plan(st_run.shape, cfg.L, cfg.lq).workspace_bytes
    assert 0 < need <= sa.STATIC_SCRATCH_BYTES
    O_ws, O_st, err = both(inp.Qq, inp.Kq, inp.Vq, cfg.L)
    assert err <= tol, err
    assert torch.equal(O_ws, O_st)                     # same kernels, same order: same bits
    # call 2, right behind it and much smaller: one decode token (streaming kernel)
    cl = cfg.L + cfg.lq
    for t in range(cfg.nd):
        print(f"call {t + 2}: decode step {t}", flush=True)
        q, k, v = (x[:, t:t + 1].contiguous() for x in (inp.Qd, inp.Kd, inp.Vd))
        O_ws, O_st, err = both(q, k, v, cl + t)
        assert err <= tol, (t, err)
        assert torch.equal(O_ws, O_st), t
    assert torch.equal(ws_run.Kc, st_run.Kc) and torch.equal(ws_run.Vc, st_run.Vc)
    # and the oracle agrees with what the static entry produced on the last step
    rep = ph.check_phase2(st_run, inp.Qd, ([inp.Kq, inp.Kd], [inp.Vq, inp.Vd]), cl,
                          torch.cat([O_st] * cfg.nd, dim=1), None, None, list(range(cfg.Hq)),
                          rows=[cfg.nd - 1], tag="static_decode")
    assert rep["static_decode_O"] <= tol, rep


def test_static_scratch_entry_fp32_and_its_size_limit():
    cfg = workloads.StarConfig("noalloc32", "fp32", 1, 2, 1, 64, 900, 256, 100, 20, 2, seed=43)
    inp, ws_run, st_run = _pair(cfg)
    O_ws, O_st = torch.empty_like(inp.Qq), torch.empty_like(inp.Qq)
    sa.phase2(ws_run.shape, cfg.L, inp.Qq, inp.Kq, inp.Vq, ws_run.Kc, ws_run.Vc, O_ws, ws_run.ws)
    sa.phase2_static(st_run.shape, cfg.L, inp.Qq, inp.Kq, inp.Vq, st_run.Kc, st_run.Vc, O_st)
    q, k, v = (x[:, :1].contiguous() for x in (inp.Qd, inp.Kd, inp.Vd))
    O1_ws, O1_st = torch.empty_like(q), torch.empty_like(q)
    sa.phase2(ws_run.shape, cfg.L + cfg.lq, q, k, v, ws_run.Kc, ws_run.Vc, O1_ws, ws_run.ws)
    sa.phase2_static(st_run.shape, cfg.L + cfg.lq, q, k, v, st_run.Kc, st_run.Vc, O1_st)
    torch.cuda.synchronize()
    assert torch.equal(O_ws, O_st) and torch.equal(O1_ws, O1_st)
    # a query call at the 128K shape needs 38 MB of partials: refused, nothing enqueued
    big = sa.StarShape.make("bf16", 1, 32, 8, 128, 131072, 16384, 16384, 131072 + 384)
    assert sa.phase2_plan(big, 131072, 256).workspace_bytes > sa.STATIC_SCRATCH_BYTES
    lib = sa.load_library()
    rc = lib.star_attn_phase2_static(ctypes.byref(big), 131072, 256, 0x1000, 0x1000, 0x1000, 0x1000,
                                     0x1000, 0x1000, None)
    assert rc == -7                                    # STAR_ATTN_ERR_WORKSPACE_TOO_SMALL


def test_static_scratch_entry_under_graph_capture():
    """The callers the entry point is for: a decode loop captured into a HIP graph
    with no workspace to bring.  Every replay (with eager work in between) gives
    the bits of the eager star_attn_phase2 loop."""
    cfg = workloads.StarConfig("noalloc-graph", "bf16", 1, 8, 2, 128, 8192, 2048, 2048, 24, 5, seed=47)
    inp, ws_run, st_run = _pair(cfg)
    Qd = [inp.Qd[:, t:t + 1].contiguous() for t in range(cfg.nd)]
    Kd = [inp.Kd[:, t:t + 1].contiguous() for t in range(cfg.nd)]
    Vd = [inp.Vd[:, t:t + 1].contiguous() for t in range(cfg.nd)]
    want = [torch.empty_like(Qd[0]) for _ in range(cfg.nd)]
    got = [torch.empty_like(Qd[0]) for _ in range(cfg.nd)]
    Oq_w, Oq_g = torch.empty_like(inp.Qq), torch.empty_like(inp.Qq)
    sa.phase2(ws_run.shape, cfg.L, inp.Qq, inp.Kq, inp.Vq, ws_run.Kc, ws_run.Vc, Oq_w, ws_run.ws)
    for t in range(cfg.nd):
        sa.phase2(ws_run.shape, cfg.L + cfg.lq + t, Qd[t], Kd[t], Vd[t], ws_run.Kc, ws_run.Vc, want[t],
                  ws_run.ws)
    torch.cuda.synchronize()
    Kc0, Vc0 = st_run.Kc.clone(), st_run.Vc.clone()

    def steps():
        sa.phase2_static(st_run.shape, cfg.L, inp.Qq, inp.Kq, inp.Vq, st_run.Kc, st_run.Vc, Oq_g)
        for t in range(cfg.nd):
            sa.phase2_static(st_run.shape, cfg.L + cfg.lq + t, Qd[t], Kd[t], Vd[t], st_run.Kc,
                             st_run.Vc, got[t])

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        steps()                                   # warm-up on the capture stream (first-call look-up)
    side.synchronize()
    st_run.Kc.copy_(Kc0)
    st_run.Vc.copy_(Vc0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        steps()
    for rep in range(3):
        print(f"replay {rep}", flush=True)
        st_run.Kc.copy_(Kc0)
        st_run.Vc.copy_(Vc0)
        for o in got:
            o.fill_(7.0)
        Oq_g.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Oq_g, Oq_w), f"replay {rep}, query call"
        for t in range(cfg.nd):
            assert torch.equal(got[t], want[t]), f"replay {rep}, decode step {t}"
        assert torch.equal(st_run.Kc, ws_run.Kc) and torch.equal(st_run.Vc, ws_run.Vc)
