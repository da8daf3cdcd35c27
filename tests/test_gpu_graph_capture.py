"""The decode loop under HIP graph capture: the library enqueues only kernels
(no allocation, no synchronisation, no memset), so a caller may capture a run of
star_attn_phase2 calls into one graph and replay it.  Every replay must give the
bits of the eager run."""
import pytest
import torch

import paper_2411_17116_amd as sa
import workloads
from tests import parity_harness as ph

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("with_query", [False, True])
def test_decode_steps_replayed_from_a_graph_match_eager(with_query):
    cfg = workloads.StarConfig("graph", "bf16", 1, 8, 2, 128, 8192, 2048, 2048, 40, 6, seed=21)
    inp = workloads.make_inputs(cfg, "cuda")
    run = ph.HipRun(cfg, inp, "cuda")
    run.phase1()
    torch.cuda.synchronize()
    Kc0, Vc0 = run.Kc.clone(), run.Vc.clone()
    Qd = [inp.Qd[:, t:t + 1].contiguous() for t in range(cfg.nd)]
    Kd = [inp.Kd[:, t:t + 1].contiguous() for t in range(cfg.nd)]
    Vd = [inp.Vd[:, t:t + 1].contiguous() for t in range(cfg.nd)]
    Oq = torch.empty_like(inp.Qq)
    Od = [torch.empty_like(Qd[0]) for _ in range(cfg.nd)]

    def steps():
        cl = cfg.L
        if with_query:       # row-tiled kernel + cache writer inside the graph as well
            sa.phase2(run.shape, cl, inp.Qq, inp.Kq, inp.Vq, run.Kc, run.Vc, Oq, run.ws)
            cl += cfg.lq
        for t in range(cfg.nd):
            sa.phase2(run.shape, cl, Qd[t], Kd[t], Vd[t], run.Kc, run.Vc, Od[t], run.ws)
            cl += 1

    print("eager run", flush=True)
    steps()
    torch.cuda.synchronize()
    want = [o.clone() for o in Od]
    want_q = Oq.clone()
    want_K = run.Kc.clone()

    print("capture", flush=True)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        steps()                                   # warm-up on the capture stream
    side.synchronize()
    with torch.cuda.graph(graph, stream=side):
        steps()
    for rep in range(3):
        print(f"replay {rep}", flush=True)
        # eager work between replays: restore the caches, scribble on the outputs
        run.Kc.copy_(Kc0)
        run.Vc.copy_(Vc0)
        for o in Od:
            o.fill_(7.0)
        Oq.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t in range(cfg.nd):
            assert torch.equal(Od[t], want[t]), f"replay {rep}, decode step {t}"
        if with_query:
            assert torch.equal(Oq, want_q), f"replay {rep}, query call"
        assert torch.equal(run.Kc, want_K)


def test_phase1_captured_with_its_own_workspace_and_refused_without():
    """Phase 1 in a graph: with a workspace the launch's work-queue counters are
    the caller's, so the captured launch can be replayed (every replay gives the
    eager bits); without one the library would have to bake one of its static
    counter sets into the graph, and refuses with STAR_ATTN_ERR_BUSY instead."""
    cfg = workloads.StarConfig("graph1", "bf16", 1, 8, 2, 128, 4000, 1024, 600, 1, 0, seed=23)
    inp = workloads.make_inputs(cfg, "cuda")
    run = ph.HipRun(cfg, inp, "cuda")
    run.phase1()
    torch.cuda.synchronize()
    want_O, want_L, want_K = run.O_ctx.clone(), run.LSE_ctx.clone(), run.Kc.clone()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run.phase1()                              # warm-up on the capture stream
    side.synchronize()
    refused = None
    with torch.cuda.graph(graph, stream=side):
        try:
            run.phase1(own_workspace=False)
        except sa.StarAttnError as e:
            refused = e.code
        run.phase1()
    assert refused == -11, refused                # STAR_ATTN_ERR_BUSY, nothing was captured for it
    for rep in range(3):
        print(f"replay {rep}", flush=True)
        run.O_ctx.fill_(7.0)
        run.LSE_ctx.fill_(7.0)
        run.Kc.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(run.O_ctx, want_O), f"replay {rep}"
        assert torch.equal(run.LSE_ctx, want_L), f"replay {rep}"
        assert torch.equal(run.Kc, want_K), f"replay {rep}"
