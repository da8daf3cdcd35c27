"""GPU parity of the per-host entry points (Algorithms 1 and 2 as one host of
several runs them): several hosts are played one after the other on the one
GPU, each with its own slice of the context, its own caches and its own shape,
and what they produce together is compared with the fp64 oracle of the whole
problem.  Tolerances as everywhere: 1e-5 (fp32) / 2e-2 (bf16) on outputs,
1e-5 / 1e-2 on log-sum-exps; caches bit-exact."""
import numpy as np
import pytest
import torch

import paper_2411_17116_amd as sa
import workloads
from oracle import star_hosts as sh
from oracle import star_oracle as so
from tests import parity_harness as ph

pytestmark = pytest.mark.gpu


class Host:
    """One simulated host: its token range, shape, caches and workspace."""

    def __init__(self, cfg, inp, run, is_query_host, tail, device):
        self.lo, self.hi = min(run[0] * cfg.b, cfg.L), min(run[1] * cfg.b, cfg.L)
        self.T = self.hi - self.lo
        self.first = run[0] == 0
        self.is_query_host = is_query_host
        if self.T == 0:
            return
        self.cap = self.T + (tail if is_query_host else 0)
        self.shape = sa.StarShape.make(cfg.dtype, cfg.B, cfg.Hq, cfg.Hkv, cfg.d, self.T, cfg.b, cfg.a,
                                       self.cap)
        self.Kc, self.Vc = sa.alloc_cache(self.shape, device)
        self.ws = sa.alloc_workspace(self.shape, max(cfg.lq, 1), device)
        self.cache_len = self.T


class Cluster:
    def __init__(self, cfg, inp, n_hosts, query_host=None, device="cuda"):
        self.cfg, self.inp, self.device = cfg, inp, device
        qh = n_hosts - 1 if query_host is None else query_host
        runs = sh.block_runs(cfg.n_blocks, n_hosts)
        self.hosts = [Host(cfg, inp, r, h == qh, cfg.lq + cfg.nd, device) for h, r in enumerate(runs)]
        assert self.hosts[qh].T > 0, "the query host owns at least one block"
        self.O_ctx = torch.empty_like(inp.Q)
        self.LSE_ctx = torch.empty((cfg.B, cfg.Hq, cfg.L), dtype=torch.float32, device=device)

    def phase1(self):
        cfg, inp = self.cfg, self.inp
        Ka = inp.K[:, :cfg.a].contiguous()
        Va = inp.V[:, :cfg.a].contiguous()
        for h in self.hosts:
            if h.T == 0:
                continue
            Q, K, V = (x[:, h.lo:h.hi].contiguous() for x in (inp.Q, inp.K, inp.V))
            O = torch.empty_like(Q)
            LSE = torch.empty((cfg.B, cfg.Hq, h.T), dtype=torch.float32, device=self.device)
            if h.first:          # the owner of the global first block runs the method as it is
                sa.phase1(h.shape, Q, K, V, O, h.Kc, h.Vc, LSE_ctx=LSE)
            else:
                n = sa.phase1_workspace_bytes(h.shape, sa.ANCHOR_ALL_BLOCKS)
                ws = torch.empty(n, dtype=torch.uint8, device=self.device) if n else None
                sa.phase1_anchor(h.shape, sa.ANCHOR_ALL_BLOCKS, Q, K, V, O, h.Kc, h.Vc, K_anchor=Ka,
                                 V_anchor=Va, LSE_ctx=LSE, workspace=ws)
            self.O_ctx[:, h.lo:h.hi] = O
            self.LSE_ctx[:, :, h.lo:h.hi] = LSE

    def phase2(self, Qn, Kn, Vn):
        """One call: every host's pair, gathered into one slab per host, merged."""
        cfg = self.cfg
        H, q_len = len(self.hosts), Qn.shape[1]
        A = torch.full((H, cfg.B, cfg.Hq, q_len, cfg.d), float("nan"), dtype=torch.float32,
                       device=self.device)
        L = torch.full((H, cfg.B, cfg.Hq, q_len), float("-inf"), dtype=torch.float32,
                       device=self.device)
        for i, h in enumerate(self.hosts):
            if h.T == 0:
                continue             # owns nothing: lse = -inf, its slab stays NaN and is ignored
            if h.is_query_host:
                sa.phase2_partial(h.shape, h.cache_len, Qn, h.Kc, h.Vc, A[i], L[i], h.ws, Kq=Kn, Vq=Vn)
                h.cache_len += q_len
            else:
                sa.phase2_partial(h.shape, h.cache_len, Qn, h.Kc, h.Vc, A[i], L[i], h.ws)
        O = torch.empty_like(Qn)
        A_all = torch.empty((cfg.B, cfg.Hq, q_len, cfg.d), dtype=torch.float32, device=self.device)
        LSE = torch.empty((cfg.B, cfg.Hq, q_len), dtype=torch.float32, device=self.device)
        sa.merge(self.hosts[0].shape if self.hosts[0].T else next(h for h in self.hosts if h.T).shape,
                 A, L, O=O, A=A_all, LSE=LSE)
        return O, A_all, LSE


def _check_caches(cl):
    inp = cl.inp
    for h in cl.hosts:
        if h.T == 0:
            continue
        assert torch.equal(h.Kc[:, :, :h.T], inp.K[:, h.lo:h.hi].transpose(1, 2))
        assert torch.equal(h.Vc[:, :, :h.T], inp.V[:, h.lo:h.hi].transpose(1, 2))


def _run_small(cfg, n_hosts, query_host):
    tol = ph.TOL[cfg.dtype]
    inp = workloads.make_inputs(cfg, "cuda")
    cl = Cluster(cfg, inp, n_hosts, query_host)
    cl.phase1()
    torch.cuda.synchronize()
    Q, K, V = (x.float().cpu().numpy() for x in (inp.Q, inp.K, inp.V))
    O_ref, LSE_ref = so.phase1_full(Q, K, V, cfg.b, cfg.a)
    assert np.abs(cl.O_ctx.float().cpu().numpy() - O_ref).max() <= tol["o"]
    assert np.abs(cl.LSE_ctx.cpu().numpy() - LSE_ref).max() <= tol["lse"]
    _check_caches(cl)
    # the whole problem's cache, for the oracle
    Kc, Vc = so.kv_cache(K, V, cfg.L + cfg.lq + cfg.nd)
    cache_len = cfg.L
    calls = [(inp.Qq, inp.Kq, inp.Vq)] + [
        tuple(x[:, t:t + 1].contiguous() for x in (inp.Qd, inp.Kd, inp.Vd)) for t in range(cfg.nd)]
    for Qn, Kn, Vn in calls:
        O, A_all, LSE = cl.phase2(Qn, Kn, Vn)
        torch.cuda.synchronize()
        so.cache_append(Kc, Vc, cache_len, Kn.float().cpu().numpy(), Vn.float().cpu().numpy())
        ref = so.phase2_rows(Qn.float().cpu().numpy(), Kc, Vc, cfg.L, cfg.b, cache_len)
        assert np.abs(O.float().cpu().numpy() - ref["O"]).max() <= tol["o"]
        assert np.abs(A_all.cpu().numpy().transpose(0, 2, 1, 3) - ref["O"]).max() <= tol["o"]
        assert np.abs(LSE.cpu().numpy() - ref["LSE"]).max() <= tol["lse"]
        cache_len += Qn.shape[1]
    # the query host's cache tail holds the appended tokens, bit-exact
    qh = next(h for h in cl.hosts if h.is_query_host)
    tailK = torch.cat([inp.Kq, inp.Kd], dim=1).transpose(1, 2)
    assert torch.equal(qh.Kc[:, :, qh.T:qh.T + cfg.lq + cfg.nd], tailK)


@pytest.mark.parametrize("n_hosts,query_host", [(1, 0), (3, 2), (8, 0), (8, 7), (11, 4)])
def test_bf16_cluster_every_row(n_hosts, query_host):
    """8 blocks (the last ragged) dealt to 1 .. 11 hosts (more hosts than blocks:
    some own nothing); the query call takes the row-tiled kernel, the decode
    steps the streaming one."""
    cfg = workloads.StarConfig("hosts", "bf16", 2, 4, 2, 128, 1000, 128, 96, 9, 2,
                               seed=50 + n_hosts, n_planted=4)
    _run_small(cfg, n_hosts, query_host)


@pytest.mark.parametrize("n_hosts,query_host", [(2, 1), (6, 3)])
def test_fp32_cluster_every_row(n_hosts, query_host):
    cfg = workloads.StarConfig("hosts32", "fp32", 1, 2, 1, 64, 600, 100, 37, 5, 2, seed=7 + n_hosts)
    _run_small(cfg, n_hosts, query_host)


def test_bf16_cluster_decode_sized_query_and_no_anchor():
    """G * lq <= 16: the query call takes the streaming kernel on every host,
    with and without an append; a = 0 is the no-anchor ablation on every host."""
    cfg = workloads.StarConfig("hosts-dec", "bf16", 1, 8, 2, 128, 2100, 512, 0, 3, 2, seed=91,
                               n_planted=4)
    _run_small(cfg, 3, 1)


def test_merge_reproduces_phase2_from_its_own_parts():
    """star_attn_phase2's per-part outputs, handed to star_attn_merge, give its O."""
    cfg = workloads.StarConfig("merge", "bf16", 1, 8, 2, 128, 1500, 400, 100, 20, 1, seed=12)
    inp = workloads.make_inputs(cfg, "cuda")
    run = ph.HipRun(cfg, inp)
    run.phase1()
    O, Op, Lp = run.phase2(inp.Qq, inp.Kq, inp.Vq, want_parts=True)
    A_parts = Op.transpose(0, 1).contiguous()            # [P, B, Hq, q, d]
    L_parts = Lp.transpose(0, 1).contiguous()
    O2 = torch.empty_like(O)
    LSE = torch.empty((cfg.B, cfg.Hq, cfg.lq), dtype=torch.float32, device="cuda")
    sa.merge(run.shape, A_parts, L_parts, O=O2, LSE=LSE)
    torch.cuda.synchronize()
    assert (O.float() - O2.float()).abs().max().item() <= 1e-2     # one bf16 rounding apart at most
    assert torch.allclose(LSE, torch.logsumexp(Lp, dim=1), atol=1e-5)
    # every pair empty -> zeros and -inf
    L_parts.fill_(float("-inf"))
    A = torch.empty((cfg.B, cfg.Hq, cfg.lq, cfg.d), dtype=torch.float32, device="cuda")
    sa.merge(run.shape, A_parts, L_parts, O=O2, A=A, LSE=LSE)
    torch.cuda.synchronize()
    assert torch.all(O2 == 0) and torch.all(A == 0) and torch.all(torch.isneginf(LSE))


def test_config3_shape_on_eight_hosts_sampled():
    """The 128K configuration as the paper deploys it: one 16K block per host,
    8 hosts.  Each host's phase-1 call is its real per-GPU share ([anchor; block]
    = 32K keys for 16K rows); phase 2 runs on 16K-row caches plus the gather."""
    cfg = workloads.CONFIGS["C3"]
    tol = ph.TOL["bf16"]
    inp = workloads.make_inputs(cfg, "cuda")
    cl = Cluster(cfg, inp, 8)
    cl.phase1()
    torch.cuda.synchronize()
    print("\n[hosts C3] phase 1 done on 8 hosts", flush=True)
    triples = workloads.phase1_sample(cfg, inp.planted_ctx, n_random=128)
    Qv, Kv, Vv = ph.LazyTensor(inp.Q), ph.LazyTensor(inp.K), ph.LazyTensor(inp.V)
    O_ref, LSE_ref = so.phase1_rows(Qv, Kv, Vv, triples, cfg.b, cfg.a)
    idx = torch.tensor(triples, dtype=torch.long, device="cuda")
    bi, hi, ri = idx.unbind(1)
    assert np.abs(cl.O_ctx[bi, ri, hi].float().cpu().numpy() - O_ref).max() <= tol["o"]
    assert np.abs(cl.LSE_ctx[bi, hi, ri].cpu().numpy() - LSE_ref).max() <= tol["lse"]
    _check_caches(cl)
    print(f"[hosts C3] phase 1 parity on {len(triples)} rows", flush=True)
    heads = workloads.phase2_heads(cfg)
    hsel = torch.tensor(heads, device="cuda")
    O, A_all, LSE = cl.phase2(inp.Qq, inp.Kq, inp.Vq)
    torch.cuda.synchronize()
    ref = so.phase2_rows(ph.LazyTensor(inp.Qq), ph.CacheView(inp.K, inp.Kq), ph.CacheView(inp.V, inp.Vq),
                         cfg.L, cfg.b, cfg.L, heads=heads)
    assert np.abs(O[:, :, hsel].float().cpu().numpy() - ref["O"]).max() <= tol["o"]
    assert np.abs(LSE[:, hsel].cpu().numpy() - ref["LSE"]).max() <= tol["lse"]
    print("[hosts C3] query call parity", flush=True)
    outs, lses = [], []
    for t in range(3):
        O1, _, L1 = cl.phase2(*(x[:, t:t + 1].contiguous() for x in (inp.Qd, inp.Kd, inp.Vd)))
        outs.append(O1)
        lses.append(L1)
    torch.cuda.synchronize()
    ref = so.phase2_rows(ph.LazyTensor(inp.Qd), ph.CacheView(inp.K, inp.Kq, inp.Kd),
                         ph.CacheView(inp.V, inp.Vq, inp.Vd), cfg.L, cfg.b, cfg.L + cfg.lq,
                         heads=list(range(cfg.Hq)), rows=[0, 1, 2])
    O_dec = torch.cat(outs, dim=1)
    assert np.abs(O_dec.float().cpu().numpy() - ref["O"]).max() <= tol["o"]
    assert np.abs(torch.cat(lses, dim=2).cpu().numpy() - ref["LSE"]).max() <= tol["lse"]
    print("[hosts C3] decode parity on 3 steps, all heads", flush=True)


def _cluster_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for k in range(n):
        dtype = "bf16" if k % 3 else "fp32"
        Hkv = int(rng.choice([1, 2]))
        G = int(rng.choice([1, 2, 4, 8])) if dtype == "bf16" else int(rng.choice([1, 2]))
        L = int(rng.choice([65, 200, 513, 1100, 1900]))
        b = int(rng.choice([16, 63, 100, 256, 700]))
        a = int(rng.integers(0, b + 1))
        lq = int(rng.choice([1, 3, 16, 17, 40]))
        nd = int(rng.choice([1, 2]))
        n_blocks = -(-L // b)
        n_hosts = int(rng.integers(1, min(n_blocks, 9) + 3))
        owners = [h for h, (i0, i1) in enumerate(sh.block_runs(n_blocks, n_hosts)) if i1 > i0]
        qh = int(rng.choice(owners))
        d = 128 if dtype == "bf16" else 64
        out.append(pytest.param(dtype, Hkv * G, Hkv, d, L, b, a, lq, nd, n_hosts, qh, 7000 + 10 * seed + k,
                                id=f"{dtype}-H{Hkv * G}/{Hkv}-L{L}-b{b}-a{a}-lq{lq}-hosts{n_hosts}-q{qh}"))
    return out


@pytest.mark.parametrize("dtype,Hq,Hkv,d,L,b,a,lq,nd,n_hosts,qh,seed", _cluster_cases(12, 3))
def test_random_clusters(dtype, Hq, Hkv, d, L, b, a, lq, nd, n_hosts, qh, seed):
    """Seeded random shapes, host counts and query hosts, every row."""
    cfg = workloads.StarConfig("hosts-fuzz", dtype, 1, Hq, Hkv, d, L, b, a, lq, nd, seed=seed, n_planted=2)
    _run_small(cfg, n_hosts, qh)
