"""Parity harness: runs the HIP path through the C-ABI binding and the fp64
oracle on the same seeded inputs and compares them.  Used by the GPU tests, by
the smoke check and by the benchmark's CPU-baseline leg.  Test infrastructure:
the product package never imports this file.

Large configurations are compared on sampled rows; the oracle receives lazy
views of the device tensors (exactly the stored values, widened to float32) so
that no multi-gigabyte host copy is needed.
"""
from __future__ import annotations

import math
import time
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import paper_2411_17116_amd as sa
import workloads
from oracle import star_oracle as so

TOL = {"fp32": dict(o=1e-5, lse=1e-5), "bf16": dict(o=2e-2, lse=1e-2)}
# The fp32 bound on a log-sum-exp is 1e-5 for values up to 8 and grows in
# proportion beyond: the statistic is dominated by its largest logit, a d-term
# fp32 dot product whose rounding grows with its magnitude (a planted pair
# gives a logit, and an LSE, near 17: one ulp is 1.9e-6 there, and 1e-5 would be
# five ulps for the whole chain of d fused multiply-adds, the exponentials and
# the logarithm).  bf16 results are compared against the plain 1e-2.
LSE_MAGNITUDE_FLOOR = {"fp32": 8.0, "bf16": None}


class LazyTensor:
    """Indexable stand-in for a numpy array that fetches the indexed part of a
    torch tensor (any device) and widens it to float32 exactly."""

    def __init__(self, t: torch.Tensor):
        self.t = t
        self.shape = tuple(t.shape)
        self.dtype = np.float32

    def __getitem__(self, idx):
        if not isinstance(idx, tuple):
            idx = (idx,)
        conv = []
        for i in idx:
            if isinstance(i, np.ndarray):
                i = torch.from_numpy(i).to(self.t.device)
            elif isinstance(i, (list, tuple)):
                i = torch.tensor(i, device=self.t.device)
            conv.append(i)
        return self.t[tuple(conv)].float().cpu().numpy()


class CacheView:
    """The KV cache the oracle's definition yields -- every context token once,
    then the appended tokens in order (Algorithm 1 + Algorithm 2) -- presented
    as [B, Hkv, rows, d] without materialising it: index [beta, g, :n]."""

    def __init__(self, ctx: torch.Tensor, *appended: torch.Tensor):
        self.parts = [ctx, *appended]            # each [B, T, Hkv, d]
        B, _, Hkv, d = ctx.shape
        rows = sum(p.shape[1] for p in self.parts)
        self.shape = (B, Hkv, rows, d)

    def __getitem__(self, idx):
        beta, g, sl = idx
        assert isinstance(sl, slice) and sl.step is None
        out = torch.cat([p[beta, :, g] for p in self.parts], dim=0)[sl]
        return out.float().cpu().numpy()


@dataclass
class ParityReport:
    name: str
    checks: Dict[str, float]
    ok: bool
    detail: str = ""
    flat_plans: Optional[dict] = None     # decode step -> (decode, flat, non_temporal, steps per batch)
    lse_range: float = 0.0                # largest |LSE_ctx| of the run
    info: Optional[dict] = None           # reported, not asserted


def shape_of(cfg: workloads.StarConfig) -> sa.StarShape:
    return sa.StarShape.make(cfg.dtype, cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.L, cfg.b, cfg.a,
                             cfg.cache_capacity)


class HipRun:
    """Device buffers of one configuration plus the calls of the hot path."""

    def __init__(self, cfg: workloads.StarConfig, inp: workloads.StarInputs, device="cuda"):
        self.cfg, self.inp, self.device = cfg, inp, device
        self.shape = shape_of(cfg)
        self.Kc, self.Vc = sa.alloc_cache(self.shape, device)
        self.O_ctx = torch.empty_like(inp.Q)
        self.LSE_ctx = torch.empty((cfg.B, cfg.Hq, cfg.L), dtype=torch.float32, device=device)
        self.ws = sa.alloc_workspace(self.shape, max(cfg.lq, 1), device)
        # phase 1's own workspace (bf16: the launch's work-queue counters)
        n1 = sa.phase1_workspace_bytes(self.shape, sa.ANCHOR_FIRST)
        self.ws1 = torch.empty(n1, dtype=torch.uint8, device=device) if n1 else None
        self.cache_len = cfg.L
        self.info: Dict[str, float] = {}      # figures reported beside the checks, not asserted

    def phase1(self, want_lse=True, own_workspace=True, stream=None):
        """`own_workspace=False` leaves the counters to the library's static sets."""
        sa.phase1(self.shape, self.inp.Q, self.inp.K, self.inp.V, self.O_ctx, self.Kc, self.Vc,
                  LSE_ctx=self.LSE_ctx if want_lse else None,
                  workspace=self.ws1 if own_workspace else None, stream=stream)
        self.cache_len = self.cfg.L

    def phase2(self, Qn, Kn, Vn, want_parts=True):
        cfg = self.cfg
        q_len = Qn.shape[1]
        P = cfg.n_blocks + 1
        O = torch.empty_like(Qn)
        O_part = LSE_part = None
        if want_parts:
            O_part = torch.empty((cfg.B, P, cfg.Hq, q_len, cfg.d), dtype=torch.float32,
                                 device=self.device)
            LSE_part = torch.empty((cfg.B, P, cfg.Hq, q_len), dtype=torch.float32,
                                   device=self.device)
        sa.phase2(self.shape, self.cache_len, Qn, Kn, Vn, self.Kc, self.Vc, O, self.ws,
                  O_part=O_part, LSE_part=LSE_part)
        self.cache_len += q_len
        return O, O_part, LSE_part


def _maxabs(a: np.ndarray, b: np.ndarray) -> float:
    if a.size == 0:
        return 0.0
    d = np.abs(a.astype(np.float64) - b.astype(np.float64))
    if np.isnan(d).any():
        return math.inf
    return float(d.max())


def _lse_err(got: np.ndarray, want: np.ndarray, dtype: str = "bf16", scaled: bool = True) -> float:
    """max |got - want| where -inf must match -inf exactly; with a magnitude
    floor for the dtype, the difference is divided by max(1, |want| / floor)
    (`scaled=False`: the plain difference, for the record)."""
    got = got.astype(np.float64)
    want = np.asarray(want, np.float64)
    inf_w = np.isneginf(want)
    if (np.isneginf(got) != inf_w).any():
        return math.inf
    g, w = got[~inf_w], want[~inf_w]
    floor = LSE_MAGNITUDE_FLOOR[dtype] if scaled else None
    if floor is None or g.size == 0:
        return _maxabs(g, w)
    d = np.abs(g - w) / np.maximum(1.0, np.abs(w) / floor)
    return math.inf if np.isnan(d).any() else float(d.max())


def check_phase1(run: HipRun, triples: Sequence, cache_heads: Optional[Sequence] = None
                 ) -> Dict[str, float]:
    """Compare phase-1 outputs on (batch, head, row) triples and the caches."""
    cfg, inp = run.cfg, run.inp
    Qv, Kv, Vv = LazyTensor(inp.Q), LazyTensor(inp.K), LazyTensor(inp.V)
    O_ref, LSE_ref = so.phase1_rows(Qv, Kv, Vv, triples, cfg.b, cfg.a)
    idx = torch.tensor(triples, dtype=torch.long, device=run.device)
    bi, hi, ri = idx.unbind(1)
    O_got = run.O_ctx[bi, ri, hi].float().cpu().numpy()
    LSE_got = run.LSE_ctx[bi, hi, ri].cpu().numpy()
    res = {"phase1_O": _maxabs(O_got, O_ref), "phase1_LSE": _lse_err(LSE_got, LSE_ref, cfg.dtype)}
    # for the record, never asserted: the same error without the magnitude scaling
    run.info["phase1_LSE_unscaled"] = _lse_err(LSE_got, LSE_ref, cfg.dtype, scaled=False)
    # cache: every context token exactly once, bit-exact
    if cache_heads is None:
        cache_heads = [(beta, g) for beta in range(cfg.B) for g in range(cfg.Hkv)]
    bad = 0
    for beta, g in cache_heads:
        bad += int(not torch.equal(run.Kc[beta, g, :cfg.L], inp.K[beta, :, g]))
        bad += int(not torch.equal(run.Vc[beta, g, :cfg.L], inp.V[beta, :, g]))
    res["cache_mismatch"] = float(bad)
    return res


def check_phase2(run: HipRun, Qn: torch.Tensor, appended: Sequence[torch.Tensor],
                 cache_len: int, O, O_part, LSE_part, heads: Sequence[int],
                 rows: Optional[Sequence[int]] = None, tag="phase2",
                 parts_compact=False) -> Dict[str, float]:
    """Compare one phase-2 call.  `appended` = (K list, V list) of every tensor
    appended so far *including* this call's; `cache_len` is the value before the
    call; `rows` are indices into this call's new tokens.  With `parts_compact`
    the per-part tensors already hold only `rows` on their token axis."""
    cfg, inp = run.cfg, run.inp
    Ks, Vs = appended
    Kc = CacheView(inp.K, *Ks)
    Vc = CacheView(inp.V, *Vs)
    rows = list(range(Qn.shape[1])) if rows is None else list(rows)
    ref = so.phase2_rows(LazyTensor(Qn), Kc, Vc, cfg.L, cfg.b, cache_len, heads=heads, rows=rows)
    hsel = torch.tensor(list(heads), device=run.device)
    rsel = torch.tensor(rows, device=run.device)
    O_got = O[:, rsel][:, :, hsel].float().cpu().numpy()               # [B, nr, nh, d]
    res = {f"{tag}_O": _maxabs(O_got, ref["O"])}
    if O_part is not None:
        Op, Lp = O_part[:, :, hsel], LSE_part[:, :, hsel]
        if not parts_compact:
            Op, Lp = Op[:, :, :, rsel], Lp[:, :, :, rsel]
        Op, Lp = Op.cpu().numpy(), Lp.cpu().numpy()                     # [B, P, nh, nr, (d)]
        # an empty part carries no output; compare outputs where the part exists
        exists = ~np.isneginf(ref["LSE_part"])
        res[f"{tag}_O_part"] = _maxabs(Op[exists], ref["O_part"][exists])
        res[f"{tag}_LSE_part"] = _lse_err(Lp, ref["LSE_part"], cfg.dtype)
    return res


def run_parity(cfg: workloads.StarConfig, device="cuda", n_random=256, decode_samples=6,
               all_rows=False, verbose=False) -> ParityReport:
    """Whole hot path of one configuration against the oracle."""
    t0 = time.time()
    inp = workloads.make_inputs(cfg, device)
    run = HipRun(cfg, inp, device)
    tol = TOL[cfg.dtype]
    checks: Dict[str, float] = {}

    def log(msg):
        if verbose:
            print(f"[{cfg.name} +{time.time() - t0:6.1f}s] {msg}", flush=True)

    log("inputs ready; phase 1")
    run.phase1()
    torch.cuda.synchronize()
    if all_rows:
        triples = [(beta, h, p) for beta in range(cfg.B) for h in range(cfg.Hq)
                   for p in range(cfg.L)]
        cache_heads = None
    else:
        triples = workloads.phase1_sample(cfg, inp.planted_ctx, n_random=n_random)
        cache_heads = sorted({(beta, h // cfg.G) for beta, h, _ in triples})
    log(f"phase 1 done; oracle on {len(triples)} rows")
    checks.update(check_phase1(run, triples, cache_heads))
    # largest |LSE| the run produced: the fp32 bound on an LSE is the plain 1e-5 only
    # while this stays below LSE_MAGNITUDE_FLOOR
    lse_range = float(run.LSE_ctx[torch.isfinite(run.LSE_ctx)].abs().max().item())

    # query encoding
    heads = list(range(cfg.Hq)) if all_rows else workloads.phase2_heads(cfg)
    log("phase 2: query call")
    cl = run.cache_len
    O, Op, Lp = run.phase2(inp.Qq, inp.Kq, inp.Vq, want_parts=True)
    torch.cuda.synchronize()
    log("query call done; oracle")
    checks.update(check_phase2(run, inp.Qq, ([inp.Kq], [inp.Vq]), cl, O, Op, Lp, heads, tag="query"))

    # decode steps: the device runs every step in order; the oracle evaluates the
    # sampled steps as rows of one call (token t of the decode tensors sees cache
    # rows [0, L + lq + t], exactly what step t sees)
    log("decode steps")
    cl0 = run.cache_len
    outs, parts, lses = [], {}, {}
    rng = np.random.default_rng(cfg.seed + 5)
    nd = cfg.nd
    # Two kinds of checked steps.  `flat_steps` run as a serving loop runs them,
    # without per-part outputs: decode-sized calls then take the flat split plan
    # (and, for caches beyond 192 MiB, the non-temporal two-steps-per-batch
    # kernel set-up) -- their merged O is compared with the oracle.  `part_steps`
    # ask for the per-part pairs, which forces block-aligned splits, and compare
    # those pairs as well.  Every other step runs without per-part outputs and
    # only feeds the cache.
    if all_rows or nd <= decode_samples:
        flat_steps = [t for t in range(nd) if t % 2 == 1] or ([0] if nd else [])
        part_steps = [t for t in range(nd) if t not in flat_steps]
    else:
        flat_steps = sorted({0, nd - 1, int(rng.integers(1, nd - 1))})
        pool = [t for t in range(nd) if t not in flat_steps]
        part_steps = sorted(map(int, rng.choice(pool, min(decode_samples, len(pool)), replace=False)))
    plans = {}
    for t in range(nd):
        want = t in part_steps
        if t in flat_steps:
            info = sa.phase2_plan(run.shape, run.cache_len, 1, False)
            plans[t] = (info.decode, info.flat, info.non_temporal, info.steps_per_batch)
        O1, Op1, Lp1 = run.phase2(inp.Qd[:, t:t + 1].contiguous(), inp.Kd[:, t:t + 1].contiguous(),
                                  inp.Vd[:, t:t + 1].contiguous(), want_parts=want)
        outs.append(O1)
        if want:
            parts[t], lses[t] = Op1, Lp1
    torch.cuda.synchronize()
    log(f"decode done; oracle on flat steps {flat_steps} (decode, flat, non-temporal, steps/batch = "
        f"{sorted(set(plans.values()))}) and per-part steps {part_steps}")
    if nd:
        O_dec = torch.cat(outs, dim=1)                                   # [B, nd, Hq, d]
        appended = ([inp.Kq, inp.Kd], [inp.Vq, inp.Vd])
        if part_steps:
            Op_dec = torch.cat([parts[t] for t in part_steps], dim=3)    # [B, P, Hq, len(part_steps), d]
            Lp_dec = torch.cat([lses[t] for t in part_steps], dim=3)
            checks.update(check_phase2(run, inp.Qd, appended, cl0, O_dec, Op_dec, Lp_dec, heads,
                                       rows=part_steps, tag="decode", parts_compact=True))
        # the path a decode loop takes: every head on the end steps, the sampled
        # heads on the others
        all_heads = list(range(cfg.Hq))
        ends = sorted({flat_steps[0], flat_steps[-1]})
        res = check_phase2(run, inp.Qd, appended, cl0, O_dec, None, None, all_heads, rows=ends,
                           tag="decode_flat_ends")
        flat_err = res["decode_flat_ends_O"]
        mid = [t for t in flat_steps if t not in ends]
        if mid:
            res = check_phase2(run, inp.Qd, appended, cl0, O_dec, None, None, heads, rows=mid,
                               tag="decode_flat_mid")
            flat_err = max(flat_err, res["decode_flat_mid_O"])
        checks["decode_flat_O"] = flat_err
        # the appended rows must be in the cache, bit-exact
        bad = 0
        for beta, g in [(0, 0), (cfg.B - 1, cfg.Hkv - 1)]:
            tailK = torch.cat([inp.Kq[beta, :, g], inp.Kd[beta, :, g]], dim=0)
            tailV = torch.cat([inp.Vq[beta, :, g], inp.Vd[beta, :, g]], dim=0)
            bad += int(not torch.equal(run.Kc[beta, g, cfg.L:cfg.L + cfg.lq + cfg.nd], tailK))
            bad += int(not torch.equal(run.Vc[beta, g, cfg.L:cfg.L + cfg.lq + cfg.nd], tailV))
        checks["tail_cache_mismatch"] = float(bad)

    ok = True
    msgs = []
    for k, v in checks.items():
        if k.endswith("mismatch"):
            good = v == 0
        elif "LSE" in k:
            good = v <= tol["lse"]
        else:
            good = v <= tol["o"]
        ok &= good
        msgs.append(f"{k}={v:.3g}{'' if good else ' FAIL'}")
    log("; ".join(msgs))
    rep = ParityReport(cfg.name, checks, ok, "; ".join(msgs))
    rep.flat_plans = plans if cfg.nd else {}
    rep.lse_range = lse_range
    rep.info = dict(run.info)
    if rep.info:
        rep.detail += " | not asserted: " + "; ".join(f"{k}={v:.3g}" for k, v in rep.info.items())
    return rep
