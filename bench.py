#!/usr/bin/env python3
"""Benchmark of the Star Attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C3]

One "step" is one pass of the whole hot path over one synthetic batch of the
chosen configuration: phase 1 over the context (anchor-block attention + KV-cache
write), the phase-2 query-encoding call, and every decode step.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line:

  value / unit        phase-1 context tokens per second (B * L / phase-1 time)
  ms_per_step         wall time of the whole step (phase 1 + query + all decodes)
  phase2              decode microseconds per step and query-encode milliseconds;
                      decode_graph = the same decode calls replayed from one HIP graph
  roofline            phase-1 attention: achieved bf16 TFLOP/s vs. 2.5 PFLOP/s dense
  roofline_decode     decode step: algorithmic KV bytes / step time vs. 8 TB/s
  full_causal         the same kernels run with block = anchor = L (one block)
  cpu_baseline        the fp64 oracle timed on this host's cores on a bounded
                      sample of the same workload (a reported baseline only)
  anchor_variants     phase 1 under the ablation study's anchor variants, ms per call
  rope                the entry points that take unrotated projections
  power               socket power and shader clock that `amd-smi` reports while
                      phase 1 runs back to back for about two seconds (the MFMA
                      peak assumes 2.4 GHz; under this load the chip runs at its
                      power limit and clocks lower)

All timings are HIP events recorded on the stream the kernels are launched on.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import statistics
import subprocess
import sys
import tempfile
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2411_17116_amd as sa  # noqa: E402
import workloads  # noqa: E402

MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "fp32": 157.3}
HBM_PEAK_GBS = 8000.0
METRIC = "phase-1 context tok/s (%MFMA peak) + phase-2 decode us/step (%HBM BW), 8B shape"


def phase1_pairs(L: int, b: int, a: int) -> int:
    """Visible (query, key) pairs of phase 1 for one head."""
    n = -(-L // b)
    pairs = 0
    for i in range(n):
        ln = min(b, L - i * b)
        pairs += ln * (ln + 1) // 2 + (a * ln if i > 0 else 0)
    return pairs


def phase1_flops(cfg, L=None, b=None, a=None) -> float:
    L = cfg.L if L is None else L
    b = cfg.b if b is None else b
    a = cfg.a if a is None else a
    return 4.0 * cfg.d * cfg.Hq * cfg.B * phase1_pairs(L, b, a)


def decode_bytes(cfg, cache_len: int) -> float:
    """K and V of every cached token (the new one included), read once."""
    return 2.0 * cfg.B * cfg.Hkv * cfg.d * cfg.elem_size * (cache_len + 1)


class Timer:
    def __init__(self):
        self.pairs = []

    def start(self):
        e = torch.cuda.Event(enable_timing=True)
        e.record()
        return e

    def stop(self, e0):
        e1 = torch.cuda.Event(enable_timing=True)
        e1.record()
        self.pairs.append((e0, e1))
        return len(self.pairs) - 1

    def ms(self, i):
        e0, e1 = self.pairs[i]
        return e0.elapsed_time(e1)


def run_step(cfg, shape, inp, bufs, timer, sections=("phase1", "query", "decode")):
    """One pass of the hot path; returns event indices (phase1, query, [decode...]).
    `sections` exists for profiling runs that isolate one part; the default (and
    the only thing the reported numbers use) is the whole path."""
    e = timer.start()
    if "phase1" in sections:
        sa.phase1(shape, inp.Q, inp.K, inp.V, bufs["O_ctx"], bufs["Kc"], bufs["Vc"], workspace=bufs["ws1"])
    i_p1 = timer.stop(e)
    cache_len = cfg.L
    e = timer.start()
    if "query" in sections:
        sa.phase2(shape, cache_len, inp.Qq, inp.Kq, inp.Vq, bufs["Kc"], bufs["Vc"], bufs["Oq"], bufs["ws"])
    i_q = timer.stop(e)
    cache_len += cfg.lq
    i_d = []
    for t in range(cfg.nd if "decode" in sections else 0):
        e = timer.start()
        sa.phase2(shape, cache_len, bufs["Qd"][t], bufs["Kd"][t], bufs["Vd"][t], bufs["Kc"], bufs["Vc"],
                  bufs["Od"][t], bufs["ws"])
        i_d.append(timer.stop(e))
        cache_len += 1
    return i_p1, i_q, i_d


def cpu_baseline(cfg, inp, budget_s=12.0):
    """Time the fp64 oracle on a bounded sample of the workload on the host cores."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import star_oracle as so
    from tests.parity_harness import LazyTensor
    cores = min(16, os.cpu_count() or 1)
    K = inp.K.float().cpu().numpy()
    V = inp.V.float().cpu().numpy()
    Qv = LazyTensor(inp.Q.cpu())
    triples = workloads.phase1_sample(cfg, [], n_random=4096)
    import numpy as np
    rng = np.random.default_rng(0)
    rng.shuffle(triples)

    def one(tr):
        beta, h, p = tr
        so.phase1_row(Qv, K, V, beta, h, p, cfg.b, cfg.a)
        return 1

    done = 0
    t0 = time.time()
    with ThreadPoolExecutor(cores) as ex:
        batch = cores * 4
        pos = 0
        while time.time() - t0 < budget_s and pos < len(triples):
            done += sum(ex.map(one, triples[pos:pos + batch]))
            pos += batch
    dt = time.time() - t0
    rows_per_s = done / dt
    tok_per_s = rows_per_s / cfg.Hq
    out = {
        "value": tok_per_s, "unit": "tok/s", "cores": cores, "kind": "oracle",
        "sample": f"phase 1, {done} seeded (batch, head, row) triples of {cfg.name} in {dt:.1f} s; "
                  f"{rows_per_s:.1f} rows/s divided by Hq={cfg.Hq} (extrapolated to whole tokens)",
    }
    if cfg.nd:
        # one decode step = Hq * B rows of global attention over the whole cache: time a
        # few (batch, head) rows of the first decode step (context + query tokens cached)
        from tests.parity_harness import CacheView
        Kc = CacheView(inp.K.cpu(), inp.Kq.cpu(), inp.Kd[:, :1].cpu())
        Vc = CacheView(inp.V.cpu(), inp.Vq.cpu(), inp.Vd[:, :1].cpu())
        heads = sorted({0, cfg.Hq // 2, cfg.Hq - 1})
        t0 = time.time()
        so.phase2_rows(LazyTensor(inp.Qd[:, :1].cpu()), Kc, Vc, cfg.L, cfg.b, cfg.L + cfg.lq,
                       heads=heads, rows=[0])
        dt2 = time.time() - t0
        out["decode_s_per_step"] = dt2 / len(heads) * cfg.Hq
        out["decode_sample"] = (f"phase 2, first decode step, {len(heads)} of {cfg.Hq} heads x {cfg.B} batch "
                                f"in {dt2:.2f} s on one core (per-part and global attention), "
                                f"extrapolated to all heads")
    return out


_POLLER = r"""
import re, subprocess, sys, time
out = open(sys.argv[1], "a", buffering=1)
while True:
    t = time.time()
    try:
        txt = subprocess.run(["amd-smi", "metric", "--power", "--clock"], capture_output=True,
                             text=True, timeout=10).stdout
    except Exception:
        break
    p = re.search(r"SOCKET_POWER:\s*(\d+)", txt)
    c = [int(x) for x in re.findall(r"GFX_\d+:\s*\n\s*CLK:\s*(\d+)", txt)]
    if not (p and c):
        break
    out.write("%.3f %.3f %s %.1f\n" % (t, time.time(), p.group(1), sum(c) / len(c)))
    time.sleep(0.1)
"""


class PowerPoller:
    """Polls `amd-smi metric --power --clock` from a child process that is started
    before this process touches the GPU.  Samples are (t_begin, t_end, socket W, shader MHz averaged over the XCDs)."""

    def __init__(self):
        self.proc = None
        self.path = None

    def start(self):
        try:
            fd, self.path = tempfile.mkstemp(prefix="star_power_", suffix=".txt")
            os.close(fd)
            self.proc = subprocess.Popen([sys.executable, "-c", _POLLER, self.path],
                                         stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        except OSError:
            self.proc = None

    def stop(self):
        if self.proc is not None:
            self.proc.terminate()
            try:
                self.proc.wait(timeout=15)
            except subprocess.TimeoutExpired:
                self.proc.kill()
            self.proc = None

    def window(self, t0, t1):
        """Samples taken entirely inside [t0, t1]."""
        rows = []
        try:
            with open(self.path) as f:
                for line in f:
                    a, b, w, mhz = line.split()
                    if float(a) >= t0 and float(b) <= t1:
                        rows.append((float(w), float(mhz)))
        except (OSError, ValueError, TypeError):
            pass
        return rows

    def cleanup(self):
        self.stop()
        if self.path:
            try:
                os.unlink(self.path)
            except OSError:
                pass


def sustained_phase1(cfg, shape, inp, bufs, poller, seconds=2.0):
    """Phase 1 back to back for about `seconds`, with the power / clock samples
    that fall inside that window."""
    t = Timer()
    e = t.start()
    sa.phase1(shape, inp.Q, inp.K, inp.V, bufs["O_ctx"], bufs["Kc"], bufs["Vc"], workspace=bufs["ws1"])
    i = t.stop(e)
    torch.cuda.synchronize()
    n = max(3, int(seconds * 1e3 / max(t.ms(i), 1e-3)))
    t0 = time.time()
    e = t.start()
    for _ in range(n):
        sa.phase1(shape, inp.Q, inp.K, inp.V, bufs["O_ctx"], bufs["Kc"], bufs["Vc"], workspace=bufs["ws1"])
    i = t.stop(e)
    torch.cuda.synchronize()
    t1 = time.time()
    ms = t.ms(i) / n
    rows = poller.window(t0 + 0.3, t1) if poller is not None else []   # skip the ramp
    res = {"phase1_calls": n, "phase1_ms": ms,
           "phase1_tflops": phase1_flops(cfg) / (ms * 1e-3) / 1e12,
           "source": "amd-smi metric --power --clock, polled while phase 1 runs back to back",
           "samples": len(rows)}
    if rows:
        res["socket_power_w"] = statistics.median(r[0] for r in rows)
        res["gfx_clock_mhz"] = statistics.median(r[1] for r in rows)
        res["mfma_peak_at_clock_tflops"] = MFMA_PEAK_TFLOPS.get(cfg.dtype, 0.0) * res["gfx_clock_mhz"] / 2400.0
    return res


def decode_graph(cfg, shape, bufs, reps=5):
    """All decode steps of the configuration captured into one HIP graph and
    replayed: microseconds per step without per-launch host work."""
    side = torch.cuda.Stream()

    def steps():
        cache_len = cfg.L + cfg.lq
        for t in range(cfg.nd):
            sa.phase2(shape, cache_len, bufs["Qd"][t], bufs["Kd"][t], bufs["Vd"][t], bufs["Kc"],
                      bufs["Vc"], bufs["Od"][t], bufs["ws"])
            cache_len += 1

    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        steps()
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        steps()
    graph.replay()
    torch.cuda.synchronize()
    times = []
    for _ in range(reps):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) * 1e3 / cfg.nd)
    us = statistics.median(times)
    gbs = decode_bytes(cfg, cfg.L + cfg.lq + cfg.nd // 2) / (us * 1e-6) / 1e9
    return {"us_per_step": us, "gb_per_s": gbs, "hbm_frac": gbs / HBM_PEAK_GBS,
            "note": f"{cfg.nd} decode calls captured into one HIP graph, median of {reps} replays"}


def rope_cost(cfg, shape, inp, bufs, theta=500000.0):
    """What unrotated inputs cost: the in-place rotation of Q alone (an HBM
    stream: Q read once and written once) and the whole phase-1 call with the
    rotation inside (Q in place, K on its way into the cache)."""
    Qs = inp.Q.clone()                 # rotated over and over; norms are preserved
    t = Timer()
    idx = []
    for _ in range(3):
        e = t.start()
        sa.rope(shape, Qs, Qs, theta)
        idx.append(t.stop(e))
    idp = []
    for _ in range(3):
        e = t.start()
        sa.phase1_rope(shape, theta, Qs, inp.K, inp.V, bufs["O_ctx"], bufs["Kc"], bufs["Vc"])
        idp.append(t.stop(e))
    torch.cuda.synchronize()
    q_ms = min(t.ms(i) for i in idx[1:])
    p_ms = min(t.ms(i) for i in idp[1:])
    q_bytes = 2.0 * Qs.numel() * Qs.element_size()
    return {"q_rotate_ms": q_ms, "q_rotate_gb_per_s": q_bytes / (q_ms * 1e-3) / 1e9,
            "q_rotate_hbm_frac": q_bytes / (q_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "phase1_rope_ms": p_ms, "theta": theta,
            "note": "star_attn_rope on Q in place (bytes = Q read + written), and star_attn_phase1_rope"}


def anchor_variants(cfg, shape, inp, bufs):
    """Phase 1 under the ablation study's anchor variants (same flops as the
    method when the anchor has `a` tokens): milliseconds per call."""
    n = cfg.n_blocks
    Ka1 = inp.K[:, :cfg.a].contiguous()
    Va1 = inp.V[:, :cfg.a].contiguous()
    KaN = Ka1[:, None].expand(cfg.B, n, cfg.a, cfg.Hkv, cfg.d).contiguous()
    VaN = Va1[:, None].expand(cfg.B, n, cfg.a, cfg.Hkv, cfg.d).contiguous()
    modes = {"previous_block": (sa.ANCHOR_PREVIOUS, None, None),
             "external": (sa.ANCHOR_EXTERNAL, Ka1, Va1),
             "per_block": (sa.ANCHOR_PER_BLOCK, KaN, VaN)}
    out = {}
    flops = phase1_flops(cfg)
    for name, (mode, Ka, Va) in modes.items():
        t = Timer()
        idx = []
        for _ in range(3):
            e = t.start()
            sa.phase1_anchor(shape, mode, inp.Q, inp.K, inp.V, bufs["O_ctx"], bufs["Kc"], bufs["Vc"],
                             K_anchor=Ka, V_anchor=Va)
            idx.append(t.stop(e))
        torch.cuda.synchronize()
        ms = min(t.ms(i) for i in idx[1:])
        out[name] = {"ms": ms, "tflops": flops / (ms * 1e-3) / 1e12}
    out["note"] = "star_attn_phase1_anchor; every variant attends a keys of anchor + the causal block, as the method does"
    return out


def block_sweep(cfg, inp, bufs):
    """Phase 1 against the block size, anchor = block, context length fixed:
    the speed side of the paper's accuracy / speed trade-off (Section 3.4; the
    method's cost is linear in the block size, full causal attention is the
    last point)."""
    out = []
    t = Timer()
    L = cfg.L
    full_ms = None
    for div in (1, 2, 4, 8, 16, 32):
        b = L // div
        shape = sa.StarShape.make(cfg.dtype, cfg.B, cfg.Hq, cfg.Hkv, cfg.d, L, b, b, cfg.cache_capacity)
        idx = []
        for _ in range(2):
            e = t.start()
            sa.phase1(shape, inp.Q, inp.K, inp.V, bufs["O_ctx"], bufs["Kc"], bufs["Vc"], workspace=bufs["ws1"])
            idx.append(t.stop(e))
        torch.cuda.synchronize()
        ms = min(t.ms(i) for i in idx)
        full_ms = ms if div == 1 else full_ms
        flops = phase1_flops(cfg, b=b, a=b)
        out.append({"block": b, "n_blocks": div, "ms": ms, "tflops": flops / (ms * 1e-3) / 1e12,
                    "speedup_vs_full_causal": full_ms / ms})
    return out


def host_share(cfg, inp):
    """One host's share when every context block lives on its own host (the
    paper's deployment: n hosts, one block each): phase 1 of a context host
    ([anchor; block]) and of the first host (its block alone), a context host's
    and the query host's pair for one decode step, and the merge of the n
    gathered pairs.  Times of single calls on this GPU; no exchange is timed."""
    n, b, a = cfg.n_blocks, cfg.b, cfg.a
    tail = cfg.lq + cfg.nd
    dev = inp.Q.device
    hshape = sa.StarShape.make(cfg.dtype, cfg.B, cfg.Hq, cfg.Hkv, cfg.d, b, b, a, b + tail)
    Kc, Vc = sa.alloc_cache(hshape)
    ws = sa.alloc_workspace(hshape, 1)
    Q, K, V = (x[:, b:2 * b].contiguous() for x in (inp.Q, inp.K, inp.V))
    Q0, K0, V0 = (x[:, :b].contiguous() for x in (inp.Q, inp.K, inp.V))
    Ka, Va = K0[:, :a].contiguous(), V0[:, :a].contiguous()
    O = torch.empty_like(Q)
    t = Timer()

    def best(fn, reps=5):
        idx = []
        for _ in range(reps):
            e = t.start()
            fn()
            idx.append(t.stop(e))
        torch.cuda.synchronize()
        return min(t.ms(i) for i in idx[1:])

    first_ms = best(lambda: sa.phase1(hshape, Q0, K0, V0, O, Kc, Vc), 3)
    ctx_ms = best(lambda: sa.phase1_anchor(hshape, sa.ANCHOR_ALL_BLOCKS, Q, K, V, O, Kc, Vc,
                                           K_anchor=Ka, V_anchor=Va), 3)
    pairs = a * b + b * (b + 1) // 2
    flops = 4.0 * cfg.d * cfg.Hq * cfg.B * pairs
    Qd, Kd, Vd = (x[:, :1].contiguous() for x in (inp.Qd, inp.Kd, inp.Vd))
    A = torch.empty((n, cfg.B, cfg.Hq, 1, cfg.d), dtype=torch.float32, device=dev)
    L = torch.empty((n, cfg.B, cfg.Hq, 1), dtype=torch.float32, device=dev)
    ctx_us = 1e3 * best(lambda: sa.phase2_partial(hshape, b, Qd, Kc, Vc, A[0], L[0], ws), 12)
    qh_us = 1e3 * best(lambda: sa.phase2_partial(hshape, b + cfg.lq, Qd, Kc, Vc, A[1], L[1], ws,
                                                 Kq=Kd, Vq=Vd), 12)
    for i in range(2, n):
        A[i].copy_(A[0])
        L[i].copy_(L[0])
    Od = torch.empty_like(Qd)
    merge_us = 1e3 * best(lambda: sa.merge(hshape, A, L, O=Od), 12)
    host_bytes = 2.0 * cfg.B * cfg.Hkv * cfg.d * 2 * b
    return {"hosts": n, "tokens_per_host": b,
            "phase1_context_host_ms": ctx_ms, "phase1_context_host_tflops": flops / (ctx_ms * 1e-3) / 1e12,
            "phase1_first_host_ms": first_ms,
            "decode_context_host_us": ctx_us, "decode_context_host_gb_per_s": host_bytes / (ctx_us * 1e-6) / 1e9,
            "decode_query_host_us": qh_us, "merge_us": merge_us,
            "note": "one host's calls at the shape it has when each of the n blocks sits on its own "
                    "host: star_attn_phase1_anchor(ALL_BLOCKS), star_attn_phase2_partial, "
                    "star_attn_merge of n pairs; single-call times, the exchange between hosts is not part of them"}


def ceilings(bufs):
    """What this machine sustains for the two resources the rooflines name,
    measured with the calibration kernels of libstarcalib.so: independent bf16
    MFMAs on register operands (random bits, as attention has them, and constant
    bits) held for about half a second each, so that the power limit has set the
    clock, and a plain 16-byte-per-lane read of as many bytes as the K and V caches hold."""
    import ctypes
    path = os.path.join(ROOT, "paper_2411_17116_amd", "libstarcalib.so")
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: build it with `python -m paper_2411_17116_amd.build`")
    lib = ctypes.CDLL(path)
    vp = ctypes.c_void_p
    lib.star_calib_seed_bytes.restype = ctypes.c_size_t
    lib.star_calib_out_words.restype = ctypes.c_size_t
    lib.star_calib_mfma_flops.restype = ctypes.c_double
    lib.star_calib_mfma_flops.argtypes = [ctypes.c_int]
    lib.star_calib_mfma.argtypes = [vp, vp, ctypes.c_int, vp]
    lib.star_calib_hbm_read.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, vp, vp]
    stream = vp(torch.cuda.current_stream().cuda_stream)
    out = torch.empty(lib.star_calib_out_words(), dtype=torch.float32, device="cuda")
    n_seed = lib.star_calib_seed_bytes() // 2
    gen = torch.Generator(device="cuda").manual_seed(7)
    seeds = {"random": torch.randn(n_seed, generator=gen, device="cuda").to(torch.bfloat16),
             "constant": torch.ones(n_seed, dtype=torch.bfloat16, device="cuda")}
    t = Timer()
    res = {}
    iters = 3_000_000
    for name, seed in seeds.items():
        idx = []
        for _ in range(2):
            e = t.start()
            rc = lib.star_calib_mfma(vp(seed.data_ptr()), vp(out.data_ptr()), iters, stream)
            idx.append(t.stop(e))
            assert rc == 0
        torch.cuda.synchronize()
        res[f"mfma_{name}_operands_tflops"] = lib.star_calib_mfma_flops(iters) / (t.ms(idx[1]) * 1e-3) / 1e12
    # MFMA and softmax-like VALU work on the two wavefronts of a SIMD: alone and together
    lib.star_calib_coexec_cycle_words.restype = ctypes.c_size_t
    lib.star_calib_coexec.argtypes = [vp, vp, ctypes.c_int, ctypes.c_int, vp]
    cyc = torch.zeros(lib.star_calib_coexec_cycle_words(), dtype=torch.int64, device="cuda")
    co_iters = 20000
    co = {}
    for mode, tag in ((1, "alone"), (2, "alone"), (3, "together")):
        assert lib.star_calib_coexec(vp(out.data_ptr()), vp(cyc.data_ptr()), co_iters, mode, stream) == 0
        torch.cuda.synchronize()
        c = cyc.view(-1, 8).double()
        if mode & 1:
            co[f"clocks_per_mfma_{tag}"] = float(c[:, :4].mean()) / (8 * co_iters)
        if mode & 2:
            co[f"clocks_per_softmax_valu_group_{tag}"] = float(c[:, 4:].mean()) / co_iters
    co["note"] = ("one wavefront per SIMD issues v_mfma_f32_16x16x32_bf16 only, its SIMD neighbour 9 v_fma_f32 + 4 "
                  "v_exp_f32 per iteration (the VALU mix of the softmax of 8 MFMAs' worth of scores); shader clocks "
                  "per MFMA and per VALU group, each stream alone and both together")
    res["mfma_valu_coexecution"] = co
    src = torch.cat([bufs["Kc"].view(-1), bufs["Vc"].view(-1)])   # as many bytes as a decode step reads
    nbytes = src.numel() * src.element_size()
    for key, nt in (("hbm_read_gb_per_s", 0), ("hbm_read_nontemporal_gb_per_s", 1)):
        idx = []
        for _ in range(6):
            e = t.start()
            rc = lib.star_calib_hbm_read(vp(src.data_ptr()), nbytes, nt, vp(out.data_ptr()), stream)
            idx.append(t.stop(e))
            assert rc == 0
        torch.cuda.synchronize()
        res[key] = nbytes / (min(t.ms(i) for i in idx[1:]) * 1e-3) / 1e9
    res["hbm_read_bytes"] = nbytes
    res["note"] = ("calibration kernels (csrc/calib.hip): v_mfma_f32_16x16x32_bf16 only, 8 wavefronts per CU, "
                   f"{iters} x 8 per wavefront per launch; grid-stride read of a copy of the K and V caches with ordinary and with non-temporal loads, best of 5 each")
    return res


def measured_traffic(kernel: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summaries
    (profiles/traffic.json), or None if that kernel/workload was not profiled."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {}).get(kernel)
    except (OSError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="C3", choices=sorted(workloads.CONFIGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-full-causal", action="store_true")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the HIP-graph replay of the decode loop")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip timing the anchor variants of the ablation study")
    ap.add_argument("--no-block-sweep", action="store_true",
                    help="skip phase 1 at other block sizes (the trade-off curve)")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the calibration kernels (sustained MFMA rate, plain HBM read)")
    ap.add_argument("--no-hosts", action="store_true",
                    help="skip the timing of one host's share (per-host entry points)")
    ap.add_argument("--no-rope", action="store_true",
                    help="skip timing the entry points that take unrotated projections")
    ap.add_argument("--no-power", action="store_true",
                    help="skip the sustained phase-1 run with power / clock polling")
    ap.add_argument("--calib-copy", action="store_true",
                    help="profiling aid: also run one device copy of the K cache (known size) "
                         "so that HBM byte counters can be scaled")
    ap.add_argument("--sections", default="phase1,query,decode",
                    help="profiling aid: comma list of phase1,query,decode to run")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the hot path of one GPU's share); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    poller = None
    if not args.no_power:
        poller = PowerPoller()
        poller.start()           # before this process initialises the GPU
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        if poller:
            poller.cleanup()
        sys.exit(1)
    sa.load_library()          # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)
    cfg = workloads.CONFIGS[args.config]
    inp = workloads.make_inputs(cfg, "cuda")
    shape = sa.StarShape.make(cfg.dtype, cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.L, cfg.b, cfg.a,
                              cfg.cache_capacity)
    Kc, Vc = sa.alloc_cache(shape)
    bufs = {
        "Kc": Kc, "Vc": Vc, "O_ctx": torch.empty_like(inp.Q), "Oq": torch.empty_like(inp.Qq),
        "ws": sa.alloc_workspace(shape, max(cfg.lq, 1)),
        # phase 1's own workspace: the launch's work-queue counters (bf16)
        "ws1": torch.empty(max(sa.phase1_workspace_bytes(shape, sa.ANCHOR_FIRST), 256),
                           dtype=torch.uint8, device="cuda"),
        "Qd": [inp.Qd[:, t:t + 1].contiguous() for t in range(cfg.nd)],
        "Kd": [inp.Kd[:, t:t + 1].contiguous() for t in range(cfg.nd)],
        "Vd": [inp.Vd[:, t:t + 1].contiguous() for t in range(cfg.nd)],
        "Od": [torch.empty_like(inp.Qd[:, :1]) for _ in range(cfg.nd)],
    }
    sections = tuple(args.sections.split(","))
    if args.calib_copy:
        calib = torch.empty_like(Kc)
        calib.copy_(Kc)
        torch.cuda.synchronize()
        print(f"calibration copy: {Kc.numel() * Kc.element_size()} bytes read and as many written",
              file=sys.stderr)
    timer = Timer()
    for _ in range(args.warmup):
        run_step(cfg, shape, inp, bufs, timer, sections)
    torch.cuda.synchronize()
    timer.pairs.clear()
    t0 = time.perf_counter()
    e_all = timer.start()
    recs = [run_step(cfg, shape, inp, bufs, timer, sections) for _ in range(args.steps)]
    i_all = timer.stop(e_all)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    total_ms = timer.ms(i_all)

    p1_ms = statistics.mean(timer.ms(r[0]) for r in recs)
    q_ms = statistics.mean(timer.ms(r[1]) for r in recs)
    dec_us = [timer.ms(i) * 1e3 for r in recs for i in r[2]]
    dec_us_med = statistics.median(dec_us) if dec_us else float("nan")
    dec_us_mean = statistics.mean(dec_us) if dec_us else float("nan")

    flops = phase1_flops(cfg)
    p1_tflops = flops / (p1_ms * 1e-3) / 1e12
    tok_s = cfg.B * cfg.L / (p1_ms * 1e-3)
    mid_len = cfg.L + cfg.lq + cfg.nd // 2
    dbytes = decode_bytes(cfg, mid_len)
    dec_gbs = dbytes / (dec_us_med * 1e-6) / 1e9 if dec_us else float("nan")
    q_flops = 4.0 * cfg.d * cfg.Hq * cfg.B * cfg.lq * (cfg.L + (cfg.lq + 1) / 2)

    out = {
        "metric": METRIC, "value": tok_s, "unit": "tok/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": total_ms / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} Hq={cfg.Hq} Hkv={cfg.Hkv} d={cfg.d} "
                               f"L={cfg.L} block={cfg.b} anchor={cfg.a} lq={cfg.lq} nd={cfg.nd}",
                   "kernel_path": sa.kernel_path(shape)},
        "phase1": {"ms": p1_ms, "tok_per_s": tok_s, "tflops": p1_tflops,
                   "mfma_frac": p1_tflops / MFMA_PEAK_TFLOPS[cfg.dtype]},
        "phase2": {"decode_us_per_step": dec_us_med, "decode_us_mean": dec_us_mean,
                   "decode_gb_per_s": dec_gbs, "hbm_frac": dec_gbs / HBM_PEAK_GBS,
                   "query_encode_ms": q_ms,
                   "query_encode_tflops": q_flops / (q_ms * 1e-3) / 1e12},
        "roofline": {"bound": "mfma", "kernel": "phase1_bf16_kernel" if cfg.dtype == "bf16" else "phase1_f32_kernel",
                     "achieved": p1_tflops, "peak": MFMA_PEAK_TFLOPS[cfg.dtype],
                     "unit": "TFLOP/s", "frac": p1_tflops / MFMA_PEAK_TFLOPS[cfg.dtype],
                     "traffic": measured_traffic("phase1", cfg.name),
                     "note": "flops = 4 d per visible (query, key) pair; time = the phase-1 call "
                             "(bf16: a 4 us kernel that clears the work-queue tickets, then one kernel that attends and files K/V in the caches)"},
        "roofline_decode": {"bound": "hbm", "kernel": "decode_bf16_kernel" if cfg.dtype == "bf16" else "phase2_f32_kernel",
                            "achieved": dec_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": dec_gbs / HBM_PEAK_GBS, "traffic": measured_traffic("decode", cfg.name),
                            "note": "bytes = K and V of every cached token once; time = whole "
                                    "decode call (append + split-KV + merge)"},
        "wall_ms_per_step": wall_ms / args.steps,
    }
    if sections != ("phase1", "query", "decode"):
        out["sections"] = list(sections)   # partial run: not a reportable result

    if not args.no_full_causal and cfg.name != "C4":
        fshape = sa.StarShape.make(cfg.dtype, cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.L, cfg.L, cfg.L,
                                   cfg.cache_capacity)
        t = Timer()
        for _ in range(2):
            e = t.start()
            sa.phase1(fshape, inp.Q, inp.K, inp.V, bufs["O_ctx"], bufs["Kc"], bufs["Vc"],
                      workspace=bufs["ws1"])
            t.stop(e)
        torch.cuda.synchronize()
        f_ms = t.ms(1)
        f_flops = phase1_flops(cfg, b=cfg.L, a=cfg.L)
        out["full_causal"] = {"ms": f_ms, "tflops": f_flops / (f_ms * 1e-3) / 1e12,
                              "time_ratio_vs_star": f_ms / p1_ms,
                              "flop_ratio_vs_star": f_flops / flops}
    if "decode" in sections and cfg.nd and not args.no_graph:
        out["phase2"]["decode_graph"] = decode_graph(cfg, shape, bufs)
    if "phase1" in sections and not args.no_variants and cfg.dtype == "bf16" and cfg.name != "C4":
        out["anchor_variants"] = anchor_variants(cfg, shape, inp, bufs)
    if "phase1" in sections and not args.no_block_sweep and cfg.dtype == "bf16" and cfg.name != "C4":
        out["block_sweep"] = block_sweep(cfg, inp, bufs)
    if not args.no_ceilings:
        try:       # calibration only: its absence must not cost the run its result
            c = ceilings(bufs)
            out["roofline"]["frac_of_measured_mfma_rate"] = p1_tflops / c["mfma_random_operands_tflops"]
            out["roofline_decode"]["frac_of_measured_hbm_read"] = dec_gbs / max(
                c["hbm_read_gb_per_s"], c["hbm_read_nontemporal_gb_per_s"])
        except (OSError, AssertionError) as exc:
            c = {"error": str(exc)}
        out["ceilings"] = c
    if sections == ("phase1", "query", "decode") and not args.no_hosts and cfg.dtype == "bf16":
        out["host_share"] = host_share(cfg, inp)
    if "phase1" in sections and not args.no_rope:
        out["rope"] = rope_cost(cfg, shape, inp, bufs)
        # the caches now hold rotated keys; nothing below reads them
    if poller is not None:
        if "phase1" in sections:
            out["power"] = sustained_phase1(cfg, shape, inp, bufs, poller)
        poller.cleanup()
    out["paper_context"] = ("paper reports only whole-model speedups vs Ring Attention on 8-32 "
                            "A100 (e.g. 2.7x at 128K, Llama-3.1-8B, block 32K); no operator-level "
                            "number exists, so vs_baseline is null")
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, inp)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
