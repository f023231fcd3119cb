#!/usr/bin/env python3
"""Benchmark of the 2D Neighborhood Attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload nat_tiny_stage1] [--k 7]

One "step" is one pass of the whole hot path over one batch of synthetic NAT-Tiny stage-1
input (B=64, heads=2, 56x56, D=32, fp16, k=7 unless overridden), inputs resident in HBM: the ten
scoped entry points, one call each,
  forward, unfused : na2d_qk_rpb -> na2d_softmax -> na2d_av
  forward, fused   : na2d_fused_fwd (with log-sum-exp)
  backward         : na2d_av_bwd_p, na2d_av_bwd_v, na2d_softmax_bwd, na2d_qk_bwd_q, na2d_qk_bwd_k, na2d_qk_bwd_rpb
`value` is the algorithmic HBM traffic of those ten calls divided by the step's time (GB/s).  The composed
backward na2d_bwd (which fuses grad-a with the softmax backward and grad-b with grad-q where it can) and the
fused backward na2d_fused_bwd are timed beside the step and reported in `kernels` and `us_per_call` with the
bytes each of them has to move; they are not part of the step or of `value`.

Timing: the step and every call are captured in HIP graphs (launches only: the library records no memset
or copy nodes) and the graphs are replayed between HIP events on the launch stream, so that the host's
issue rate is not part of a kernel's time; `--eager` times Python-issued launches instead.  Every kernel
is timed over at least 200 launches: `us` is the median over the graph replays, `us_min` the fastest
replay.  Buffers rotate over several disjoint sets so that successive launches of one kernel do not find
their operands in the 256 MB Infinity Cache.  A plain device copy of 128 MiB is timed the same way as the
practical ceiling of the memory system (`copy_ceiling_GBps`).
Prints exactly one JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
METRIC = "2D NA fwd+bwd us/call and achieved HBM GB/s (% peak), NAT-Tiny shapes, k=7"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(p) -> dict:
    """Bytes each call must move per launch: what the method itself reads and writes
    (never the gathered-neighbourhood tensor it avoids)."""
    e, D, kk, nq = p.elem_bytes, p.D, p.kk, p.n_queries
    contraction = nq * (2 * D * e + kk * e)
    return {
        "qk_rpb": contraction, "softmax": nq * 2 * kk * e, "av": contraction,
        "fused_fwd": nq * (4 * D * e + 4),
        "av_bwd_p": contraction, "av_bwd_v": contraction, "softmax_bwd": nq * 3 * kk * e,
        "qk_bwd_q": contraction, "qk_bwd_k": contraction, "qk_bwd_rpb": nq * kk * e,
        # q, k, v, dout and lse in; dq, dk, dv out (the bias gradient is a few hundred bytes)
        "fused_bwd": nq * (7 * D * e + 4),
        # the composed backward on stored weights; where it fuses grad-a with the softmax backward (16-bit, k <= 9, D = 32) dp is never stored and
        # ds is read by grad-q and grad-k only: grad-a + softmax backward (attn, dout, v in; ds out), grad-v,
        # grad-q (+ grad-b), grad-k.  Elsewhere it is the six steps one after the other.
        "bwd": (nq * ((2 * D * e + 2 * kk * e) + 3 * (2 * D * e + kk * e))
                if (p.dtype != "f32" and p.k <= 9 and p.D == 32) else 4 * contraction + nq * 4 * kk * e),
    }


STEP_CALLS = ("qk_rpb", "softmax", "av", "fused_fwd", "av_bwd_p", "av_bwd_v", "softmax_bwd", "qk_bwd_q", "qk_bwd_k", "qk_bwd_rpb")


class BufferSet:
    def __init__(self, p, host, na, synth, torch):
        dev = lambda x: synth.to_device(x, p.dtype)
        self.q, self.k, self.v, self.rpb, self.dout = (dev(host[n]) for n in ("q", "k", "v", "rpb", "dout"))
        td = synth.TORCH_DTYPES[p.dtype]
        attn_shape = (p.B, p.heads, p.H, p.W, p.kk)
        self.logits = torch.empty(attn_shape, dtype=td, device="cuda")
        self.attn = torch.empty(attn_shape, dtype=td, device="cuda")
        self.dpds = torch.empty(attn_shape, dtype=td, device="cuda")
        self.out, self.out_fused, self.dq, self.dk, self.dv = (torch.empty_like(self.q) for _ in range(5))
        self.lse = torch.empty(self.q.shape[:4], dtype=torch.float32, device="cuda")
        nb = 2 * p.k - 1
        self.d_rpb = torch.empty((p.heads, nb, nb), dtype=torch.float32, device="cuda")
        prob = na.problem(p.B, p.heads, p.H, p.W, p.D, p.k, td)
        self.ws = torch.empty(na.na2d_workspace_bytes(prob, na.WS_BWD), dtype=torch.uint8, device="cuda")
        self.ws_rpb = torch.empty(na.na2d_workspace_bytes(prob, na.WS_QK_BWD_RPB), dtype=torch.uint8, device="cuda")
        self.ws_fused = torch.empty(na.na2d_workspace_bytes(prob, na.WS_FUSED_BWD), dtype=torch.uint8, device="cuda")


def make_calls(p, na, scale):
    k = p.k
    return {
        "qk_rpb": lambda s: na.na2d_qk_rpb(s.q, s.k, s.rpb, scale, k, s.logits),
        "softmax": lambda s: na.na2d_softmax(s.logits, k, s.q, s.attn),
        "av": lambda s: na.na2d_av(s.attn, s.v, k, s.out),
        "fused_fwd": lambda s: na.na2d_fused_fwd(s.q, s.k, s.v, s.rpb, scale, k, s.out_fused, s.lse),
        "av_bwd_p": lambda s: na.na2d_av_bwd_p(s.dout, s.v, k, s.dpds),
        "av_bwd_v": lambda s: na.na2d_av_bwd_v(s.attn, s.dout, k, s.dv),
        "softmax_bwd": lambda s: na.na2d_softmax_bwd(s.attn, s.dpds, k, s.q, s.dpds),
        "qk_bwd_q": lambda s: na.na2d_qk_bwd_q(s.dpds, s.k, scale, k, s.dq),
        "qk_bwd_k": lambda s: na.na2d_qk_bwd_k(s.dpds, s.q, scale, k, s.dk),
        "qk_bwd_rpb": lambda s: na.na2d_qk_bwd_rpb(s.dpds, k, s.q, s.d_rpb, s.ws_rpb),
        "fused_bwd": lambda s: na.na2d_fused_bwd(s.q, s.k, s.v, s.rpb, scale, s.lse, s.dout, k, s.dq, s.dk, s.dv,
                                                 s.d_rpb, s.ws_fused),
        "bwd": lambda s: na.na2d_bwd(s.q, s.k, s.v, s.attn, s.dout, scale, k, s.dq, s.dk, s.dv, s.d_rpb, s.ws),
    }


def step(s, calls):
    """One pass of the hot path: the ten scoped entry points, one call each."""
    for n in STEP_CALLS:
        calls[n](s)


class Timer:
    """Times a sequence of launches between HIP events on the launch stream.  With graphs (the default) the
    sequence is captured once and replayed: `launches` launches per replay, `replays` replays, each replay
    between its own pair of events; otherwise the launches are issued from Python between one pair of events
    per replay.  Returns (median, min) microseconds per launch over the replays."""

    def __init__(self, torch, use_graphs: bool):
        self.torch, self.use_graphs = torch, use_graphs
        self.mode = "hip graph replays" if use_graphs else "python-issued launches"

    def per_launch_us(self, fn, sets, launches: int, replays: int):
        torch = self.torch
        for st in sets:   # untimed: the first launch of a kernel loads its code object and sets its LDS limit
            fn(st)
        torch.cuda.synchronize()
        run = None
        if self.use_graphs:
            try:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    for i in range(launches):
                        fn(sets[i % len(sets)])
                run = g.replay
            except Exception as e:   # capture refused: say so once and go on with python-issued launches
                log(f"  (graph capture failed: {e!r}; timing python-issued launches)")
                self.use_graphs, self.mode = False, "python-issued launches (graph capture failed)"
                torch.cuda.synchronize()
        if run is None:
            def run():
                for i in range(launches):
                    fn(sets[i % len(sets)])
        run()   # untimed replay
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream()
        times = []
        for _ in range(replays):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            run()
            b.record(stream)
            torch.cuda.synchronize()
            times.append(a.elapsed_time(b) * 1e3 / launches)
        times.sort()
        return times[len(times) // 2], times[0]


def launches_for(us_guess: float) -> int:
    """Launches per graph: enough that a replay lasts about a millisecond (its own launch cost then vanishes)."""
    return max(24, min(240, int(1000.0 / max(us_guess, 1.0))))


def cpu_baseline(p, synth, budget_s: float = 20.0) -> dict:
    """The oracle as it stands, timed on this machine's host cores over a bounded sample (a few
    batch items of the same workload), reported in the metric's unit."""
    import numpy as np
    from oracle import na2d_oracle as o
    o.build()
    cores = o.num_threads()
    scale = p.default_scale

    inputs = {}

    def run(bs: int) -> float:
        if bs not in inputs:
            inputs.clear()
            sp = synth.Problem(bs, p.heads, p.H, p.W, p.D, p.k, p.dtype)
            inputs[bs] = {n: x.astype(np.float64) for n, x in synth.make_inputs(sp, 4242).items()}
        h = inputs[bs]
        t0 = time.perf_counter()
        logits = o.qk_rpb(h["q"], h["k"], h["rpb"], scale, p.k)
        attn = o.softmax(logits)
        o.av(attn, h["v"], p.k)
        o.fwd(h["q"], h["k"], h["v"], h["rpb"], scale, p.k)          # the fused forward's counterpart
        dp = o.av_bwd_p(h["dout"], h["v"], p.k)
        o.av_bwd_v(attn, h["dout"], p.k)
        ds = o.softmax_bwd(attn, dp)
        o.qk_bwd_q(ds, h["k"], scale, p.k)
        o.qk_bwd_k(ds, h["q"], scale, p.k)
        o.qk_bwd_rpb(ds, p.k)
        return time.perf_counter() - t0

    bs = 1
    t = run(bs)
    while t < budget_s / 4 and bs * 2 <= p.B:
        bs *= 2
        t = run(bs)
    reps, total = 1, t
    while total < budget_s / 2 and reps < 64:   # the whole batch fits the budget: repeat it and take the mean
        total += run(bs)
        reps += 1
    t = total / reps
    sp = synth.Problem(bs, p.heads, p.H, p.W, p.D, p.k, p.dtype)
    step_bytes = lambda q: sum(algorithmic_bytes(q)[n] for n in STEP_CALLS)
    out = {"value": round(step_bytes(sp) / t / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
           "sample": f"one full step (same 10 calls) on batch {bs} of {p.B}, mean of {reps} runs, {t:.2f} s each",
           "us_per_step_extrapolated": round(t * p.B / bs * 1e6, 1)}
    # the same on one thread, on one batch item (best of 3)
    o.set_threads(1)
    try:
        t1, spent = run(1), 0.0
        while spent < 3.0:   # best of about three seconds of runs
            t = run(1)
            t1, spent = min(t1, t), spent + t
    finally:
        o.set_threads(cores)
    s1 = synth.Problem(1, p.heads, p.H, p.W, p.D, p.k, p.dtype)
    out["single_thread"] = {"value": round(step_bytes(s1) / t1 / 1e9, 4), "unit": "GB/s", "cores": 1,
                            "sample": f"one full step on batch 1 of {p.B}, best run of about 3 s of runs, {t1 * 1e3:.1f} ms",
                            "us_per_step_extrapolated": round(t1 * p.B * 1e6, 1)}
    return out


def measured_traffic(workload: str, p, kernel_group: str):
    """HBM bytes per launch of the dominant kernel as counted by rocprofv3 (FETCH_SIZE + WRITE_SIZE,
    scaled by what the same counters read for a plain copy of known size), from the summary kept
    under profiles/ for this workload; None when there is no summary for it."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}_k{p.k}_{p.dtype}.txt")
    if not os.path.exists(path):
        return None
    key = kernel_group.split(" ")[0]
    for line in open(path):
        f = line.split()
        if len(f) >= 4 and f[0] == key:
            return int(float(f[3]))   # columns: kernel, fetch bytes, write bytes, fetch + write bytes per launch
    return None


def composite_nat_tiny(p1, na, synth, torch, timer, replays: int) -> dict:
    """One NAT-Tiny forward's (and forward + backward's) worth of neighbourhood attention at the bench
    batch: the four stages of the model (Section 3.2: 3, 4, 18 and 5 layers on 56, 28, 14 and 7 wide
    maps with 2, 4, 8 and 16 heads of dim 32), each layer one fused forward (plus one fused backward),
    every stage timed on its own over rotating buffer sets and weighted by its layer count."""
    layers = (3, 4, 18, 5)
    stages, fwd_us, bwd_us, fwd_bytes, bwd_bytes = [], 0.0, 0.0, 0, 0
    for i, nl in enumerate(layers):
        sp = synth.Problem(p1.B, p1.heads << i, p1.H >> i, p1.W >> i, p1.D, p1.k, p1.dtype)
        host = synth.make_inputs(sp, seed=1100 + i)
        sets = [BufferSet(sp, host, na, synth, torch) for _ in range(3)]
        calls = make_calls(sp, na, sp.default_scale)
        ab = algorithmic_bytes(sp)
        us = {}
        for name, guess in (("fused_fwd", 15.0), ("fused_bwd", 50.0)):
            us[name], _ = timer.per_launch_us(calls[name], sets, launches_for(guess), replays)
        stages.append({"map": f"{sp.H}x{sp.W}", "heads": sp.heads, "layers": nl, "fused_fwd_us": round(us["fused_fwd"], 2),
                       "fused_bwd_us": round(us["fused_bwd"], 2)})
        fwd_us += nl * us["fused_fwd"]
        bwd_us += nl * us["fused_bwd"]
        fwd_bytes += nl * ab["fused_fwd"]
        bwd_bytes += nl * ab["fused_bwd"]
        del sets
    log(f"  composite NAT-Tiny (30 layers, batch {p1.B}): NA forward {fwd_us:.0f} us, forward + backward {fwd_us + bwd_us:.0f} us")
    return {"what": f"NAT-Tiny's 30 NA layers at batch {p1.B}, {p1.dtype}, k={p1.k}: fused forward (+ fused backward) per layer",
            "fwd_us": round(fwd_us, 1), "fwd_bwd_us": round(fwd_us + bwd_us, 1),
            "fwd_GBps": round(fwd_bytes / fwd_us / 1e3, 1), "fwd_bwd_GBps": round((fwd_bytes + bwd_bytes) / (fwd_us + bwd_us) / 1e3, 1),
            "stages": stages}


def bench_na1d(na, synth, torch, timer, replays: int) -> dict:
    """The 1D entry points on the sequence workload (NAT-Tiny's first-stage tokens read as a sequence:
    B=64, heads=2, L=3136, D=32, k=7, f16), each call timed on its own over rotating buffer sets.
    Algorithmic bytes per query: contractions 2*D*e + k*e, softmax 2*k*e, softmax backward 3*k*e, bias
    gradient k*e, fused forward 4*D*e + 4."""
    p = synth.CONFIGS_1D["seq_3136_k7"]
    host = synth.make_inputs_1d(p, seed=1200)
    td, k, e, scale = synth.TORCH_DTYPES[p.dtype], p.k, p.elem_bytes, p.default_scale
    prob = na.problem_1d(p.B, p.heads, p.L, p.D, k, td)

    class S:
        pass
    sets = []
    for _ in range(3):
        s = S()
        s.q, s.k, s.v, s.rpb, s.dout = (synth.to_device(host[n], p.dtype) for n in ("q", "k", "v", "rpb", "dout"))
        attn_like = lambda: torch.empty((p.B, p.heads, p.L, k), dtype=td, device="cuda")
        s.logits, s.attn, s.dp = attn_like(), attn_like(), attn_like()
        s.out, s.dq, s.dk, s.dv = (torch.empty_like(s.q) for _ in range(4))
        s.lse = torch.empty((p.B, p.heads, p.L), dtype=torch.float32, device="cuda")
        s.d_rpb = torch.empty((p.heads, 2 * k - 1), dtype=torch.float32, device="cuda")
        s.ws = torch.empty(na.na1d_workspace_bytes(prob), dtype=torch.uint8, device="cuda")
        s.ws_fused = torch.empty(na.na1d_fused_bwd_workspace_bytes(prob), dtype=torch.uint8, device="cuda")
        sets.append(s)
    nq = p.n_queries
    contraction = nq * (2 * p.D * e + k * e)
    calls = {
        "qk_rpb": (lambda s: na.na1d_qk_rpb(s.q, s.k, s.rpb, scale, k, s.logits), contraction),
        "softmax": (lambda s: na.na1d_softmax(s.logits, k, s.q, s.attn), nq * 2 * k * e),
        "av": (lambda s: na.na1d_av(s.attn, s.v, k, s.out), contraction),
        "fused_fwd": (lambda s: na.na1d_fused_fwd(s.q, s.k, s.v, s.rpb, scale, k, s.out, s.lse), nq * (4 * p.D * e + 4)),
        "av_bwd_p": (lambda s: na.na1d_av_bwd_p(s.dout, s.v, k, s.dp), contraction),
        "av_bwd_v": (lambda s: na.na1d_av_bwd_v(s.attn, s.dout, k, s.dv), contraction),
        "softmax_bwd": (lambda s: na.na1d_softmax_bwd(s.attn, s.dp, k, s.q, s.dp), nq * 3 * k * e),
        "qk_bwd_q": (lambda s: na.na1d_qk_bwd_q(s.dp, s.k, scale, k, s.dq), contraction),
        "qk_bwd_k": (lambda s: na.na1d_qk_bwd_k(s.dp, s.q, scale, k, s.dk), contraction),
        "qk_bwd_rpb": (lambda s: na.na1d_qk_bwd_rpb(s.dp, k, s.q, s.d_rpb, s.ws), nq * k * e),
        # q, k, v, dout and lse in; dq, dk, dv out
        "fused_bwd": (lambda s: na.na1d_fused_bwd(s.q, s.k, s.v, s.rpb, scale, s.lse, s.dout, k, s.dq, s.dk, s.dv, s.d_rpb,
                                                  s.ws_fused), nq * (7 * p.D * e + 4)),
    }
    res, total_us, total_bytes = {}, 0.0, 0
    for name, (fn, nbytes) in calls.items():
        us, us_min = timer.per_launch_us(fn, sets, launches_for(80.0 if name == "fused_bwd" else 12.0), replays)
        res[name] = {"us": round(us, 2), "us_min": round(us_min, 2), "GBps": round(nbytes / us / 1e3, 1),
                     "pct_hbm_peak": round(100 * nbytes / us / 1e3 / HBM_PEAK_GBPS, 1), "MB": round(nbytes / 1e6, 2)}
        if name != "fused_bwd":   # the fused backward is an alternative to the six unfused steps, not one more call
            total_us += us
            total_bytes += nbytes
        log(f"  na1d {name:12s} {us:9.2f} us  {nbytes / us / 1e3:8.1f} GB/s")
    return {"workload": f"seq_3136_k7 (B={p.B}, heads={p.heads}, L={p.L}, D={p.D}, k={k}, {p.dtype})",
            "us_all_calls": round(total_us, 1), "GBps_all_calls": round(total_bytes / total_us / 1e3, 1), "kernels": res}


def inverse_kernel_name(workload: str, p) -> str:
    """grad-v / grad-k run one of three device kernels, chosen by the library from the map and kernel
    size (the column-walking `inverse_ring`, the tile kernel `inverse_mfma` or the row-streaming
    `inverse_rows`); the name reported is the one the profile summary of this workload recorded, else
    the neutral `inverse`."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}_k{p.k}_{p.dtype}.txt")
    if os.path.exists(path):
        for line in open(path):
            f = line.split()
            if f and f[0] in ("inverse_ring", "inverse_mfma", "inverse_rows"):
                return f[0]
    return "inverse"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="nat_tiny_stage1")
    ap.add_argument("--k", type=int, default=None, help="override the kernel size (config 5 sweeps 3..13)")
    ap.add_argument("--sets", type=int, default=3, help="disjoint buffer sets rotated between launches")
    ap.add_argument("--replays", type=int, default=10, help="timed graph replays per kernel (each at least 24 launches)")
    ap.add_argument("--eager", action="store_true", help="time python-issued launches instead of HIP graph replays")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--skip-composite", action="store_true",
                    help="leave out the NAT-Tiny composite and the 1D workload (their maps launch the same kernels: "
                         "per-kernel averages of a profiler then mix shapes)")
    ap.add_argument("--only", default=None,
                    help="comma-separated entry points (of the `kernels` table) to launch, nothing else: for counter runs")
    ap.add_argument("--lib", default=None,
                    help="time another build of the library (the memory-only measurement build of "
                         "`python -m paper_2204_07143_amd.build --probe`); its results are not the method's")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch plain device copies of known size (calibration of rocprofv3's HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives or sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2204_07143_amd import binding as na
    from paper_2204_07143_amd import synth

    na.load(args.lib)  # raises if the HIP library is missing: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    base = synth.CONFIGS[args.workload]
    p = base if args.k is None else synth.Problem(base.B, base.heads, base.H, base.W, base.D, args.k, base.dtype)
    scale = p.default_scale
    host = synth.make_inputs(p, seed=1002)
    sets = [BufferSet(p, host, na, synth, torch) for _ in range(args.sets)]
    calls = make_calls(p, na, scale)
    abytes = algorithmic_bytes(p)
    step_bytes = sum(abytes[n] for n in STEP_CALLS)
    log(f"workload {args.workload}: {p}  step = {step_bytes / 1e6:.1f} MB algorithmic, {args.sets} buffer sets")

    # populate every set once (also the warm-up of every kernel: code objects, LDS limits)
    for s in sets:
        step(s, calls)
        calls["fused_bwd"](s)
        calls["bwd"](s)
    torch.cuda.synchronize()

    if args.only:   # a bare run of the named entry points for a profiler: 30 launches each, no timing, no JSON
        for name in args.only.split(","):
            for i in range(30):
                calls[name](sets[i % len(sets)])
        if args.copy_probe:
            src = torch.empty(128 << 20, dtype=torch.uint8, device="cuda")
            dst = torch.empty_like(src)
            for _ in range(3):
                dst.copy_(src)
        torch.cuda.synchronize()
        return 0

    timer = Timer(torch, use_graphs=not args.eager)
    stream = torch.cuda.current_stream()

    # W untimed warm-up steps, then the timed region: exactly K steps between events, one device synchronisation
    # on each side.  With graphs, one graph per buffer set holds the ten launches of a step and the K steps are K
    # graph replays, rotating over the sets.
    step_graphs = None
    if timer.use_graphs:
        try:
            step_graphs = []
            for st in sets:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    step(st, calls)
                step_graphs.append(g)
        except Exception as e:
            log(f"  (graph capture of the step failed: {e!r}; python-issued launches)")
            step_graphs = None
            timer.use_graphs, timer.mode = False, "python-issued launches (graph capture failed)"
            torch.cuda.synchronize()

    def run_step(i):
        if step_graphs is not None:
            step_graphs[i % len(sets)].replay()
        else:
            step(sets[i % len(sets)], calls)

    for i in range(args.warmup):
        run_step(i)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    a.record(stream)
    for i in range(args.steps):
        run_step(i)
    b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    us_step = a.elapsed_time(b) * 1e3 / args.steps
    log(f"step: {us_step:.1f} us  ({step_bytes / us_step / 1e3:.1f} GB/s algorithmic; wall {wall * 1e3:.1f} ms for {args.steps} steps; {timer.mode})")
    # the same K steps issued from Python, for comparison (host issue rate included)
    torch.cuda.synchronize()
    a2, b2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a2.record(stream)
    for i in range(args.steps):
        step(sets[i % len(sets)], calls)
    b2.record(stream)
    torch.cuda.synchronize()
    us_step_eager = a2.elapsed_time(b2) * 1e3 / args.steps

    # the practical ceiling of the memory system: a plain device copy of 128 MiB (read + write), timed the same way
    # (four source / destination pairs in rotation, 1 GiB in all, so that no copy finds its source in the 256 MB
    # Infinity Cache)
    class _C:
        pass
    csets = []
    for _ in range(4):
        c = _C()
        c.src = torch.empty(128 << 20, dtype=torch.uint8, device="cuda")
        c.dst = torch.empty_like(c.src)
        csets.append(c)
    copy_us, copy_us_min = timer.per_launch_us(lambda c: c.dst.copy_(c.src), csets, 24, args.replays)
    copy_ceiling = 2 * (128 << 20) / copy_us / 1e3
    log(f"  device copy of 128 MiB: {copy_us:.1f} us = {copy_ceiling:.0f} GB/s (read + write)")
    del csets

    # per-kernel: every entry point over rotating buffer sets, at least 200 launches each
    kernels = {}
    guess = {"softmax": 14.0, "softmax_bwd": 18.0, "qk_bwd_rpb": 10.0, "fused_bwd": 100.0, "bwd": 110.0}
    for name, fn in calls.items():
        n = launches_for(guess.get(name, 22.0) * (p.kk / 49.0 if p.kk > 49 else 1.0))
        us, us_min = timer.per_launch_us(fn, sets, n, max(args.replays, (200 + n - 1) // n))
        gbps = abytes[name] / us / 1e3
        kernels[name] = {"us": round(us, 2), "us_min": round(us_min, 2), "GBps": round(gbps, 1),
                         "pct_hbm_peak": round(100 * gbps / HBM_PEAK_GBPS, 1), "MB": round(abytes[name] / 1e6, 2)}
        log(f"  {name:12s} {us:9.2f} us (min {us_min:7.2f})  {gbps:8.1f} GB/s  {100 * gbps / HBM_PEAK_GBPS:5.1f}% of 8 TB/s")
    unfused_fwd = sum(kernels[n]["us"] for n in ("qk_rpb", "softmax", "av"))
    bwd = sum(kernels[n]["us"] for n in ("av_bwd_p", "av_bwd_v", "softmax_bwd", "qk_bwd_q", "qk_bwd_k", "qk_bwd_rpb"))
    log(f"  unfused fwd {unfused_fwd:.1f} us, fused fwd {kernels['fused_fwd']['us']:.1f} us, bwd (six calls) {bwd:.1f} us, "
        f"na2d_bwd {kernels['bwd']['us']:.1f} us, fused bwd {kernels['fused_bwd']['us']:.1f} us")

    # Entry points that run the same device kernel are grouped; the dominant kernel is the group with the most
    # time in the step.  Its launch duration for the roofline is the median measured above (events on the launch
    # stream around graph replays), which is what a kernel trace of the same command reports.
    inv = inverse_kernel_name(args.workload, p)
    groups = {"qk_mfma_small (qk_rpb, av_bwd_p)": ["qk_rpb", "av_bwd_p"], "av_mfma_small (av, qk_bwd_q)": ["av", "qk_bwd_q"],
              f"{inv} (av_bwd_v, qk_bwd_k)": ["av_bwd_v", "qk_bwd_k"], "fused_mfma_small (fused_fwd)": ["fused_fwd"],
              "softmax": ["softmax"], "softmax_bwd": ["softmax_bwd"], "rpb_partial + rpb_final (qk_bwd_rpb)": ["qk_bwd_rpb"]}
    dominant = max(groups, key=lambda g: sum(kernels[n]["us"] for n in groups[g]))
    members = groups[dominant]
    avg_us = sum(kernels[n]["us"] for n in members) / len(members)
    avg_bytes = sum(abytes[n] for n in members) / len(members)
    achieved = avg_bytes / avg_us / 1e3
    log(f"  dominant kernel: {dominant}: {avg_us:.2f} us per launch, {achieved:.0f} GB/s algorithmic")
    traffic_file = f"profiles/hbm_traffic_{args.workload}_k{p.k}_{p.dtype}.txt"
    traffic = measured_traffic(args.workload, p, dominant)
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "traffic_source": (f"{traffic_file}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this "
                                   "workload, scaled by a plain copy; not measured in this run") if traffic is not None else None,
                "us_per_launch": round(avg_us, 2), "algorithmic_bytes_per_launch": int(avg_bytes),
                "frac_of_copy_ceiling": round(achieved / copy_ceiling, 4)}

    composite, na1d = None, None
    if args.workload == "nat_tiny_stage1" and args.k is None:
        if not args.skip_composite:
            composite = composite_nat_tiny(p, na, synth, torch, timer, args.replays)
            na1d = bench_na1d(na, synth, torch, timer, args.replays)

    result = {
        "metric": METRIC, "value": round(step_bytes / us_step / 1e3, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us_step / 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": p.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload} (B={p.B}, heads={p.heads}, {p.H}x{p.W}, D={p.D}, k={p.k}, {p.dtype}): "
                               "the ten scoped calls (unfused fwd, fused fwd, six backward steps), one call each",
                   "buffer_sets": args.sets, "timing": timer.mode,
                   **({"library": os.path.relpath(args.lib, ROOT) + " (measurement build: not the method's results)"} if args.lib else {})},
        "step_MB": round(step_bytes / 1e6, 1), "us_per_step_python_issued": round(us_step_eager, 1),
        "copy_ceiling_GBps": round(copy_ceiling, 1),
        "us_per_call": {"unfused_fwd": round(unfused_fwd, 1), "fused_fwd": kernels["fused_fwd"]["us"],
                        "bwd_six_calls": round(bwd, 1), "bwd": kernels["bwd"]["us"], "fused_bwd": kernels["fused_bwd"]["us"],
                        "fwd_bwd_unfused": round(unfused_fwd + bwd, 1),
                        "fwd_bwd_fused": round(kernels["fused_fwd"]["us"] + kernels["fused_bwd"]["us"], 1)},
        "kernels": kernels, "roofline": roofline,
    }
    if composite is not None:
        result["composite"] = composite
    if na1d is not None:
        result["na1d"] = na1d
    if not args.no_cpu_baseline:
        log("timing the oracle on the host cores (bounded sample) ...")
        result["cpu_baseline"] = cpu_baseline(p, synth)
        log(f"  oracle: {result['cpu_baseline']}")
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
