#!/usr/bin/env python3
"""Benchmark of the Streaming DiLoCo fragment outer step on one MI355X.

A "step" is one outer step of one fragment: for every run of the fragment, the outer
gradient of each of the M bf16 replicas, its E3M0 (or other) encoding, decode + fp32
mean, Nesterov update of the fp32 global parameters and momentum, and the alpha-merge
into the M locally advanced replicas -- one call of sdl_fragment_outer_step_plan, which
is a single kernel launch for the decoder shapes used here.  Inputs are resident in HBM
before the timed region starts.

Prints ONE JSON line.  `value` is parameters of the fragment per second; `roofline`
prices the fused kernel against the 8 TB/s HBM peak using the algorithmic bytes
(16 + 6*M bytes per parameter with an overlap delay, 16 + 4*M without); `cpu_baseline`
is the CPU oracle timed on a bounded sample of the same workload on the host cores.
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
DEFAULT_FRAGMENT = {"tiny": 0, "100m": 1, "1b": 1, "4b_p6": 1, "4b_p1": 0, "stress": 1}
# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, each scaled by
# the reading of the copy kernel); see profiles/.  None = not measured for that workload.
MEASURED_TRAFFIC_BYTES = {     # (workload, M, format), default fragment of the workload
    # profiles/fused_all_configs_hbm_traffic.txt: bytes fetched + bytes written per launch
    ("1b", 4, "e3m0"): 7.2483e9 + 4.8322e9,
    ("stress", 8, "e3m0"): 12.0806e9 + 7.2483e9,
    ("4b_p6", 2, "e3m0"): 10.8721e9 + 8.1543e9,
    ("4b_p1", 2, "e3m0"): 68.3781e9 + 51.2844e9,
    ("100m", 2, "e3m0"): 0.4531e9 + 0.3399e9,
}


def algorithmic_bytes_per_param(M: int, tau: int) -> float:
    # read g, mom (8) + w_send (2M) [+ w_now (2M) if it is a different array]; write g, mom (8) + w_now (2M)
    return 16.0 + (6.0 if tau > 0 else 4.0) * M


class State:
    """Flat model arrays in HBM and the plan of one workload.  The arrays are carved from one allocation as
    sdl_flat_layout says (what the library recommends); separate=True allocates them one by one instead."""

    def __init__(self, wl, sdl, workloads, torch, fragment: int, M: int, separate: bool = False):
        self.wl, self.M, self.fragment = wl, M, fragment
        dev = "cuda"
        if wl.shape is None:
            numel, block, L = [wl.flat_numel], [0], 1
        else:
            shape = workloads.SHAPES[wl.shape]
            numel, block, _ = shape.units()
            L = shape.n_layers
        self.plan = sdl.sdl_fragment_plan(numel, block, L, wl.P, sdl.PATTERN_STRIDED, wl.H, wl.tau)
        total = self.plan.total_numel
        if separate:
            self.g = torch.empty(total, dtype=torch.float32, device=dev)
            self.mom = torch.empty(total, dtype=torch.float32, device=dev)
            self.w_send = [torch.empty(total, dtype=torch.bfloat16, device=dev) for _ in range(M)]
            self.w_now = self.w_send if wl.tau == 0 else \
                [torch.empty(total, dtype=torch.bfloat16, device=dev) for _ in range(M)]
        else:
            self.g, self.mom, self.w_send, self.w_now, self.pool = sdl.alloc_flat_model(total, M, wl.tau > 0, device=dev)
        self.spans = sdl.sdl_plan_fragment_spans(self.plan, fragment)
        self.runs = sdl.sdl_plan_fragment_runs(self.plan, fragment)
        self.n = sum(n for _, n, _ in self.spans)
        for off, n, unit in self.spans:
            sl = slice(off, off + n)
            workloads.fill_span(self.g[sl], self.mom[sl], [w[sl] for w in self.w_send],
                                [w[sl] for w in self.w_now], unit=unit, tau=wl.tau, delta=wl.delta,
                                base_seed=wl.seed)


def time_gpu(torch, fn, steps: int, warmup: int) -> float:
    """Average milliseconds per call of fn, HIP events on the current stream around `steps` calls."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(steps):
        fn()
    end.record()
    torch.cuda.synchronize()
    return start.elapsed_time(end) / steps


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="1b", choices=sorted(DEFAULT_FRAGMENT))
    ap.add_argument("--fragment", type=int, default=None)
    ap.add_argument("--format", default=None,
                    choices=["e3m0", "e4m3", "bf16", "fp32", "e3m0_b64", "e3m0_b128", "e3m0_span", "e3m0_rn"])
    ap.add_argument("--workers", type=int, default=None, help="override M")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-allocations", action="store_true",
                    help="allocate every flat array on its own instead of carving them from one allocation")
    ap.add_argument("--no-extras", action="store_true", help="skip the unfused / copy side measurements")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the other target configurations (100M, 4B P=6, 4B P=1, stress) and the stress curve")
    ap.add_argument("--sweep", action="store_true",
                    help="also time the receive side and the fused step over M in {1,2,4,8} x {e3m0,e4m3,bf16}")
    ap.add_argument("--offload", action="store_true",
                    help="also time the fragment step with g / mom staged from pinned host memory")
    ap.add_argument("--graph", action="store_true",
                    help="also time the same steps replayed from one captured HIP graph (launch-bound small cases)")
    ap.add_argument("--engine", action="store_true",
                    help="also walk the schedule driver over whole outer rounds (all P fragments, messages in HBM)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the M workers are M replicas resident in one "
              "GPU's HBM; there is no multi-GPU path). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch

    import paper_2501_18512_amd as sdl
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path.", file=sys.stderr)
        return 2
    wl = workloads.WORKLOADS[args.workload]
    M = args.workers or wl.M
    fmt_name = args.format or wl.fmt
    fmt = sdl.FORMATS[fmt_name]
    frag = DEFAULT_FRAGMENT[args.workload] if args.fragment is None else args.fragment
    st = State(wl, sdl, workloads, torch, frag, M, separate=args.separate_allocations)
    torch.cuda.synchronize()

    # ---- CPU baseline sample is taken from the untouched inputs (before any GPU step)
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(st, fmt, torch, workloads)

    # the whole-span scale needs its scale words (one per span and replica) as workspace
    span_words = None
    if fmt == sdl.FMT_E3M0_SPAN:
        span_words = [torch.zeros(max(sdl.sdl_plan_message_bytes(st.plan, frag, fmt)[1], 4), dtype=torch.uint8,
                                  device="cuda") for _ in range(M)]

    def step():
        sdl.sdl_fragment_outer_step_plan_ex(st.plan, frag, st.g, st.mom, st.w_send, st.w_now, fmt, wl.lr, wl.mu,
                                            wl.alpha, None, span_words)

    n_launch = -(-len(st.runs) // 16)
    ms = time_gpu(torch, step, args.steps, args.warmup)
    bpp = algorithmic_bytes_per_param(M, wl.tau)
    kernel_name = "sdl_kernel<fused>"
    if fmt == sdl.FMT_E3M0_SPAN:
        # one scale per span: an extra read pass over g and w_send for the grid-wide maximum, and one
        # launch group per 16 spans; the step is reported as a whole
        bpp += 4.0 + 2.0 * M
        n_launch = 1
        kernel_name = "sdl_kernel<absmax> + sdl_kernel<fused>, all launches of the step"
    launch_ms = ms / n_launch
    achieved = bpp * st.n / n_launch / (launch_ms * 1e-3) / 1e9
    out = {
        "metric": "fragment_outer_step_params_per_s",
        "value": st.n / (ms * 1e-3),
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{wl.name}: fragment {frag} of P={wl.P} strided ({wl.shape or 'flat'} decoder shape), "
                        f"{st.n} params in {len(st.runs)} runs, M={M} bf16 replicas, {fmt_name} exchange, "
                        f"tau={wl.tau}, alpha={wl.alpha}, lr={wl.lr}, mu={wl.mu}, deltas={wl.delta}",
            "fragment_params": st.n, "M": M, "format": fmt_name, "tau": wl.tau, "alpha": wl.alpha,
            "launches_per_step": n_launch,
            "array_layout": "separate allocations" if args.separate_allocations else
                            "one allocation, sdl_flat_layout (2 MiB slots, bases staggered by 32 KiB)",
        },
        "roofline": {
            "bound": "hbm", "kernel": kernel_name, "achieved": achieved, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, M, fmt_name))
            if frag == DEFAULT_FRAGMENT[args.workload] else None,
            "algorithmic_bytes_per_param": bpp, "bytes_per_launch": bpp * st.n / n_launch,
            "launch_ms": launch_ms,
        },
        "cpu_baseline": cpu,
    }
    if not args.no_extras:
        out["extras"] = extras(st, fmt, wl, M, torch, sdl, args)
        # the practical ceiling: a non-temporal copy of 1.2 GB (what fraction of it the fused kernel reaches)
        out["roofline"]["copy_nt_GB/s"] = out["extras"]["memory_probes"]["copy_nt"]["GB/s"]
        out["roofline"]["frac_of_copy"] = achieved / out["extras"]["memory_probes"]["copy_nt"]["GB/s"]
    if args.sweep:
        out["sweep"] = sweep(st, frag, wl, M, torch, sdl, args)
    if args.offload:
        out["offload"] = offload_timing(st, frag, fmt, wl, M, torch, sdl, args)
    if args.graph:
        out["graph"] = graph_timing(step, st, bpp, torch, args)
    if args.engine:
        out["engine"] = engine_timing(st, fmt, wl, M, torch, sdl, workloads)
    if not args.no_configs and args.workload == "1b" and args.fragment is None and args.format is None \
            and args.workers is None:
        # the other target configurations, each timed with the same loop on a state of its own
        del st, step
        torch.cuda.empty_cache()
        out.setdefault("extras", {})
        out["extras"]["configs"], out["extras"]["stress_curve"] = other_configs(torch, sdl, workloads, args)
    print(json.dumps(out))
    return 0


def cpu_baseline(st, fmt, torch, workloads):
    """The oracle's fused step on the first 2^27 parameters of the fragment's largest run (block
    aligned), with the host threads the box offers to one GPU job (at most 16)."""
    import oracle

    off, n, _ = max(st.runs, key=lambda r: r[1])
    n = min(n, 1 << 27)
    sl = slice(off, off + n)
    hg, hmom = st.g[sl].cpu().numpy().copy(), st.mom[sl].cpu().numpy().copy()
    hs = [workloads.bf16_bits(w[sl]) for w in st.w_send]
    hn = hs if st.wl.tau == 0 else [workloads.bf16_bits(w[sl]) for w in st.w_now]
    threads = max(1, min(16, os.cpu_count() or 1))
    oracle.build()
    t0 = time.perf_counter()
    used = oracle.fragment_outer_step_chunked(hg, hmom, hs, hn, fmt, st.wl.lr, st.wl.mu, st.wl.alpha, threads)
    dt = time.perf_counter() - t0
    # one thread, on a smaller piece of the same data (the arrays above were advanced in place:
    # a second outer step on them is as good an input as the first)
    n1 = min(n, 1 << 23)
    hs1 = [w[:n1] for w in hs]
    hn1 = hs1 if hn is hs else [w[:n1] for w in hn]
    t0 = time.perf_counter()
    oracle.fragment_outer_step_chunked(hg[:n1], hmom[:n1], hs1, hn1, fmt, st.wl.lr, st.wl.mu, st.wl.alpha, 1)
    dt1 = time.perf_counter() - t0
    return {"value": n / dt, "unit": "params/s", "cores": min(threads, used), "kind": "oracle",
            "sample": f"first {n} parameters of the fragment's largest run, M={st.M}, same inputs, "
                      f"{dt:.2f} s wall on {min(threads, used)} threads",
            "single_thread": {"value": n1 / dt1, "unit": "params/s", "cores": 1,
                              "sample": f"first {n1} parameters, {dt1:.2f} s"}}


def extras(st, fmt, wl, M, torch, sdl, args):
    """Side measurements on the largest run of the fragment: the three unfused calls and the
    plain copy kernel (the practical HBM ceiling)."""
    off, n, _ = max(st.runs, key=lambda r: r[1])
    sl = slice(off, off + n)
    g, mom = st.g[sl], st.mom[sl]
    ws, wn = [w[sl] for w in st.w_send], [w[sl] for w in st.w_now]
    codes, scales = sdl.alloc_exchange(fmt, n, M)
    cb, sb = sdl.sdl_exchange_bytes(fmt, n)
    steps, warm = max(5, args.steps // 2), 3
    res = {"run_params": n}
    t = time_gpu(torch, lambda: sdl.sdl_quantize_outer_grad(g, ws, n, fmt, codes, scales), steps, warm)
    res["quantize"] = {"ms": t, "GB/s": (4 + 2 * M) * n / t / 1e6 + M * (cb + sb) / t / 1e6}
    t = time_gpu(torch, lambda: sdl.sdl_dequant_reduce_nesterov(g, mom, codes, scales, n, fmt, wl.lr, wl.mu),
                 steps, warm)
    res["dequant_reduce_nesterov"] = {"ms": t, "GB/s": (16 * n + M * (cb + sb)) / t / 1e6}
    t = time_gpu(torch, lambda: sdl.sdl_merge_overlap(g, wn, n, wl.alpha), steps, warm)
    res["merge_overlap"] = {"ms": t, "GB/s": (4 + 4 * M) * n / t / 1e6}
    work = scales if fmt == sdl.FMT_E3M0_SPAN else None          # the whole-span scale needs its scale words
    t = time_gpu(torch, lambda: sdl.sdl_fragment_outer_step(g, mom, ws, wn, n, fmt, wl.lr, wl.mu, wl.alpha, None, work),
                 steps, warm)
    res["fused_single_run"] = {"ms": t, "GB/s": algorithmic_bytes_per_param(M, wl.tau) * n / t / 1e6}
    res["memory_probes"] = memory_probes(torch, sdl, steps, warm)
    # the unfused calls once more on the whole fragment (what the schedule driver launches when tau > 0)
    if fmt != sdl.FMT_E3M0_SPAN:
        fcb, fsb = sdl.sdl_plan_message_bytes(st.plan, st.fragment, fmt)
        fc = [torch.empty(max(fcb, 16), dtype=torch.uint8, device="cuda") for _ in range(M)]
        fs = [torch.empty(max(fsb, 16), dtype=torch.uint8, device="cuda") for _ in range(M)]
        msg = M * (fcb + fsb)
        frag_calls = {}
        for name, fn, nbytes in (
                ("quantize", lambda: sdl.sdl_quantize_outer_grad_plan(st.plan, st.fragment, st.g, st.w_send, fmt, fc, fs),
                 (4 + 2 * M) * st.n + msg),
                ("dequant_reduce_nesterov", lambda: sdl.sdl_dequant_reduce_nesterov_plan(
                    st.plan, st.fragment, st.g, st.mom, fc, fs, fmt, wl.lr, wl.mu), 16 * st.n + msg),
                ("merge_overlap", lambda: sdl.sdl_merge_overlap_plan(st.plan, st.fragment, st.g, st.w_now, wl.alpha),
                 (4 + 4 * M) * st.n),
                ("receive_outer_step", lambda: sdl.sdl_receive_outer_step_plan(
                    st.plan, st.fragment, st.g, st.mom, fc, fs, st.w_now, fmt, wl.lr, wl.mu, wl.alpha),
                 (16 + 4 * M) * st.n + msg)):
            t = time_gpu(torch, fn, steps, warm)
            frag_calls[name] = {"ms": t, "GB/s": nbytes / t / 1e6, "frac": nbytes / t / 1e6 / HBM_PEAK_GBS}
        res["fragment_calls"] = frag_calls
        del fc, fs
        # the fused step in the whole-span (per-tensor) scale, the 4.0 bits per parameter of the paper's accounting:
        # one more read pass over g and w_send for the grid-wide maxima (pre-pass + fused launch timed together)
        span_fmt = sdl.FMT_E3M0_SPAN
        words = [torch.zeros(max(sdl.sdl_plan_message_bytes(st.plan, st.fragment, span_fmt)[1], 4), dtype=torch.uint8,
                             device="cuda") for _ in range(M)]
        t = time_gpu(torch, lambda: sdl.sdl_fragment_outer_step_plan_ex(
            st.plan, st.fragment, st.g, st.mom, st.w_send, st.w_now, span_fmt, wl.lr, wl.mu, wl.alpha, None, words),
            steps, warm)
        sbpp = algorithmic_bytes_per_param(M, wl.tau) + 4.0 + 2.0 * M
        res["fused_whole_span_scale"] = {"ms": t, "GB/s": sbpp * st.n / t / 1e6, "frac": sbpp * st.n / t / 1e6 / HBM_PEAK_GBS,
                                         "algorithmic_bytes_per_param": sbpp}
    # parameters handed to evaluation: fp32 mean of the replicas, written as bf16 (2M + 2 bytes per parameter)
    ev = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    t = time_gpu(torch, lambda: sdl.sdl_evaluation_params(sdl.EVAL_REPLICA_MEAN, None, ws, n, ev), steps, warm)
    res["evaluation_params_replica_mean"] = {"ms": t, "GB/s": (2 * M + 2) * n / t / 1e6}
    # diagnostics: cosine similarity of the replicas' outer gradients, per span and for the whole fragment
    # (reads 4 + 2M bytes per parameter)
    frag = st.fragment
    n_spans = len(st.spans)
    span_res, work = sdl.alloc_cosine(M, n_spans)
    frag_res = torch.empty(sdl.cosine_result_doubles(M), dtype=torch.float64, device="cuda")
    t = time_gpu(torch, lambda: sdl.sdl_outer_grad_cosine_plan(st.plan, frag, st.g, st.w_send, span_res, frag_res, work),
                 steps, warm)
    res["outer_grad_cosine_fragment"] = {"ms": t, "GB/s": (4 + 2 * M) * st.n / t / 1e6, "spans": n_spans}
    return res


def memory_probes(torch, sdl, steps, warm, nbytes=1207959552):
    """What the memory system gives a kernel that does nothing else, on buffers far larger than the
    256 MB of Infinity Cache (1.2 GB each): a plain copy, and a copy, a read-only pass and a write-only
    pass with the non-temporal policy of the method's kernels.  GB/s counts every byte read or written."""
    # both buffers in one allocation, 2 MiB-aligned slots with a 32 KiB stagger, like the model arrays
    slot = (nbytes + (1 << 21) - 1) // (1 << 21) * (1 << 21)
    pool = torch.empty(2 * slot + (1 << 22), dtype=torch.uint8, device="cuda")
    base = (-pool.data_ptr()) % (1 << 21)
    src = pool[base:base + nbytes].fill_(1)
    dst = pool[base + slot + 32768:base + slot + 32768 + nbytes].fill_(2)
    res = {"bytes": nbytes}
    for name, kind, traffic in (("copy", sdl.PROBE_COPY, 2 * nbytes), ("copy_nt", sdl.PROBE_COPY_NT, 2 * nbytes),
                                ("read_nt", sdl.PROBE_READ_NT, nbytes), ("fill_nt", sdl.PROBE_FILL_NT, nbytes)):
        t = time_gpu(torch, lambda: sdl.sdl_memory_probe(kind, dst, src, nbytes), steps, warm)
        res[name] = {"ms": t, "GB/s": traffic / t / 1e6}
    return res


def other_configs(torch, sdl, workloads, args):
    """The target configurations besides the headline one, each on a state of its own that is freed before
    the next: fused step of the default fragment, same timing loop; then, on the stress state, the curve over
    replica counts and formats."""
    configs, curve = {}, None
    # "1b_separate_allocations": the headline workload once more with every array allocated on its own, which is
    # how a caller that does not follow sdl_flat_layout holds them
    for name in ("1b_separate_allocations", "100m", "4b_p6", "4b_p1", "stress"):
        separate = name.endswith("_separate_allocations")
        wl = workloads.WORKLOADS[name.split("_separate")[0]]
        frag = DEFAULT_FRAGMENT[wl.name]
        st = State(wl, sdl, workloads, torch, frag, wl.M, separate=separate)
        fmt = sdl.FORMATS[wl.fmt]
        torch.cuda.synchronize()
        ms = time_gpu(torch, lambda: sdl.sdl_fragment_outer_step_plan(st.plan, frag, st.g, st.mom, st.w_send, st.w_now,
                                                                      fmt, wl.lr, wl.mu, wl.alpha),
                      args.steps, args.warmup)
        bpp = algorithmic_bytes_per_param(wl.M, wl.tau)
        gbs = bpp * st.n / ms / 1e6
        configs[name] = {"fragment": frag, "fragment_params": st.n, "M": wl.M, "format": wl.fmt, "tau": wl.tau,
                         "launches_per_step": -(-len(st.runs) // 16), "ms": ms, "params_per_s": st.n / (ms * 1e-3),
                         "GB/s": gbs, "frac": gbs / HBM_PEAK_GBS, "algorithmic_bytes_per_param": bpp,
                         "traffic": MEASURED_TRAFFIC_BYTES.get((wl.name, wl.M, wl.fmt))}
        if name == "stress":
            curve = sweep(st, frag, wl, wl.M, torch, sdl, args)
        del st
        torch.cuda.empty_cache()
    return configs, curve


def sweep(st, frag, wl, M, torch, sdl, args):
    """Bandwidth curve of the stress configuration: replica counts 1, 2, 4, 8 (up to the M that was
    allocated) and exchange formats E3M0 / E4M3 / BF16, for the receive side alone
    (sdl_dequant_reduce_nesterov_plan: 16 + M*c bytes per parameter) and for the fused step."""
    res = {}
    steps, warm = max(10, args.steps // 2), 3
    # fp32 (no quantisation) rides along as the codec-free reference: same arrays and launch shape, trivial arithmetic
    for fmt_name in ("e3m0", "e4m3", "bf16", "fp32"):
        f = sdl.FORMATS[fmt_name]
        cb, sb = sdl.sdl_plan_message_bytes(st.plan, frag, f)
        codes = [torch.zeros(max(cb, 16), dtype=torch.uint8, device="cuda") for _ in range(M)]
        scales = [torch.zeros(max(sb, 16), dtype=torch.uint8, device="cuda") for _ in range(M)]
        sdl.sdl_quantize_outer_grad_plan(st.plan, frag, st.g, st.w_send, f, codes, scales)
        for m in (1, 2, 4, 8):
            if m > M:
                continue
            t_r = time_gpu(torch, lambda: sdl.sdl_dequant_reduce_nesterov_plan(
                st.plan, frag, st.g, st.mom, codes[:m], scales[:m], f, wl.lr, wl.mu), steps, warm)
            t_f = time_gpu(torch, lambda: sdl.sdl_fragment_outer_step_plan(
                st.plan, frag, st.g, st.mom, st.w_send[:m], st.w_now[:m], f, wl.lr, wl.mu, wl.alpha), steps, warm)
            r_gbs = (16.0 * st.n + m * (cb + sb)) / t_r / 1e6
            f_gbs = algorithmic_bytes_per_param(m, wl.tau) * st.n / t_f / 1e6
            res[f"{fmt_name}_M{m}"] = {"reduce_ms": t_r, "reduce_GB/s": r_gbs, "reduce_frac": r_gbs / HBM_PEAK_GBS,
                                       "fused_ms": t_f, "fused_GB/s": f_gbs, "fused_frac": f_gbs / HBM_PEAK_GBS}
    return res


def offload_timing(st, frag, fmt, wl, M, torch, sdl, args):
    """Outer parameters and momentum in pinned host memory (Section 2.5 of the paper): copy-in of the
    fragment, staged fused step, write-back -- each timed alone, then the whole round trip."""
    g_host = st.g.cpu().pin_memory()
    mom_host = st.mom.cpu().pin_memory()
    pool = sdl.sdl_offload_create(st.plan, 1)
    slot_g = [torch.empty(pool.slot_numel, dtype=torch.float32, device="cuda")]
    slot_mom = [torch.empty(pool.slot_numel, dtype=torch.float32, device="cuda")]
    sdl.sdl_offload_bind(pool, g_host, mom_host, slot_g, slot_mom)
    copy = torch.cuda.Stream()
    res = {"state_bytes": 8 * st.n}
    t_in, t_step, t_out = [], [], []
    for _ in range(max(3, args.steps // 10)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        sdl.sdl_offload_prefetch(pool, frag, copy)
        copy.synchronize()
        t1 = time.perf_counter()
        sdl.sdl_offload_acquire(pool, frag, copy)
        sdl.sdl_fragment_outer_step_staged(st.plan, frag, slot_g[0], slot_mom[0], st.w_send, st.w_now, fmt, wl.lr,
                                           wl.mu, wl.alpha)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        sdl.sdl_offload_release(pool, frag, copy)
        copy.synchronize()
        t3 = time.perf_counter()
        t_in.append(t1 - t0), t_step.append(t2 - t1), t_out.append(t3 - t2)
    for name, ts in (("copy_in", t_in), ("staged_step", t_step), ("write_back", t_out)):
        ms = 1e3 * sorted(ts)[len(ts) // 2]
        res[name] = {"ms": ms, "GB/s": (8 * st.n if name != "staged_step" else
                                        algorithmic_bytes_per_param(M, wl.tau) * st.n) / ms / 1e6}
    return res


def graph_timing(step, st, bpp, torch, args):
    """The timed loop once more, as one captured graph of `steps` launches replayed from the host with a
    single call: what is left of the per-step time when the launch overhead is taken out (the calls
    allocate nothing and use no memset, so they can be captured as they are)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(args.steps):
            step()
    for _ in range(2):
        graph.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 5
    e0.record()
    for _ in range(reps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / (reps * args.steps)
    return {"ms_per_step": ms, "params_per_s": st.n / (ms * 1e-3), "GB/s": bpp * st.n / ms / 1e6,
            "steps_per_graph": args.steps}


def engine_timing(st, fmt, wl, M, torch, sdl, workloads):
    """Algorithm 2's outer schedule for the whole model: the engine is stepped through three periods of
    H inner steps (inner steps themselves are not part of this build: nothing runs between the calls),
    every fragment sends once and receives once per period.  Reports the device time of one period's
    outer work and the host time the driver spends per inner step."""
    P = st.plan.num_fragments
    for p in range(P):                     # fill the fragments the main measurement left empty
        if p == st.fragment:
            continue
        for off, n, unit in sdl.sdl_plan_fragment_spans(st.plan, p):
            sl = slice(off, off + n)
            workloads.fill_span(st.g[sl], st.mom[sl], [w[sl] for w in st.w_send], [w[sl] for w in st.w_now],
                                unit=unit, tau=wl.tau, delta=wl.delta, base_seed=wl.seed)
    eng = sdl.sdl_engine_create(st.plan, wl.H, [wl.tau] * M, fmt, wl.lr, wl.mu, wl.alpha)
    codes, scales = [], []
    for p in range(P):
        cb, sb = sdl.sdl_plan_message_bytes(st.plan, p, fmt)
        for _ in range(M):
            codes.append(torch.empty(max(cb, 16), dtype=torch.uint8, device="cuda"))
            scales.append(torch.empty(max(sb, 16), dtype=torch.uint8, device="cuda"))
    # the engine works on the live replicas: the same arrays serve as w at the send and at the receive step
    sdl.sdl_engine_bind(eng, st.g, st.mom, st.w_now, codes, scales)
    total = st.plan.total_numel
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    periods, host = [], []
    t = 0
    for period in range(3):
        torch.cuda.synchronize()
        ev0.record()
        h0 = time.perf_counter()
        events = 0
        for _ in range(wl.H):
            t += 1
            sent, received = sdl.sdl_engine_step(eng, t)
            events += sent + received
        host.append((time.perf_counter() - h0) / wl.H)
        ev1.record()
        torch.cuda.synchronize()
        periods.append((ev0.elapsed_time(ev1), events))
    ms, events = periods[-1]               # a steady-state period: P sends and P receives
    c = sum(sdl.sdl_plan_message_bytes(st.plan, p, fmt)[i] for p in range(P) for i in (0, 1)) / total
    bytes_per_param = (4 + 2 * M + M * c) + (16 + M * c + 4 * M) if wl.tau > 0 else algorithmic_bytes_per_param(M, 0)
    return {"fragments": P, "model_params": total, "H": wl.H, "tau": wl.tau, "events_per_period": events,
            "outer_work_ms_per_period": ms, "params_per_s": total / (ms * 1e-3),
            "GB/s": bytes_per_param * total / ms / 1e6, "bytes_per_param": bytes_per_param,
            "host_us_per_inner_step": 1e6 * host[-1]}


if __name__ == "__main__":
    sys.exit(main())
