#!/usr/bin/env python3
"""Benchmark of the fused AsyncMesh stage update on one MI355X.

A step = one am_step call = local optimizer step + look-ahead + asynchronous sparse averaging
with EMA correction for all R replicas of the stage (subset offsets, then the fused kernel).
Inputs (weights, optimizer state, gradients) are resident in HBM before the timed region.
The K timed steps run as REPEATS consecutive segments, each bracketed by a device synchronisation;
the median segment gives `value` and `ms_per_step`, the spread is reported beside it.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import statistics
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
REPEATS = 5

# name -> (n, R, tau, p, lookahead, bf16)
WORKLOADS = {
    "tiny":      dict(n=1_048_576,     R=4,  tau=1, p=0.05, lookahead=False, bf16=False),
    "small":     dict(n=7_077_888,     R=4,  tau=2, p=0.10, lookahead=True,  bf16=False),
    "stage125m": dict(n=125_829_120,   R=8,  tau=4, p=0.05, lookahead=True,  bf16=False),
    "bf16":      dict(n=125_829_120,   R=16, tau=8, p=0.01, lookahead=False, bf16=True),
    "model1b":   dict(n=1_000_000_000, R=8,  tau=4, p=0.10, lookahead=True,  bf16=False),
}
DESCRIPTION = {
    "stage125m": "one stage of 125,829,120 fp32 params (2.5 layers at d=2048), R=8 replicas, staleness 4, "
                 "subset 5%, AdamW, look-ahead and EMA correction on",
}

# HBM bytes per launch of the fused kernel measured with rocprofv3 hardware counters (FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for a plain copy of known size: x2.0 and
# x1.0 on gfx950); the runs are in profiles/.  Keyed by the digest of the library sources the
# figures were measured on and by (workload, layout of the EMA vectors): a library built from other
# sources gets no traffic figure from here.
MEASURED_TRAFFIC = {
    "source_hash": "34f3f7fd58f7c77c",
    "bytes": {"stage125m/interleaved": 34.24e9, "stage125m/per-replica": 39.23e9,
              "bf16/interleaved": 57.54e9, "model1b/interleaved": 285.41e9},
}


def algorithmic_bytes_per_param(w) -> float:
    """HBM bytes the method itself must move per parameter per replica per step: read w, g, m, v and
    write w, m, v (28 B with fp32 gradients), the forward copy (4 B, or 2 B in bf16), and per
    selected coordinate 4 B sent, 4 B received, 4+4 B of the EMA vector read and written (16 p)."""
    g = 2 if w["bf16"] else 4
    fwd = (2 if w["bf16"] else 4) if (w["lookahead"] or w["bf16"]) else 0
    return 4 + g + 4 + 4 + 4 + 4 + 4 + fwd + 16 * w["p"]


def tiled_on_device(torch, pool, n, offset):
    reps = (n + offset) // pool.numel() + 2
    return pool.repeat(reps)[offset:offset + n].clone()


def fill_tiled(torch, out, pool, offset):
    """out[k] = pool[(k + offset) mod len(pool)], written in place in pieces of one pool length, so that
    no temporary of the size of a state array is ever allocated (the big arrays are the first and only
    large allocations of the process and get whole, aligned stretches of memory)."""
    n, m = out.numel(), pool.numel()
    start = offset % m
    rolled = torch.roll(pool, -start).to(out.dtype)
    for lo in range(0, n, m):
        k = min(m, n - lo)
        out[lo:lo + k].copy_(rolled[:k])


def sample_windows(n):
    """Coordinate ranges on which the oracle replays the run: the whole stage when it is small, else its
    head, an unaligned stretch in the middle and its tail."""
    ln = 2_000_000
    if n <= 3 * ln:
        return [(0, n)]
    return [(0, ln), (n // 2 - ln // 2 + 3, ln), (n - ln, ln)]


def rel_err(got, ref):
    """max |got - ref| over max(|ref|, rms(ref)), the measure the parity tests use."""
    import numpy as np
    ref = ref.astype(np.float64)
    scale = np.maximum(np.abs(ref), np.sqrt(np.mean(ref * ref)) if ref.size else 0.0)
    scale = np.where(scale > 0, scale, 1.0)
    return float(np.max(np.abs(got.astype(np.float64) - ref) / scale)) if ref.size else 0.0


def cpu_baseline(w, args, st, gsets, steps_done, w_pool, seconds_target=12.0):
    """The oracle as it stands, on the host cores, on windows of the same run: it replays the
    steps_done steps the GPU has just made on those coordinate ranges with the same inputs (the
    method is coordinate-wise given (seed, step, global coordinate), so a window is exact), is
    compared with the GPU's state there, and then keeps stepping until about seconds_target of
    timed work is done."""
    import numpy as np
    import torch

    import synth_inputs as si
    from oracle import oracle as O

    n, R, tau, p, bf16 = w["n"], w["R"], w["tau"], w["p"], w["bf16"]
    windows = sample_windows(n)
    oracles, grads = [], []
    for lo, ln in windows:
        orc = O.Oracle(ln, R, delay=tau, avg_interval=args.avg_interval, fraction=p, seed=0, lookahead=w["lookahead"],
                       gamma=0.9, fwd_bf16=bf16, grad_bf16=bf16, mu0=lo, subset_granule=args.subset_granule,
                       subset_kind=O.SUBSET_STRATIFIED if args.subset_kind == "stratified" else O.SUBSET_BERNOULLI,
                       correction=O.CORR_NONE if args.no_correction else O.CORR_EMA)
        orc.set_w(si.tiled(w_pool, ln, lo))
        oracles.append(orc)
        per_set = []
        for gs in gsets:
            sl = [g[lo:lo + ln] for g in gs]
            per_set.append([(x.view(torch.int16).cpu().numpy().view(np.uint16) if bf16 else x.cpu().numpy()) for x in sl])
        grads.append(per_set)
    nsets = len(gsets)
    coords = sum(ln for _, ln in windows)
    t_used, done, t, worst = 0.0, 0, 0, None
    while True:
        t += 1
        t0 = time.perf_counter()
        for orc, per_set in zip(oracles, grads):
            orc.step(t, per_set[t % nsets], 3e-4, 0.5)
        dt = time.perf_counter() - t0
        if t > tau * args.avg_interval + 1:       # count only steps after the ring has filled
            t_used += dt
            done += 1
        if t == steps_done:
            worst = 0.0
            for (lo, ln), orc in zip(windows, oracles):
                for i in range(R):
                    for name in ("w", "m", "v", "d", "fwd"):
                        dev = getattr(st, name)
                        if dev is None:
                            continue
                        e = rel_err(dev[i][lo:lo + ln].float().cpu().numpy(), getattr(orc, name)(i))
                        tol = 1e-2 if (bf16 and name == "fwd") else 1e-6
                        if e >= tol:
                            raise SystemExit(f"bench.py: GPU and oracle disagree on {name}[{i}] in window {lo}: {e:.3e}")
                        if not (bf16 and name == "fwd"):
                            worst = max(worst, e)
        if t >= steps_done and (t_used > seconds_target or t > steps_done + 2000):
            break
    return {
        "value": R * coords * done / t_used, "unit": "params/s", "cores": O.threads(), "kind": "oracle",
        "sample": f"{len(windows)} windows ({coords} coordinates) of the stage, all {R} replicas, {done} steps after "
                  f"start-up ({t_used:.1f} s of CPU time), same inputs as the GPU run",
        "parity": {"steps_compared": steps_done, "windows": windows, "max_rel_err_fp32": worst, "tol_fp32": 1e-6},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="stage125m", choices=sorted(WORKLOADS))
    ap.add_argument("--skip-cpu", action="store_true", help="leave out the CPU oracle leg (profiling runs)")
    ap.add_argument("--avg-interval", type=int, default=1, help="K: average every K-th step (1 = the paper's default)")
    ap.add_argument("--fraction", type=float, default=None, help="override the workload's subset fraction p")
    ap.add_argument("--delay", type=int, default=None, help="override the workload's delay tau")
    ap.add_argument("--no-correction", action="store_true", help="plain delayed averaging (no EMA vector)")
    ap.add_argument("--d-layout", default="interleaved", choices=("interleaved", "per-replica"),
                    help="memory layout of the EMA vectors: replicas side by side per coordinate (one-GPU simulation, "
                         "the headline) or one array per replica")
    ap.add_argument("--subset-granule", type=int, default=1, choices=(1, 32),
                    help="1: coordinates drawn independently (the paper); 32: variant, whole 128-byte lines drawn")
    ap.add_argument("--subset-kind", default="bernoulli", choices=("bernoulli", "stratified"),
                    help="bernoulli: independent draws (the paper); stratified: variant, one coordinate per block of round(1/p)")
    ap.add_argument("--averaging-only", action="store_true",
                    help="time am_sparse_average (the averaging alone, on weights the caller steps itself) instead of the "
                         "fused step; not the headline metric, no CPU leg")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (replicas are simulated as HBM-resident copies on it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2601_22442_amd as am
    import synth_inputs as si
    from paper_2601_22442_amd.build import check_library_is_current

    digest = check_library_is_current(am.version())      # refuses a library not built from the sources beside it

    w = dict(WORKLOADS[args.workload])
    if args.fraction is not None:
        w["p"] = args.fraction
    if args.delay is not None:
        w["tau"] = args.delay
    n, R, tau, p = w["n"], w["R"], w["tau"], w["p"]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = am.make_config(n, R, delay=tau, avg_interval=args.avg_interval, fraction=p, seed=0, optimizer=am.OPT_ADAMW,
                         correction=am.CORR_NONE if args.no_correction else am.CORR_EMA,
                         subset_granule=args.subset_granule,
                         subset_kind=am.SUBSET_STRATIFIED if args.subset_kind == "stratified" else am.SUBSET_BERNOULLI,
                         d_layout=am.D_INTERLEAVED if args.d_layout == "interleaved" else am.D_PER_REPLICA,
                         lookahead=w["lookahead"], gamma=0.9,
                         fwd_dtype=am.BF16 if w["bf16"] else am.F32,
                         grad_dtype=am.BF16 if w["bf16"] else am.F32)
    pool_n = 1 << 20
    w_pool_host = si.stage_weights(pool_n, 0)
    # the big arrays first (state, then gradients), each its own allocation, filled in place afterwards
    st = am.init_state(cfg, None)
    nsets = 1 if n * R * 4 > 24e9 else 2        # two gradient sets per replica, cycled (traffic per step is unchanged); one where two do not fit
    gdt = torch.bfloat16 if w["bf16"] else torch.float32
    if args.averaging_only:
        nsets = 0
    gsets = [[torch.empty(n, dtype=gdt, device=dev) for _ in range(R)] for _ in range(nsets)]
    w_pool = torch.from_numpy(w_pool_host).to(dev)
    for i in range(R):
        fill_tiled(torch, st.w[i], w_pool, 0)
    for s in range(nsets):
        pools = si.replica_grads(pool_n, R, s + 1, 0)
        for i in range(R):
            fill_tiled(torch, gsets[s][i], torch.from_numpy(pools[i]).to(dev), (7919 * (i + 1) * (s + 1)) % pool_n)
    torch.cuda.synchronize()

    if args.averaging_only:
        def one_step(t):
            st.sparse_average(t, 0.5)
    else:
        def one_step(t):
            st.step(t, gsets[t % nsets], 3e-4, 0.5)

    warm = max(args.warmup, tau + 1)          # timed region starts with send and receive both live
    t = 0
    for _ in range(warm):
        t += 1
        one_step(t)
    torch.cuda.synchronize()

    # exactly args.steps timed steps, as up to REPEATS consecutive segments
    repeats = max(1, min(REPEATS, args.steps))
    seg_steps = [args.steps // repeats + (1 if k < args.steps % repeats else 0) for k in range(repeats)]
    st.set_profiling(True)
    seg_ms, launch_ms = [], []
    for k in seg_steps:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        events = []
        for _ in range(k):
            t += 1
            if args.averaging_only:              # events on the library's stream (torch's current one, named at init)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                one_step(t)
                e1.record()
                events.append((e0, e1))
            else:
                one_step(t)
        torch.cuda.synchronize()
        seg_ms.append((time.perf_counter() - t0) * 1e3 / k)
        if args.averaging_only:                  # the whole call: offsets pass + scan + k_average
            launch_ms += [e0.elapsed_time(e1) for e0, e1 in events]
        else:
            launch_ms += st.get_profile_times()      # HIP events around each launch of the fused kernel, on its stream
    st.set_profiling(False)
    assert len(launch_ms) == args.steps
    assert st.read_flags() == 0, "a subset overflowed its ring slot"

    bpp = algorithmic_bytes_per_param(w)
    if args.averaging_only:
        # per selected coordinate and replica: read w^ 4 + write w 4 + sent 4 + received 4 + d 4 + 4 (no d without correction)
        bpp = (16.0 if args.no_correction else 24.0) * p
    bytes_per_launch = bpp * R * n
    ms_per_step = statistics.median(seg_ms)
    kernel_ms_mean = sum(launch_ms) / len(launch_ms)
    achieved = bytes_per_launch / (kernel_ms_mean * 1e-3) / 1e9
    out = {
        "metric": ("am_sparse_average alone: params/s and achieved HBM GB/s (% peak)" if args.averaging_only else
                   "fused AsyncMesh step: params/s and achieved HBM GB/s (% peak), 125M stage"),
        "value": R * n / (ms_per_step * 1e-3),
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": warm, "ms_per_step": ms_per_step,
        "ms_per_step_segments": {"repeats": repeats, "steps_per_segment": seg_steps, "median": ms_per_step,
                                 "min": min(seg_ms), "max": max(seg_ms), "mean": sum(a * b for a, b in zip(seg_ms, seg_steps)) / args.steps},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 gradients and forward weights, f32 state" if w["bf16"] else "f32", "data": "synthetic",
        "library": am.version(), "source_hash": digest,
        "config": {"workload": DESCRIPTION.get(args.workload, args.workload), "name": args.workload,
                   "n": n, "replicas": R, "delay": tau, "fraction": p, "lookahead": w["lookahead"],
                   "avg_interval": args.avg_interval,
                   "correction": "none" if args.no_correction else "ema", "d_layout": args.d_layout,
                   "subset_granule": args.subset_granule, "subset_kind": args.subset_kind, "bf16": w["bf16"], "algorithmic_bytes_per_param": bpp},
        "step_GBps": bytes_per_launch / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": bytes_per_launch / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "roofline": {"kernel": "k_average (+ offsets pass)" if args.averaging_only else "k_step", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": None,
                     "kernel_ms": kernel_ms_mean, "kernel_ms_median": statistics.median(launch_ms),
                     "kernel_ms_min": min(launch_ms), "kernel_ms_max": max(launch_ms), "launches": len(launch_ms),
                     "algorithmic_bytes_per_launch": bytes_per_launch},
    }
    default_settings = (p == WORKLOADS[args.workload]["p"] and tau == WORKLOADS[args.workload]["tau"] and args.avg_interval == 1
                        and not args.no_correction and args.subset_granule == 1 and args.subset_kind == "bernoulli")
    traffic = MEASURED_TRAFFIC["bytes"].get(f"{args.workload}/{args.d_layout}")
    if args.averaging_only:
        # what whole 128-byte lines make of it: every line of w (and of a per-replica d) that holds a selected
        # coordinate is read and rewritten, ring lines and interleaved d lines hold 32 / rb coordinates
        rb = min(8, 1 << max(0, R - 1).bit_length())
        q_w = 1.0 - (1.0 - p) ** 32
        q_d = 0.0 if args.no_correction else (1.0 - (1.0 - p) ** (32 // rb) if args.d_layout == "interleaved" else q_w)
        out["config"]["entry"] = "am_sparse_average"
        out["roofline"]["line_granular_bytes_per_launch"] = R * n * 4.0 * (2.0 * q_w + 2.0 * q_d + 2.0 * p)
        traffic = None
    if traffic is not None and default_settings and MEASURED_TRAFFIC["source_hash"] == digest:
        # counter-measured bytes of this very configuration and this very library, over this run's kernel time
        out["roofline"]["traffic"] = traffic
        out["roofline"]["traffic_from_profile_GBps"] = traffic / (kernel_ms_mean * 1e-3) / 1e9
        out["roofline"]["traffic_from_profile_frac"] = traffic / (kernel_ms_mean * 1e-3) / 1e9 / HBM_PEAK_GBPS
    if not args.skip_cpu and not args.averaging_only:
        out["cpu_baseline"] = cpu_baseline(w, args, st, gsets, t, w_pool_host)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
