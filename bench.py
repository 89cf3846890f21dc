#!/usr/bin/env python3
"""Benchmark of the Markovian next-scale attention hot path on one MI355X.

A step is one forward plus one backward of the whole path over one batch of the 256px
large-model training shape (10 scales, L = 680, B = 32, H = 24, D = 64, bf16).  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

  value      useful TFLOP/s, fwd+bwd: (4 + 10) * D * A * B * H flops per step, A = number of
             unmasked (query, key) pairs per head; element-exact, independent of tile sizes
  roofline   the kernel with the largest share of the step, against the roof that bounds it
  cpu_baseline  the fp64 oracle timed on the host cores on the same workload (every head once)
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

MFMA_PEAK_TFLOPS = 2516.6      # MI355X dense bf16: 256 CU x 2.4 GHz x 4096 flop/clk/CU
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
WORKLOAD = "256px_b32_h24"
SPIN_UP_S = 0.15               # untimed load before each timed region (clock settling)
METRIC = "useful TFLOP/s fwd+bwd (680 tok, H=24, D=64) and % of bf16 MFMA peak"


def kernel_models(n_heads: int, L: int, D: int, A: int):
    """Algorithmic bytes and flops of one launch of each kernel (inputs read once, outputs
    written once; re-reads served by cache are not counted).
    `flops` are the contractions the kernel EXECUTES over the unmasked pairs; `useful_flops`
    what the method needs of them: the backward's scores and dP are formed by both of its
    kernels but count once (with the dQ kernel, which runs first), so the dK/dV kernel
    executes four contractions of which two are useful: 2 + 5 useful per pair and D in all."""
    row = D * 2                                  # one bf16 row
    rows = n_heads * L
    pair_flops = 2 * D * A * n_heads             # one contraction over all unmasked pairs
    return {
        "hmar_fwd_kernel": {"bytes": rows * (4 * row + 4), "flops": 2 * pair_flops, "useful_flops": 2 * pair_flops},
        "hmar_dkdv_kernel": {"bytes": rows * (6 * row + 8), "flops": 4 * pair_flops, "useful_flops": 2 * pair_flops},
        # dQ also reads O and LSE and writes the two per-row statistics of the backward
        "hmar_dq_kernel": {"bytes": rows * (6 * row + 12), "flops": 3 * pair_flops, "useful_flops": 3 * pair_flops},
    }


def read_traffic(kernel: str, workload: str = WORKLOAD):
    """HBM bytes per launch measured offline with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE),
    kept as `kernel = bytes` lines in profiles/hbm_traffic_<workload>.txt; None if absent."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.strip().startswith("#") or "=" not in line:
                    continue
                k, v = line.split("=", 1)
                if k.strip() == kernel:
                    return float(v.split()[0])
    except OSError:
        pass
    return None


def cpu_baseline(w, A: int, budget_s: float = 30.0, chunk: int = 16):
    """Time the oracle (as it stands) on the host cores: the WHOLE workload, every head once, in
    chunks of heads so that the fp64 tensors stay small.  Should the budget run out first, the
    heads done so far are the sample and the line says so."""
    import torch
    import synth_inputs as si
    from oracle import hmar_attn_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    Q, K, V, dO = si.make_inputs(w)
    n_heads = w.B * w.H
    flat = [t.reshape(1, n_heads, w.L, w.D) for t in (Q, K, V, dO)]

    def run(h0, h1):
        q, k, v, g = (si.to_f64(t[:, h0:h1]) for t in flat)
        orc.attn_fwd(q, k, v, w.sides)
        orc.attn_bwd(q, k, v, g, w.sides)

    run(0, min(chunk, n_heads))                   # warm-up (BLAS threads, page faults), untimed
    done, spent = 0, 0.0
    while done < n_heads and spent < budget_s:
        h1 = min(done + chunk, n_heads)
        t0 = time.perf_counter()
        run(done, h1)
        spent += time.perf_counter() - t0
        done = h1
    flops = 14 * w.D * A * done
    whole = "the whole workload" if done == n_heads else f"the first {done} heads (time budget {budget_s:.0f} s)"
    return {"value": flops / spent / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{whole}: {done} of {n_heads} heads of {w.name}, fp64 dense masked fwd+bwd, once, "
                      f"{chunk} heads per call, {spent:.2f} s (input widening to fp64 included)",
            "seconds": spent, "seconds_per_head": spent / done}


def other_workloads(hm, si, torch, dev, reps: int = 24):
    """Context figures for the other shapes and entry points (GPU time from HIP events on the
    launch stream, eager launches): not the headline, not part of `value`.  Each shape rotates
    through enough buffer sets that a launch never finds its operands in the 256 MB last-level
    cache from the launch before (working sets: 180 MB to 670 MB per set)."""
    def gpu_ms(fn, n=reps):
        # the same untimed load first, so that the clocks have settled (see SPIN_UP_S)
        t0, i = time.perf_counter(), 0
        while time.perf_counter() - t0 < 0.08:
            fn(i)
            i += 1
            if i % 8 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / n

    res = {}
    g = torch.Generator(device=dev)
    g.manual_seed(0)

    def rnd(shape):
        return torch.randn(shape, device=dev, generator=g).to(torch.bfloat16)

    for name, mask in (("256px_b16_h16", 0), ("256px_b32_h30", 0), ("512px_b8_h24", 0), ("256px_b32_h24", 1),
                       ("512px_b8_h24", 1), ("large_synthetic_b2_h24", 0), ("large_synthetic_b2_h24", 1)):
        w = si.WORKLOADS[name]
        shape = (w.B, w.H, w.L, w.D)
        one_set = 8 * w.B * w.H * w.L * w.D * 2
        n_sets = max(2, min(4, -(-600_000_000 // one_set)))
        sets = []
        for _ in range(n_sets):
            q, k, v, do = rnd(shape), rnd(shape), rnd(shape), rnd(shape)
            O, LSE = hm.hmar_attn_fwd_masked(q, k, v, w.sides, mask)
            sets.append((q, k, v, do, O, LSE, torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)))
        ws = torch.empty(hm.hmar_attn_bwd_workspace_bytes(w.sides, w.B, w.H, w.D), dtype=torch.uint8, device=dev)

        def f(i):
            q, k, v, do, O, LSE, dq, dk, dv = sets[i % n_sets]
            hm.hmar_attn_fwd_masked(q, k, v, w.sides, mask, 0.0, O, LSE)

        def b(i):
            q, k, v, do, O, LSE, dq, dk, dv = sets[i % n_sets]
            hm.hmar_attn_bwd_masked(q, k, v, O, do, LSE, w.sides, mask, 0.0, dq, dk, dv, ws)
        f_ms, b_ms = gpu_ms(f), gpu_ms(b)
        n = [s * s for s in w.sides]
        if mask == 0:
            A = sum(n[i] * (n[i] + (n[i - 1] if i else 0)) for i in range(len(n)))
        else:
            A = sum(n[i] * sum(n[:i + 1]) for i in range(len(n)))
        flops = 2 * w.D * A * w.B * w.H
        res[name + ("_block_causal" if mask else "")] = {
            "fwd_ms": f_ms, "bwd_ms": b_ms, "fwd_tflops": 2 * flops / f_ms / 1e9, "bwd_tflops": 5 * flops / b_ms / 1e9,
            "fwd_bwd_tflops": 7 * flops / (f_ms + b_ms) / 1e9, "buffer_sets": n_sets}
        del sets, ws
    # KV-cache-free inference: the 10 steps of the 256px schedule, B = 64, H = 24, forward only
    # (706 MB per sweep, two buffer sets): all ten steps in ONE call, and one call per step
    w = si.WORKLOADS["256px_b32_h24"]
    B, H, D = 64, 24, 64
    n = [s * s for s in w.sides]
    n_prevs = [n[i - 1] if i else 0 for i in range(len(n))]
    sweeps = []
    for _ in range(2):
        qs = [rnd((B, H, c, D)) for c in n]
        ks = [rnd((B, H, p + c, D)) for p, c in zip(n_prevs, n)]
        vs = [rnd((B, H, p + c, D)) for p, c in zip(n_prevs, n)]
        os_ = [torch.empty_like(q) for q in qs]
        ls = [torch.empty((B, H, c), dtype=torch.float32, device=dev) for c in n]
        sweeps.append((qs, ks, vs, os_, ls))

    def batched(i):
        qs, ks, vs, os_, ls = sweeps[i % 2]
        hm.hmar_attn_steps_fwd(qs, ks, vs, n_prevs, 0.0, os_, ls)

    def one_by_one(i):
        qs, ks, vs, os_, ls = sweeps[i % 2]
        for j in range(len(n)):
            hm.hmar_attn_step_fwd(qs[j], ks[j], vs[j], n_prevs[j], 0.0, os_[j], ls[j])

    def last_only(i):
        qs, ks, vs, os_, ls = sweeps[i % 2]
        hm.hmar_attn_step_fwd(qs[-1], ks[-1], vs[-1], n_prevs[-1], 0.0, os_[-1], ls[-1])
    ms, ms_single, last = gpu_ms(batched), gpu_ms(one_by_one), gpu_ms(last_only)
    pairs = sum(n[i] * (n[i] + n_prevs[i]) for i in range(len(n)))
    flops = 4 * D * pairs * B * H
    nbytes = B * H * sum((2 * n[i] + 2 * (n[i] + n_prevs[i])) * D * 2 + 4 * n[i] for i in range(len(n)))
    res["inference_steps_256px_b64_h24"] = {
        "all_10_steps_ms": ms, "launch": "one hmar_attn_steps_fwd call (one kernel launch)",
        "tflops": flops / ms / 1e9, "hbm_gbs": nbytes / ms / 1e6,
        "ten_single_step_calls_ms": ms_single,
        "last_step_ms": last, "last_step_tflops": 4 * D * n[-1] * (n[-1] + n[-2]) * B * H / last / 1e9}
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--spin-up-ms", type=float, default=SPIN_UP_S * 1e3,
                    help="untimed load before each timed region, for the clocks to settle")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the secondary workloads (context only)")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of HIP graph replays")
    ap.add_argument("--workload", default=WORKLOAD,
                    help="time another training shape of synth_inputs.WORKLOADS instead (for profiling it; the "
                         "headline line is the default workload's)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch the plain copy kernel (for rocprofv3 --pmc traffic calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path shards over (batch, head) without communication; "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_2506_04421_amd as hm
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("no GPU visible: this benchmark has no CPU path", file=sys.stderr)
        return 3
    w = si.WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    offs, A = hm.hmar_schedule_describe(w.sides)
    n_heads = w.B * w.H

    # three rotating buffer sets (3 x 0.54 GB): no step finds its operands in the 256 MB
    # last-level cache from the previous step
    host = si.make_inputs(w)
    sets = []
    for i in range(3):
        q, k, v, g = (torch.roll(t, shifts=i, dims=0).contiguous().to(dev) for t in host)
        sets.append(dict(q=q, k=k, v=v, g=g, o=torch.empty_like(q),
                         lse=torch.empty((w.B, w.H, w.L), dtype=torch.float32, device=dev),
                         dq=torch.empty_like(q), dk=torch.empty_like(q), dv=torch.empty_like(q)))
    del host
    ws = torch.empty(hm.hmar_attn_bwd_workspace_bytes(w.sides, w.B, w.H, w.D), dtype=torch.uint8, device=dev)

    def fwd(s):
        hm.hmar_attn_fwd(s["q"], s["k"], s["v"], w.sides, 0.0, O=s["o"], LSE=s["lse"])

    def bwd(s):
        hm.hmar_attn_bwd(s["q"], s["k"], s["v"], s["o"], s["g"], s["lse"], w.sides, 0.0,
                         dQ=s["dq"], dK=s["dk"], dV=s["dv"], workspace=ws)

    def step(i):
        s = sets[i % len(sets)]
        fwd(s)
        bwd(s)

    if args.calibration_copy:
        # a plain copy kernel of known size (256 MiB read + 256 MiB written per launch): the
        # reference against which rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled
        src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            hm.hmar_calibration_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    def timed_steps(run_step):
        # An idle MI355X needs some tens of milliseconds under load before its clocks settle
        # (the first ~10 ms after a pause run 20-25 % slower): bring the device to its working
        # state first, untimed, then the W warm-up steps and the K timed steps.
        t_end = time.perf_counter() + args.spin_up_ms * 1e-3
        i = 0
        while args.spin_up_ms > 0 and time.perf_counter() < t_end:
            for _ in range(16):
                run_step(i)
                i += 1
            torch.cuda.synchronize()
        for i in range(args.warmup):
            run_step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            run_step(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    ms_eager = timed_steps(step)
    # The step is three short kernels: launched one by one from Python the host can become
    # the limit, so the same K steps are also timed as replays of one captured HIP graph per
    # buffer set (same kernels, same work, launch cost off the critical path); the faster of
    # the two ways of launching is the headline, both are reported.
    ms_per_step, launch, ms_graph = ms_eager, "eager launches", None
    if not args.no_graph:
        side = torch.cuda.Stream(device=dev)
        graphs = []
        with torch.cuda.stream(side):
            for s_ in sets:
                g_ = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g_, stream=side):
                    fwd(s_)
                    bwd(s_)
                graphs.append(g_)
        torch.cuda.synchronize()
        ms_graph = timed_steps(lambda i: graphs[i % len(graphs)].replay())
        if ms_graph <= ms_eager:
            ms_per_step, launch = ms_graph, "hipGraph replay (one graph per buffer set)"

    # forward and backward separately, HIP events on the launch stream
    def timed(fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(args.steps):
            fn(sets[i % len(sets)])
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / args.steps
    fwd_ms = timed(fwd)
    bwd_ms = timed(bwd)

    # spread of the individual repetitions: one HIP event between consecutive calls
    def spread(fn, n=50):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        ev[0].record()
        for i in range(n):
            fn(sets[i % len(sets)])
            ev[i + 1].record()
        ev[n].synchronize()
        t = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(n))
        return {"median_ms": t[n // 2], "min_ms": t[0], "max_ms": t[-1], "n": n}
    spreads = {"fwd": spread(fwd), "bwd": spread(bwd), "fwd_bwd": spread(lambda s_: (fwd(s_), bwd(s_)))}

    # per-kernel durations: the same steps again with every launch bracketed by HIP events
    hm.hmar_profile_begin()
    for i in range(args.steps):
        step(i)
    prof = hm.hmar_profile_end()
    kern_ms = {k: (ms / n if n else 0.0) for k, (ms, n) in prof.items()}
    models = kernel_models(n_heads, w.L, w.D, A)
    dominant = max(kern_ms, key=lambda k: kern_ms[k])
    m = models[dominant]
    t_dom = kern_ms[dominant] * 1e-3
    hbm_time = m["bytes"] / (HBM_PEAK_GBS * 1e9)
    mfma_time = m["flops"] / (MFMA_PEAK_TFLOPS * 1e12)
    if hbm_time >= mfma_time:
        achieved = m["bytes"] / t_dom / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS}
    else:
        achieved = m["flops"] / t_dom / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / MFMA_PEAK_TFLOPS}
    roof["traffic"] = read_traffic(dominant, w.name)
    roof["kernel"] = dominant
    roof["kernel_ms"] = kern_ms[dominant]
    roof["algorithmic_bytes"] = m["bytes"]
    roof["executed_flops"] = m["flops"]
    roof["useful_flops"] = m["useful_flops"]
    roof["mfma_frac_executed"] = m["flops"] / t_dom / 1e12 / MFMA_PEAK_TFLOPS
    roof["mfma_frac_useful"] = m["useful_flops"] / t_dom / 1e12 / MFMA_PEAK_TFLOPS
    roof["hbm_frac"] = m["bytes"] / t_dom / 1e9 / HBM_PEAK_GBS

    flops_fwd = 4 * w.D * A * n_heads
    flops_bwd = 10 * w.D * A * n_heads
    value = (flops_fwd + flops_bwd) / (ms_per_step * 1e-3) / 1e12
    step_bytes = n_heads * w.L * ((4 * 128 + 4) + (8 * 128 + 4 + 8))   # compulsory fwd + bwd
    out = {
        "metric": METRIC, "value": value, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: sides {list(w.sides)}, L={w.L}, B={w.B}, H={w.H}, D={w.D}, "
                               f"Markovian mask, fwd+bwd, iid N(0,1) bf16 seed {w.seed}",
                   "allowed_pairs_per_head": A, "buffer_sets": len(sets), "launch": launch,
                   "spin_up_ms": args.spin_up_ms},
        "ms_per_step_eager": ms_eager, "ms_per_step_graph": ms_graph,
        "pct_mfma_peak": 100.0 * value / MFMA_PEAK_TFLOPS,
        "fwd_ms": fwd_ms, "bwd_ms": bwd_ms, "repetition_spread": spreads,
        "fwd_tflops": flops_fwd / (fwd_ms * 1e-3) / 1e12, "bwd_tflops": flops_bwd / (bwd_ms * 1e-3) / 1e12,
        "step_hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "kernel_ms": kern_ms,
        "roofline": roof,
    }
    if not args.no_extras:
        out["other_workloads"] = other_workloads(hm, si, torch, dev)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, A)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
