#!/usr/bin/env python3
"""Benchmark of the ROCKET transform hot path on one MI355X.

A step is one rocket_transform call (zero-pad copy + conv/pooling kernel) on
the paper's headline workload: a batch of 64 examples of 20 channels x 50,000
timesteps through K = 10,000 random kernels, two pooled features per kernel
(max + PPV).  Inputs are synthetic (seeded AR(1) channels, z-normalised) and
resident in HBM before the timed region.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP32_VECTOR_PEAK_TFLOPS = 157.3   # MI355X datasheet, packed FP32 on the vector ALUs
# HBM-side bytes per launch of the dominant kernel, from the two `rocprofv3 --pmc` runs (FETCH_SIZE,
# WRITE_SIZE, each scaled by what the counter reads for the padding copy of known size) whose summaries
# are under profiles/: (workload, batch, feature mask) -> bytes.  Other shapes report null.
MEASURED_TRAFFIC = {
    # profiles/rk_forward_multivariate-20x50k.md: 12,581,194 KiB x 1.968 fetched + 59,074 KiB x 1.001 written
    ("multivariate-20x50k", 64, 3): 25414576462,
    # profiles/rk_backward_multivariate-20x50k-grad.md: 20,025,199 KiB x 1.968 + 168,805 KiB x 1.001
    ("multivariate-20x50k-grad", 60, 5): 40528449964,
}

WORKLOADS = {
    # name: (synth config, feature mask or None = the config's, description)
    "multivariate-20x50k": 2,
    "multivariate-20x50k-grad": 3,
    "multivariate-20x50k-train": 3,   # whole training step: transform, linear head, loss gradient, backward, update
    "multivariate-20x50k-u8": 2,      # the same batch as raw 8-bit samples, normalised inside the call
    "univariate-standard": 1,
    "univariate-tiny": 0,
    "long-20x200k": 4,
    "ridge-677x20000": None,          # the regressor at the paper's sizes: one step = one fit + one 64-row predict
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="multivariate-20x50k", choices=sorted(WORKLOADS))
    ap.add_argument("--batch", type=int, default=None, help="override the workload's batch size")
    ap.add_argument("--features", type=int, default=None, help="feature mask override (1=max, 2=PPV, 4=softPPV)")
    ap.add_argument("--lam", type=float, default=10.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--lean", action="store_true",
                    help="only the timed region: no extra workloads, no H2D-inclusive run, no FMA calibration "
                         "(for profiler runs, so that the trace holds the timed launches only)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time its replays (for launch-bound small workloads)")
    ap.add_argument("--cpu-examples", type=int, default=None, help="examples in the oracle's timed sample")
    return ap.parse_args()


def cpu_baseline(cfg_id, x_host, kr, mask, lam, n_examples):
    """Times the oracle (all host threads) on the first n_examples examples x all kernels."""
    import oracle
    xs = x_host[:n_examples]
    t0 = time.perf_counter()
    if xs.dtype == np.uint8:
        xs = oracle.znormalize_u8(xs)
    oracle.transform(xs, kr, lam=lam, shift=-3.0)
    dt = time.perf_counter() - t0
    return {
        "value": n_examples / dt, "unit": "examples/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "%d example(s) x all %d kernels of the same workload, %.1f s, fp64, all features at once"
                  % (n_examples, len(kr["length"]), dt),
    }


def quick_rate(rocket, synth, torch, cfg_id, lam, steps=20, warmup=3):
    """series/s and conv TFLOP/s of a small workload, whole batch resident, same timing rules."""
    cfg = synth.CONFIGS[cfg_id]
    B, mask = cfg["B"], cfg["features"]
    h = rocket.rocket_make_kernels(synth.seed_k(cfg_id), cfg["K"], cfg["C"], cfg["L"])
    fma, _ = rocket.rocket_work_per_series(h)
    x = torch.from_numpy(synth.make_input(cfg_id)).cuda()
    out = torch.empty((B, rocket.rocket_num_features(mask) * cfg["K"]), dtype=torch.float32, device="cuda")
    ws = torch.empty(rocket.rocket_workspace_bytes(h, B, mask), dtype=torch.uint8, device="cuda")
    for _ in range(warmup):
        rocket.rocket_transform(h, x, mask, lam, -3.0, out=out, workspace=ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        rocket.rocket_transform(h, x, mask, lam, -3.0, out=out, workspace=ws)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    h.free()
    return {"workload": cfg["name"], "B": B, "C": cfg["C"], "L": cfg["L"], "K": cfg["K"], "features": mask,
            "value": B / dt, "unit": "series/s", "ms_per_step": 1e3 * dt, "conv_tflops": 2.0 * fma * B / dt / 1e12}


def ridge_bench(args, torch, rocket):
    """The ridge regressor at the paper's sizes (677 training examples x 20,000 features):
    a step is one fit followed by one prediction of 64 rows."""
    n, p, m = 677, 20000, 64
    rng = np.random.Generator(np.random.PCG64(677))
    X = torch.from_numpy(rng.standard_normal((n, p)).astype(np.float32)).cuda()
    y = torch.from_numpy((0.6 + 1.2 * rng.random(n)).astype(np.float32)).cuda()
    ws = torch.empty(rocket.rocket_ridge_workspace_bytes(n, p), dtype=torch.uint8, device="cuda")

    def step():
        coef, b = rocket.rocket_ridge_fit(X, y, 1.0, workspace=ws)
        return rocket.rocket_ridge_predict(X[:m], coef, b)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    print(json.dumps({
        "metric": "ridge fits/sec (677 x 20,000, fp64, dual form) with a 64-row predict each",
        "value": 1.0 / dt, "unit": "fits/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * dt, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": args.workload, "n": n, "p": p, "predict_rows": m, "alpha": 1.0},
    }))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    from paper_2301_08527_amd import rocket

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the transform has no CPU path", file=sys.stderr)
        sys.exit(1)

    if args.workload == "ridge-677x20000":
        ridge_bench(args, torch, rocket)
        return
    cfg_id = WORKLOADS[args.workload]
    cfg = synth.CONFIGS[cfg_id]
    B = cfg["B"] if args.batch is None else args.batch
    mask = cfg["features"] if args.features is None else args.features
    K, C, L = cfg["K"], cfg["C"], cfg["L"]

    from_u8 = args.workload.endswith("-u8")
    x_host = synth.make_input_u8(cfg_id, B=B) if from_u8 else synth.make_input(cfg_id, B=B)
    h = rocket.rocket_make_kernels(synth.seed_k(cfg_id), K, C, L)
    fma_per_series, outputs_per_series = rocket.rocket_work_per_series(h)
    F = rocket.rocket_num_features(mask)

    dev = torch.device("cuda:0")
    x = torch.from_numpy(x_host).to(dev)
    out = torch.empty((B, F * K), dtype=torch.float32, device=dev)
    ws = torch.empty(rocket.rocket_workspace_bytes(h, B, mask), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    with_grad = cfg_id == 3
    if with_grad:
        # forward (max + softPPV), then the backward pass from a seeded N(0,1) upstream gradient
        view = rocket.rocket_kernels_view_get(h)
        gout = torch.from_numpy(synth.make_upstream_grad(cfg_id, B, F * K)).to(dev)
        gw = torch.empty(len(view["weights"]), dtype=torch.float32, device=dev)
        gb = torch.empty(K, dtype=torch.float32, device=dev)
        ws = torch.empty(rocket.rocket_workspace_bytes(h, B, mask, True), dtype=torch.uint8, device=dev)

    def backward():
        rocket.rocket_soft_ppv_backward(h, x, mask, gout, args.lam, -3.0, True, grad_w=gw, grad_b=gb,
                                        workspace=ws, stream=stream)

    transform = rocket.rocket_transform_u8 if from_u8 else rocket.rocket_transform

    train = args.workload.endswith("-train")
    if train:
        # a fixed random linear head and roughness-like targets; a small learning rate, re-centred rows
        rng = np.random.Generator(np.random.PCG64(synth.seed_g(cfg_id)))
        coef = torch.from_numpy(rng.standard_normal(F * K) * 0.01).to(dev)
        icpt = torch.tensor([1.2], dtype=torch.float64, device=dev)
        targets = torch.from_numpy((0.6 + 1.2 * rng.random(B)).astype(np.float32)).to(dev)
        train_ws = torch.empty(rocket.rocket_train_workspace_bytes(h, B, mask), dtype=torch.uint8, device=dev)

    def step():
        if train:
            rocket.rocket_train_step(h, x, mask, coef, icpt, targets, 1e-3, args.lam, -3.0, True,
                                     workspace=train_ws, stream=stream)
            return
        transform(h, x, mask, args.lam, -3.0, out=out, workspace=ws, stream=stream)
        if with_grad:
            backward()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    run = step
    if args.graph:
        # the parameters are on the device after the warm-up: a step only launches kernels
        side = torch.cuda.Stream()
        stream = side
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        run = graph.replay
        run()
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream()

    rocket.rocket_profile_enable(h, not with_grad and not args.graph)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    if args.graph and not with_grad:
        # kernel time for the roofline figure: eager launches after the timed region
        rocket.rocket_profile_enable(h, True)
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
    if with_grad:
        # the dominant kernel of this workload is the backward one: time it alone, after the timed region
        rocket.rocket_profile_enable(h, True)
        for _ in range(args.steps):
            backward()
        torch.cuda.synchronize()
    launches, kernel_ms = rocket.rocket_profile_read(h)
    rocket.rocket_profile_enable(h, False)
    assert launches == args.steps

    ms_per_step = 1e3 * elapsed / args.steps
    value = B * args.steps / elapsed
    kernel_ms_avg = kernel_ms / launches
    # conv FMAs only, as the method defines them; the backward kernel recomputes the conv
    # and does as many multiply-adds again for the weight gradient
    flops_per_launch = 2.0 * fma_per_series * B * (2.0 if with_grad else 1.0)
    achieved = flops_per_launch / (kernel_ms_avg * 1e-3) / 1e12
    # pooling, counted as the method defines it: max 1, PPV 2 (compare, add), softPPV 6
    # (fma = 2, exp, add, rcp, add) flop per position; the backward kernel's sigmoid derivative 10
    pool_per_pos = (1 if mask & 1 else 0) + (2 if mask & 2 else 0) + (6 if mask & 4 else 0)
    pool_flops = outputs_per_series * B * (10.0 if with_grad else pool_per_pos)
    achieved_with_pooling = (flops_per_launch + pool_flops) / (kernel_ms_avg * 1e-3) / 1e12
    plain_fma_ceiling = None if args.lean else rocket.rocket_calibrate_fma()
    traffic = MEASURED_TRAFFIC.get((args.workload, B, mask))

    line = {
        "metric": ("examples/sec (20ch x 50k, K=10k) and % of FP32 vector peak" if cfg_id == 2 else
                   "examples/sec, whole training step through softPPV (20ch x 50k, K=10k)" if train else
                   "examples/sec, forward + softPPV backward (20ch x 50k, K=10k)" if cfg_id == 3 else
                   "series/sec" if cfg_id in (0, 1) else "examples/sec"),
        "value": value, "unit": "examples/s" if cfg_id != 1 and cfg_id != 0 else "series/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "launch": "hip-graph replay" if args.graph else "eager", "B": B, "C": C, "L": L, "K": K, "features": mask,
                   "lambda": args.lam, "shift": -3.0, "seed_x": synth.seed_x(cfg_id), "seed_k": synth.seed_k(cfg_id)},
        "roofline": {
            "bound": "alu", "achieved": achieved, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / FP32_VECTOR_PEAK_TFLOPS, "traffic": traffic,
            "kernel": "rk_backward" if with_grad else "rk_forward", "kernel_ms": kernel_ms_avg,
            "flop_per_launch": flops_per_launch, "fma_per_example": fma_per_series,
            "pooled_positions_per_example": outputs_per_series,
            "achieved_with_pooling": achieved_with_pooling,
            "plain_fma_measured": plain_fma_ceiling,
            "frac_of_plain_fma_measured": achieved / plain_fma_ceiling if plain_fma_ceiling else None,
            "note": "peak is the data-sheet figure, which assumes packed FP32; this build issues plain v_fma_f32, "
                    "whose rate measured in this run by a kernel of nothing but FMAs is plain_fma_measured",
        },
        "percent_of_fp32_vector_peak": 100.0 * achieved / FP32_VECTOR_PEAK_TFLOPS,
    }

    if traffic:
        line["roofline"]["hbm_GBps"] = traffic / (kernel_ms_avg * 1e-3) / 1e9
    if cfg_id == 2 and not from_u8 and not args.lean:
        # the univariate workloads of the classic ROCKET setting, in series/s, in the same run
        line["series_per_s"] = [quick_rate(rocket, synth, torch, i, args.lam) for i in (1, 0)]

    if cfg_id == 2 and not train and not args.lean:
        # once with the host-to-device copy of the batch inside the timed region (pinned source)
        x_pin = torch.from_numpy(x_host).pin_memory()
        for _ in range(2):
            x.copy_(x_pin, non_blocking=True)
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            x.copy_(x_pin, non_blocking=True)
            step()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        line["with_h2d_copy"] = {"value": B / dt, "unit": "examples/s", "ms_per_step": 1e3 * dt,
                                 "bytes": int(x_pin.numel() * x_pin.element_size())}
        # and with the copy of the next batch on a second stream while this one is transformed
        # (two input buffers, two workspaces, two outputs; events order copy -> transform -> next copy)
        copy_stream, work_stream = torch.cuda.Stream(), torch.cuda.Stream()
        xs = [x, torch.empty_like(x)]
        wss = [ws, torch.empty_like(ws)]
        outs = [out, torch.empty_like(out)]
        copied = [torch.cuda.Event(), torch.cuda.Event()]
        used = [torch.cuda.Event(), torch.cuda.Event()]
        torch.cuda.synchronize()

        def pipelined(n):
            for i in range(n):
                s = i & 1
                with torch.cuda.stream(copy_stream):
                    if i >= 2:
                        copy_stream.wait_event(used[s])          # buffer s is free again
                    xs[s].copy_(x_pin, non_blocking=True)
                    copied[s].record(copy_stream)
                with torch.cuda.stream(work_stream):
                    work_stream.wait_event(copied[s])
                    transform(h, xs[s], mask, args.lam, -3.0, out=outs[s], workspace=wss[s], stream=work_stream)
                    used[s].record(work_stream)
            torch.cuda.synchronize()

        pipelined(2)
        t0 = time.perf_counter()
        pipelined(args.steps)
        dt = (time.perf_counter() - t0) / args.steps
        line["with_h2d_copy"]["overlapped"] = {"value": B / dt, "unit": "examples/s", "ms_per_step": 1e3 * dt}

    if not args.no_cpu_baseline and not with_grad:
        kr = rocket.rocket_kernels_view_get(h)
        n_ex = args.cpu_examples
        if n_ex is None:
            # aim at 10-30 s of oracle time: the oracle does roughly 1.4 GFMA/s per thread
            import oracle
            rate = 1.4e9 * oracle.num_threads()
            n_ex = int(max(1, min(B, round(15.0 * rate / fma_per_series))))
        line["cpu_baseline"] = cpu_baseline(cfg_id, x_host, kr, mask, args.lam, n_ex)
        # the same oracle on one core, on a sample that takes about 10 s
        import oracle
        threads = oracle.num_threads()
        oracle.set_threads(1)
        one = cpu_baseline(cfg_id, x_host, kr, mask, args.lam, int(max(1, round(10.0 * 1.4e9 / fma_per_series))))
        oracle.set_threads(threads)
        line["cpu_baseline"]["one_core"] = {"value": one["value"], "unit": one["unit"], "sample": one["sample"]}

    print(json.dumps(line))
    h.free()


if __name__ == "__main__":
    main()
