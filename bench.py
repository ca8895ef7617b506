#!/usr/bin/env python3
"""Benchmark of the ROCKET transform hot path on one MI355X.

A step is one rocket_transform call (zero-pad copy + conv/pooling kernel + feature kernel) on
the paper's headline workload: a batch of 64 examples of 20 channels x 50,000
timesteps through K = 10,000 random kernels, two pooled features per kernel
(max + PPV).  Inputs are synthetic (seeded AR(1) channels, z-normalised) and
resident in HBM before the timed region.  Prints one JSON line; the default run also
carries the other workloads (univariate series/s, forward + backward, long series) as
sub-records, each timed the same way.
"""
import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP32_VECTOR_PEAK_TFLOPS = 157.3   # MI355X datasheet, packed FP32 on the vector ALUs
# Memory-side bytes per launch of the dominant kernel.  These are not measured by this program: they come
# from `rocprofv3 --pmc` runs of this same command whose summaries are under profiles/ (the file and the
# commit it was taken on are repeated in the JSON line).  `l2_fill` = FETCH_SIZE + WRITE_SIZE (traffic between
# L2 and the fabric: Infinity Cache hits and DRAM together), each scaled by what the counter reads for the
# padding copy of known size; `dram` = TCC_EA0_RDREQ_DRAM (128-byte) + TCC_EA0_WRREQ_DRAM (64-byte) requests: the
# requests that the L2's fabric interface labels DRAM -- all of them here; the Infinity Cache sits on the memory
# side of that interface and is not told apart from HBM by any counter of the compute dies.
# (workload, batch, feature mask) -> figures; other shapes report null.
MEASURED_TRAFFIC = {
    # 9,547,000 KiB x 1.968 fetched + 56,700 KiB written; 1.527e8 read requests x 128 B + 1.05e6 write requests x 64 B
    ("multivariate-20x50k", 64, 3): {
        "l2_fill_bytes": 19298000000, "dram_bytes": 19613000000,
        "source": "profiles/rk_forward_multivariate-20x50k.md", "commit": "e304e0a"},
    # 16,320,000 KiB x 1.968 fetched + 153,600 KiB written; 2.61e8 read requests x 128 B + 2.94e6 write requests x 64 B
    ("multivariate-20x50k-grad", 60, 5): {
        "l2_fill_bytes": 33046000000, "dram_bytes": 33596000000,
        "source": "profiles/rk_backward_multivariate-20x50k-grad.md", "commit": "e304e0a"},
}

WORKLOADS = {
    # name: synth config
    "multivariate-20x50k": 2,
    "multivariate-20x50k-grad": 3,
    "multivariate-20x50k-train": 3,   # whole training step: transform, linear head, loss gradient, backward, update
    "multivariate-20x50k-u8": 2,      # the same batch as raw 8-bit samples, normalised inside the call
    "univariate-standard": 1,
    "univariate-tiny": 0,
    "long-20x200k": 4,
    "ridge-677x20000": None,          # the regressor at the paper's sizes: one step = one fit + one 64-row predict
    "minirocket-20x50k": None,        # MINIROCKET-style variant on the same batch: 119 groups x 84 kernels, PPV only
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
                    help="only the timed region: no extra workloads, no H2D-inclusive run, no unit calibration "
                         "(for profiler runs, so that the trace holds the timed launches only)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time its replays (for launch-bound small workloads)")
    ap.add_argument("--cpu-examples", type=int, default=None, help="examples in the oracle's timed sample")
    return ap.parse_args()


def cpu_baseline(x_host, kr, lam, n_examples):
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


def time_steps(torch, run, steps):
    """Runs `steps` steps between two device synchronisations.  Returns the wall-clock seconds of the whole
    region (what the headline rate is computed from) and the per-step milliseconds from events recorded on the
    current stream around every step (median and minimum are taken from those)."""
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        run()
        marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
    return elapsed, per_step


class Workload:
    """One workload set up on the device: kernels, resident input, outputs, workspace, and its step."""

    def __init__(self, torch, rocket, synth, name, lam, batch=None, features=None):
        self.torch, self.rocket, self.name, self.lam = torch, rocket, name, lam
        self.cfg_id = WORKLOADS[name]
        cfg = synth.CONFIGS[self.cfg_id]
        self.B = cfg["B"] if batch is None else batch
        self.mask = cfg["features"] if features is None else features
        self.K, self.C, self.L = cfg["K"], cfg["C"], cfg["L"]
        self.from_u8 = name.endswith("-u8")
        self.train = name.endswith("-train")
        self.with_grad = self.cfg_id == 3
        self.x_host = synth.make_input_u8(self.cfg_id, B=self.B) if self.from_u8 else synth.make_input(self.cfg_id, B=self.B)
        self.h = rocket.rocket_make_kernels(synth.seed_k(self.cfg_id), self.K, self.C, self.L)
        self.fma_per_series, self.outputs_per_series = rocket.rocket_work_per_series(self.h)
        self.F = rocket.rocket_num_features(self.mask)
        dev = torch.device("cuda:0")
        self.x = torch.from_numpy(self.x_host).to(dev)
        self.out = torch.empty((self.B, self.F * self.K), dtype=torch.float32, device=dev)
        self.ws = torch.empty(rocket.rocket_workspace_bytes(self.h, self.B, self.mask, self.with_grad),
                              dtype=torch.uint8, device=dev)
        self.stream = torch.cuda.current_stream()
        if self.with_grad:
            # forward (max + softPPV), then the backward pass from a seeded N(0,1) upstream gradient
            self.gout = torch.from_numpy(synth.make_upstream_grad(self.cfg_id, self.B, self.F * self.K)).to(dev)
            self.gw = torch.empty(self.h.total_weights, dtype=torch.float32, device=dev)
            self.gb = torch.empty(self.K, dtype=torch.float32, device=dev)
        if self.train:
            # a fixed random linear head and roughness-like targets; a small learning rate, re-centred rows
            rng = np.random.Generator(np.random.PCG64(synth.seed_g(self.cfg_id)))
            self.coef = torch.from_numpy(rng.standard_normal(self.F * self.K) * 0.01).to(dev)
            self.icpt = torch.tensor([1.2], dtype=torch.float64, device=dev)
            self.targets = torch.from_numpy((0.6 + 1.2 * rng.random(self.B)).astype(np.float32)).to(dev)
            self.train_ws = torch.empty(rocket.rocket_train_workspace_bytes(self.h, self.B, self.mask),
                                        dtype=torch.uint8, device=dev)
        self.transform = rocket.rocket_transform_u8 if self.from_u8 else rocket.rocket_transform

    def backward(self, include_max=True):
        self.rocket.rocket_soft_ppv_backward(self.h, self.x, self.mask, self.gout, self.lam, -3.0, include_max,
                                             grad_w=self.gw, grad_b=self.gb, workspace=self.ws, stream=self.stream)

    def step(self):
        if self.train:
            self.rocket.rocket_train_step(self.h, self.x, self.mask, self.coef, self.icpt, self.targets, 1e-3,
                                          self.lam, -3.0, True, workspace=self.train_ws, stream=self.stream)
            return
        self.transform(self.h, self.x, self.mask, self.lam, -3.0, out=self.out, workspace=self.ws, stream=self.stream)
        if self.with_grad:
            self.backward()

    def kernel_time(self, steps, include_max=True):
        """Average duration (ms) of the dominant kernel over `steps` launches, from the HIP events the library
        records on the call's stream around that kernel (the backward kernel for the gradient workloads)."""
        self.rocket.rocket_profile_enable(self.h, True)
        for _ in range(steps):
            if self.with_grad:
                self.backward(include_max)
            else:
                self.transform(self.h, self.x, self.mask, self.lam, -3.0, out=self.out, workspace=self.ws,
                               stream=self.stream)
        self.torch.cuda.synchronize()
        launches, ms = self.rocket.rocket_profile_read(self.h)
        self.rocket.rocket_profile_enable(self.h, False)
        assert launches == steps
        return ms / launches

    def roofline(self, kernel_ms):
        # conv FMAs only, as the method defines them; the backward kernel recomputes the conv
        # and does as many multiply-adds again for the weight gradient
        flops = 2.0 * self.fma_per_series * self.B * (2.0 if self.with_grad else 1.0)
        achieved = flops / (kernel_ms * 1e-3) / 1e12
        # pooling, counted as the method defines it: max 1, PPV 2 (compare, add), softPPV 6
        # (fma = 2, exp, add, rcp, add) flop per position; the backward kernel's sigmoid derivative 10
        pool_per_pos = (1 if self.mask & 1 else 0) + (2 if self.mask & 2 else 0) + (6 if self.mask & 4 else 0)
        pool_flops = self.outputs_per_series * self.B * (10.0 if self.with_grad else pool_per_pos)
        traffic = MEASURED_TRAFFIC.get((self.name, self.B, self.mask))
        r = {
            "bound": "alu", "achieved": achieved, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / FP32_VECTOR_PEAK_TFLOPS,
            "traffic": traffic["l2_fill_bytes"] if traffic else None,
            "kernel": "rk_backward" if self.with_grad else ("rk_forward<64>" if self.L <= 8192 else "rk_forward<256>"),
            "kernel_ms": kernel_ms, "flop_per_launch": flops, "fma_per_example": self.fma_per_series,
            "pooled_positions_per_example": self.outputs_per_series,
            "achieved_with_pooling": (flops + pool_flops) / (kernel_ms * 1e-3) / 1e12,
        }
        if traffic:
            # traffic is the figure of an earlier profiler run, not of this run (see MEASURED_TRAFFIC)
            r["traffic_kind"] = "L2 fill (Infinity Cache + DRAM), from " + traffic["source"] + " @ " + traffic["commit"]
            r["l2_fill_GBps"] = traffic["l2_fill_bytes"] / (kernel_ms * 1e-3) / 1e9
            r["dram_labelled_bytes"] = traffic["dram_bytes"]      # Infinity Cache hits included (see MEASURED_TRAFFIC)
            r["dram_labelled_GBps"] = traffic["dram_bytes"] / (kernel_ms * 1e-3) / 1e9 if traffic["dram_bytes"] else None
        return r

    def free(self):
        self.h.free()


def sub_record(torch, rocket, synth, name, lam, min_steps=10, min_seconds=2.0, max_steps=400):
    """A secondary workload timed like the main one: at least `min_steps` steps and `min_seconds` seconds
    (short steps are repeated up to `max_steps` times), mean / median / minimum, and its own roofline."""
    w = Workload(torch, rocket, synth, name, lam)
    for _ in range(3):
        w.step()
    torch.cuda.synchronize()
    elapsed, per_step = time_steps(torch, w.step, min_steps)
    more = int(min(max_steps, np.ceil(min_seconds / (elapsed / min_steps)))) - min_steps
    if more > 0:
        e2, p2 = time_steps(torch, w.step, more)
        elapsed, per_step = elapsed + e2, per_step + p2
    steps = len(per_step)
    kernel_ms = w.kernel_time(min(steps, 10))
    unit = "series/s" if w.cfg_id in (0, 1) else "examples/s"
    rec = {"workload": name, "B": w.B, "C": w.C, "L": w.L, "K": w.K, "features": w.mask,
           "what": "forward + softPPV backward (max sub-gradient included)" if w.with_grad else "forward",
           "value": w.B * steps / elapsed, "unit": unit, "steps": steps, "ms_per_step": 1e3 * elapsed / steps,
           "ms_per_step_median": statistics.median(per_step), "ms_per_step_min": min(per_step),
           "roofline": w.roofline(kernel_ms)}
    if w.with_grad:
        # the same backward kernel without the max plane's sub-gradient (no arg-max bookkeeping)
        rec["backward_kernel_ms_without_max"] = w.kernel_time(5, include_max=False)
    w.free()
    return rec


def ridge_record(torch, rocket, steps, warmup):
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

    for _ in range(warmup):
        step()
    elapsed, per_step = time_steps(torch, step, steps)
    dt = elapsed / steps
    return {"workload": "ridge-677x20000", "n": n, "p": p, "predict_rows": m, "alpha": 1.0,
            "what": "one fit (fp64, dual form, Gram matrix on the fp64 matrix cores) and one 64-row predict",
            "value": 1.0 / dt, "unit": "fits/s", "steps": steps, "ms_per_step": 1e3 * dt,
            "ms_per_step_median": statistics.median(per_step), "ms_per_step_min": min(per_step)}


def ridge_bench(args, torch, rocket):
    rec = ridge_record(torch, rocket, args.steps, args.warmup)
    print(json.dumps({
        "metric": "ridge fits/sec (677 x 20,000, fp64, dual form) with a 64-row predict each",
        "value": rec["value"], "unit": "fits/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rec["ms_per_step"], "ms_per_step_median": rec["ms_per_step_median"],
        "ms_per_step_min": rec["ms_per_step_min"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": args.workload, "n": rec["n"], "p": rec["p"], "predict_rows": rec["predict_rows"], "alpha": 1.0},
    }))


MINIROCKET_GROUPS = 119          # 9,996 kernels, the nearest multiple of 84 below the paper's 10,000
# vector operations per (group, output position) as the method defines them: the sum of the nine taps (8 adds),
# nine U_j = 9 T_j - sum (multiply-add: 2 flop each), 36 pair sums, 84 third additions, 84 comparisons; plus
# n_ch - 1 additions for the channel sum of the position's sample
MINIROCKET_FLOP_PER_POSITION = 8 + 18 + 36 + 84 + 84


def minirocket_record(torch, rocket, synth, steps, warmup, lam, cpu_seconds=12.0, extend=True):
    """The MINIROCKET-style variant on the batch of the main workload: biases fitted on the first 8 series, then a
    step is one rocket_minirocket_transform of all 64.  Also times rocket_transform's PPV plane on the same handle
    (the general multiply-add kernel on the same kernels) and the oracle on a sample."""
    cfg = synth.CONFIGS[2]
    B, C, L = cfg["B"], cfg["C"], cfg["L"]
    x_host = synth.make_input(2, B=B)
    x = torch.from_numpy(x_host).cuda()
    h = rocket.rocket_minirocket_kernels(synth.seed_k(2), MINIROCKET_GROUPS, C, L)
    rocket.rocket_minirocket_fit_bias(h, x[:8], synth.seed_k(2) + 1)
    torch.cuda.synchronize()
    v = rocket.rocket_kernels_view_get(h)
    K = len(v["length"])
    n_out = (L + 2 * v["padding"].astype(np.int64) - 8 * v["dilation"].astype(np.int64))[::84]
    n_ch = v["n_ch"].astype(np.int64)[::84]
    flop = float(np.sum(n_out * (MINIROCKET_FLOP_PER_POSITION + n_ch - 1))) * B
    out = torch.empty((B, K), dtype=torch.float32, device="cuda")
    ws = torch.empty(rocket.rocket_minirocket_workspace_bytes(h, B), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        rocket.rocket_minirocket_transform(h, x, out=out, workspace=ws, stream=stream)

    for _ in range(warmup):
        step()
    elapsed, per_step = time_steps(torch, step, steps)
    more = int(min(400, np.ceil(2.0 / (elapsed / steps)))) - steps if extend else 0
    if more > 0:
        e2, p2 = time_steps(torch, step, more)
        elapsed, per_step = elapsed + e2, per_step + p2
    steps = len(per_step)
    rocket.rocket_profile_enable(h, True)
    for _ in range(10):
        step()
    torch.cuda.synchronize()
    launches, ms = rocket.rocket_profile_read(h)
    rocket.rocket_profile_enable(h, False)
    kernel_ms = ms / launches
    achieved = flop / (kernel_ms * 1e-3) / 1e12
    rec = {
        "workload": "minirocket-20x50k", "B": B, "C": C, "L": L, "K": K, "groups": MINIROCKET_GROUPS, "features": 2,
        "what": "PPV of 84 predetermined two-valued kernels per group, biases fitted to data (group kernel)",
        "value": B * steps / elapsed, "unit": "examples/s", "steps": steps, "ms_per_step": 1e3 * elapsed / steps,
        "ms_per_step_median": statistics.median(per_step), "ms_per_step_min": min(per_step),
        "roofline": {
            "bound": "alu", "achieved": achieved, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / FP32_VECTOR_PEAK_TFLOPS,
            # 599,750 KiB x 1.968 fetched + 31,602 KiB written per launch (L2 fill: Infinity Cache + DRAM), from
            # profiles/rk_mr_forward_minirocket-20x50k.md; not measured by this run
            "traffic": 1240980000 if (B, MINIROCKET_GROUPS) == (64, 119) else None,
            "traffic_kind": "L2 fill (Infinity Cache + DRAM), from profiles/rk_mr_forward_minirocket-20x50k.md",
            "kernel": "rk_mr_forward",
            "kernel_ms": kernel_ms, "flop_per_launch": flop,
            "note": "additions and comparisons count one flop and run one per lane and clock: their ceiling is a "
                    "quarter of the packed-FMA peak (39.3 TFLOP/s)", "plain_op_ceiling": FP32_VECTOR_PEAK_TFLOPS / 4.0,
            "frac_of_plain_op_ceiling": achieved / (FP32_VECTOR_PEAK_TFLOPS / 4.0),
        },
    }
    # the same features from the general kernel (9 n_ch multiply-adds per output)
    fma, _ = rocket.rocket_work_per_series(h)
    ws2 = torch.empty(rocket.rocket_workspace_bytes(h, B, 2, False), dtype=torch.uint8, device="cuda")
    out2 = torch.empty((B, K), dtype=torch.float32, device="cuda")

    def general():
        rocket.rocket_transform(h, x, 2, lam, -3.0, out=out2, workspace=ws2, stream=stream)

    general()
    e3, p3 = time_steps(torch, general, 5)
    rec["general_kernel"] = {"value": B * 5 / e3, "unit": "examples/s", "ms_per_step": 1e3 * e3 / 5,
                             "conv_TFLOPs": 2.0 * fma * B / (e3 / 5) / 1e12,
                             "speedup_of_group_kernel": (e3 / 5) / (elapsed / steps)}
    if cpu_seconds > 0:
        import oracle
        kr = oracle.minirocket_kernels(synth.seed_k(2), MINIROCKET_GROUPS, C, L)
        kr["bias"] = v["bias"]
        n_ex = int(max(1, min(B, round(cpu_seconds * 1.4e9 * oracle.num_threads() / fma))))
        t0 = time.perf_counter()
        oracle.minirocket_transform(x_host[:n_ex], kr)
        dt = time.perf_counter() - t0
        rec["cpu_baseline"] = {"value": n_ex / dt, "unit": "examples/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "%d example(s) x all %d kernels, %.1f s, fp64" % (n_ex, K, dt)}
    h.free()
    return rec


def minirocket_bench(args, torch, rocket, synth):
    rec = minirocket_record(torch, rocket, synth, args.steps, args.warmup, args.lam,
                            0.0 if args.no_cpu_baseline else 12.0, extend=False)
    line = {
        "metric": "examples/sec, MINIROCKET-style PPV features (20ch x 50k, 119 groups x 84 kernels)",
        "value": rec["value"], "unit": "examples/s", "n_gpus": 1, "steps": rec["steps"], "warmup": args.warmup,
        "ms_per_step": rec["ms_per_step"], "ms_per_step_median": rec["ms_per_step_median"],
        "ms_per_step_min": rec["ms_per_step_min"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "B": rec["B"], "C": rec["C"], "L": rec["L"], "K": rec["K"],
                   "groups": rec["groups"], "features": 2},
        "roofline": rec["roofline"], "general_kernel": rec["general_kernel"],
    }
    if "cpu_baseline" in rec:
        line["cpu_baseline"] = rec["cpu_baseline"]
    print(json.dumps(line))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    from paper_2301_08527_amd import rocket

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the transform has no CPU path", file=sys.stderr)
        sys.exit(1)

    if args.workload == "ridge-677x20000":
        ridge_bench(args, torch, rocket)
        return
    if args.workload == "minirocket-20x50k":
        minirocket_bench(args, torch, rocket, synth)
        return
    w = Workload(torch, rocket, synth, args.workload, args.lam, args.batch, args.features)
    cfg_id, B, mask, K, C, L = w.cfg_id, w.B, w.mask, w.K, w.C, w.L

    for _ in range(args.warmup):
        w.step()
    torch.cuda.synchronize()

    run = w.step
    if args.graph:
        # the parameters are on the device after the warm-up: a step only launches kernels
        side = torch.cuda.Stream()
        w.stream = side
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            w.step()
        run = graph.replay
        run()
        torch.cuda.synchronize()
        w.stream = torch.cuda.current_stream()

    elapsed, per_step = time_steps(torch, run, args.steps)
    # duration of the dominant kernel: eager launches after the timed region, HIP events on their stream
    kernel_ms_avg = w.kernel_time(args.steps)

    ms_per_step = 1e3 * elapsed / args.steps
    value = B * args.steps / elapsed
    roofline = w.roofline(kernel_ms_avg)
    if not args.lean:
        plain = rocket.rocket_calibrate_fma()
        roofline["plain_fma_measured"] = plain
        roofline["frac_of_plain_fma_measured"] = roofline["achieved"] / plain
        roofline["units_measured"] = rocket.rocket_calibrate_units()
    roofline["note"] = ("peak is the data-sheet figure, which assumes packed FP32; this build issues plain v_fma_f32, "
                        "whose rate measured in this run by a kernel of nothing but FMAs is plain_fma_measured; "
                        "units_measured are whole-device rates of the load, LDS and matrix units from micro-kernels")

    line = {
        "metric": ("examples/sec (20ch x 50k, K=10k) and % of FP32 vector peak" if cfg_id == 2 else
                   "examples/sec, whole training step through softPPV (20ch x 50k, K=10k)" if w.train else
                   "examples/sec, forward + softPPV backward (20ch x 50k, K=10k)" if cfg_id == 3 else
                   "series/sec" if cfg_id in (0, 1) else "examples/sec"),
        "value": value, "unit": "examples/s" if cfg_id != 1 and cfg_id != 0 else "series/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": statistics.median(per_step), "ms_per_step_min": min(per_step),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "launch": "hip-graph replay" if args.graph else "eager", "B": B, "C": C,
                   "L": L, "K": K, "features": mask, "lambda": args.lam, "shift": -3.0,
                   "seed_x": synth.seed_x(cfg_id), "seed_k": synth.seed_k(cfg_id)},
        "roofline": roofline,
        "percent_of_fp32_vector_peak": 100.0 * roofline["achieved"] / FP32_VECTOR_PEAK_TFLOPS,
    }

    main_run = cfg_id == 2 and not w.from_u8 and not args.lean and args.batch is None and args.features is None
    if main_run:
        # the other workloads, each timed for at least 10 steps and 2 seconds: the univariate ones of the classic
        # ROCKET setting in series/s, the forward + backward step and the long-series stress in examples/s
        line["series_per_s"] = [sub_record(torch, rocket, synth, n, args.lam) for n in ("univariate-standard", "univariate-tiny")]
        line["fwd_bwd"] = sub_record(torch, rocket, synth, "multivariate-20x50k-grad", args.lam)
        line["long"] = sub_record(torch, rocket, synth, "long-20x200k", args.lam)
        line["minirocket"] = minirocket_record(torch, rocket, synth, 10, 2, args.lam, cpu_seconds=0.0)
        line["ridge"] = ridge_record(torch, rocket, 200, 5)

    if cfg_id == 2 and not w.train and not args.lean:
        # once with the host-to-device copy of the batch inside the timed region (pinned source)
        x, ws, out = w.x, w.ws, w.out
        x_pin = torch.from_numpy(w.x_host).pin_memory()
        for _ in range(2):
            x.copy_(x_pin, non_blocking=True)
            w.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            x.copy_(x_pin, non_blocking=True)
            w.step()
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
                    w.transform(w.h, xs[s], mask, args.lam, -3.0, out=outs[s], workspace=wss[s], stream=work_stream)
                    used[s].record(work_stream)
            torch.cuda.synchronize()

        pipelined(2)
        t0 = time.perf_counter()
        pipelined(args.steps)
        dt = (time.perf_counter() - t0) / args.steps
        line["with_h2d_copy"]["overlapped"] = {"value": B / dt, "unit": "examples/s", "ms_per_step": 1e3 * dt}

    if not args.no_cpu_baseline and not w.with_grad:
        import oracle
        # the oracle computes with kernels from its own sampler (bit-identical to the library's, as the tests check)
        kr = oracle.sample_kernels(synth.seed_k(cfg_id), K, C, L)
        n_ex = args.cpu_examples
        if n_ex is None:
            # aim at 10-30 s of oracle time: the oracle does roughly 1.4 GFMA/s per thread
            rate = 1.4e9 * oracle.num_threads()
            n_ex = int(max(1, min(B, round(15.0 * rate / w.fma_per_series))))
        line["cpu_baseline"] = cpu_baseline(w.x_host, kr, args.lam, n_ex)
        # the same oracle on one core, on a sample that takes about 10 s
        threads = oracle.num_threads()
        oracle.set_threads(1)
        one = cpu_baseline(w.x_host, kr, args.lam, int(max(1, round(10.0 * 1.4e9 / w.fma_per_series))))
        oracle.set_threads(threads)
        line["cpu_baseline"]["one_core"] = {"value": one["value"], "unit": one["unit"], "sample": one["sample"]}

    print(json.dumps(line))
    w.free()


if __name__ == "__main__":
    main()
