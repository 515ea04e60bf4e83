#!/usr/bin/env python3
"""Benchmark of the Tune-mode ConvBN block (fold -> conv -> dgrad/wgrad -> fold-back) on one
MI355X, synthetic ResNet-50 shapes.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2]

One "step" = one forward + backward pass of the Tune-mode block over one batch for every
shape of the workload (default: the two ResNet-50 3x3 shapes, 64->64 @56x56 and
512->512 @7x7, bf16 with fp32 accumulation).  Inputs are resident in HBM before the timed
region; the step rotates through a pool of independent buffer sets larger than the last-
level cache so that it does not measure cache-resident reruns.

Prints ONE JSON line: whole-job TFLOP/s (useful conv FLOPs only: 3 x 2 M K Cout per block),
the Eval-mode time and saved-activation bytes for comparison, a roofline object for the
dominant kernel and the CPU oracle timed on a bounded sample as a baseline.
"""
import argparse
import json
import os
import sys
import time
from dataclasses import replace

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E peak

WORKLOADS = {
    "c1": ["c1"], "c2": ["c2a", "c2b"], "c2a": ["c2a"], "c2b": ["c2b"],
    "c3": ["c3a", "c3b"], "c3a": ["c3a"], "c3b": ["c3b"],
    "all": ["c1", "c2a", "c2b", "c3a", "c3b"],
}

# HBM bytes per launch of the dominant kernels, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of this script (summaries under profiles/); None where not measured.
MEASURED_TRAFFIC_BYTES = {}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=sorted(WORKLOADS))
    ap.add_argument("--pool-mb", type=int, default=768,
                    help="minimum total size of the rotating buffer pool per shape")
    ap.add_argument("--kernel-reps", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-eval", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    return ap.parse_args()


def tensor_bytes(run):
    n = 0
    for v in vars(run).values():
        if hasattr(v, "element_size") and hasattr(v, "numel"):
            n += v.numel() * v.element_size()
    return n


def make_pool(inp, mode, pool_mb):
    from paper_2305_11624_amd.runner import BlockRun
    first = BlockRun(inp, mode=mode)
    per = max(1, tensor_bytes(first))
    count = max(2, min(64, -(-pool_mb * (1 << 20) // per)))
    return [first] + [BlockRun(inp, mode=mode) for _ in range(count - 1)]


def time_steps(pools, steps, warmup):
    import torch
    it = 0

    def one_step():
        nonlocal it
        for pool in pools:
            pool[it % len(pool)].step()
        it += 1

    for _ in range(warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3


def kernel_times(pool, reps):
    """Average duration (ms) of each step's kernel for one shape: `reps` back-to-back
    launches through the per-step entry points, bracketed by HIP events recorded on the
    stream the kernels run on (torch's current stream)."""
    import torch
    from paper_2305_11624_amd import binding as B
    r0 = pool[0]
    d = r0.desc
    dev = r0.x.device
    s = r0.shape
    P = s.Cout * s.K
    scratch = []
    for r in pool:
        scratch.append(dict(
            w_fprop=torch.empty(P, dtype=r.dt, device=dev),
            w_t=torch.empty(P, dtype=r.dt, device=dev),
            bfold=torch.empty(s.Cout, dtype=torch.float32, device=dev),
            ws_f=torch.empty(max(16, B.convbn_conv_workspace_bytes(d, B.PASS_FWD)), dtype=torch.uint8, device=dev),
            ws_d=torch.empty(max(16, B.convbn_conv_workspace_bytes(d, B.PASS_BWD)), dtype=torch.uint8, device=dev),
            dw_part=torch.empty(B.convbn_wgrad_parts(d) * P, dtype=torch.float32, device=dev),
            r_part=torch.empty(B.convbn_rsum_parts(d) * s.Cout, dtype=torch.float32, device=dev)))
    calls = {
        "fold": lambda r, w: B.convbn_fold(d, r.W, r.b, r.gamma, r.beta, r.mean, r.var,
                                            w["w_fprop"], w["w_t"], w["bfold"]),
        "fprop": lambda r, w: B.convbn_conv_fprop(d, r.x, w["w_fprop"], w["bfold"], r.z, w["ws_f"]),
        "dgrad": lambda r, w: B.convbn_conv_dgrad(d, r.dz, w["w_t"], r.dx, w["ws_d"]),
        "wgrad": lambda r, w: B.convbn_conv_wgrad(d, r.x, r.dz, w["dw_part"], None, w["ws_d"]),
        "wgrad+rsum": lambda r, w: B.convbn_conv_wgrad(d, r.x, r.dz, w["dw_part"], w["r_part"], w["ws_d"]),
        "fold_back": lambda r, w: B.convbn_fold_back(d, w["dw_part"], w["r_part"], r.W, r.b,
                                                     r.gamma, r.mean, r.var, r.dW, r.db,
                                                     r.dgamma, r.dbeta),
    }
    out = {}
    for name, fn in calls.items():
        for i in range(min(3, len(pool))):
            fn(pool[i], scratch[i])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            fn(pool[i % len(pool)], scratch[i % len(pool)])
        e1.record()
        torch.cuda.synchronize()
        out[name] = e0.elapsed_time(e1) / reps
    return out


def cpu_baseline(shapes, seconds):
    """The CPU oracle (fp64 direct loops, OpenMP) on a bounded sample: a slice of the batch
    of each shape sized so the whole leg takes roughly `seconds`."""
    import numpy as np
    import oracle
    from paper_2305_11624_amd import synth
    cores = oracle.num_threads()
    assumed = 0.6e9 * cores             # rough direct-loop rate, FLOP/s, to size the sample
    flops, secs, desc = 0.0, 0.0, []
    for name in shapes:
        s = synth.CONFIGS[name]
        per_image = s.step_flop / s.N
        n = int(max(1, min(s.N, seconds / len(shapes) * assumed / per_image)))
        inp = synth.make_inputs(s, batch=n)
        s2 = inp["shape"]
        d = oracle.Dims(s2.N, s2.Cin, s2.Hin, s2.Win, s2.Cout, s2.k, s2.k, s2.stride, s2.stride,
                        s2.pad, s2.pad)
        f = lambda t: None if t is None else t.double().numpy()
        a = {k: f(inp[k]) for k in ("x", "W", "b", "gamma", "beta", "rmean", "rvar", "dy")}
        t0 = time.perf_counter()
        Y, Z = oracle.eval_fwd(d, a["x"], a["W"], a["b"], a["gamma"], a["beta"], a["rmean"],
                               a["rvar"], inp["eps"])
        oracle.eval_bwd(d, a["x"], a["W"], a["b"], a["gamma"], a["rmean"], a["rvar"], inp["eps"],
                        Y, a["dy"])
        secs += time.perf_counter() - t0
        flops += s2.step_flop
        desc.append(f"{name} with N={n} of {s.N}")
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": "one fwd+bwd of " + ", ".join(desc) + f" ({secs:.1f} s)"}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus %d is not supported "
              "(the block shards over the batch, see DESIGN.md)." % a.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2305_11624_amd import binding as B
    from paper_2305_11624_amd import synth
    B.lib()                                    # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    names = WORKLOADS[a.workload]
    shapes = [synth.CONFIGS[n] for n in names]
    inputs = [synth.make_inputs(s) for s in shapes]
    flop = sum(s.step_flop for s in shapes)

    tune_pools = [make_pool(inp, "tune", a.pool_mb) for inp in inputs]
    ms_tune = time_steps(tune_pools, a.steps, a.warmup)

    ktimes = {n: kernel_times(p, a.kernel_reps) for n, p in zip(names, tune_pools)}
    saved_tune = sum(p[0].saved_bytes() for p in tune_pools)
    del tune_pools
    torch.cuda.empty_cache()

    ms_eval, saved_eval = None, None
    if not a.no_eval:
        eval_pools = [make_pool(inp, "eval", a.pool_mb) for inp in inputs]
        ms_eval = time_steps(eval_pools, a.steps, a.warmup)
        saved_eval = sum(p[0].saved_bytes() for p in eval_pools)
        del eval_pools
        torch.cuda.empty_cache()

    # dominant kernel by time among the three convolutions of every shape
    dom = max(((n, k, ktimes[n][k]) for n in names for k in ("fprop", "dgrad", "wgrad")),
              key=lambda t: t[2])
    dshape = synth.CONFIGS[dom[0]]
    achieved = dshape.fwd_flop / (dom[2] * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": f"{dom[1]} igemm @ {dom[0]}", "achieved": achieved,
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                "avg_launch_ms": dom[2],
                "traffic": MEASURED_TRAFFIC_BYTES.get(f"{dom[1]}@{dom[0]}")}

    per_shape = {}
    for n, s in zip(names, shapes):
        kt = ktimes[n]
        e = s.elem_bytes
        per_shape[n] = {
            "kernel_ms": {k: round(v, 5) for k, v in kt.items()},
            "conv_tflops": {k: round(s.fwd_flop / (kt[k] * 1e-3) / 1e12, 1)
                            for k in ("fprop", "dgrad", "wgrad")},
            "fold_gbs": round((2 * s.P * e + s.P * e + 24 * s.Cout) / (kt["fold"] * 1e-3) / 1e9, 1),
        }

    line = {
        "metric": "ConvBN Tune fwd+bwd TFLOP/s (% bf16 MFMA peak) + activation MB vs Eval",
        "value": flop / (ms_tune * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_tune,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "ResNet-50 3x3 ConvBN blocks, bf16: " + ", ".join(
            f"{s.name} x[{s.N},{s.Cin},{s.Hin},{s.Win}] {s.k}x{s.k} {s.Cin}->{s.Cout} s{s.stride} p{s.pad}"
            for s in shapes), "mode": "tune", "layout": "NHWC", "step": "fwd+bwd of every shape"},
        "pct_of_bf16_mfma_peak": 100.0 * flop / (ms_tune * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "eval_ms_per_step": ms_eval,
        "tune_speedup_vs_eval": (ms_eval / ms_tune) if ms_eval else None,
        "saved_activation_mb": {"tune": saved_tune / 1e6,
                                "eval": saved_eval / 1e6 if saved_eval is not None else None},
        "per_shape": per_shape,
        "roofline": roofline,
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(names, a.cpu_seconds)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
