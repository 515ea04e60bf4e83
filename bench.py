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
    "resnet50": [],          # the whole 53-block backbone, Tune vs Eval (time and activation memory)
    "tconv": [],             # TransposedConv-BN up-sampling blocks in Tune mode
    "depthwise": [],         # depthwise ConvBN blocks in Tune mode (memory-bound)
    "grouped": [],           # grouped ConvBN blocks in Tune mode (memory-bound)
}

# depthwise 3x3 layers of an inverted-residual network at N = 32 (stand-ins for the mobile-network rows of the
# paper's model tables): name, N, C, H, W, window, stride, padding
DW_SHAPES = [("dw_112_s2", 32, 96, 112, 112, 3, 2, 1), ("dw_56", 32, 144, 56, 56, 3, 1, 1),
             ("dw_14", 32, 576, 14, 14, 3, 1, 1)]

# grouped 3x3 layers of an aggregated-transform network (32 groups of 4, 8, 16, 32 channels in its four stages, and
# the stride-2 layer that opens its second stage) at
# N = 32 (stand-ins for the ResNeXt / RegNet rows of the paper's model tables): name, N, C, H, W, window, stride,
# padding, groups
GROUPED_SHAPES = [("gx_56", 32, 128, 56, 56, 3, 1, 1, 32), ("gx_56_s2", 32, 256, 56, 56, 3, 2, 1, 32),
                  ("gx_28", 32, 256, 28, 28, 3, 1, 1, 32), ("gx_14", 32, 512, 14, 14, 3, 1, 1, 32),
                  ("gx_7", 32, 1024, 7, 7, 3, 1, 1, 32)]

# 2x up-sampling blocks of an encoder-decoder network (stand-ins for the UNet rows of Sec. 4.3): name, N, Cin, Hin,
# Win, Cout, window, stride, padding
TCONV_SHAPES = [("up_k2", 32, 256, 28, 28, 128, 2, 2, 0), ("up_k4", 32, 512, 14, 14, 256, 4, 2, 1)]

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "c2_default_bench_hbm_traffic.txt")
KERNEL_SOURCES = os.path.join(ROOT, "paper_2305_11624_amd", "csrc")


def sources_digest():
    """Digest of the kernel sources: the traffic table names the digest of the build it was measured on."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(KERNEL_SOURCES)):
        if name.endswith((".hip", ".h")):
            with open(os.path.join(KERNEL_SOURCES, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(key):
    """HBM bytes per launch (fetched + written) of `key` ("pass@shape") from the tracked rocprofv3 counter summary,
    or None when the summary has no such row or was measured on other kernel sources than the ones in the tree."""
    try:
        rows, digest = {}, None
        with open(TRAFFIC_TABLE) as f:
            for ln in f:
                if ln.startswith("sources-digest:"):
                    digest = ln.split(":", 1)[1].strip()
                elif ln.startswith("traffic|"):
                    _, k, fetch, write = [t.strip() for t in ln.split("|")[:4]]
                    rows[k] = float(fetch) + float(write)
        return rows.get(key) if digest == sources_digest() else None
    except (OSError, ValueError):
        return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=sorted(WORKLOADS))
    ap.add_argument("--only", default=None, help="depthwise / grouped workloads: comma-separated shape names to keep")
    ap.add_argument("--pool-mb", type=int, default=768,
                    help="minimum total size of the rotating buffer pool per shape")
    ap.add_argument("--kernel-reps", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-eval", action="store_true")
    ap.add_argument("--eager", action="store_true", help="time eager launches only (no HIP graph replay)")
    ap.add_argument("--no-hbm-shapes", action="store_true", help="skip the memory-bound configurations 1 and 3a")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also launch a plain streaming kernel of known size (in-place ReLU over 256 MiB: "
                         "reads and writes 268435456 bytes each) so that rocprofv3 --pmc FETCH_SIZE / "
                         "WRITE_SIZE readings of the other kernels can be scaled to bytes")
    ap.add_argument("--group-fold", action="store_true",
                    help="resnet50 workload: also run Tune mode with all blocks folded in one launch")
    ap.add_argument("--batch", type=int, default=32, help="batch of the resnet50 workload")
    ap.add_argument("--image", type=int, default=224, help="image size of the resnet50 workload")
    return ap.parse_args()


def tensor_bytes(run):
    n = 0
    for v in vars(run).values():
        if hasattr(v, "element_size") and hasattr(v, "numel"):
            n += v.numel() * v.element_size()
    return n


def keeps_folded(shape):
    """Keep w' between forward and backward only where it is smaller than the Y that Eval mode keeps (P <= A_z,
    App. K.1); elsewhere backward folds again and nothing but x is kept."""
    return shape.P <= shape.A_z


def make_pool(inp, mode, pool_mb):
    from paper_2305_11624_amd.runner import BlockRun
    keep = keeps_folded(inp["shape"])
    first = BlockRun(inp, mode=mode, keep_folded=keep)
    per = max(1, tensor_bytes(first))
    count = max(2, min(64, -(-pool_mb * (1 << 20) // per)))
    return [first] + [BlockRun(inp, mode=mode, keep_folded=keep) for _ in range(count - 1)]


def time_steps(pools, steps, warmup):
    """Eager launches: K steps enqueued from Python, one library call after the other."""
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


def time_steps_graph(pools, steps, warmup):
    """The same K steps replayed from HIP graphs: one captured graph per buffer set of the rotation (the library
    only enqueues kernels on the caller's stream, so a step is capturable as it is).  Returns None if capture is
    not available."""
    import torch
    rot = max(len(p) for p in pools)
    graphs = []
    try:
        side = torch.cuda.Stream()
        for i in range(rot):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for pool in pools:
                    pool[i % len(pool)].step()
            graphs.append(g)
    except Exception as e:   # capture refused: report eager numbers only
        print(f"bench.py: graph capture not available ({e})", file=sys.stderr)
        return None
    for k in range(max(warmup, 1)):
        graphs[k % rot].replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        graphs[k % rot].replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3


def hbm_bound_shapes(pool_mb, steps):
    """Configurations 1 and 3a are bound by memory traffic, not by the matrix cores: their Tune step against the
    HBM peak, in algorithmic bytes (x read by forward and weight gradient, z written, dz read by both gradient
    passes, dx written; the weight passes are negligible there)."""
    from paper_2305_11624_amd import synth
    out = {}
    for name in ("c1", "c3a"):
        s = synth.CONFIGS[name]
        pool = make_pool(synth.make_inputs(s), "tune", pool_mb)
        ms = time_steps([pool], steps, 5)
        e = s.elem_bytes
        nbytes = e * (3 * s.A_x + 3 * s.A_z) + s.P * (6 * e + 8)
        out[name] = {"ms_per_step": ms, "algorithmic_mb": nbytes / 1e6, "gbs": nbytes / (ms * 1e-3) / 1e9,
                     "pct_of_hbm_peak": 100.0 * nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     "tflops": s.step_flop / (ms * 1e-3) / 1e12}
        del pool
    return out


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
    # blocks whose backward runs weight gradient and fold-back as one launch: that launch (no dx: nothing else runs)
    if B.convbn_tune_bwd_is_fused(d):
        calls["wgrad_fused_fold_back"] = lambda r, w: B.convbn_tune_bwd(
            d, r.x, r.W, r.b, r.gamma, r.mean, r.var, None, r.dz, None, r.dW, r.db, r.dgamma, r.dbeta, r.ws_bwd)
    # the ablation of the fold (unfolded weight, scale applied in the convolution's epilogue): where it is built
    if B.convbn_tune_fwd_scale_epilogue(d, r0.x, r0.W, r0.b, r0.gamma, r0.beta, r0.mean, r0.var, r0.z,
                                        check=False) == B.OK:
        calls["fprop_scale_epilogue"] = lambda r, w: B.convbn_tune_fwd_scale_epilogue(
            d, r.x, r.W, r.b, r.gamma, r.beta, r.mean, r.var, r.z)
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


def backbone_flop(shapes):
    """Useful convolution FLOPs of one fwd+bwd: fprop + wgrad everywhere, dgrad except for the
    stem (nothing upstream of the images needs a gradient)."""
    return sum(s.fwd_flop * (2 if s.name == "stem" else 3) for s in shapes)


def run_backbone(mode, N, image, steps, warmup, group_fold=False, group_units=False):
    import torch
    from paper_2305_11624_amd.resnet50 import ResNet50
    net = ResNet50(N, image, "bf16", mode, group_fold=group_fold, group_units=group_units)
    g = torch.Generator(device="cpu").manual_seed(0)
    x = torch.randn(N, image, image, 3, generator=g).to("cuda", torch.bfloat16)
    h = image // 32
    dout = torch.randn(N, h, h, 2048, generator=g).to("cuda", torch.bfloat16)
    torch.cuda.synchronize()
    base = torch.cuda.memory_allocated()
    torch.cuda.reset_peak_memory_stats()
    for _ in range(max(1, warmup)):
        net.forward(x)
        net.backward(dout)
    torch.cuda.synchronize()
    peak = torch.cuda.max_memory_allocated() - base
    # Workspace (the library's scratch and, with per-unit grouping, the arena of a unit's w' and partial sums) is
    # allocated once before `base` and reported on its own; the w' that per-unit grouping keeps between the passes is
    # preallocated too and belongs to the activation figure, as the w' a single block allocates in forward does.
    workspace = net.ws.numel() + net.arena_bytes
    if group_units:
        peak += net.kept_bytes
    t0 = time.perf_counter()
    for _ in range(steps):
        net.forward(x)
        net.backward(dout)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    # forward alone and backward alone, HIP events on the stream the kernels run on
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ev[0].record(); net.forward(x); ev[1].record(); net.backward(dout); ev[2].record()
    torch.cuda.synchronize()
    out = dict(ms=ms, peak_activation_mb=peak / 1e6, workspace_mb=workspace / 1e6,
               saved_model_mb=net.saved_bytes_model() / 1e6,
               fwd_ms=ev[0].elapsed_time(ev[1]), bwd_ms=ev[1].elapsed_time(ev[2]),
               refold_blocks=sum(1 for b in net.blocks.values() if mode == "tune" and not b.keep_folded))
    if group_fold:
        # the grouped fold alone: every block's w -> w' (both orders) and b' in one launch
        items, n, table, grid = net._group
        byts = sum(3 * b.shape.Cout * b.shape.K * 2 + 24 * b.shape.Cout for b, _ in items)
        from paper_2305_11624_amd import binding as B
        e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        e[0].record()
        for _ in range(20):
            B.convbn_fold_group(n, table, grid)
        e[1].record()
        torch.cuda.synchronize()
        fms = e[0].elapsed_time(e[1]) / 20
        out.update(fold_group_blocks=n, fold_group_ms=fms, fold_group_mb=byts / 1e6, fold_group_gbs=byts / fms / 1e6,
                   saved_model_mb=net.group_bytes / 1e6, refold_blocks=0)
    del net
    torch.cuda.empty_cache()
    return out


def backbone_cpu_baseline(image, seconds):
    """The backbone oracle (fp64, OpenMP direct loops) on one fwd+bwd of a batch sized to
    roughly `seconds`."""
    import numpy as np
    import oracle
    from oracle.resnet import ResNet50Oracle
    from paper_2305_11624_amd import synth
    cores = oracle.num_threads()
    per_image = backbone_flop(synth.resnet50_blocks(1, image, "bf16"))
    n = int(max(1, min(8, seconds * 1.5e9 * cores / per_image)))
    shapes = synth.resnet50_blocks(n, image, "bf16")
    params = {}
    for sh in shapes:
        p = synth.make_params(sh)
        params[sh.name] = {k: (v.double().numpy() if hasattr(v, "numpy") else v) for k, v in p.items()}
    stages = [[f"l{st}.{i}" for i in range(k)] for st, k in enumerate((3, 4, 6, 3), start=1)]
    rng = np.random.default_rng(0)
    x = rng.standard_normal((n, 3, image, image))
    dout = rng.standard_normal((n, 2048, image // 32, image // 32))
    ref = ResNet50Oracle(params, stages)
    t0 = time.perf_counter()
    ref.forward(x)
    ref.backward(dout)
    secs = time.perf_counter() - t0
    return {"value": backbone_flop(shapes) / secs / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"one fwd+bwd of the backbone with N={n}, {image}x{image} ({secs:.1f} s)"}


def main_backbone(a):
    import torch
    from paper_2305_11624_amd import binding as B
    from paper_2305_11624_amd import synth
    B.lib()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    N, image = a.batch, a.image
    shapes = synth.resnet50_blocks(N, image, "bf16")
    flop = backbone_flop(shapes)
    # Tune mode with one fold launch and one fold-back launch per bottleneck unit (the default), and with one of
    # each per block for comparison
    tune = run_backbone("tune", N, image, a.steps, a.warmup, group_units=True)
    tune_pb = run_backbone("tune", N, image, a.steps, a.warmup)
    ev = None if a.no_eval else run_backbone("eval", N, image, a.steps, a.warmup)
    grouped = run_backbone("tune", N, image, a.steps, a.warmup, group_fold=True) if a.group_fold else None
    tf = flop / (tune["ms"] * 1e-3) / 1e12
    line = {
        "metric": "ConvBN Tune fwd+bwd TFLOP/s (% bf16 MFMA peak) + activation MB vs Eval",
        "value": tf, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": tune["ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"ResNet-50 backbone, 53 ConvBN blocks + ReLU + residual adds + max-pool, "
                               f"bf16, N={N}, {image}x{image}x3, frozen BN statistics; residual sums applied by the convolutions; fold and fold-back grouped per "
                               f"bottleneck unit", "mode": "tune",
                   "layout": "NHWC", "step": "fwd+bwd of the backbone (no gradient w.r.t. the images)"},
        "pct_of_bf16_mfma_peak": 100.0 * tf / PEAK_BF16_TFLOPS,
        "tune": tune, "tune_fold_per_block": tune_pb, "eval": ev, "tune_group_fold": grouped,
        "eval_ms_per_step": ev["ms"] if ev else None,
        "tune_speedup_vs_eval": ev["ms"] / tune["ms"] if ev else None,
        "peak_activation_mb": {"tune": tune["peak_activation_mb"], "eval": ev["peak_activation_mb"] if ev else None},
        "peak_with_workspace_mb": {"tune": tune["peak_activation_mb"] + tune["workspace_mb"],
                                   "eval": ev["peak_activation_mb"] + ev["workspace_mb"] if ev else None},
        "roofline": {"bound": "mfma", "kernel": "whole backbone step (all kernels)", "achieved": tf,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": tf / PEAK_BF16_TFLOPS, "traffic": None},
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = backbone_cpu_baseline(image, a.cpu_seconds)
    print(json.dumps(line))


def main_tconv(a):
    """TransposedConv-BN blocks in Tune mode: whole-step time, the forward pass and the two backward convolutions
    timed one by one (the latter through the step entry points of the convolution each block is the adjoint
    of), and the CPU oracle."""
    import torch
    import oracle
    from paper_2305_11624_amd import binding as B
    from paper_2305_11624_amd import synth
    from paper_2305_11624_amd.runner import TconvRun
    B.lib()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    shapes = [synth.BlockShape(n, N, ci, h, w, co, k, st, pd, "bf16", 90 + i)
              for i, (n, N, ci, h, w, co, k, st, pd) in enumerate(TCONV_SHAPES)]
    flops = [3.0 * 2.0 * s.N * s.Hin * s.Win * s.Cin * s.Cout * s.k * s.k for s in shapes]
    inputs = [synth.make_tconv_inputs(s) for s in shapes]
    pools = []
    for inp in inputs:
        first = TconvRun(inp)
        count = max(2, min(32, -(-a.pool_mb * (1 << 20) // max(1, tensor_bytes(first)))))
        pools.append([first] + [TconvRun(inp) for _ in range(count - 1)])
    ms = time_steps(pools, a.steps, a.warmup)
    per_shape = {}
    best = None
    for s, fl, pool in zip(shapes, flops, pools):
        r0 = pool[0]
        ho, wo = synth.tconv_out(s)
        d = B.make_desc(s.N, s.Cout, ho, wo, s.Cin, s.k, s.k, s.stride, s.pad, dtype=B.BF16)   # the adjoint convolution
        P = s.Cin * s.Cout * s.k * s.k
        dev = r0.x.device
        ws_f = torch.empty(max(16, B.convbn_conv_workspace_bytes(d, B.PASS_FWD)), dtype=torch.uint8, device=dev)
        ws_b = torch.empty(max(16, B.convbn_conv_workspace_bytes(d, B.PASS_BWD)), dtype=torch.uint8, device=dev)
        part = torch.empty(B.convbn_wgrad_parts(d) * P, dtype=torch.float32, device=dev)
        r0.forward()                                            # fills w_folded (read by the input-gradient pass)
        calls = {
            "forward (fold + transposed conv)": lambda r: r.forward(),
            "input gradient (conv)": lambda r: B.convbn_conv_fprop(d, r.dz, r0.w_folded, None, r.dx, ws_f),
            "weight gradient": lambda r: B.convbn_conv_wgrad(d, r.dz, r.x, part, None, ws_b),
        }
        kt = {}
        for name, fn in calls.items():
            for i in range(min(3, len(pool))):
                fn(pool[i])
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(a.kernel_reps):
                fn(pool[i % len(pool)])
            e1.record()
            torch.cuda.synchronize()
            kt[name] = e0.elapsed_time(e1) / a.kernel_reps
            if best is None or kt[name] > best[2]:
                best = (s.name, name, kt[name], fl / 3.0)
        per_shape[s.name] = {"kernel_ms": {k: round(v, 5) for k, v in kt.items()},
                             "conv_tflops": {k: round(fl / 3.0 / (v * 1e-3) / 1e12, 1) for k, v in kt.items()}}
    achieved = best[3] / (best[2] * 1e-3) / 1e12
    saved_tune = sum(p[0].saved_bytes() for p in pools)
    ms_eval, saved_eval = None, None
    if not a.no_eval:
        counts = [len(p) for p in pools]
        del pools, pool, r0
        torch.cuda.empty_cache()
        epools = [[TconvRun(inp, mode="eval") for _ in range(n)] for inp, n in zip(inputs, counts)]
        ms_eval = time_steps(epools, a.steps, a.warmup)
        saved_eval = sum(p[0].saved_bytes() for p in epools)
        del epools
        torch.cuda.empty_cache()
    line = {
        "metric": "TransposedConv-BN Tune fwd+bwd TFLOP/s", "value": sum(flops) / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "TransposedConv-BN up-sampling blocks, bf16: " + ", ".join(
            f"{s.name} x[{s.N},{s.Cin},{s.Hin},{s.Win}] {s.k}x{s.k} {s.Cin}->{s.Cout} s{s.stride} p{s.pad}"
            for s in shapes), "mode": "tune", "layout": "NHWC", "step": "fwd+bwd of every shape"},
        "eval_ms_per_step": ms_eval, "tune_speedup_vs_eval": (ms_eval / ms) if ms_eval else None,
        "saved_activation_mb": {"tune": saved_tune / 1e6, "eval": saved_eval / 1e6 if saved_eval is not None else None},
        "per_shape": per_shape,
        "roofline": {"bound": "mfma", "kernel": f"{best[1]} @ {best[0]}", "achieved": achieved,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "avg_launch_ms": best[2], "traffic": None},
    }
    if not a.no_cpu_baseline:
        cores = oracle.num_threads()
        fl, secs, desc = 0.0, 0.0, []
        for s, f1 in zip(shapes, flops):
            n = int(max(1, min(s.N, a.cpu_seconds / len(shapes) * 0.6e9 * cores / (f1 / s.N))))
            inp = synth.make_tconv_inputs(replace(s, N=n))
            d = oracle.Dims(n, s.Cin, s.Hin, s.Win, s.Cout, s.k, s.k, s.stride, s.stride, s.pad, s.pad)
            f = lambda t: None if t is None else t.double().numpy()
            v = {k: f(inp[k]) for k in ("x", "W", "b", "gamma", "beta", "rmean", "rvar", "dy")}
            t0 = time.perf_counter()
            Y, _ = oracle.teval_fwd(d, v["x"], v["W"], v["b"], v["gamma"], v["beta"], v["rmean"], v["rvar"], inp["eps"])
            oracle.teval_bwd(d, v["x"], v["W"], v["b"], v["gamma"], v["rmean"], v["rvar"], inp["eps"], Y, v["dy"])
            secs += time.perf_counter() - t0
            fl += f1 * n / s.N
            desc.append(f"{s.name} with N={n} of {s.N}")
        line["cpu_baseline"] = {"value": fl / secs / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                                "sample": "one fwd+bwd of " + ", ".join(desc) + f" ({secs:.1f} s)"}
    print(json.dumps(line))


def main_depthwise(a, kind="depthwise"):
    """Depthwise (or, kind = "grouped", grouped) ConvBN blocks in Tune mode.  With at most 2 k^2 cg FLOP per output
    element they are bound by memory traffic, so the figure of merit is the algorithmic bytes of a step (x read by the
    forward pass and the weight gradient, z written, dz read by both gradient passes, dx written: 3 A_x + 3 A_z
    elements) over its time, against the HBM peak."""
    import torch
    import oracle
    from paper_2305_11624_amd import binding as B
    from paper_2305_11624_amd import synth
    from paper_2305_11624_amd.runner import DepthwiseRun, GroupedRun
    B.lib()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    grouped = kind == "grouped"
    keep = (lambda rows: [t for t in rows if a.only is None or t[0] in a.only.split(",")])
    if grouped:
        shapes = [synth.BlockShape(n, N, c, h, w, c, k, st, pd, "bf16", 130 + i)
                  for i, (n, N, c, h, w, k, st, pd, _) in enumerate(keep(GROUPED_SHAPES))]
        groups = [t[-1] for t in keep(GROUPED_SHAPES)]
        inputs = [synth.make_grouped_inputs(s, g) for s, g in zip(shapes, groups)]
        DepthwiseRun = GroupedRun
    else:
        shapes = [synth.BlockShape(n, N, c, h, w, c, k, st, pd, "bf16", 110 + i)
                  for i, (n, N, c, h, w, k, st, pd) in enumerate(keep(DW_SHAPES))]
        groups = [s.Cin for s in shapes]
        inputs = [synth.make_dw_inputs(s) for s in shapes]
    step_bytes = [2.0 * (3 * s.A_x + 3 * s.A_z) for s in shapes]
    step_flop = [3.0 * 2.0 * s.A_z * s.k * s.k * (s.Cin // g) for s, g in zip(shapes, groups)]

    def pools_of(mode, **kw):
        out = []
        for inp in inputs:
            first = DepthwiseRun(inp, mode=mode, **kw)
            count = max(2, min(32, -(-a.pool_mb * (1 << 20) // max(1, tensor_bytes(first)))))
            out.append([first] + [DepthwiseRun(inp, mode=mode, **kw) for _ in range(count - 1)])
        return out

    def timed(fn, pool):
        for i in range(min(3, len(pool))):
            fn(pool[i])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(a.kernel_reps):
            fn(pool[i % len(pool)])
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / a.kernel_reps

    pools = pools_of("tune")
    ms = time_steps(pools, a.steps, a.warmup)
    saved_tune = sum(p[0].saved_bytes() for p in pools)
    per_shape, best = {}, None
    for s, pool in zip(shapes, pools):
        fwd = timed(lambda r: r.forward(), pool)
        bwd = timed(lambda r: r.backward(), pool)
        # passes: forward reads x and writes z; backward reads dz twice and x once and writes dx
        fb, bb = 2.0 * (s.A_x + s.A_z), 2.0 * (2 * s.A_x + 2 * s.A_z)
        per_shape[s.name] = {"pass_ms": {"forward (fold + conv)": round(fwd, 5), "backward (dgrad + wgrad + fold-back)": round(bwd, 5)},
                             "pass_gbs": {"forward": round(fb / (fwd * 1e-3) / 1e9, 1), "backward": round(bb / (bwd * 1e-3) / 1e9, 1)}}
        for name, t, nb in (("forward", fwd, fb), ("backward", bwd, bb)):
            if best is None or t > best[2]:
                best = (s.name, name, t, nb)
    del pools, pool
    torch.cuda.empty_cache()
    ms_eval, saved_eval = None, None
    if not a.no_eval:
        epools = pools_of("eval")
        ms_eval = time_steps(epools, a.steps, a.warmup)
        saved_eval = sum(p[0].saved_bytes() for p in epools)
        del epools
        torch.cuda.empty_cache()
    achieved = best[3] / (best[2] * 1e-3) / 1e9
    line = {
        "metric": ("Grouped" if grouped else "Depthwise") + " ConvBN Tune fwd+bwd GB/s (algorithmic bytes)", "value": sum(step_bytes) / (ms * 1e-3) / 1e9,
        "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": kind + " ConvBN blocks, bf16: " + ", ".join(
            f"{s.name} x[{s.N},{s.Cin},{s.Hin},{s.Win}] {s.k}x{s.k} s{s.stride} p{s.pad}" + (f" groups {g}" if grouped else "")
            for s, g in zip(shapes, groups)),
            "mode": "tune", "layout": "NHWC", "step": "fwd+bwd of every shape"},
        "pct_of_hbm_peak": 100.0 * sum(step_bytes) / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "useful_tflops": sum(step_flop) / (ms * 1e-3) / 1e12,
        "eval_ms_per_step": ms_eval, "tune_speedup_vs_eval": (ms_eval / ms) if ms_eval else None,
        "saved_activation_mb": {"tune": saved_tune / 1e6, "eval": saved_eval / 1e6 if saved_eval is not None else None},
        "per_shape": per_shape,
        "roofline": {"bound": "hbm", "kernel": f"{best[1]} pass @ {best[0]}", "achieved": achieved, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS, "avg_launch_ms": best[2], "traffic": None},
    }
    if not a.no_cpu_baseline:
        cores = oracle.num_threads()
        nb, secs, desc = 0.0, 0.0, []
        for s, b1, flop1, g in zip(shapes, step_bytes, step_flop, groups):
            n = int(max(1, min(s.N, a.cpu_seconds / len(shapes) * 0.3e9 * cores / (flop1 / s.N))))
            inp = synth.make_grouped_inputs(replace(s, N=n), g) if grouped else synth.make_dw_inputs(replace(s, N=n))
            d = oracle.Dims(n, s.Cin, s.Hin, s.Win, s.Cout, s.k, s.k, s.stride, s.stride, s.pad, s.pad)
            f = lambda t: None if t is None else t.double().numpy()
            v = {k: f(inp[k]) for k in ("x", "W", "b", "gamma", "beta", "rmean", "rvar", "dy")}
            t0 = time.perf_counter()
            if grouped:
                Y, _ = oracle.g_eval_fwd(d, g, v["x"], v["W"], v["b"], v["gamma"], v["beta"], v["rmean"], v["rvar"], inp["eps"])
                oracle.g_eval_bwd(d, g, v["x"], v["W"], v["b"], v["gamma"], v["rmean"], v["rvar"], inp["eps"], Y, v["dy"])
            else:
                Y, _ = oracle.dw_eval_fwd(d, v["x"], v["W"], v["b"], v["gamma"], v["beta"], v["rmean"], v["rvar"], inp["eps"])
                oracle.dw_eval_bwd(d, v["x"], v["W"], v["b"], v["gamma"], v["rmean"], v["rvar"], inp["eps"], Y, v["dy"])
            secs += time.perf_counter() - t0
            nb += b1 * n / s.N
            desc.append(f"{s.name} with N={n} of {s.N}")
        line["cpu_baseline"] = {"value": nb / secs / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
                                "sample": "one fwd+bwd of " + ", ".join(desc) + f" ({secs:.1f} s)"}
    print(json.dumps(line))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus %d is not supported "
              "(the block would shard over the batch; only the one-GPU path is built)." % a.gpus, file=sys.stderr)
        sys.exit(2)
    if a.workload == "resnet50":
        return main_backbone(a)
    if a.workload == "tconv":
        return main_tconv(a)
    if a.workload == "depthwise":
        return main_depthwise(a)
    if a.workload == "grouped":
        return main_depthwise(a, kind="grouped")
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
    ms_eager = time_steps(tune_pools, a.steps, a.warmup)
    ms_graph = None if a.eager else time_steps_graph(tune_pools, a.steps, a.warmup)
    ms_tune = min(ms_eager, ms_graph) if ms_graph is not None else ms_eager   # whichever way of launching is faster

    ktimes = {n: kernel_times(p, a.kernel_reps) for n, p in zip(names, tune_pools)}
    saved_tune = sum(p[0].saved_bytes() for p in tune_pools)
    saved_by_shape = {n: {"tune": p[0].saved_bytes() / 1e6, "kept": "w'" if p[0].keep_folded else "nothing (backward folds again)"}
                      for n, p in zip(names, tune_pools)}
    del tune_pools
    torch.cuda.empty_cache()

    ms_eval, saved_eval = None, None
    if not a.no_eval:
        eval_pools = [make_pool(inp, "eval", a.pool_mb) for inp in inputs]
        ms_eval = time_steps(eval_pools, a.steps, a.warmup)
        if not a.eager:
            ms_eval = min(ms_eval, time_steps_graph(eval_pools, a.steps, a.warmup) or ms_eval)
        saved_eval = sum(p[0].saved_bytes() for p in eval_pools)
        for n, p in zip(names, eval_pools):
            saved_by_shape[n]["eval"] = p[0].saved_bytes() / 1e6
        del eval_pools
        torch.cuda.empty_cache()

    # dominant kernel by time among the three convolutions of every shape, as the step launches them (the weight
    # gradient with the fold-back inside where the library fuses the two)
    def conv_legs(n):
        return ("fprop", "dgrad", "wgrad_fused_fold_back" if "wgrad_fused_fold_back" in ktimes[n] else "wgrad")
    dom = max(((n, k, ktimes[n][k]) for n in names for k in conv_legs(n)), key=lambda t: t[2])
    dshape = synth.CONFIGS[dom[0]]
    achieved = dshape.fwd_flop / (dom[2] * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": f"{dom[1]} @ {dom[0]}", "achieved": achieved,
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                "avg_launch_ms": dom[2],
                "traffic": measured_traffic(f"{dom[1]}@{dom[0]}")}

    per_shape = {}
    for n, s in zip(names, shapes):
        kt = ktimes[n]
        e = s.elem_bytes
        per_shape[n] = {
            "kernel_ms": {k: round(v, 5) for k, v in kt.items()},
            "conv_tflops": {k: round(s.fwd_flop / (kt[k] * 1e-3) / 1e12, 1)
                            for k in ("fprop", "dgrad", "wgrad", "wgrad_fused_fold_back") if k in kt},
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
            for s in shapes), "mode": "tune", "layout": "NHWC", "step": "fwd+bwd of every shape",
            "launch": "HIP graph replay, one graph per buffer set" if (ms_graph is not None and ms_graph < ms_eager) else "eager"},
        "pct_of_bf16_mfma_peak": 100.0 * flop / (ms_tune * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "eager_ms_per_step": ms_eager, "graph_replay_ms_per_step": ms_graph,
        "eval_ms_per_step": ms_eval,
        "tune_speedup_vs_eval": (ms_eval / ms_tune) if ms_eval else None,
        "saved_activation_mb": {"tune": saved_tune / 1e6,
                                "eval": saved_eval / 1e6 if saved_eval is not None else None},
        "saved_activation_mb_per_shape": saved_by_shape,
        "per_shape": per_shape,
        "roofline": roofline,
    }
    if a.workload == "c2" and not a.no_hbm_shapes:
        line["hbm_bound_configs"] = hbm_bound_shapes(a.pool_mb, max(20, a.steps // 4))
    if a.traffic_calibration:
        buf = torch.zeros(256 << 19, dtype=torch.bfloat16, device="cuda")     # 256 MiB
        for _ in range(3):
            B.convbn_aux_eltwise(B.OP_RELU, buf)
        torch.cuda.synchronize()
        del buf
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(names, a.cpu_seconds)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
