"""Seeded sweep of randomly drawn (valid) shapes through the four blocks (the dense one also as a first layer), each against the oracle: windows 1-7,
strides 1-3, all paddings, channel counts that do and do not fit the MFMA tiles, ragged images.  Catches planner
corner cases the hand-picked shapes miss; every draw is reproducible from the seed."""
import random

import pytest

from paper_2305_11624_amd import synth
from paper_2305_11624_amd.synth import BlockShape

from helpers import compare, oracle_block, oracle_dw_block, oracle_grouped_block, oracle_tconv_block

pytestmark = pytest.mark.gpu

CHANS = [8, 16, 24, 32, 40, 64, 72, 96, 128, 136, 192, 256, 320, 512]


def _bounded(n, h, cin, work):
    """Shrink until the oracle's multiply count `work(n, h, cin)` is small."""
    while work(n, h, cin) > 2e9:
        if n > 1:
            n -= 1
        elif h > 8:
            h //= 2
        else:
            cin = max(8, cin // 2)
    return n, h, cin


def test_dense_block_random_shapes():
    from paper_2305_11624_amd.runner import BlockRun
    rng = random.Random(20230511)
    for it in range(48):
        k = rng.choice([1, 1, 3, 3, 3, 5, 7])
        s = rng.choice([1, 1, 2])
        p = rng.randint(0, k // 2)
        cin, cout = rng.choice(CHANS), rng.choice(CHANS)
        h, w = rng.randint(max(k, 4), 48), rng.randint(max(k, 4), 48)
        n, h, cin = _bounded(rng.randint(1, 8), h, cin, lambda n_, h_, c_: n_ * h_ * w * c_ * cout * k * k)
        h = max(h, k)
        shape = BlockShape(f"r{it}", n, cin, h, w, cout, k, s, p, "bf16", 4000 + it)
        mode, keep, bias = rng.choice(["tune", "tune", "eval"]), rng.random() < 0.7, rng.random() < 0.5
        inp = synth.make_inputs(shape, bias=bias)
        r = BlockRun(inp, mode=mode, keep_folded=keep, poison=True)
        r.step()
        compare(r.results(), oracle_block(inp), "bf16", tag=f"{shape} {mode} keep={keep}")


def test_transposed_block_random_shapes():
    from paper_2305_11624_amd.runner import TconvRun
    rng = random.Random(20230512)
    for it in range(32):
        k = rng.choice([1, 2, 2, 3, 4, 4])
        s = rng.choice([1, 2, 2, 3]) if k > 1 else 1
        p = rng.randint(0, (k - 1) // 2)
        cin, cout = rng.choice(CHANS[:12]), rng.choice(CHANS[:12])
        h, w = rng.randint(3, 40), rng.randint(3, 40)
        n, h, cin = _bounded(rng.randint(1, 8), h, cin, lambda n_, h_, c_: n_ * h_ * w * c_ * cout * k * k)
        h = max(h, 3)
        shape = BlockShape(f"rt{it}", n, cin, h, w, cout, k, s, p, "bf16", 5000 + it)
        mode, keep, bias = rng.choice(["tune", "tune", "eval"]), rng.random() < 0.7, rng.random() < 0.5
        inp = synth.make_tconv_inputs(shape, bias=bias)
        r = TconvRun(inp, mode=mode, keep_folded=keep, poison=True)
        r.step()
        compare(r.results(), oracle_tconv_block(inp), "bf16", tag=f"{shape} {mode} keep={keep}")


def test_depthwise_block_random_shapes():
    from paper_2305_11624_amd.runner import DepthwiseRun
    rng = random.Random(20230513)
    for it in range(32):
        k = rng.choice([1, 3, 3, 3, 5, 7])
        s = rng.choice([1, 1, 2])
        p = rng.randint(0, k // 2)
        c = rng.choice(CHANS[:12] + [12, 20, 144, 576])
        h, w = rng.randint(max(k, 4), 60), rng.randint(max(k, 4), 60)
        shape = BlockShape(f"rd{it}", rng.randint(1, 8), c, h, w, c, k, s, p, "bf16", 6000 + it)
        mode, keep, bias = rng.choice(["tune", "tune", "eval"]), rng.random() < 0.7, rng.random() < 0.5
        inp = synth.make_dw_inputs(shape, bias=bias)
        r = DepthwiseRun(inp, mode=mode, keep_folded=keep, poison=True)
        r.step()
        compare(r.results(), oracle_dw_block(inp), "bf16", tag=f"{shape} {mode} keep={keep}")


def test_grouped_block_random_shapes():
    """Mostly shapes the matrix-core kernels take (equal channel counts, groups of 4-32 channels, 3x3 or 1x1: wide and
    tall images, both strides, paddings 0-1, so that every column split, tile height and chunk count of their planner
    comes up), some the any-shape kernels take (other widths, unequal counts, 5x5)."""
    from paper_2305_11624_amd.runner import GroupedRun
    rng = random.Random(20230514)
    for it in range(40):
        fast = rng.random() < 0.75
        if fast:
            cg = rng.choice([4, 8, 16, 32])
            cin = cout = 32 * rng.choice([1, 2, 3, 4, 6, 8])
            groups = cin // cg
            k = rng.choice([3, 3, 3, 1])
        else:
            groups = rng.choice([2, 3, 4, 6])
            cin, cout = groups * rng.choice([2, 6, 12, 24]), groups * rng.choice([4, 8, 12])
            k = rng.choice([1, 3, 5])
        s = rng.choice([1, 1, 2])
        p = rng.randint(0, k // 2)
        h, w = rng.randint(max(k, 4), 40), rng.randint(max(k, 4), 150 if it % 5 == 0 else 40)
        shape = BlockShape(f"rg{it}", rng.randint(1, 3), cin, h, w, cout, k, s, p, "bf16", 7000 + it)
        mode, keep, bias = rng.choice(["tune", "tune", "eval"]), rng.random() < 0.7, rng.random() < 0.5
        inp = synth.make_grouped_inputs(shape, groups, bias=bias)
        r = GroupedRun(inp, mode=mode, keep_folded=keep, poison=True)
        r.step()
        compare(r.results(), oracle_grouped_block(inp), "bf16", tag=f"{shape} G={groups} {mode} keep={keep}")


def test_first_layer_random_shapes():
    """1-4 input channels: the first-layer kernels (forward, input gradient, weight gradient) where their plans fit,
    the padded generic route elsewhere; row lengths that do and do not allow whole 16-byte pieces."""
    from paper_2305_11624_amd.runner import BlockRun
    rng = random.Random(20230515)
    for it in range(32):
        k = rng.choice([1, 3, 3, 5, 7, 7])
        s = rng.choice([1, 2, 2])
        p = rng.randint(0, k // 2)
        cin, cout = rng.choice([1, 2, 3, 3, 3, 4]), rng.choice([32, 64, 64, 96, 128])
        h, w = rng.randint(max(k, 6), 70), rng.choice([rng.randint(max(k, 6), 70), 4 * rng.randint(2, 40)])
        shape = BlockShape(f"rs{it}", rng.randint(1, 3), cin, h, w, cout, k, s, p, "bf16", 8000 + it)
        mode, keep, bias = rng.choice(["tune", "tune", "eval"]), rng.random() < 0.7, rng.random() < 0.5
        inp = synth.make_inputs(shape, bias=bias)
        r = BlockRun(inp, mode=mode, keep_folded=keep, poison=True)
        r.step()
        compare(r.results(), oracle_block(inp), "bf16", tag=f"{shape} {mode} keep={keep}")
