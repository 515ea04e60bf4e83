"""GPU parity of the grouped ConvBN block (channels split into groups), Tune mode and the Eval comparison path,
against the fp64 Eval-mode definition of the CPU oracle, through the C ABI."""
import pytest
import torch

from paper_2305_11624_amd import binding as B, synth
from paper_2305_11624_amd.synth import BlockShape

from helpers import compare, oracle_grouped_block

pytestmark = pytest.mark.gpu

KEYS = ("Z", "dX", "dW", "db", "dgamma", "dbeta", "Wf")
EVAL_KEYS = ("Z", "dX", "dW", "db", "dgamma", "dbeta", "Y")


def _run(inp, **kw):
    from paper_2305_11624_amd.runner import GroupedRun
    r = GroupedRun(inp, poison=True, **kw)
    r.step()
    return r.results()


SHAPES = [
    #           name            N  Cin  H   W  Cout k s p             groups
    (BlockShape("g32_3x3", 2, 6, 9, 8, 9, 3, 1, 1, "f32", 111), 3),
    (BlockShape("g32_3x3_s2", 2, 8, 9, 9, 4, 3, 2, 1, "f32", 112), 2),
    (BlockShape("g32_5x5_mult", 1, 4, 11, 10, 12, 5, 1, 2, "f32", 113), 4),       # one input channel per group, 3 outputs
    # bf16: the widths of an aggregated-transform network's four stages (32 groups of 4, 8, 16, 32 channels) and of a
    # network with a fixed group width; several tiles and ragged tails in every dimension
    (BlockShape("g_w4", 3, 128, 20, 19, 128, 3, 1, 1, "bf16", 114), 32),
    (BlockShape("g_w8", 2, 256, 17, 17, 256, 3, 1, 1, "bf16", 115), 32),
    (BlockShape("g_w16", 3, 512, 14, 14, 512, 3, 1, 1, "bf16", 116), 32),
    (BlockShape("g_w32", 5, 1024, 7, 7, 1024, 3, 1, 1, "bf16", 117), 32),
    (BlockShape("g_w8_s2", 2, 256, 29, 27, 256, 3, 2, 1, "bf16", 118), 32),
    (BlockShape("g_w24", 2, 144, 15, 14, 144, 3, 1, 1, "bf16", 119), 6),          # group width not a power of two
    (BlockShape("g_w48_s2", 2, 96, 18, 18, 96, 3, 2, 1, "bf16", 120), 2),
    (BlockShape("g_w64", 2, 128, 12, 13, 128, 3, 1, 1, "bf16", 121), 2),
    (BlockShape("g_w64_s2", 2, 192, 17, 18, 192, 3, 2, 1, "bf16", 130), 3),       # groups of 64, stride 2
    (BlockShape("g_uneven", 2, 64, 10, 10, 32, 3, 1, 1, "bf16", 122), 4),         # 16 inputs and 8 outputs per group
    (BlockShape("g_1x1", 2, 64, 9, 9, 64, 1, 1, 0, "bf16", 123), 8),
    (BlockShape("g_5x5", 2, 32, 11, 11, 32, 5, 1, 2, "bf16", 124), 4),
    (BlockShape("g_odd", 2, 20, 9, 9, 30, 3, 1, 1, "bf16", 125), 5),              # group widths 4 and 6
]


@pytest.mark.parametrize("shape,groups", SHAPES, ids=lambda v: v.name if isinstance(v, BlockShape) else f"G{v}")
def test_shapes(shape, groups):
    inp = synth.make_grouped_inputs(shape, groups, bias=shape.dtype == "f32" or shape.name in ("g_w8", "g_w24", "g_odd"))
    ref = oracle_grouped_block(inp)
    compare(_run(inp), ref, shape.dtype, keys=KEYS, tag=shape.name)
    compare(_run(inp, mode="eval"), ref, shape.dtype, keys=EVAL_KEYS, tag=shape.name + "/eval")


def test_refold_input_gradient_only_and_wide_scale():
    shape = BlockShape("g_refold", 2, 128, 12, 12, 128, 3, 1, 1, "bf16", 126)
    inp = synth.make_grouped_inputs(shape, 16, wide_scale=True, bias=True)
    ref = oracle_grouped_block(inp)
    compare(_run(inp), ref, "bf16", keys=KEYS, tag="g_wide_scale")
    compare(_run(inp, keep_folded=False), ref, "bf16", keys=KEYS[:-1], tag="g_refold")
    res = _run(inp, params=False)
    compare(res, ref, "bf16", keys=("Z", "dX"), tag="g_dx_only")
    assert res["dW"] is None and res["dgamma"] is None


def test_one_group_matches_the_dense_block():
    from paper_2305_11624_amd.runner import BlockRun
    shape = BlockShape("g_dense", 2, 32, 10, 10, 48, 3, 1, 1, "bf16", 127)
    inp = synth.make_grouped_inputs(shape, 1, bias=True)
    res = _run(inp)
    ref = oracle_grouped_block(inp)
    compare(res, ref, "bf16", keys=KEYS, tag="g_dense")
    r = BlockRun(inp)
    r.step()
    dense = r.results()
    for k in ("Z", "dX", "dW"):
        assert (res[k] - dense[k]).abs().max() <= 2e-2 * ref[k].__abs__().max()


def test_groups_equal_to_channels_is_the_depthwise_block():
    from paper_2305_11624_amd.runner import DepthwiseRun
    shape = BlockShape("g_dw", 2, 48, 13, 12, 48, 3, 2, 1, "bf16", 129)
    inp = synth.make_grouped_inputs(shape, 48, bias=True)
    ref = oracle_grouped_block(inp)
    res = _run(inp)
    compare(res, ref, "bf16", keys=KEYS[:-1], tag="g_dw")
    compare(_run(inp, mode="eval"), ref, "bf16", keys=EVAL_KEYS, tag="g_dw/eval")
    r = DepthwiseRun(inp)
    r.step()
    dw = r.results()
    for k in ("Z", "dX", "dW", "dgamma"):
        assert torch.equal(res[k], dw[k]), k          # the same kernels: the grouped calls pass this limit on


@pytest.mark.parametrize("name,C,H,stride", [("gx_56", 128, 56, 1), ("gx_56_s2", 256, 56, 2), ("gx_14", 512, 14, 1),
                                             ("gx_7", 1024, 7, 1), ("gx_7_w64", 2048, 7, 1)])
def test_full_size_layers(name, C, H, stride):
    """The benchmark's grouped layers at their full size (32 groups, N = 32, the launch configuration the benchmark
    times), sampled against the oracle run on the first two images (the block is independent across images except
    for the parameter gradients, compared on a two-image problem of their own)."""
    shape = BlockShape(name, 32, C, H, H, C, 3, stride, 1, "bf16", 128)
    inp = synth.make_grouped_inputs(shape, 32)
    res = _run(inp)
    small = {k: (v[:2] if k in ("x", "dy") else v) for k, v in inp.items()}
    small["shape"] = BlockShape(name + "_n2", 2, C, H, H, C, 3, stride, 1, "bf16", 128)
    ref = oracle_grouped_block(small)
    compare({k: res[k][:2] for k in ("Z", "dX")}, ref, "bf16", keys=("Z", "dX"), tag=name + "[:2]")
    compare(_run(small), ref, "bf16", keys=KEYS, tag=name + "_n2")


def test_errors():
    d = B.make_desc(2, 16, 8, 8, 32, 3, 3, 1, 1)
    assert B.convbn_grouped_workspace_bytes(d, 3, B.MODE_TUNE, B.PASS_FWD) == 0      # 3 divides neither count
    assert B.convbn_grouped_workspace_bytes(d, 0, B.MODE_TUNE, B.PASS_FWD) == 0
    x = torch.zeros(8192, device="cuda", dtype=torch.bfloat16)
    v = torch.zeros(32, device="cuda")
    assert B.convbn_grouped_tune_fwd(d, 3, x, x, None, v, v, v, v, x, None, x, check=False) == B.ERR_SHAPE
    assert B.convbn_grouped_tune_fwd(d, 4, x, x, None, v, v, v, v, x, None, None, check=False) == B.ERR_WORKSPACE
    assert B.convbn_grouped_tune_fwd(d, 4, x, None, None, v, v, v, v, x, None, x, check=False) == B.ERR_NULL
