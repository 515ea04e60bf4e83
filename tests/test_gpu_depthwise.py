"""GPU parity of the depthwise ConvBN block (one filter per channel), Tune mode and the Eval comparison path,
against the fp64 Eval-mode definition of the CPU oracle, through the C ABI."""
import pytest
import torch

from paper_2305_11624_amd import binding as B, synth
from paper_2305_11624_amd.synth import BlockShape

from helpers import compare, oracle_dw_block

pytestmark = pytest.mark.gpu

KEYS = ("Z", "dX", "dW", "db", "dgamma", "dbeta", "Wf")
EVAL_KEYS = ("Z", "dX", "dW", "db", "dgamma", "dbeta", "Y")


def _run(inp, **kw):
    from paper_2305_11624_amd.runner import DepthwiseRun
    r = DepthwiseRun(inp, poison=True, **kw)
    r.step()
    return r.results()


SHAPES = [
    #          name          N  C   H   W   C  k s p
    BlockShape("d32_3x3", 2, 6, 9, 8, 6, 3, 1, 1, "f32", 91),
    BlockShape("d32_3x3_s2", 2, 5, 9, 9, 5, 3, 2, 1, "f32", 92),
    BlockShape("d32_5x5", 1, 4, 11, 10, 4, 5, 1, 2, "f32", 93),
    # bf16, channel counts of inverted-residual / ghost modules; several slices and a ragged tail in every dimension
    BlockShape("d_3x3", 3, 144, 28, 28, 144, 3, 1, 1, "bf16", 94),
    BlockShape("d_3x3_s2", 2, 96, 29, 27, 96, 3, 2, 1, "bf16", 95),
    BlockShape("d_5x5", 2, 72, 14, 14, 72, 5, 1, 2, "bf16", 96),       # more window positions than one pass accumulates
    BlockShape("d_5x5_s2", 2, 40, 17, 17, 40, 5, 2, 2, "bf16", 97),
    BlockShape("d_wide", 2, 960, 7, 7, 960, 3, 1, 1, "bf16", 98),
    BlockShape("d_odd_ch", 2, 20, 9, 9, 20, 3, 1, 1, "bf16", 99),      # channels not a multiple of 8: scalar path
    BlockShape("d_1x1", 2, 32, 6, 6, 32, 1, 1, 0, "bf16", 100),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
def test_shapes(shape):
    inp = synth.make_dw_inputs(shape, bias=shape.dtype == "f32" or shape.name in ("d_3x3_s2", "d_5x5"))
    ref = oracle_dw_block(inp)
    compare(_run(inp), ref, shape.dtype, keys=KEYS, tag=shape.name)
    compare(_run(inp, mode="eval"), ref, shape.dtype, keys=EVAL_KEYS, tag=shape.name + "/eval")


def test_refold_input_gradient_only_and_wide_scale():
    shape = BlockShape("d_refold", 2, 64, 12, 12, 64, 3, 1, 1, "bf16", 101)
    inp = synth.make_dw_inputs(shape, wide_scale=True, bias=True)
    ref = oracle_dw_block(inp)
    compare(_run(inp), ref, "bf16", keys=KEYS, tag="d_wide_scale")
    compare(_run(inp, keep_folded=False), ref, "bf16", keys=KEYS[:-1], tag="d_refold")
    res = _run(inp, params=False)
    compare(res, ref, "bf16", keys=("Z", "dX"), tag="d_dx_only")
    assert res["dW"] is None and res["dgamma"] is None


def test_full_size_layer():
    """A depthwise layer at network size: 144 channels, 56x56, N = 32 (an inverted-residual stage), sampled against
    the oracle run on the first two images (the block is independent across images except for the parameter gradients,
    which are compared on a two-image problem of their own)."""
    shape = BlockShape("d_full", 32, 144, 56, 56, 144, 3, 1, 1, "bf16", 102)
    inp = synth.make_dw_inputs(shape)
    res = _run(inp)
    small = {k: (v[:2] if k in ("x", "dy") else v) for k, v in inp.items()}
    small["shape"] = BlockShape("d_full2", 2, 144, 56, 56, 144, 3, 1, 1, "bf16", 102)
    ref = oracle_dw_block(small)
    compare({k: res[k][:2] for k in ("Z", "dX")}, ref, "bf16", keys=("Z", "dX"), tag="d_full[:2]")
    compare(_run(small), ref, "bf16", keys=KEYS, tag="d_full2")


def test_errors():
    d = B.make_desc(2, 16, 8, 8, 32, 3, 3, 1, 1)     # Cin != Cout
    assert B.convbn_dw_workspace_bytes(d, B.MODE_TUNE, B.PASS_FWD) == 0
    x = torch.zeros(4096, device="cuda", dtype=torch.bfloat16)
    v = torch.zeros(32, device="cuda")
    assert B.convbn_dw_tune_fwd(d, x, x, None, v, v, v, v, x, None, x, check=False) == B.ERR_SHAPE
    d = B.make_desc(2, 16, 8, 8, 16, 3, 3, 1, 1)
    assert B.convbn_dw_tune_fwd(d, x, x, None, v, v, v, v, x, None, None, check=False) == B.ERR_WORKSPACE
