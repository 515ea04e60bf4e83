"""GPU parity of the TransposedConv-BN block (Sec. 3.2.1, closing remark), Tune mode and the Eval comparison
path, against the fp64 Eval-mode definition of the CPU oracle, through the C ABI."""
import pytest
import torch

from paper_2305_11624_amd import binding as B, synth
from paper_2305_11624_amd.synth import BlockShape

from helpers import compare, oracle_tconv_block

pytestmark = pytest.mark.gpu

KEYS = ("Z", "dX", "dW", "db", "dgamma", "dbeta", "Wf")
EVAL_KEYS = ("Z", "dX", "dW", "db", "dgamma", "dbeta", "Y")


def _run(inp, **kw):
    from paper_2305_11624_amd.runner import TconvRun
    r = TconvRun(inp, poison=True, **kw)
    r.step()
    return r.results()


F32 = [
    #          name        N Cin H  W Cout k s p
    BlockShape("t32_k2s2", 2, 6, 5, 4, 5, 2, 2, 0, "f32", 61),
    BlockShape("t32_k4s2p1", 2, 5, 6, 7, 4, 4, 2, 1, "f32", 62),
    BlockShape("t32_k3s1p1", 1, 4, 7, 6, 6, 3, 1, 1, "f32", 63),
    BlockShape("t32_k3s2p1", 2, 3, 5, 5, 7, 3, 2, 1, "f32", 64),
    BlockShape("t32_k1", 3, 6, 4, 5, 9, 1, 1, 0, "f32", 65),
    BlockShape("t32_k3s3p1", 1, 4, 4, 4, 3, 3, 3, 1, "f32", 66),
]


@pytest.mark.parametrize("shape", F32, ids=lambda s: s.name)
def test_fp32_shapes(shape):
    inp = synth.make_tconv_inputs(shape, bias=True)
    ref = oracle_tconv_block(inp)
    compare(_run(inp), ref, "f32", keys=KEYS, tag=shape.name)
    compare(_run(inp, mode="eval"), ref, "f32", keys=EVAL_KEYS, tag=shape.name + "/eval")


BF16 = [
    # the 2x up-sampling blocks of encoder-decoder networks (window 2 / stride 2, and window 4 / stride 2 / pad 1),
    # several tiles and ragged tails in every dimension
    BlockShape("t_k2s2", 3, 128, 14, 14, 64, 2, 2, 0, "bf16", 71),
    BlockShape("t_k4s2p1", 2, 64, 13, 11, 72, 4, 2, 1, "bf16", 72),
    BlockShape("t_k3s1p1", 2, 72, 12, 12, 136, 3, 1, 1, "bf16", 73),
    BlockShape("t_k3s2p1", 2, 64, 9, 9, 64, 3, 2, 1, "bf16", 74),
    BlockShape("t_k1", 2, 256, 12, 12, 64, 1, 1, 0, "bf16", 75),
    BlockShape("t_k2s3", 2, 32, 6, 6, 40, 2, 3, 0, "bf16", 76),      # stride > window: output positions no tap reaches
    BlockShape("t_odd_out", 2, 64, 8, 8, 20, 2, 2, 0, "bf16", 77),   # output channels not a multiple of 8
    BlockShape("t_odd_in", 2, 12, 8, 8, 32, 3, 2, 1, "bf16", 78),    # input channels not a multiple of 8
    # stride = window over enough pixels for the single-product forward (depth-to-space store), ragged last tile
    BlockShape("t_d2s_k2", 6, 64, 37, 37, 64, 2, 2, 0, "bf16", 79),
    BlockShape("t_d2s_k3", 2, 32, 41, 41, 64, 3, 3, 0, "bf16", 80),
    # 1x1 over a long pixel range: the persistent 1x1 kernel in its input-gradient role, with the folded bias
    BlockShape("t_k1_long", 8, 64, 48, 48, 64, 1, 1, 0, "bf16", 84),
]


@pytest.mark.parametrize("shape", BF16, ids=lambda s: s.name)
def test_bf16_shapes(shape):
    inp = synth.make_tconv_inputs(shape, bias=shape.name in ("t_k2s3", "t_k4s2p1", "t_d2s_k2", "t_d2s_k3", "t_k1_long"))
    ref = oracle_tconv_block(inp)
    compare(_run(inp), ref, "bf16", keys=KEYS, tag=shape.name)
    compare(_run(inp, mode="eval"), ref, "bf16", keys=EVAL_KEYS, tag=shape.name + "/eval")


def test_refold_and_input_gradient_only():
    shape = BlockShape("t_refold", 2, 64, 10, 10, 32, 2, 2, 0, "bf16", 81)
    inp = synth.make_tconv_inputs(shape)
    ref = oracle_tconv_block(inp)
    compare(_run(inp, keep_folded=False), ref, "bf16", keys=KEYS[:-1], tag="t_refold")
    res = _run(inp, params=False)
    compare(res, ref, "bf16", keys=("Z", "dX"), tag="t_dx_only")
    assert res["dW"] is None and res["dgamma"] is None
    compare(_run(inp, mode="eval", params=False), ref, "bf16", keys=("Z", "dX"), tag="t_dx_only/eval")


def test_wide_scale_with_zero_channels():
    """Scales from 0 to 30 with exact zeros (the range of pretrained backbones, Fig. 2a): Tune mode never divides by s."""
    shape = BlockShape("t_wide", 2, 64, 8, 8, 64, 2, 2, 0, "bf16", 82)
    inp = synth.make_tconv_inputs(shape, wide_scale=True, bias=True)
    compare(_run(inp), oracle_tconv_block(inp), "bf16", keys=KEYS, tag="t_wide")


def test_decoder_block_full_size():
    """An up-sampling block at the size of a segmentation decoder stage: 256 -> 128 channels, 28x28 -> 56x56, N = 8."""
    shape = BlockShape("t_dec", 8, 256, 28, 28, 128, 2, 2, 0, "bf16", 83)
    inp = synth.make_tconv_inputs(shape)
    compare(_run(inp), oracle_tconv_block(inp), "bf16", keys=KEYS, tag="t_dec")


def test_errors():
    d = B.make_desc(1, 8, 2, 2, 8, 1, 1, stride=1, pad=1, dtype=B.BF16)   # padding removes the whole output
    assert B.convbn_tconv_workspace_bytes(d, B.MODE_TUNE, B.PASS_FWD) == 0
    x = torch.zeros(64, device="cuda", dtype=torch.bfloat16)
    v = torch.zeros(8, device="cuda")
    st = B.convbn_tconv_tune_fwd(d, x, x, None, v, v, v, v, x, None, None, check=False)
    assert st == B.ERR_SHAPE
    d = B.make_desc(1, 8, 2, 2, 8, 2, 2, stride=2, pad=0, dtype=B.BF16)
    st = B.convbn_tconv_tune_fwd(d, x, x, None, v, v, v, v, x, None, None, check=False)
    assert st == B.ERR_WORKSPACE
