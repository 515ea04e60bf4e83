"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle, element
by element on identical seeded inputs.  Sizes span several tiles and ragged tails while
the oracle still finishes in seconds."""
import dataclasses

import pytest
import torch

from paper_2305_11624_amd import synth
from paper_2305_11624_amd.synth import BlockShape

from helpers import compare, oracle_block

pytestmark = pytest.mark.gpu


def _run(inp, mode, keep_folded=True, need_dx=True):
    from paper_2305_11624_amd.runner import BlockRun
    r = BlockRun(inp, mode=mode, keep_folded=keep_folded, need_dx=need_dx, poison=True)
    r.step()
    return r.results()


def test_config0_fp32_tune_and_eval():
    """Benchmark configuration 0 exactly as stated (fp32, seed 0), both modes."""
    inp = synth.make_inputs(synth.CONFIGS["c0"])
    ref = oracle_block(inp)
    for mode in ("tune", "eval"):
        res = _run(inp, mode)
        compare(res, ref, "f32", tag=f"c0/{mode}")
        if mode == "tune":
            compare(res, ref, "f32", keys=("Wf",), tag="c0/fold")
        else:
            compare(res, ref, "f32", keys=("Y",), tag="c0/Y")


F32_SHAPES = [
    BlockShape("f32_bias_s2", 2, 5, 9, 8, 7, 3, 2, 1, "f32", 21),
    BlockShape("f32_1x1", 3, 6, 5, 7, 10, 1, 1, 0, "f32", 22),
    BlockShape("f32_7x7", 1, 3, 20, 20, 8, 7, 2, 3, "f32", 23),
    BlockShape("f32_nopad", 2, 4, 8, 8, 4, 3, 1, 0, "f32", 24),
    BlockShape("f32_linear_bn", 33, 20, 1, 1, 12, 1, 1, 0, "f32", 25),
]


@pytest.mark.parametrize("shape", F32_SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("mode", ["tune", "eval"])
def test_fp32_odd_shapes(shape, mode):
    inp = synth.make_inputs(shape, bias=True)
    ref = oracle_block(inp)
    compare(_run(inp, mode), ref, "f32", tag=f"{shape.name}/{mode}")


BF16_SHAPES = [
    # MFMA path: several tiles + ragged tails in every GEMM dimension
    BlockShape("b_3x3_64", 3, 64, 14, 14, 64, 3, 1, 1, "bf16", 31),
    BlockShape("b_3x3_ragged", 2, 72, 13, 11, 136, 3, 1, 1, "bf16", 32),
    BlockShape("b_1x1", 2, 256, 12, 12, 64, 1, 1, 0, "bf16", 33),
    BlockShape("b_1x1_s2", 2, 64, 14, 14, 128, 1, 2, 0, "bf16", 34),
    BlockShape("b_3x3_s2", 2, 32, 15, 15, 40, 3, 2, 1, "bf16", 35),
    BlockShape("b_7x7_cin8", 1, 8, 30, 30, 16, 7, 2, 3, "bf16", 36),
    BlockShape("b_small7", 4, 128, 7, 7, 160, 3, 1, 1, "bf16", 37),
    # a Linear layer followed by BatchNorm is the 1x1 block on a 1x1 image (Sec. 3.2.1, closing remark)
    BlockShape("b_linear_bn", 200, 512, 1, 1, 264, 1, 1, 0, "bf16", 44),
    # long pixel ranges (more than 512 tiles of 128 pixels, ragged last tile): the persistent pointwise
    # kernel, 32- and 64-channel chunks, one and several chunks, ragged channel tiles, forward and dgrad
    BlockShape("b_pw_long32", 8, 32, 95, 97, 96, 1, 1, 0, "bf16", 47),
    BlockShape("b_pw_long64", 8, 64, 95, 97, 128, 1, 1, 0, "bf16", 48),
    # direct path (channels not multiples of 8), incl. a stem-like 7x7/2 with Cin=3
    BlockShape("b_stem", 2, 3, 32, 32, 64, 7, 2, 3, "bf16", 38),
    BlockShape("b_odd_ch", 2, 12, 9, 9, 20, 3, 1, 1, "bf16", 39),
    # first-layer kernel: rows that are not whole groups of four pixels (4-channel copy), a 4-channel and a
    # 1-channel input, 32 and 128 output channels, 3x3 and 5x5 windows, stride 1, two tiles per output row
    BlockShape("b_stem_w30", 2, 3, 30, 30, 64, 7, 2, 3, "bf16", 40),
    BlockShape("b_stem_c4", 2, 4, 24, 24, 32, 3, 1, 1, "bf16", 41),
    BlockShape("b_stem_c1", 2, 1, 20, 28, 128, 5, 2, 2, "bf16", 42),
    BlockShape("b_stem_wide", 1, 3, 23, 300, 64, 7, 2, 3, "bf16", 43),
]


@pytest.mark.parametrize("shape", BF16_SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("mode", ["tune", "eval"])
def test_bf16_shapes(shape, mode):
    inp = synth.make_inputs(shape)
    ref = oracle_block(inp)
    res = _run(inp, mode)
    compare(res, ref, "bf16", tag=f"{shape.name}/{mode}")
    if mode == "tune":
        compare(res, ref, "bf16", keys=("Wf",), tag=f"{shape.name}/fold")


def test_bf16_bias_refold_and_no_dx():
    shape = BlockShape("b_bias", 2, 64, 10, 10, 72, 3, 1, 1, "bf16", 41)
    inp = synth.make_inputs(shape, bias=True)
    ref = oracle_block(inp)
    a = _run(inp, "tune", keep_folded=True)
    b = _run(inp, "tune", keep_folded=False)
    c = _run(inp, "tune", need_dx=False)
    compare(a, ref, "bf16", tag="bias/keep")
    compare(b, ref, "bf16", tag="bias/refold")
    for k in ("Z", "dX", "dW", "db", "dgamma", "dbeta"):
        assert torch.equal(a[k], b[k]), k          # re-folding reproduces the kept w' bit for bit
    assert c["dX"] is None
    for k in ("dW", "dgamma", "dbeta"):
        assert torch.equal(a[k], c[k]), k
    compare(_run(inp, "eval"), ref, "bf16", tag="bias/eval")


def test_bf16_wide_scale_with_zero_channels():
    """BN scales spread over [0, 30] with exact zeros (the range of pretrained
    backbones, Fig. 2a): Tune mode never divides by gamma."""
    shape = BlockShape("b_wide", 2, 32, 12, 12, 32, 3, 1, 1, "bf16", 42)
    inp = synth.make_inputs(shape, wide_scale=True)
    ref = oracle_block(inp)
    compare(_run(inp, "tune"), ref, "bf16", tag="wide/tune")
    compare(_run(inp, "eval"), ref, "bf16", tag="wide/eval")


def test_tune_matches_eval_on_gpu():
    """Same library, two routes (Sec. 3.4.1): outputs agree to bf16 rounding."""
    shape = BlockShape("b_te", 2, 64, 14, 14, 64, 3, 1, 1, "bf16", 43)
    inp = synth.make_inputs(shape)
    t, e = _run(inp, "tune"), _run(inp, "eval")
    for k in ("Z", "dX", "dW", "dgamma", "dbeta"):
        ref = e[k].numpy()
        compare({k: t[k]}, {k: ref}, "bf16", keys=(k,), tag=f"tune-vs-eval/{k}")


@pytest.mark.parametrize("mode", ["tune", "eval"])
@pytest.mark.parametrize("shape", [BlockShape("b_dxonly", 2, 64, 14, 14, 72, 3, 1, 1, "bf16", 45),
                                   BlockShape("f32_dxonly", 2, 5, 9, 8, 7, 3, 2, 1, "f32", 46)],
                         ids=lambda s: s.name)
def test_input_gradient_only(shape, mode):
    """Backward for the input alone (frozen model, Sec. 4.3): dW, dgamma, dbeta NULL.  dX equals the full
    backward's bit for bit; any other mix of NULL outputs is refused before anything is launched."""
    from paper_2305_11624_amd import binding as B
    from paper_2305_11624_amd.runner import BlockRun
    inp = synth.make_inputs(shape)
    ref = oracle_block(inp)
    full = BlockRun(inp, mode=mode, poison=True)
    full.step()
    r = BlockRun(inp, mode=mode, poison=True)
    r.forward()
    fn = B.convbn_tune_bwd if mode == "tune" else B.convbn_eval_bwd
    saved = r.w_folded if mode == "tune" else r.y_saved
    fn(r.desc, r.x, r.W, None, r.gamma, r.mean, r.var, saved, r.dz, r.dx, None, None, None, None, r.ws_bwd)
    torch.cuda.synchronize()
    assert torch.equal(r.dx, full.dx)
    compare({"dX": B.act_from_device(r.dx)}, ref, shape.dtype, keys=("dX",), tag=f"{shape.name}/{mode}/dx-only")
    # refused mixes: dW without dgamma, dgamma without dW, nothing at all
    before = r.dx.clone()
    for dx, dW, dg, dbt in ((r.dx, r.dW, None, r.dbeta), (r.dx, None, r.dgamma, None), (None, None, None, None)):
        st = fn(r.desc, r.x, r.W, None, r.gamma, r.mean, r.var, saved, r.dz, dx, dW, None, dg, dbt, r.ws_bwd,
                check=False)
        assert st == B.ERR_NULL, st
    torch.cuda.synchronize()
    assert torch.equal(r.dx, before)


STRIDED = [
    # strided input gradients run as one stride-1 sweep per residue class of input positions when the
    # reduction (Cout) fits one channel chunk: odd sizes, classes without taps (1x1), even and large
    # windows, stride 3, no padding, rows / columns no window reaches
    BlockShape("b_s2_3x3", 2, 64, 15, 13, 64, 3, 2, 1, "bf16", 61),
    BlockShape("b_s2_1x1", 2, 72, 14, 11, 64, 1, 2, 0, "bf16", 62),
    BlockShape("b_s2_5x5", 2, 16, 17, 17, 64, 5, 2, 2, "bf16", 63),
    BlockShape("b_s2_2x2", 3, 24, 12, 12, 32, 2, 2, 0, "bf16", 64),
    BlockShape("b_s3_3x3", 2, 32, 16, 16, 64, 3, 3, 0, "bf16", 65),
    BlockShape("b_s3_5x5", 2, 40, 19, 14, 64, 5, 3, 1, "bf16", 66),
    BlockShape("b_s2_nopad", 2, 64, 10, 10, 32, 3, 2, 0, "bf16", 67),
    # several channel chunks with 1-, 2- and 4-tap class windows (fewer taps than the copy pipeline is
    # deep: the activation tiles then sit in a ring of three or more buffers)
    BlockShape("b_s2_3x3_deep", 2, 64, 15, 13, 192, 3, 2, 1, "bf16", 69),
    BlockShape("b_s3_5x5_deep", 2, 40, 19, 14, 128, 5, 3, 1, "bf16", 70),
    # more than 64 taps: the tile kernel keeps one table entry per tap in a lane and declines
    BlockShape("b_9x9", 1, 8, 20, 20, 16, 9, 1, 4, "bf16", 68),
]


@pytest.mark.parametrize("shape", STRIDED, ids=lambda s: s.name)
def test_bf16_strided_and_large_windows(shape):
    inp = synth.make_inputs(shape)
    ref = oracle_block(inp)
    compare(_run(inp, "tune"), ref, "bf16", tag=f"{shape.name}/tune")
