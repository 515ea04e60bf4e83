"""GPU parity of the activation bits of the descriptor: a ReLU behind the block (forward output) and the backward mask
of a ReLU in front of it (input gradient), for every convolution kernel family the planner picks -- the ones that apply
them in their epilogue and the ones that get a pass of their own.  Reference: the oracle's block, with max(., 0) on its
Z and its dX zeroed where the block's input is not positive; and, bit for bit, the same calls without the bits followed
by the stand-alone element-wise kernels."""
import numpy as np
import pytest
import torch

from paper_2305_11624_amd import binding as B
from paper_2305_11624_amd import synth
from paper_2305_11624_amd.synth import BlockShape

from helpers import compare, oracle_block

pytestmark = pytest.mark.gpu

SHAPES = [
    BlockShape("act_pw_1x1", 6, 256, 20, 20, 64, 1, 1, 0, "bf16", 301),          # pointwise kernel
    BlockShape("act_pw_1x1_wide", 5, 64, 28, 28, 256, 1, 1, 0, "bf16", 302),
    BlockShape("act_pw_strided", 4, 256, 28, 28, 512, 1, 2, 0, "bf16", 303),      # a downsampling shortcut
    BlockShape("act_shallow_3x3", 9, 64, 47, 53, 64, 3, 1, 1, "bf16", 304),       # weight and window resident in LDS
    BlockShape("act_deep_3x3", 10, 512, 7, 7, 512, 3, 1, 1, "bf16", 305),         # deep-layer kernel, fused weight gradient
    BlockShape("act_mid_3x3", 6, 128, 28, 28, 128, 3, 1, 1, "bf16", 306),         # LDS-tile kernel
    BlockShape("act_mid_3x3_s2", 6, 128, 28, 28, 128, 3, 2, 1, "bf16", 307),      # strided: residue classes in the input gradient
    BlockShape("act_split_sums", 2, 256, 14, 14, 256, 3, 1, 1, "bf16", 308),      # split sums + their reduction
    BlockShape("act_stem", 2, 3, 64, 64, 64, 7, 2, 3, "bf16", 309),               # first layer: padded channels
    BlockShape("act_odd_bf16", 2, 24, 9, 11, 40, 3, 1, 1, "bf16", 310),           # generic kernels
    BlockShape("act_gm_fwd_256", 5, 128, 31, 33, 1024, 1, 1, 0, "bf16", 313),    # tiled matrix product, 256-pixel tiles, ragged tail
    BlockShape("act_gm_fwd_128", 5, 192, 31, 33, 512, 1, 1, 0, "bf16", 314),     # ... 128-pixel tiles, three chunks
    BlockShape("act_gm_bwd", 5, 1024, 31, 33, 128, 1, 1, 0, "bf16", 315),        # ... in the input gradient
    BlockShape("act_gm_one_fwd", 10, 64, 56, 55, 256, 1, 1, 0, "bf16", 316),     # ... single-chunk variant (64 reduced channels, long pixel range)
    BlockShape("act_gm_one_bwd", 10, 256, 56, 55, 64, 1, 1, 0, "bf16", 317),     # ... in the input gradient
    BlockShape("act_gm_two_fwd", 5, 128, 56, 55, 512, 1, 1, 0, "bf16", 318),     # ... two resident chunks
    BlockShape("act_gm_two_bwd", 5, 512, 56, 55, 128, 1, 1, 0, "bf16", 319),
    BlockShape("act_gm_64_one", 20, 64, 56, 55, 64, 1, 1, 0, "bf16", 320),       # ... 64-channel tiles, one resident chunk
    BlockShape("act_gm_64_two", 20, 128, 56, 55, 64, 1, 1, 0, "bf16", 321),      # ... two
    BlockShape("act_gm_strided", 30, 256, 27, 29, 512, 1, 2, 0, "bf16", 322),    # ... a downsampling shortcut: gathered / scattered rows
    BlockShape("act_f32", 2, 16, 12, 10, 24, 3, 1, 1, "f32", 311),
    BlockShape("act_f32_ragged", 1, 5, 7, 9, 7, 3, 2, 1, "f32", 312),             # element counts that are not multiples of 8
]
BOTH = B.ACT_RELU_OUT | B.ACT_RELU_IN


def _inputs(shape):
    inp = synth.make_inputs(shape, bias=True)
    inp["x"] = torch.clamp(inp["x"], min=0)   # the block's input is a ReLU's output: about half of it zero
    return inp


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("mode,keep", [("tune", True), ("tune", False), ("eval", True)],
                         ids=["tune_keeps_w", "tune_keeps_nothing", "eval"])
def test_activation_bits_against_oracle_and_unfused_calls(shape, mode, keep):
    from paper_2305_11624_amd.runner import BlockRun
    inp = _inputs(shape)
    ref = oracle_block(inp)
    x = inp["x"].double().numpy()
    ref["Z"] = np.maximum(ref["Z"], 0)
    ref["dX"] = ref["dX"] * (x > 0)
    run = BlockRun(inp, mode=mode, keep_folded=keep, poison=True, act=BOTH)
    run.step()
    got = run.results()
    compare(got, ref, shape.dtype, tag=shape.name + "/" + mode)

    plain = BlockRun(inp, mode=mode, keep_folded=keep, poison=True, act=0)
    plain.step()
    B.convbn_aux_eltwise(B.OP_RELU, plain.z)
    B.convbn_aux_eltwise(B.OP_RELU_BWD, plain.dx, plain.x)
    want = plain.results()
    for k in ("Z", "dX", "dW", "dgamma", "dbeta", "db"):
        assert torch.equal(got[k], want[k]), k


@pytest.mark.parametrize("shape", [SHAPES[0], SHAPES[3], SHAPES[5], SHAPES[8], SHAPES[10], SHAPES[12], SHAPES[13], SHAPES[14], SHAPES[15], SHAPES[18]], ids=lambda s: s.name)
def test_step_entry_points_with_activation(shape):
    """convbn_conv_fprop with the output bit and convbn_conv_dgrad_masked, against the same calls plus element-wise passes."""
    from paper_2305_11624_amd.runner import BlockRun
    inp = _inputs(shape)
    r = BlockRun(inp, "tune")
    d = r.desc
    P = shape.Cout * shape.K
    dev = r.x.device
    w_fprop = torch.empty(P, dtype=r.dt, device=dev)
    w_t = torch.empty(P, dtype=r.dt, device=dev)
    bfold = torch.empty(shape.Cout, dtype=torch.float32, device=dev)
    B.convbn_fold(d, r.W, r.b, r.gamma, r.beta, r.mean, r.var, w_fprop, w_t, bfold)
    ws = torch.empty(max(16, B.convbn_conv_workspace_bytes(d, B.PASS_FWD), B.convbn_conv_workspace_bytes(d, B.PASS_BWD)),
                     dtype=torch.uint8, device=dev)
    z0, z1 = torch.empty_like(r.z), torch.empty_like(r.z)
    dx0, dx1 = torch.empty_like(r.dx), torch.empty_like(r.dx)
    B.convbn_conv_fprop(d, r.x, w_fprop, bfold, z0, ws)
    B.convbn_aux_eltwise(B.OP_RELU, z0)
    B.convbn_conv_dgrad(d, r.dz, w_t, dx0, ws)
    B.convbn_aux_eltwise(B.OP_RELU_BWD, dx0, r.x)
    d.act = B.ACT_RELU_OUT
    B.convbn_conv_fprop(d, r.x, w_fprop, bfold, z1, ws)
    B.convbn_conv_dgrad(d, r.dz, w_t, dx1, ws, x_mask=r.x)
    torch.cuda.synchronize()
    assert torch.equal(z0, z1)
    assert torch.equal(dx0, dx1)
    assert (z1.float() >= 0).all() and (dx1.float()[r.x.float() <= 0] == 0).all()


def _addends(shape, run_like):
    """Seeded tensors laid out like z and dx (a shortcut branch and the gradient of a second consumer of x)."""
    g = torch.Generator().manual_seed(shape.seed + 7000)
    a_out = torch.randn((shape.N, shape.Cout, shape.Hout, shape.Wout), generator=g, dtype=torch.float32)
    a_in = torch.randn((shape.N, shape.Cin, shape.Hin, shape.Win), generator=g, dtype=torch.float32)
    if shape.dtype == "bf16":
        a_out, a_in = a_out.bfloat16().float(), a_in.bfloat16().float()
    dev = "cuda"
    return (a_out, a_in, B.act_to_device(a_out, run_like, dev), B.act_to_device(a_in, run_like, dev))


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("mode,keep", [("tune", True), ("tune", False), ("eval", True)],
                         ids=["tune_keeps_w", "tune_keeps_nothing", "eval"])
@pytest.mark.parametrize("relu", [True, False], ids=["add_relu", "add_only"])
def test_residual_addends_against_oracle_and_unfused_calls(shape, mode, keep, relu):
    """ACT_ADD_OUT / ACT_ADD_IN: a residual sum behind the block and a second gradient branch at its input, with and
    without the ReLU bits.  Reference: the oracle's block with the addends applied to its Z and dX in fp64; and, bit for
    bit, the plain calls followed by the stand-alone element-wise kernels."""
    from paper_2305_11624_amd.runner import BlockRun
    inp = _inputs(shape)
    dt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
    a_out, a_in, d_out, d_in = _addends(shape, dt)
    ref = oracle_block(inp)
    x = inp["x"].double().numpy()
    ref["Z"] = ref["Z"] + a_out.double().numpy()
    ref["dX"] = ref["dX"] + a_in.double().numpy()
    if relu:
        ref["Z"] = np.maximum(ref["Z"], 0)
        ref["dX"] = ref["dX"] * (x > 0)
    act = B.ACT_ADD_OUT | B.ACT_ADD_IN | (BOTH if relu else 0)
    run = BlockRun(inp, mode=mode, keep_folded=keep, poison=True, act=act, add_out=d_out, add_in=d_in)
    run.step()
    got = run.results()
    compare(got, ref, shape.dtype, tag=shape.name + "/" + mode + ("/relu" if relu else ""))

    plain = BlockRun(inp, mode=mode, keep_folded=keep, poison=True, act=0)
    plain.step()
    if relu:
        B.convbn_aux_eltwise(B.OP_ADD_RELU, plain.z, d_out)
        B.convbn_aux_add_relu_bwd(plain.dx, d_in, plain.x)
    else:
        B.convbn_aux_eltwise(B.OP_ADD, plain.z, d_out)
        B.convbn_aux_eltwise(B.OP_ADD, plain.dx, d_in)
    want = plain.results()
    for k in ("Z", "dX", "dW", "dgamma", "dbeta", "db"):
        assert torch.equal(got[k], want[k]), k


def test_addend_bit_without_a_tensor_is_refused():
    from paper_2305_11624_amd.runner import BlockRun
    run = BlockRun(_inputs(SHAPES[0]), mode="tune")
    run.desc.act = B.ACT_ADD_OUT
    with pytest.raises(B.ConvBNError):
        run.forward()
    run.desc.act = B.ACT_ADD_IN
    with pytest.raises(B.ConvBNError):
        run.backward()
