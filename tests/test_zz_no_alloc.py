"""The forward entry point that allocates nothing (its workspace is a device array built into the library): called
through the C ABI twice in a row, the second time on a smaller block, and compared with convbn_tune_fwd on the same
inputs and with the oracle."""
import pytest
import torch

from paper_2305_11624_amd import synth
from paper_2305_11624_amd.synth import BlockShape

from helpers import TOL, oracle_block, rel_err

pytestmark = pytest.mark.gpu

FIRST = BlockShape("na_big", 8, 256, 14, 14, 256, 3, 1, 1, "bf16", 71)      # split sums: part of the workspace is fp32 partials
SECOND = BlockShape("na_small", 2, 64, 9, 11, 72, 3, 1, 1, "bf16", 72)


def _run(shape, B):
    inp = synth.make_inputs(shape, bias=True)
    desc = B.desc_from_shape(shape, eps=inp["eps"])
    dt = torch.bfloat16
    x = B.act_to_device(inp["x"], dt)
    W = B.weight_to_device(inp["W"], dt)
    vec = {k: B.vec_to_device(inp[k]) for k in ("b", "gamma", "beta", "rmean", "rvar")}
    P = shape.Cout * shape.K
    outs = []
    for static in (False, True):
        z = torch.full((shape.N, shape.Hout, shape.Wout, shape.Cout), float("nan"), dtype=dt, device="cuda")
        wf = torch.full((P,), float("nan"), dtype=dt, device="cuda")
        args = (desc, x, W, vec["b"], vec["gamma"], vec["beta"], vec["rmean"], vec["rvar"], z, wf)
        if static:
            before = torch.cuda.memory_allocated()
            B.convbn_tune_fwd_static(*args)
            assert torch.cuda.memory_allocated() == before
        else:
            n = B.convbn_workspace_bytes(desc, B.MODE_TUNE, B.PASS_FWD)
            assert n <= B.convbn_static_workspace_limit()
            ws = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
            B.convbn_tune_fwd(*args, ws)
        torch.cuda.synchronize()
        outs.append((z, wf))
    (z0, w0), (z1, w1) = outs
    assert torch.equal(w0, w1)
    assert rel_err(z1.float().cpu(), z0.float().cpu().numpy()) <= TOL["bf16"]
    ref = oracle_block(inp, need_dx=False)
    assert rel_err(B.act_from_device(z1), ref["Z"]) <= TOL["bf16"]
    assert rel_err(B.folded_from_device(w1.view(shape.Cin, shape.k, shape.k, shape.Cout)), ref["Wf"]) <= TOL["bf16"]


def test_static_workspace_forward_two_calls_in_a_row():
    from paper_2305_11624_amd import binding as B
    _run(FIRST, B)
    _run(SECOND, B)     # a smaller block right after: the array still holds the first call's bytes


def test_static_workspace_forward_refuses_blocks_beyond_its_limit():
    from paper_2305_11624_amd import binding as B
    d = B.make_desc(1, 4096, 4, 4, 4096, 3, 3, 1, 1)      # w' alone is 302 MB
    assert B.convbn_workspace_bytes(d, B.MODE_TUNE, B.PASS_FWD) > B.convbn_static_workspace_limit()
    t = torch.zeros(16, device="cuda", dtype=torch.bfloat16)
    v = torch.zeros(16, device="cuda")
    st = B.convbn_tune_fwd_static(d, t, t, None, v, v, v, v, t, None, check=False)
    assert st == B.ERR_WORKSPACE
    assert "built-in" in B.convbn_last_error()
