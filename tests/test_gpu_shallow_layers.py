"""GPU parity of shallow 3x3 / stride-1 layers (64 -> 64 channels, long pixel streams), whose forward convolution and
input gradient keep the whole weight and a workgroup's window rows in LDS: whole blocks against the oracle, with pixel
counts that leave ragged subtiles and ragged last workgroups, one or several rounds of workgroups, other paddings, a
bias and wide scales, and twice in a row on one workspace."""
import pytest
import torch

from paper_2305_11624_amd import synth
from paper_2305_11624_amd.synth import BlockShape

from helpers import compare, oracle_block

pytestmark = pytest.mark.gpu

SHAPES = [
    (BlockShape("shallow_47x53", 9, 64, 47, 53, 64, 3, 1, 1, "bf16", 81), dict()),                 # 88 pixels per workgroup
    (BlockShape("shallow_56x56", 11, 64, 56, 56, 64, 3, 1, 1, "bf16", 82), dict(bias=True)),       # 135: one wave takes two subtiles
    (BlockShape("shallow_56x56_rounds", 37, 64, 56, 56, 64, 3, 1, 1, "bf16", 83), dict(wide_scale=True)),   # two rounds
    (BlockShape("shallow_40x64_pad0", 13, 64, 40, 64, 64, 3, 1, 0, "bf16", 84), dict(bias=True)),
    (BlockShape("shallow_33x70_pad2", 10, 64, 33, 70, 64, 3, 1, 2, "bf16", 85), dict(bias=True, wide_scale=True)),
]


@pytest.mark.parametrize("shape,kw", SHAPES, ids=lambda v: v.name if hasattr(v, "name") else "")
@pytest.mark.parametrize("keep", [True, False], ids=["keeps_w", "keeps_nothing"])
def test_shallow_layer_block(shape, kw, keep):
    from paper_2305_11624_amd.runner import BlockRun
    inp = synth.make_inputs(shape, **kw)
    ref = oracle_block(inp)
    run = BlockRun(inp, mode="tune", keep_folded=keep, poison=True)
    run.step()
    compare(run.results(), ref, "bf16", tag=shape.name + "/first")
    first = {k: (None if v is None else v.clone()) for k, v in run.results().items()}
    run.step()   # same workspace again
    second = run.results()
    for k in ("Z", "dX", "dW", "dgamma", "dbeta"):
        assert torch.equal(first[k], second[k]), k
