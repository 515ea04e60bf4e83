"""GPU parity of deep 3x3 layers (many channels, few pixels), whose backward runs the weight gradient and the
fold-back in one launch (partial dot products exchanged between workgroups through slots that carry the launch's
tag, finished by the workgroup that finds all of them in place): whole blocks against the oracle with ragged pixel
tails, other paddings, a bias and wide scales, twice in a row on one workspace (the slots of the first call are
stale for the second), and replayed from a captured graph."""
import pytest
import torch

from paper_2305_11624_amd import synth
from paper_2305_11624_amd.synth import BlockShape

from helpers import compare, oracle_block

pytestmark = pytest.mark.gpu

SHAPES = [
    (BlockShape("deep_7x7_512", 37, 512, 7, 7, 512, 3, 1, 1, "bf16", 61), dict()),               # ragged tail
    (BlockShape("deep_7x7_512_bias", 19, 512, 7, 7, 512, 3, 1, 1, "bf16", 66), dict(bias=True, wide_scale=True)),
    (BlockShape("deep_14x14_256", 41, 256, 14, 14, 256, 3, 1, 1, "bf16", 62), dict(bias=True)),   # 4 splits
    (BlockShape("deep_28x28_128", 21, 128, 28, 28, 128, 3, 1, 1, "bf16", 63), dict(wide_scale=True)),   # 2 splits
    (BlockShape("deep_13x11_pad0", 70, 256, 13, 11, 128, 3, 1, 0, "bf16", 64), dict()),
    (BlockShape("deep_9x12_pad2", 56, 128, 9, 12, 384, 3, 1, 2, "bf16", 65), dict(bias=True)),
]


@pytest.mark.parametrize("shape,kw", SHAPES, ids=lambda v: v.name if hasattr(v, "name") else "")
def test_deep_layer_block(shape, kw):
    from paper_2305_11624_amd.runner import BlockRun
    inp = synth.make_inputs(shape, **kw)
    ref = oracle_block(inp)
    run = BlockRun(inp, mode="tune", poison=True)
    run.step()
    compare(run.results(), ref, "bf16", tag=shape.name + "/first")
    first = {k: (None if v is None else v.clone()) for k, v in run.results().items()}
    run.step()   # same workspace again
    second = run.results()
    compare(second, ref, "bf16", tag=shape.name + "/second")
    for k in ("Z", "dX", "dW", "dgamma", "dbeta"):   # split sums and partial dot products are combined in a fixed order
        assert torch.equal(first[k], second[k]), k


@pytest.mark.parametrize("kw", [dict(), dict(bias=True, wide_scale=True)], ids=["plain", "bias_wide_scale"])
def test_deep_layer_that_keeps_nothing(kw):
    """A block whose w' is larger than its output keeps nothing between the passes (P > A_z): forward then needs no
    folded weight at all (the scale and the folded bias are applied in the convolution's epilogue) and backward folds
    again.  Same definition, same tolerances."""
    from paper_2305_11624_amd.runner import BlockRun
    shape = BlockShape("deep_refold", 35, 512, 7, 7, 512, 3, 1, 1, "bf16", 67)
    assert shape.P > shape.A_z
    inp = synth.make_inputs(shape, **kw)
    ref = oracle_block(inp)
    run = BlockRun(inp, mode="tune", keep_folded=False, poison=True)
    run.step()
    res = run.results()
    assert res["Wf"] is None
    compare(res, ref, "bf16", tag="deep_refold")


def test_deep_layer_replayed_from_a_graph():
    """A captured step replays with the same arguments, the launch tag of the workgroup exchange among them: each
    replay must find the slots of the previous one cleared.  Three replays over changing inputs, eager work and
    synchronisations in between, each compared bit for bit with an eager step on the same inputs."""
    from paper_2305_11624_amd import binding as B
    from paper_2305_11624_amd.runner import BlockRun
    shapes = [BlockShape("deep_graph", 33, 512, 7, 7, 512, 3, 1, 1, "bf16", 70 + i) for i in range(2)]
    inps = [synth.make_inputs(s, bias=True) for s in shapes]
    assert B.convbn_tune_bwd_is_fused(B.desc_from_shape(shapes[0], eps=inps[0]["eps"]))
    eager = []
    for inp in inps:
        run = BlockRun(inp, mode="tune", keep_folded=False)
        run.step()
        eager.append(run.results())
    sources = [BlockRun(inp, mode="tune", keep_folded=False) for inp in inps]
    run = BlockRun(inps[0], mode="tune", keep_folded=False, poison=True)
    fields = ("x", "dz", "W", "b", "gamma", "beta", "mean", "var")
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        run.step()
    for which in (0, 1, 1, 0):
        for f in fields:
            getattr(run, f).copy_(getattr(sources[which], f))
        for t in (run.z, run.dx, run.dW, run.dgamma, run.dbeta, run.db):
            t.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        got = run.results()
        for k in ("Z", "dX", "dW", "dgamma", "dbeta", "db"):
            assert torch.equal(got[k], eager[which][k]), (which, k)
