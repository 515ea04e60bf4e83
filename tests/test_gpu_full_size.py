"""GPU parity at the benchmark's full sizes and launch configurations (the single-block
configurations 1-3 of the benchmark), every output element against the oracle."""
import pytest

from paper_2305_11624_amd import synth

from helpers import compare, oracle_block

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["c1", "c2a", "c2b", "c3a", "c3b"])
def test_full_size_tune(name):
    from paper_2305_11624_amd.runner import BlockRun
    inp = synth.make_inputs(synth.CONFIGS[name])
    ref = oracle_block(inp)
    run = BlockRun(inp, mode="tune", poison=True)
    run.step()
    compare(run.results(), ref, "bf16", tag=f"{name}/tune")


@pytest.mark.parametrize("name", ["c2a", "c3b"])
def test_full_size_eval(name):
    from paper_2305_11624_amd.runner import BlockRun
    inp = synth.make_inputs(synth.CONFIGS[name])
    ref = oracle_block(inp)
    run = BlockRun(inp, mode="eval", poison=True)
    run.step()
    compare(run.results(), ref, "bf16", tag=f"{name}/eval")


def test_wide_image_128_channels():
    """A 3x3 layer on a wide image with 128 output channels (not among the benchmark's shapes): whole-row
    tiles with four channel subtiles per wave forward, whole-row tiles with two channel chunks backward."""
    from paper_2305_11624_amd.runner import BlockRun
    from paper_2305_11624_amd.synth import BlockShape
    inp = synth.make_inputs(BlockShape("wide_128", 32, 64, 56, 56, 128, 3, 1, 1, "bf16", 91))
    ref = oracle_block(inp)
    run = BlockRun(inp, mode="tune", poison=True)
    run.step()
    compare(run.results(), ref, "bf16", tag="wide_128/tune")


def _distinct_backbone_shapes():
    """One block per distinct layer shape of the ResNet-50 backbone at the benchmarked batch (N = 32, 224 x 224)."""
    seen, out = set(), []
    for s in synth.resnet50_blocks(32, 224, "bf16"):
        key = (s.Cin, s.Hin, s.Cout, s.k, s.stride)
        if key not in seen:
            seen.add(key)
            out.append(s)
    return out


BACKBONE_SHAPES = _distinct_backbone_shapes()


def test_backbone_has_23_distinct_shapes():
    assert len(BACKBONE_SHAPES) == 23


@pytest.mark.parametrize("shape", BACKBONE_SHAPES, ids=lambda s: s.name)
def test_backbone_layer_at_bench_size(shape):
    """Every distinct layer shape of the backbone workload at the batch the benchmark times, so that the plan the
    host picks for it (tile shape, split sums, pointwise or window kernel) is the one compared: Z, dX, dW, dgamma
    and dbeta against the definition, every element, in Tune mode and on the Eval comparison path."""
    from paper_2305_11624_amd.runner import BlockRun
    inp = synth.make_inputs(shape)
    ref = oracle_block(inp)
    for mode in ("tune", "eval"):
        run = BlockRun(inp, mode=mode, poison=True)
        run.step()
        compare(run.results(), ref, "bf16", tag=f"{shape.name}/{mode}")
        del run
