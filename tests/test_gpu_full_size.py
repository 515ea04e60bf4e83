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
