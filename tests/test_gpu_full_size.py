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
