"""The whole stack in one loop: LVF decides, the block table rotates with eager
copies, the reader stands in for model execution on its own stream.  Short run
on a small cache so that requests really rotate."""
import pytest

from paper_2601_20309_amd import experiments as X

pytestmark = pytest.mark.gpu


def test_cross_iteration_pipeline_runs_and_keeps_synced_blocks_valid():
    # a fixed link budget: derived from measured times it would make the schedule depend on the box's timing
    out = X.serve(rps=400.0, seconds=0.8, seed=3, b_xfer=64, hbm_blocks=768, host_slots=4096)
    c = out["counts"]
    assert out["iterations"] > 50
    assert c["swapped_in"] > 0 and c["dropped_synced"] > 0 and c["copied_eager"] > 0
    # eager rotation makes most preemptions free of copies (Section 4.3.2)
    assert c["dropped_synced"] > 4 * c["copied_preempt"]
