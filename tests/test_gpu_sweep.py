"""Three cells of the asynchrony sweep (Section 6, "Asynchrony", Figure 7; Appendix B on the greedy controller):
an 8-replica RNN on the synthetic list reduction, trained until 96 % validation accuracy.

  * a moderate setting (8 keys in flight per replica, an update every 16 gradients) converges in a few epochs;
  * 64 keys in flight with an update after every gradient does not under the greedy controller: the gradients are
    too stale (the paper's instability at a high max_active_keys);
  * the same cell with the staleness-bounded admission converges, with far fewer keys in flight than allowed.

With AMP_SWEEP_OUT set the cell results are also written there as JSON."""
import json
import os

import pytest

from paper_1705_09786_amd import sweep, synth

pytestmark = pytest.mark.gpu


def test_three_cells_of_the_asynchrony_sweep():
    dims = synth.DEFAULT_DIMS["rnn"]
    data = synth.make_rnn(10000, synth.BASE_SEED + 20, dims, 2, 10, reduction="max")
    valid = synth.make_rnn(1000, synth.BASE_SEED + 1020, dims, 2, 10, reduction="max")
    fp = synth.init_params("rnn", dims, 102)
    good = sweep.run_one(data, valid, dims, fp, 8, 8, 16, 0.001, 15)
    stale = sweep.run_one(data, valid, dims, fp, 8, 64, 1, 0.001, 15)
    bounded = sweep.run_one(data, valid, dims, fp, 8, 64, 1, 0.001, 15, bounded=8.0)
    rows = dict(moderate=good, greedy_stale=stale, bounded=bounded)
    print(json.dumps(rows))
    if os.environ.get("AMP_SWEEP_OUT"):
        with open(os.environ["AMP_SWEEP_OUT"], "w") as f:
            json.dump(rows, f, indent=1)
    assert good["converged"] and good["epochs"] <= 10, good
    assert not stale["converged"] and stale["valid_accuracy"] < 0.9, stale
    assert bounded["converged"] and bounded["epochs"] <= 12, bounded
    assert bounded["max_in_flight"] < 32, bounded           # the controller held the number in flight down
    assert stale["max_in_flight"] == 64
