"""The parity comparison itself, checked on the CPU: a result that differs from the checker's by one lost row
scatter of a lookup table, or by one wrong element of a dense tensor, must fail it, although the tensor's 2-norm
hides both."""
import numpy as np
import pytest

from oracle import amp as oamp
from paper_1705_09786_amd import synth

from util import compare


def _reference_run():
    dims = dict(vocab=2000, emb=24, hidden=16, n_class=5)
    data = synth.make_tree(12, 3, dims, max_leaves=8)
    fp = synth.init_params("tree", dims, 4)
    rt = oamp.Runtime("tree", dims, fp)
    rt.set_muf(3)
    rt.set_optimizer(kind="sgd", lr=0.05)
    rt.run(data, mak=4)
    as_gpu = dict(params=[p.astype(np.float32) for p in rt.params()], init=[np.asarray(v, np.float32) for v in fp],
                  losses=np.array([np.float32(rt.loss[s]) for s in range(len(data))], np.float64))
    return dims, data, rt, as_gpu


def test_compare_accepts_the_checkers_own_result_rounded_to_fp32():
    _, data, rt, g = _reference_run()
    compare(g, rt, len(data))


def test_compare_catches_one_lost_lookup_row():
    dims, data, rt, g = _reference_run()
    tok = int(data[0]["tokens"][0])
    table = g["params"][0].reshape(dims["vocab"], dims["emb"]).copy()
    init = g["init"][0].reshape(dims["vocab"], dims["emb"])
    assert not np.array_equal(table[tok], init[tok]), "the row was trained"
    table[tok] = init[tok]   # the scatter-add of this row never happened
    bad = dict(g, params=[table.reshape(-1)] + g["params"][1:])
    ref = rt.params()[0]
    assert np.linalg.norm(bad["params"][0] - ref) / np.linalg.norm(ref) < 1e-2   # small in the norm of the whole table
    with pytest.raises(AssertionError):
        compare(bad, rt, len(data))


def test_compare_catches_a_write_to_an_untouched_row():
    dims, data, rt, g = _reference_run()
    used = set(int(t) for i in data for t in i["tokens"])
    free = next(r for r in range(dims["vocab"]) if r not in used)
    table = g["params"][0].reshape(dims["vocab"], dims["emb"]).copy()
    table[free, 3] = np.nextafter(table[free, 3], np.float32(1))   # one bit, far below any tolerance
    bad = dict(g, params=[table.reshape(-1)] + g["params"][1:])
    with pytest.raises(AssertionError, match="untouched"):
        compare(bad, rt, len(data))


def test_compare_catches_one_wrong_element_of_a_dense_tensor():
    dims, data, rt, g = _reference_run()
    w = g["params"][2].copy()
    w[17] += np.float32(3e-4) * np.sqrt(np.mean(w.astype(np.float64) ** 2)).astype(np.float32)
    bad = dict(g, params=g["params"][:2] + [w] + g["params"][3:])
    ref = rt.params()[2]
    assert np.linalg.norm(w - ref) / np.linalg.norm(ref) <= 1e-5   # passes the per-tensor norm
    with pytest.raises(AssertionError):
        compare(bad, rt, len(data))
