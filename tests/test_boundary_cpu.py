"""Host-side checks of the C boundary that need no GPU: the library loads,
exports every declared symbol, and turns bad input into error codes."""
import ctypes as ct
import os
import re

import numpy as np
import pytest

from paper_1705_09786_amd import binding as B
from paper_1705_09786_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_ARENA = 0x10000000          # never dereferenced on the host


def new_ctx(nbytes=1 << 30):
    return B.Amp(FAKE_ARENA, nbytes)


def test_every_declared_symbol_is_exported_and_bound():
    text = open(os.path.join(ROOT, "include", "amp.h")).read()
    declared = set(re.findall(r"\b(amp_[a-z_]+)\s*\(", text))
    assert declared, "no declarations found"
    lib = ct.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.SIGNATURES), declared ^ set(B.SIGNATURES)


def test_create_rejects_bad_arena():
    h = ct.c_void_p()
    L = B.lib()
    assert L.amp_create(ct.byref(h), None, 1 << 30, None) == B.AMP_EINVAL
    assert L.amp_create(ct.byref(h), ct.c_void_p(FAKE_ARENA + 4), 1 << 30, None) == B.AMP_EINVAL
    assert L.amp_create(ct.byref(h), ct.c_void_p(FAKE_ARENA), 1000, None) == B.AMP_EINVAL


def expect(code, fn, *a, **k):
    with pytest.raises(B.AmpError) as e:
        fn(*a, **k)
    assert e.value.code == code, e.value


def test_phase_and_argument_errors():
    a = new_ctx()
    expect(B.AMP_ESTATE, a.finalize, 4, 8, 0, 10)                     # before build
    expect(B.AMP_EINVAL, a.build, "mlp", dict(d_in=0, hidden=4, n_class=3))
    a.build("mlp", dict(d_in=5, hidden=4, n_class=3))
    expect(B.AMP_ESTATE, a.build, "mlp", dict(d_in=5, hidden=4, n_class=3))
    a.model = B.MODEL_MLP
    expect(B.AMP_ESTATE, a.submit, dict(x=np.zeros(5), label=0))      # before finalize
    expect(B.AMP_EINVAL, a.finalize, 0, 1, 0, 10)                     # mak < 1
    expect(B.AMP_EINVAL, a.set_min_update_frequency, -1, 0)           # muf < 1
    expect(B.AMP_EINVAL, a.set_min_update_frequency, 7, 1)            # no such node
    expect(B.AMP_EUNSUPPORTED, a.set_tiles, 0, 2)
    a.finalize(4, 1, 0, 3)
    expect(B.AMP_ESTATE, a.finalize, 4, 1, 0, 3)
    expect(B.AMP_EINVAL, a.set_max_active_keys, 5)
    expect(B.AMP_EINVAL, a.set_max_active_keys, 0)
    expect(B.AMP_EINVAL, a.set_params, 0, np.zeros(7))                # wrong size
    expect(B.AMP_EINVAL, a.submit, dict(x=np.zeros(4), label=0))      # wrong input size
    expect(B.AMP_EINVAL, a.submit, dict(x=np.zeros(5), label=3))      # label out of range
    for _ in range(3):
        a.submit(dict(x=np.zeros(5), label=1))
    expect(B.AMP_EFULL, a.submit, dict(x=np.zeros(5), label=1))
    expect(B.AMP_ESTATE, a.get_loss)
    expect(B.AMP_ESTATE, a.get_staleness_hist)
    # parameters set before training read back unchanged, with no device involved
    v = np.arange(4 * 5 + 4, dtype=np.float32)
    a.set_params(0, v)
    assert np.array_equal(a.get_params(0), v)


def test_arena_too_small_for_stash():
    a = new_ctx(1 << 20)
    a.build("rnn", synth.DEFAULT_DIMS["rnn"])
    expect(B.AMP_ENOMEM, a.finalize, 64, 32, 0, 100)


def test_tree_needs_tiles_that_fit_lds():
    a = new_ctx()
    a.build("tree", synth.DEFAULT_DIMS["tree"])
    a.set_tiles(1, 1)
    expect(B.AMP_EUNSUPPORTED, a.finalize, 4, 60, 0, 100)


def test_malformed_trees_and_graphs():
    a = new_ctx()
    a.build("tree", dict(vocab=10, emb=4, hidden=3, n_class=3))
    a.finalize(2, 4, 0, 10)
    good = dict(n_leaves=3, tokens=[1, 2, 3], left=[-1, -1, -1, 0, 3], right=[-1, -1, -1, 1, 2], labels=[0] * 5)
    a.submit(good)
    for patch in (dict(left=[-1, -1, -1, 0, 0]),          # node 3 never used, node 0 twice
                  dict(right=[-1, -1, -1, 1, 4]),         # child id not smaller than the node
                  dict(left=[-1, -1, -1, 3, 3]),          # child id not smaller than the node
                  dict(labels=[0] * 4),                   # wrong label count
                  dict(tokens=[1, 2, 10]),                # token out of range
                  dict(right=[-1, -1, -1, 0, 2])):        # both children the same
        bad = dict(good)
        bad.update(patch)
        expect(B.AMP_EINVAL, a.submit, bad)
    expect(B.AMP_EINVAL, a.submit, dict(n_leaves=5, tokens=[1] * 5, left=[-1] * 9, right=[-1] * 9, labels=[0] * 9))
    g = new_ctx()
    g.build("ggnn", dict(n_node_types=4, hidden=3, n_edge_types=2, n_steps=2))
    g.finalize(2, 4, 8, 10)
    ok = dict(n_nodes=3, node_type=[0, 1, 2], src=[0, 1, 1, 2], dst=[1, 0, 2, 1], etype=[0, 0, 1, 1], target=0.5)
    g.submit(ok)
    for patch in (dict(dst=[1, 0, 3, 1]),                 # edge index >= N
                  dict(etype=[0, 0, 2, 1]),               # edge type out of range
                  dict(src=[0, 1, 1, 1], dst=[1, 0, 0, 1]),   # node 2 has no incoming edge
                  dict(node_type=[0, 1, 4]),
                  dict(target=float("nan"))):
        bad = dict(ok)
        bad.update(patch)
        expect(B.AMP_EINVAL, g.submit, bad)


def test_replica_and_weight_placement_setters():
    a = new_ctx()
    expect(B.AMP_ESTATE, a.set_replicas, 2)                            # before build
    expect(B.AMP_ESTATE, a.set_weights_in_hbm, 1, True)
    a.build("tree", dict(vocab=11, emb=8, hidden=6, n_class=3))
    expect(B.AMP_EINVAL, a.set_replicas, 0)
    expect(B.AMP_EINVAL, a.set_replicas, 129)
    expect(B.AMP_EINVAL, a.set_weights_in_hbm, 9, True)                # no such node
    expect(B.AMP_EUNSUPPORTED, a.set_weights_in_hbm, 0, True)          # the lookup
    expect(B.AMP_EUNSUPPORTED, a.set_weights_in_hbm, 3, True)          # the output layer
    expect(B.AMP_EUNSUPPORTED, a.set_weights_in_hbm, 1, True)          # hidden 6 is no multiple of 4
    a.set_replicas(3)
    a.finalize(4, 5, 0, 10)
    expect(B.AMP_ESTATE, a.set_replicas, 2)                            # after finalize
    assert a.num_workers() == 3 * (1 + 1 + 5 + 8 + 1)                  # controller, lookup, leaf / branch tiles, output
    b = new_ctx()
    b.build("mlp", dict(d_in=5, hidden=4, n_class=3))
    expect(B.AMP_EUNSUPPORTED, b.set_weights_in_hbm, 1, True)          # only the tree cells
    c = new_ctx()
    c.build("tree", dict(vocab=11, emb=8, hidden=6, n_class=3))
    c.set_replicas(17)
    expect(B.AMP_EUNSUPPORTED, c.finalize, 4, 5, 0, 10)                # 17 x 16 workers exceed 256 workgroups


def test_admission_setter():
    a = new_ctx()
    expect(B.AMP_EINVAL, a.set_admission, 2, 1.0)                      # no such policy
    expect(B.AMP_EINVAL, a.set_admission, B.ADMIT_BOUNDED, -1.0)
    expect(B.AMP_EINVAL, a.set_admission, B.ADMIT_BOUNDED, float("nan"))
    a.set_admission(B.ADMIT_BOUNDED, 0.0)
    a.set_admission(B.ADMIT_GREEDY)
    assert a.get_admission() == dict(max_in_flight=0, final_limit=0)   # nothing trained yet


def test_measure_peaks_needs_a_buffer():
    import ctypes as ct
    x, y = ct.c_double(), ct.c_double()
    assert B.lib().amp_measure_peaks(None, 1 << 30, None, ct.byref(x), ct.byref(y)) == B.AMP_EINVAL
    assert B.lib().amp_measure_peaks(ct.c_void_p(4096), 1 << 20, None, ct.byref(x), ct.byref(y)) == B.AMP_EINVAL
