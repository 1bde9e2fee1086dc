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


# ---------------------------------------------------------------- generic graph construction
def mlp_graph(a, d_in=5, hidden=4, n_class=3, hidden2=None):
    """The pipelined MLP as a caller describes it: controller -> Linear+ReLU -> Linear+ReLU -> Linear -> loss."""
    l1 = a.add_node("linear", hidden, d_in, aux=B.ACT_RELU)
    l2 = a.add_node("linear", hidden, hidden2 or hidden, aux=B.ACT_RELU)
    l3 = a.add_node("linear", n_class, hidden)
    loss = a.add_node("softmax_xent", n_class)
    a.connect(0, 0, l1, 0)
    a.connect(l1, 0, l2, 0)
    a.connect(l2, 0, l3, 0)
    a.connect(l3, 0, loss, 0)
    a.connect(0, 1, loss, 1)
    return l1, l2, l3, loss


def rnn_graph(a, vocab=6, emb=3, hidden=4, n_class=3, loop_through_phi=True):
    """Figure 2's loop, nodes added in another order than the model numbers them."""
    out = a.add_node("linear", n_class, hidden)
    loss = a.add_node("softmax_xent", n_class)
    cond = a.add_node("cond", n_out=2)
    isu = a.add_node("isu")
    cell = a.add_node("rnn_tanh", hidden, emb + hidden)
    cat = a.add_node("concat", n_in=2)
    lk = a.add_node("lookup", vocab, emb)
    a.connect(0, 0, lk, 0)
    if loop_through_phi:
        phi = a.add_node("phi", n_in=2)
        a.connect(0, 1, phi, 0)
        a.connect(0, 2, loss, 1)
        a.connect(phi, 0, cat, 1)
        a.connect(cond, 0, phi, 1)
    else:
        a.connect(0, 1, loss, 1)
        a.connect(cond, 0, cat, 1)      # the loop closes without a Phi
    a.connect(lk, 0, cat, 0)
    a.connect(cat, 0, cell, 0)
    a.connect(cell, 0, isu, 0)
    a.connect(isu, 0, cond, 0)
    a.connect(cond, 1, out, 0)
    a.connect(out, 0, loss, 0)
    return dict(lookup=lk, cell=cell, out=out, loss=loss)


def test_hand_built_graphs_are_recognised():
    a = new_ctx()
    l1, l2, l3, loss = mlp_graph(a)
    a.validate_graph("mlp")
    assert a.num_nodes() == 3
    assert [a.get_node_index(n) for n in (l1, l2, l3, loss, 0)] == [0, 1, 2, -1, -1]
    a.finalize(4, 1, 0, 3)
    a.set_params(1, np.zeros(4 * 4 + 4, np.float32))
    # the recurrent model, nodes added back to front: the parameterized nodes still carry the model's numbering
    b = new_ctx()
    ids = rnn_graph(b)
    b.finalize(4, 8, 0, 3)                 # finalize validates a graph that has not been validated yet
    assert b.num_nodes() == 3
    assert [b.get_node_index(ids[k]) for k in ("lookup", "cell", "out", "loss")] == [0, 1, 2, -1]
    b.set_params(1, np.zeros(4 * 7 + 4, np.float32))


def test_graph_errors_the_host_can_force():
    # dangling port: the label never reaches the loss layer
    a = new_ctx()
    l1 = a.add_node("linear", 4, 5, aux=B.ACT_RELU)
    loss = a.add_node("softmax_xent", 4)
    a.connect(0, 0, l1, 0)
    a.connect(l1, 0, loss, 0)
    with pytest.raises(B.AmpError, match="dangling port") as e:
        a.validate_graph()
    assert e.value.code == B.AMP_EINVAL
    # dimension mismatch: the second layer takes 6 values, the first sends 4
    a = new_ctx()
    mlp_graph(a, hidden2=6)
    with pytest.raises(B.AmpError, match="dimension mismatch") as e:
        a.validate_graph()
    assert e.value.code == B.AMP_EINVAL
    # a cycle that does not pass through a Phi
    a = new_ctx()
    rnn_graph(a, loop_through_phi=False)
    with pytest.raises(B.AmpError, match="cycle without a Phi") as e:
        a.finalize(4, 8, 0, 3)
    assert e.value.code == B.AMP_EINVAL
    # a port connected twice; nodes and ports that do not exist; the controller's ports go in order
    a = new_ctx()
    l1 = a.add_node("linear", 4, 5)
    l2 = a.add_node("linear", 4, 4)
    a.connect(0, 0, l1, 0)
    a.connect(l1, 0, l2, 0)
    a.connect(l1, 0, l2, 0)
    with pytest.raises(B.AmpError, match="connected twice"):
        a.validate_graph()
    a = new_ctx()
    l1 = a.add_node("linear", 4, 5)
    expect(B.AMP_EINVAL, a.connect, l1, 0, 9, 0)
    expect(B.AMP_EINVAL, a.connect, 0, 3, l1, 0)
    expect(B.AMP_EINVAL, a.connect, l1, 0, 0, 0)          # nothing connects into the controller
    d = B.NodeDesc(1, 1, 1, 1, 0)
    nid = ct.c_int()
    assert a.L.amp_add_node(a.h, 99, ct.byref(d), ct.byref(nid)) == B.AMP_EINVAL
    assert a.L.amp_add_node(a.h, 0, ct.byref(d), ct.byref(nid)) == B.AMP_EINVAL   # the controller exists already
    # a valid graph the kernel has no workers for: a perceptron with one more layer
    a = new_ctx()
    ls = [a.add_node("linear", 4, 5, aux=B.ACT_RELU)] + [a.add_node("linear", 4, 4, aux=B.ACT_RELU) for _ in range(2)]
    ls.append(a.add_node("linear", 3, 4))
    loss = a.add_node("softmax_xent", 3)
    a.connect(0, 0, ls[0], 0)
    for x, y in zip(ls[:-1], ls[1:]):
        a.connect(x, 0, y, 0)
    a.connect(ls[-1], 0, loss, 0)
    a.connect(0, 1, loss, 1)
    with pytest.raises(B.AmpError) as e:
        a.validate_graph()
    assert e.value.code == B.AMP_EUNSUPPORTED
    # phases: no nodes after a model is built, no canned model on top of added nodes
    a = new_ctx()
    a.build("mlp", dict(d_in=5, hidden=4, n_class=3))
    expect(B.AMP_ESTATE, a.add_node, "linear", 4, 4)
    expect(B.AMP_ESTATE, a.connect, 0, 0, 1, 0)
    a = new_ctx()
    a.add_node("linear", 4, 4)
    expect(B.AMP_ESTATE, a.build, "mlp", dict(d_in=5, hidden=4, n_class=3))


def test_hand_built_tree_and_graph_network():
    """The two larger graphs written out by a caller: Tree-LSTM (Section 6) and the gated graph network of Figure
    4(a) with two edge types and three propagation steps."""
    H, E, V, C = 6, 5, 11, 3
    a = new_ctx()
    lk, leaf, br = a.add_node("lookup", V, E), a.add_node("leaf_lstm", H, E), a.add_node("branch_lstm", H)
    out, loss = a.add_node("linear", C, H), a.add_node("softmax_xent", C)
    phi, bc, sp = a.add_node("phi", n_in=2), a.add_node("bcast", n_out=2), a.add_node("split", n_out=2)
    csink, cond, rsink = a.add_node("sink"), a.add_node("cond", n_out=2), a.add_node("sink")
    isu, cat = a.add_node("isu"), a.add_node("concat", n_in=1, aux=2)
    a.connect(0, 0, lk, 0)
    a.connect(0, 1, loss, 1)
    for s, sp_, d, dp in [(lk, 0, leaf, 0), (leaf, 0, phi, 0), (br, 0, phi, 1), (phi, 0, bc, 0), (bc, 0, sp, 0), (sp, 0, out, 0),
                          (sp, 1, csink, 0), (out, 0, loss, 0), (bc, 1, cond, 0), (cond, 0, rsink, 0), (cond, 1, isu, 0),
                          (isu, 0, cat, 0), (cat, 0, br, 0)]:
        a.connect(s, sp_, d, dp)
    a.validate_graph("tree")
    assert a.num_nodes() == 4 and [a.get_node_index(n) for n in (lk, leaf, br, out)] == [0, 1, 2, 3]
    n = ct.c_size_t()
    assert a.L.amp_param_count(a.h, 2, ct.byref(n)) == 0 and n.value == 5 * H * 2 * H + 5 * H

    g = new_ctx()
    T, S, ne = 4, 3, 2
    lk = g.add_node("lookup", T, H)
    lin = [g.add_node("ggnn_edge_linear", H, H) for _ in range(ne)]
    gru, ro, loss = g.add_node("gru", H), g.add_node("sum_readout", 1, H), g.add_node("squared_err")
    phi_h, bc, ung, fm = g.add_node("phi", n_in=2), g.add_node("bcast", n_out=2), g.add_node("ungroup"), g.add_node("flatmap")
    bytype, phi_e = g.add_node("cond", n_out=ne), g.add_node("phi", n_in=ne)
    bydst, sm, alln, isu = g.add_node("group"), g.add_node("sum"), g.add_node("group"), g.add_node("isu")
    done = g.add_node("cond", n_out=2, aux=S)
    g.connect(0, 0, lk, 0)
    g.connect(0, 1, loss, 1)
    edges = [(lk, 0, phi_h, 0), (phi_h, 0, bc, 0), (bc, 0, ung, 0), (ung, 0, fm, 0), (fm, 0, bytype, 0)]
    for c in range(ne):
        grp, ungc = g.add_node("group"), g.add_node("ungroup")
        edges += [(bytype, c, grp, 0), (grp, 0, lin[c], 0), (lin[c], 0, ungc, 0), (ungc, 0, phi_e, c)]
    edges += [(phi_e, 0, bydst, 0), (bydst, 0, sm, 0), (sm, 0, alln, 0), (alln, 0, gru, 0), (bc, 1, gru, 1), (gru, 0, isu, 0),
              (isu, 0, done, 0), (done, 0, phi_h, 1), (done, 1, ro, 0), (ro, 0, loss, 0)]
    for e in edges:
        g.connect(*e)
    g.validate_graph("ggnn")
    assert g.num_nodes() == 1 + ne + 3 + 1
    assert [g.get_node_index(x) for x in [lk] + lin + [gru, ro]] == [0, 1, 2, 3, 6]
    g.finalize(4, 9, 24, 5)
    g.submit(dict(n_nodes=2, node_type=np.array([0, 1]), src=np.array([0, 1]), dst=np.array([1, 0]), etype=np.array([1, 1]),
                  target=0.5))


def test_node_replicas_on_the_host():
    """Replicas of one heavy node (Section 5): built for the RNN's cell; the copies are nodes of their own that
    follow what is set on the node they copy."""
    rnn = dict(vocab=6, emb=3, hidden=4, n_class=3)
    a = new_ctx()
    expect(B.AMP_ESTATE, a.set_node_replicas, 1, 2)                    # before build
    expect(B.AMP_ESTATE, a.set_group_sync, 10)
    a.build("mlp", dict(d_in=5, hidden=4, n_class=3))
    expect(B.AMP_EUNSUPPORTED, a.set_node_replicas, 1, 2)              # another model
    a.close()
    a = new_ctx()
    a.build("rnn", rnn)
    expect(B.AMP_EUNSUPPORTED, a.set_node_replicas, 2, 2)              # the output layer
    expect(B.AMP_EINVAL, a.set_node_replicas, 1, 0)
    expect(B.AMP_EINVAL, a.set_node_replicas, 1, 65)
    a.set_node_replicas(1, 3)
    assert a.num_nodes() == 7
    a.set_node_replicas(1, 2)                                          # asked again: replaces the earlier copies
    assert a.num_nodes() == 5
    expect(B.AMP_EINVAL, a.set_group_sync, -1)
    a.set_group_sync(50)                                               # a synchronisation request every 50 retirements
    a.set_replicas(2)
    expect(B.AMP_EUNSUPPORTED, a.finalize, 4, 5, 0, 10)                # both kinds of replica at once
    a.set_replicas(1)
    a.finalize(4, 5, 0, 10)
    assert a.num_workers() == 4                                        # controller, cell, output layer, one copy
    expect(B.AMP_ESTATE, a.set_node_replicas, 1, 2)                    # after finalize
    fp = synth.init_params("rnn", rnn, 3)
    a.set_params(1, fp[1])
    assert np.array_equal(a.get_params(4), fp[1]) and np.array_equal(a.get_params(1), fp[1])   # the copy follows
    a.set_params(4, fp[1] + 1)                                         # a copy's own id works too
    assert np.array_equal(a.get_params(4), fp[1] + 1) and np.array_equal(a.get_params(1), fp[1])
    a.close()
