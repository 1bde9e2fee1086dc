"""The boundary's diagnostics on the GPU: the staleness histogram (Section 3's definition: the number of updates
a node applies between a message's forward and backward pass) and the per-worker utilisation counters."""
import numpy as np
import pytest

from oracle import amp as oamp
from paper_1705_09786_amd import synth

from util import gpu_train, named_logs, oracle_replay, oracle_runtime

pytestmark = pytest.mark.gpu

SGD = dict(kind="sgd", lr=0.05)


def hist_of(values, nbins):
    h = [0] * nbins
    for v in values:
        h[min(int(v), nbins - 1)] += 1
    return h


@pytest.mark.parametrize("mak", [1, 4, 7])
def test_mlp_staleness_is_bounded_by_max_active_keys(mak):
    """MLP with an update after every gradient: a gradient's staleness is at most max_active_keys - 1, because only
    the other instances in flight can update a layer between an instance's forward and backward pass.  The
    library's histogram must also equal the staleness the checker measures when it replays the same record."""
    model, dims, data = synth.workload(1, n=512)
    fp = synth.init_params(model, dims, 5)
    g = gpu_train(model, dims, fp, data, mak, 1, SGD)
    a = g["trainer"].amp
    nbins = 16
    hist = a.get_staleness_hist(nbins)
    assert sum(hist) == 3 * len(data)                      # one gradient per layer and instance
    assert sum(hist[mak:]) == 0, hist                      # all mass in bins 0 .. mak - 1
    if mak == 1:
        assert hist[0] == 3 * len(data)
    else:
        assert sum(hist[1:]) > 0, "with several instances in flight some gradient is stale"
    rt = oracle_replay(model, dims, fp, data, g["logs"], 1, SGD)
    ref = [v for vs in rt.staleness().values() for v in vs]
    assert hist == hist_of(ref, nbins)


def test_staleness_histogram_with_replicas_and_tiles():
    """Tree-LSTM with tiled cells and three replicas: every replica's nodes are counted apart, a tiled node once
    (its first tile keeps the record); the histogram equals the sum of the per-replica checker replays'."""
    dims = dict(vocab=97, emb=50, hidden=37, n_class=5)
    data = synth.make_tree(45, 27, dims, max_leaves=16)
    fp = synth.init_params("tree", dims, 12)
    R, mak, muf, lmuf = 3, 6, 3, 5
    g = gpu_train("tree", dims, fp, data, mak, muf, SGD, lookup_muf=lmuf, replicas=R, tiles={1: 2, 2: 3})
    a = g["trainer"].amp
    nbins = 12
    hist = a.get_staleness_hist(nbins)
    wpr = a.num_workers() // R
    parts = oamp.replica_subsets(data, R)
    ref = []
    for r in range(R):
        rt = oracle_runtime("tree", dims, fp, muf, SGD, lookup_muf=lmuf)
        rt.replay(parts[r], named_logs("tree", dims, g["logs"][r * wpr + 1:(r + 1) * wpr]))
        ref += [v for vs in rt.staleness().values() for v in vs]
    assert sum(hist) == len(ref)
    assert hist == hist_of(ref, nbins)


def test_worker_statistics():
    """Fractions lie in [0, 1]; the messages a worker took equal its node's visits: forward and backward for a
    cell tile and the lookup, one (the loss turns it round in place) for the output layer."""
    dims = dict(vocab=200, emb=300, hidden=150, n_class=5)
    data = synth.make_tree(64, 99, dims, max_leaves=24)
    fp = synth.init_params("tree", dims, 3)
    g = gpu_train("tree", dims, fp, data, 16, 10, SGD, lookup_muf=100, log=False)
    stats = g["trainer"].amp.get_worker_stats()
    leaves = sum(i["n_leaves"] for i in data)
    nodes = sum(2 * i["n_leaves"] - 1 for i in data)
    expect = {0: 2 * leaves, 1: 2 * leaves, 2: 2 * (nodes - leaves), 3: nodes}
    assert stats[0]["node"] == -1                          # the controller
    assert len(stats) == 1 + 1 + 5 + 8 + 1
    for w in stats:
        assert 0.0 <= w["wait_fraction"] <= 1.0, w
        assert all(0.0 <= p <= 1.0 for p in w["phases"]), w
        if w["node"] >= 0:
            assert w["messages"] == expect[w["node"]], w
            assert 1 <= w["batches"] <= w["messages"], w


def test_graph_workers_take_several_messages_per_pass():
    """The graph model's dense workers count messages and passes; every message is counted once (4 steps x forward
    and backward per graph at the GRU nodes, the same for an edge type where the graph has such edges), split
    nodes' tiles all see every message, and with 32 graphs in flight a pass holds more than one message on average."""
    model, dims, data = synth.workload(4, n=600)
    fp = synth.init_params(model, dims, 5)
    g = gpu_train(model, dims, fp, data, 32, 20, dict(kind="adam", lr=0.0002, beta1=0.9, beta2=0.999, eps=1e-6),
                  tiles={1: 2, 5: 2, 7: 3}, log=False)
    stats = g["trainer"].amp.get_worker_stats()
    S, T = dims["n_steps"], dims["n_edge_types"]
    with_type = [sum(1 for d in data if (np.asarray(d["etype"]) == c).any()) for c in range(T)]
    dense = [w for w in stats if 1 <= w["node"] <= T + 3]
    assert len(dense) == (T + 1) + 2 + 1 + 3
    for w in dense:
        graphs = with_type[w["node"] - 1] if w["node"] <= T else len(data)
        assert w["messages"] == 2 * S * graphs, w
        assert 1 <= w["batches"] <= w["messages"], w
    gru = [w for w in dense if w["node"] > T]
    assert sum(w["messages"] for w in gru) / sum(w["batches"] for w in gru) >= 1.3, gru


def test_workers_run_on_the_dies_the_launch_assumes():
    """The launch maps workgroups to the eight dies (XCDs) by their index -- block b is expected on die b % 8 -- and
    packs each replica's workers onto one die when whole replicas fit its 32 compute units.  Every workgroup reads
    the die it really ran on from the hardware; this checks the assumption instead of trusting it."""
    # three replicas of a 9-worker tree pipeline (packed: replica r on die r), and a single MLP (4 workers, packed)
    dims = dict(vocab=97, emb=50, hidden=37, n_class=5)
    data = synth.make_tree(45, 27, dims, max_leaves=16)
    fp = synth.init_params("tree", dims, 12)
    g = gpu_train("tree", dims, fp, data, 6, 3, SGD, lookup_muf=5, replicas=3, tiles={1: 2, 2: 4}, log=False)
    a = g["trainer"].amp
    xcc = a.get_worker_placement()
    wpr = a.num_workers() // 3
    assert wpr == 9 and len(xcc) == 27
    for r in range(3):
        assert set(xcc[r * wpr:(r + 1) * wpr]) == {r}, xcc
    model, mdims, mdata = synth.workload(1, n=64)
    g = gpu_train(model, mdims, synth.init_params(model, mdims, 5), mdata, 4, 1, SGD, log=False)
    assert set(g["trainer"].amp.get_worker_placement()) == {0}
    # a single pipeline of many workers is spread over the dies: worker w = block w on die w % 8
    dims2 = dict(vocab=200, emb=300, hidden=150, n_class=5)
    data2 = synth.make_tree(32, 99, dims2, max_leaves=24)
    g = gpu_train("tree", dims2, synth.init_params("tree", dims2, 3), data2, 16, 10, SGD, lookup_muf=100, log=False)
    xcc = g["trainer"].amp.get_worker_placement()
    assert xcc == [w % 8 for w in range(len(xcc))], xcc
