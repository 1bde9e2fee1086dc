"""GPU parity: the HIP path, called through the C boundary, against the CPU
checker replaying the order in which the GPU's workers executed their
events.  Parameters and per-instance losses must agree to 1e-5 (relative)."""
import numpy as np
import pytest

from oracle import direct
from paper_1705_09786_amd import synth

from oracle import amp as oamp

from util import (check_controller_log, compare, compare_up_to_relu_decisions, elem_tol, elementwise_err, gpu_train,
                  named_logs, oracle_replay, oracle_runtime, rel_err)

pytestmark = pytest.mark.gpu

SGD = dict(kind="sgd", lr=0.05)
# Adam's step lr * m / (sqrt(v) + eps) has slope lr / eps at a zero gradient: with the customary eps = 1e-8 an
# fp32 rounding difference of 1e-9 in one near-zero gradient element moves that parameter by a full step, and a
# single such element is enough to exceed 1e-5 in the norm.  The replay cases therefore use eps = 1e-6, which keeps
# the optimizer's own amplification of rounding noise below the tolerance; the checker's Adam is pinned with the
# customary eps against torch.optim.Adam in the CPU suite.
# The step size is 5e-4: at 2e-3 several of these short training runs amplify a 1e-7 perturbation of the
# initial parameters 5..10 times in the checker itself (and the recurrent and graph models far more), which
# leaves fp32 rounding too little room under 1e-5; each run has its own event order, so a case close to the
# limit fails now and then.
ADAM = dict(kind="adam", lr=0.0005, beta1=0.9, beta2=0.999, eps=1e-6)


# Momentum 0.9 at lr = 0.02 is an unstable training run on this task (losses spike to twice their initial value);
# at lr = 0.005 a 1e-7 perturbation stays at 1e-7 (checked on the CPU in test_oracle_models.py).  The MLP's ReLUs
# make one more thing necessary: see compare_up_to_relu_decisions.
@pytest.mark.parametrize("mak,muf,opt", [(1, 1, SGD), (4, 1, SGD), (4, 3, ADAM), (8, 5, dict(kind="momentum", lr=0.005, momentum=0.9))])
def test_mlp_replay_parity(mak, muf, opt):
    model, dims, data = synth.workload(1)
    fp = synth.init_params(model, dims, 5)
    g = gpu_train(model, dims, fp, data, mak, muf, opt)
    check_controller_log(g["logs"], mak, len(data))
    compare_up_to_relu_decisions(model, dims, fp, data, g, muf, opt)


def test_mlp_mak1_is_synchronous_sgd():
    """max_active_keys = 1 on the MLP is plain per-instance SGD (Section 6,
    Table 1 caption): compare with the checker's direct trainer, no log."""
    model, dims, data = synth.workload(1)
    fp = synth.init_params(model, dims, 5)
    g = gpu_train(model, dims, fp, data, 1, 1, SGD, log=False)
    P = direct.unpack(model, dims, fp)
    ref = direct.train(model, dims, P, data, lr=float(np.float32(0.05)))
    assert np.abs(g["losses"] - np.array(ref)).max() <= 1e-5 * max(1.0, np.abs(ref).max())
    for k in range(3):
        refv = np.concatenate([P[k]["W"].reshape(-1), P[k]["b"]])
        assert np.linalg.norm(g["params"][k] - refv) / np.linalg.norm(refv) <= 1e-5


# The recurrent model under Adam at lr = 0.002 is a chaotic training run: the checker's own result moves by O(1)
# when its initial parameters are perturbed by 1e-7 (relative), so no fp32 implementation can follow it to 1e-5.
# At lr = 5e-4 over 300 sequences the same perturbation stays at 1e-7 (the CPU suite checks this), and that
# is the setting the recurrent Adam case uses.
RNN_ADAM = dict(ADAM)
# an update every 3 gradients amplifies more: the same check asks for lr = 2e-4 there
RNN_ADAM_MUF3 = dict(RNN_ADAM, lr=0.0002)


# With an update per gradient the cell's weights are rounded to fp32 after every one of about 18 updates per
# sequence, while the checker keeps them in float64: the rounding of one stored element accumulates like a random walk,
# about 3.4e-8 x sqrt(updates) relative, and the largest of the cell's 49k elements lies four to five times above that.
# Measured: 600 sequences (10,800 updates) sit at 8.4e-6 and exceed the element-wise 1e-5 in one run of eight
# (1.08e-5), with the tensor's 2-norm a steady 2.0e-6; 300 sequences reach 6.2e-6 to 7.7e-6 depending on the event
# order -- so the cases with an update per gradient have 200 sequences (3,600 updates), and the 600-sequence run keeps
# an update every 7 gradients.
@pytest.mark.parametrize("mak,muf,opt,n", [(1, 1, SGD, 200), (16, 1, SGD, 200), (16, 7, SGD, 600), (4, 3, RNN_ADAM_MUF3, 300),
                                           (16, 7, RNN_ADAM, 300)])
def test_rnn_replay_parity(mak, muf, opt, n):
    model, dims, data = synth.workload(2, n=n)
    fp = synth.init_params(model, dims, 6)
    g = gpu_train(model, dims, fp, data, mak, muf, opt)
    check_controller_log(g["logs"], mak, len(data))
    rt = oracle_replay(model, dims, fp, data, g["logs"], muf, opt)
    compare(g, rt, len(data), opt=opt)


def test_hand_built_graph_trains_like_the_canned_one():
    """The recurrent model described node by node through amp_add_node / amp_connect (Figure 2's graph, nodes added
    in another order than the model numbers them) and lowered by amp_finalize: same replay parity as the canned
    builder's."""
    from test_boundary_cpu import rnn_graph
    dims = dict(vocab=13, emb=20, hidden=44, n_class=7)
    data = synth.make_rnn(120, 31, dims, min_len=1, max_len=12)
    fp = synth.init_params("rnn", dims, 7)
    g = gpu_train("rnn", dims, fp, data, 8, 3, SGD, graph=lambda a: rnn_graph(a, **dims))
    check_controller_log(g["logs"], 8, len(data))
    rt = oracle_replay("rnn", dims, fp, data, g["logs"], 3, SGD)
    compare(g, rt, len(data), opt=SGD)


def max_in_flight(log):
    active = worst = 0
    for (_, kind, _, _) in log:
        active += 1 if kind == "A" else -1
        worst = max(worst, active)
    return worst


def test_staleness_bounded_admission():
    """The controller's own limit on the instances in flight (Appendix B, MNIST: a better schedule than the greedy
    one).  The event record is replayed as for any other admission order; bound 0 keeps one instance in flight and
    so repeats the max_active_keys = 1 run bit for bit; a bound nothing reaches ends at max_active_keys."""
    model, dims, data = synth.workload(2, n=200)   # an update per gradient: see the note at test_rnn_replay_parity
    fp = synth.init_params(model, dims, 6)
    seq = gpu_train(model, dims, fp, data, 1, 1, SGD)
    for bound, lo, hi in ((0.0, 1, 1), (60.0, 2, 15), (1e9, 16, 16)):
        g = gpu_train(model, dims, fp, data, 16, 1, SGD, max_staleness=bound)
        check_controller_log(g["logs"], 16, len(data))
        assert lo <= max_in_flight(g["logs"][0]) <= hi, (bound, max_in_flight(g["logs"][0]))
        assert g["admission"]["max_in_flight"] == max_in_flight(g["logs"][0])
        assert 1 <= g["admission"]["final_limit"] <= 16
        rt = oracle_replay(model, dims, fp, data, g["logs"], 1, SGD)
        compare(g, rt, len(data), opt=SGD)
        if bound == 0.0:
            for a, b in zip(g["params"], seq["params"]):
                assert np.array_equal(a, b)
            assert np.array_equal(g["losses"], seq["losses"])
        if bound == 1e9:
            assert g["admission"]["final_limit"] == 16
    # a tree run under the bound: tiles, joins and the lookup count their updates too
    tdims = TREE_ODD
    tdata = synth.make_tree(48, 5, tdims)
    tfp = synth.init_params("tree", tdims, 8)
    g = gpu_train("tree", tdims, tfp, tdata, 8, 3, SGD, tiles={1: 3, 2: 5}, lookup_muf=5, max_staleness=4.0)
    check_controller_log(g["logs"], 8, len(tdata))
    rt = oracle_replay("tree", tdims, tfp, tdata, g["logs"], 3, SGD, lookup_muf=5)
    compare(g, rt, len(tdata), opt=SGD)


def test_rnn_edge_lengths():
    """Length-1 sequences, the maximum length, and a ragged mix."""
    dims = synth.DEFAULT_DIMS["rnn"]
    data = synth.make_rnn(40, 3, dims, min_len=1, max_len=1) + synth.make_rnn(40, 4, dims, min_len=32, max_len=32) \
        + synth.make_rnn(40, 5, dims, min_len=1, max_len=32)
    fp = synth.init_params("rnn", dims, 6)
    g = gpu_train("rnn", dims, fp, data, 5, 2, SGD)
    rt = oracle_replay("rnn", dims, fp, data, g["logs"], 2, SGD)
    compare(g, rt, len(data), opt=SGD)


@pytest.mark.parametrize("dims,opt", [(dict(vocab=13, emb=50, hidden=37, n_class=7), SGD),
                                      (dict(vocab=13, emb=20, hidden=44, n_class=7), RNN_ADAM_MUF3),
                                      (dict(vocab=5, emb=128, hidden=64, n_class=3), SGD)])
def test_rnn_unequal_and_odd_sizes(dims, opt):
    """Embedding and hidden size differ (the cell's two input segments have their own widths), sizes that are
    no multiples of 4 or 16, and an embedding as wide as the padded segment next to a narrower hidden state."""
    data = synth.make_rnn(150, 31, dims, min_len=1, max_len=12)
    fp = synth.init_params("rnn", dims, 7)
    g = gpu_train("rnn", dims, fp, data, 8, 3, opt)
    check_controller_log(g["logs"], 8, len(data))
    rt = oracle_replay("rnn", dims, fp, data, g["logs"], 3, opt)
    compare(g, rt, len(data), opt=opt)


TREE_SMALLVOCAB = dict(vocab=64, emb=300, hidden=150, n_class=5)
TREE_ODD = dict(vocab=97, emb=50, hidden=37, n_class=5)


@pytest.mark.parametrize("dims,tiles,mak,muf,lmuf,opt,n", [
    (TREE_SMALLVOCAB, None, 1, 1, 1, SGD, 16),
    (synth.DEFAULT_DIMS["tree"], None, 16, 50, 1000, SGD, 96),
    (synth.DEFAULT_DIMS["tree"], None, 64, 7, 333, ADAM, 96),
    (synth.DEFAULT_DIMS["tree"], {1: 8, 2: 16}, 32, 50, 1000, SGD, 96),   # tiles of 4 and 3 row blocks
    (synth.DEFAULT_DIMS["tree"], {1: 10, 2: 17}, 64, 50, 1000, SGD, 96),  # the benchmark's tiling: 3 row blocks, 45 of 48 rows used
    (TREE_ODD, {1: 3, 2: 5}, 8, 3, 5, SGD, 64),
    # an update every 3 gradients under Adam: lr 2e-4 as in the recurrent case of that kind -- at 5e-4 four of forty
    # runs put a single element of the branch matrix 5e-5 .. 7e-5 off (median 1.8e-5), at 2e-4 forty runs stay within 7.1e-6
    (TREE_ODD, {1: 1, 2: 1}, 8, 3, 5, dict(ADAM, lr=0.0002), 64),
    (TREE_ODD, {1: 2, 2: 3}, 8, 4, 5, dict(kind="momentum", lr=0.005, momentum=0.9), 64),
])
def test_tree_replay_parity(dims, tiles, mak, muf, lmuf, opt, n):
    data = synth.make_tree(n, 21, dims)
    fp = synth.init_params("tree", dims, 8)
    g = gpu_train("tree", dims, fp, data, mak, muf, opt, tiles=tiles, lookup_muf=lmuf)
    check_controller_log(g["logs"], mak, len(data))
    rt = oracle_replay("tree", dims, fp, data, g["logs"], muf, opt, lookup_muf=lmuf)
    compare(g, rt, len(data), opt=opt)


TREE_HBM = dict(vocab=97, emb=40, hidden=36, n_class=5)


@pytest.mark.parametrize("tiles,mak,muf,opt,n", [({1: 2, 2: 3}, 8, 3, SGD, 64), ({1: 1, 2: 2}, 16, 5, ADAM, 64)])
def test_tree_weights_in_hbm_replay_parity(tiles, mak, muf, opt, n):
    """Leaf and branch tiles that read their rows from HBM as they go and update them in place (the mode for
    cells too large for LDS), at sizes the checker replays in seconds: several tiles, ragged last row block."""
    dims = TREE_HBM
    data = synth.make_tree(n, 23, dims)
    fp = synth.init_params("tree", dims, 8)
    g = gpu_train("tree", dims, fp, data, mak, muf, opt, tiles=tiles, lookup_muf=7, in_hbm=(1, 2))
    check_controller_log(g["logs"], mak, len(data))
    rt = oracle_replay("tree", dims, fp, data, g["logs"], muf, opt, lookup_muf=7)
    compare(g, rt, len(data), opt=opt)


def test_tree_hidden_1024_replay_parity():
    """The scale-up shape (hidden = embedding = 1024, weights streamed from HBM, leaf / branch split over 16 / 64
    workgroups as the benchmark runs it) on a handful of trees the checker can still replay."""
    dims = synth.DEFAULT_DIMS["tree_big"]
    data = synth.make_tree(6, 31, dims, min_leaves=2, max_leaves=12)
    fp = synth.init_params("tree", dims, 8)
    g = gpu_train("tree", dims, fp, data, 4, 5, SGD, tiles={1: 16, 2: 64}, lookup_muf=9, arena_bytes=3 << 30)
    check_controller_log(g["logs"], 4, len(data))
    rt = oracle_replay("tree", dims, fp, data, g["logs"], 5, SGD, lookup_muf=9)
    compare(g, rt, len(data), opt=SGD)


TREE_512 = dict(vocab=2000, emb=512, hidden=512, n_class=5)


@pytest.mark.parametrize("tiles,opt", [({1: 4, 2: 6}, SGD), ({1: 8, 2: 16}, dict(kind="momentum", lr=0.005, momentum=0.9))])
def test_tree_streamed_weights_large_batches_replay_parity(tiles, opt):
    """The streamed-weight kernels in their steady state, with a real learning rate: hidden = embedding = 512, 64
    instances in flight and 40 trees of up to 60 leaves, so that the forward and input-gradient products run with
    two to four 16-message blocks, the chunk loop over the input columns makes 8 (leaf) and 16 (branch) rounds with
    both staging buffers in use, and the update reads pending lists of 50 pairs.  Four leaf tiles have 24 row
    blocks (three per wave), six branch tiles 27 (two passes: three per wave, then one); 8 + 16 tiles have 12 and
    10 (two per wave)."""
    dims = TREE_512
    data = synth.make_tree(40, 41, dims)
    fp = synth.init_params("tree", dims, 8)
    g = gpu_train("tree", dims, fp, data, 64, 50, opt, tiles=tiles, lookup_muf=300, in_hbm=(1, 2), arena_bytes=3 << 30)
    check_controller_log(g["logs"], 64, len(data))
    stats = g["trainer"].amp.get_worker_stats()
    leaf = next(w for w in stats if w["node"] == 1)
    assert leaf["messages"] / max(leaf["batches"], 1) >= 20, "batches stayed small: %r" % (leaf,)
    rt = oracle_replay("tree", dims, fp, data, g["logs"], 50, opt, lookup_muf=300)
    compare(g, rt, len(data), opt=opt)


def test_tree_hidden_1024_large_batches_replay_parity():
    """The scale-up shape itself (hidden = embedding = 1024, 16 + 64 tiles as the benchmark runs it) with 64
    instances in flight, a real learning rate and updates every 50 gradients."""
    dims = dict(synth.DEFAULT_DIMS["tree_big"], vocab=2000)
    data = synth.make_tree(16, 43, dims, min_leaves=8, max_leaves=40)
    fp = synth.init_params("tree", dims, 8)
    g = gpu_train("tree", dims, fp, data, 64, 50, SGD, tiles={1: 16, 2: 64}, lookup_muf=200, arena_bytes=5 << 30)
    check_controller_log(g["logs"], 64, len(data))
    rt = oracle_replay("tree", dims, fp, data, g["logs"], 50, SGD, lookup_muf=200)
    compare(g, rt, len(data), opt=SGD)


def test_threshold_lowered_between_training_calls():
    """min_update_frequency changed between two training calls: the gradients a node still holds stay with it
    (Section 3), so a threshold at or below a held count is refused (it would already have been reached; letting
    it through would also run the pending-gradient list past its end), and a lower threshold above every held
    count is taken: both calls are then replayed as one run."""
    from paper_1705_09786_amd import binding as B
    model, dims, _ = synth.workload(2, n=1)
    data = synth.make_rnn(61, 77, dims, min_len=3, max_len=9)
    fp = synth.init_params(model, dims, 6)
    g = gpu_train(model, dims, fp, data, 8, 7, SGD)
    a = g["trainer"].amp
    tokens = sum(len(i["tokens"]) for i in data)
    held = {0: tokens % 7, 1: tokens % 7, 2: len(data) % 7}    # lookup, cell, out
    assert max(held.values()) >= 1, "pick data that leaves gradients behind"
    for node, h in held.items():
        if h >= 1:
            with pytest.raises(B.AmpError) as ei:
                a.set_min_update_frequency(node, h)
            assert ei.value.code == B.AMP_ESTATE
    with pytest.raises(B.AmpError):
        a.set_min_update_frequency(-1, 1)
    new = max(held.values()) + 1
    assert new < 7
    a.set_min_update_frequency(-1, new)
    rt = oracle_replay(model, dims, fp, data, g["logs"], 7, SGD)
    first = compare(g, rt, len(data), opt=SGD)
    a.train(1)
    rt.set_muf(new)
    rt.replay(data, named_logs(model, dims, a.get_event_log()[1:]), first_seq=len(data))
    g2 = dict(g, params=g["trainer"].params(), losses=a.get_instance_losses().astype(np.float64))
    ref_loss = np.array([rt.loss[len(data) + s] for s in range(len(data))])
    assert np.abs(g2["losses"] - ref_loss).max() <= 1e-5 * max(1.0, np.abs(ref_loss).max())
    for k, node in enumerate(rt.ppt):
        assert rel_err(g2["params"][k], oamp.C.pack_node(node.P)) <= 1e-5, node.name
        assert elementwise_err(g2["params"][k], oamp.C.pack_node(node.P))[0] <= 1e-5, node.name
    assert first is not None


@pytest.mark.parametrize("model", ["tree", "ggnn"])
def test_strict_join_build_replay_parity(model):
    """The library built with explicitly ordered join completion (acquire on the completing arrival, release before
    its post) instead of the fence-free shortcut: the same replay parity must hold for both builds, so that a
    mismatch in one of them can be attributed.  Trees and graphs are the models with joins."""
    if model == "tree":
        dims, muf, lmuf, opt = TREE_ODD, 3, 5, SGD
        data = synth.make_tree(64, 21, dims)
        fp = synth.init_params("tree", dims, 8)
        kw = dict(tiles={1: 3, 2: 5}, lookup_muf=lmuf)
    else:
        _, dims, data = synth.workload(4, n=120)
        fp = synth.init_params("ggnn", dims, 9)
        muf, lmuf, opt, kw = 8, None, G_ADAM, {}
    for strict in (True, False):
        g = gpu_train(model, dims, fp, data, 8, muf, opt, strict=strict, **kw)
        check_controller_log(g["logs"], 8, len(data))
        rt = oracle_replay(model, dims, fp, data, g["logs"], muf, opt, lookup_muf=lmuf)
        compare(g, rt, len(data), opt=opt)


def test_tree_edge_shapes():
    """Single-leaf trees (the root is a leaf), two leaves, the maximum size,
    left and right combs, with repeated tokens inside a tree."""
    dims = TREE_ODD
    data = synth.make_tree(6, 1, dims, min_leaves=1, max_leaves=1) + synth.make_tree(6, 2, dims, min_leaves=2, max_leaves=2) \
        + synth.make_tree(4, 3, dims, min_leaves=60, max_leaves=60)
    L = 9
    comb_l = dict(n_leaves=L, tokens=np.full(L, 5, np.int32),
                  left=np.array([-1] * L + [0] + list(range(L, 2 * L - 2)), np.int32),
                  right=np.array([-1] * L + list(range(1, L)), np.int32),
                  labels=np.arange(2 * L - 1, dtype=np.int32) % 5)
    comb_r = dict(comb_l, left=comb_l["right"], right=comb_l["left"])
    data += [comb_l, comb_r]
    fp = synth.init_params("tree", dims, 8)
    g = gpu_train("tree", dims, fp, data, 4, 2, SGD, tiles={1: 2, 2: 3}, lookup_muf=3)
    rt = oracle_replay("tree", dims, fp, data, g["logs"], 2, SGD, lookup_muf=3)
    compare(g, rt, len(data), opt=SGD)


MOM = dict(kind="momentum", lr=0.0005, momentum=0.9)
GG_ODD = dict(n_node_types=5, hidden=37, n_edge_types=3, n_steps=3)


# The graph model under Adam at lr = 0.002 trains at the edge of stability: repeated runs (each with its own
# event order) put the worst per-graph loss between 2e-6 and 4e-5 off the checker while the parameters agree to
# 1e-6, whatever eps is.  At lr = 5e-4 the outcome depends on the schedule the workers happen to follow: when every
# worker took one message at a time, 118 of 120 runs (60 with each build of the join) stayed within 1.3e-6 and two
# reached 6e-6 and 1.3e-5; with several messages per pass the median run of 200 is 1.4e-5 off in its worst graph.
# At lr = 2e-4 thirty runs, each with its own event order, all stayed within 4e-7: the case runs there.
G_ADAM = dict(ADAM, lr=0.0002)


@pytest.mark.parametrize("mak,muf,opt,n", [(1, 1, dict(kind="sgd", lr=0.01), 40), (32, 20, G_ADAM, 300), (8, 3, MOM, 150),
                                           (64, 5, dict(kind="sgd", lr=0.01), 256)])   # long queues: passes of four messages
def test_ggnn_replay_parity(mak, muf, opt, n):
    model, dims, data = synth.workload(4, n=n)
    fp = synth.init_params(model, dims, 9)
    g = gpu_train(model, dims, fp, data, mak, muf, opt)
    check_controller_log(g["logs"], mak, len(data))
    rt = oracle_replay(model, dims, fp, data, g["logs"], muf, opt)
    compare(g, rt, len(data), opt=opt)


@pytest.mark.parametrize("dims,tiles,mak,muf,opt,n", [
    (synth.DEFAULT_DIMS["ggnn"], {1: 2, 5: 2, 6: 2, 7: 3}, 32, 20, G_ADAM, 300),   # the benchmark's split: 52 + 48 and 36 + 32 + 32 units
    (GG_ODD, {1: 2, 2: 3, 4: 2, 5: 3, 6: 4}, 6, 4, dict(kind="sgd", lr=0.01), 0),  # uneven splits of 37 units, scalar path
    (dict(n_node_types=5, hidden=40, n_edge_types=2, n_steps=2), {1: 4, 2: 1, 3: 3, 4: 2, 5: 4}, 8, 3, MOM, 120),
])
def test_ggnn_tiled_nodes_replay_parity(dims, tiles, mak, muf, opt, n):
    """Edge linears and GRU nodes split by hidden unit over several workgroups (Section 5's tiling of a linear
    layer): every tile writes its units on the way forward and hands back a partial W^T delta that the consumers
    add up.  Hidden 100 in two and three tiles (52 + 48 and 36 + 32 + 32 units, the fixed-shape products), 37 units in uneven tiles of 2, 3
    and 4 (no 16-byte moves) on two-node and 29-node graphs, 40 units in tiles of 1 to 4 (12 + 8 + ... units)."""
    if n:
        data = synth.make_ggnn(n, 5, dims)[0]
    else:
        data = synth.make_ggnn(30, 5, dims, min_nodes=2, max_nodes=3)[0] + synth.make_ggnn(30, 6, dims, min_nodes=29, max_nodes=29)[0]
    fp = synth.init_params("ggnn", dims, 9)
    g = gpu_train("ggnn", dims, fp, data, mak, muf, opt, tiles=tiles)
    check_controller_log(g["logs"], mak, len(data))
    assert g["trainer"].amp.num_workers() == 3 + dims["n_edge_types"] + 3 + sum(t - 1 for t in tiles.values())
    rt = oracle_replay("ggnn", dims, fp, data, g["logs"], muf, opt)
    compare(g, rt, len(data), opt=opt)


def test_ggnn_odd_sizes_and_tiny_graphs():
    """Hidden size not a multiple of anything, three edge types of which some
    graphs use only one, graphs of two nodes next to the largest ones."""
    dims = GG_ODD
    data = synth.make_ggnn(30, 5, dims, min_nodes=2, max_nodes=3)[0] + synth.make_ggnn(30, 6, dims, min_nodes=29, max_nodes=29)[0]
    pair = dict(n_nodes=2, node_type=np.array([0, 4], np.int32), src=np.array([0, 1], np.int32),
                dst=np.array([1, 0], np.int32), etype=np.array([2, 2], np.int32), target=0.25)
    data += [pair, pair]
    fp = synth.init_params("ggnn", dims, 9)
    g = gpu_train("ggnn", dims, fp, data, 6, 4, ADAM)
    rt = oracle_replay("ggnn", dims, fp, data, g["logs"], 4, ADAM)
    compare(g, rt, len(data), opt=ADAM)


@pytest.mark.parametrize("cfg,n,nv", [(1, 256, 128), (2, 200, 100), (3, 48, 32), (4, 100, 50)])
def test_eval_matches_direct_forward(cfg, n, nv):
    """Forward-only pass (Section 1: training and inference through the same
    graph): after some training, evaluation of a held-out set must equal the
    checker's plain forward with the trained parameters."""
    from paper_1705_09786_amd import runner
    model, dims, data = synth.workload(cfg, n=n)
    _, _, valid = synth.workload(cfg, n=nv, valid=True)
    fp = synth.init_params(model, dims, 10 + cfg)
    ml, me = runner.max_len_of(model, data + valid)
    tr = runner.Trainer(model, dims, fp, 8, ml, me, len(data))
    a = tr.amp
    a.set_watchdog(5.0)
    a.set_min_update_frequency(-1, 4)
    a.set_optimizer(-1, 0, lr=0.002 if model == "ggnn" else 0.02)   # sum-pooled regression needs a small step
    tr.submit_all(data)
    tr.submit_all(valid, which=1)
    a.train(1)
    ev = a.eval()
    P = direct.unpack(model, dims, tr.params())
    ref_loss, ref_acc = direct.evaluate(model, dims, P, valid)
    assert ev["n_instances"] == len(valid)
    assert abs(ev["mean_loss"] - ref_loss) <= 1e-5 * max(1.0, abs(ref_loss))
    if model != "ggnn":
        assert abs(ev["accuracy"] - ref_acc) < 1e-9
    # evaluation changes nothing: a second call gives the same numbers (a tree's loss is
    # summed over its nodes in arrival order, hence fp32 rounding differences)
    ev2 = a.eval()
    assert abs(ev2["mean_loss"] - ev["mean_loss"]) <= 1e-6 * abs(ev["mean_loss"])
    assert ev2["accuracy"] == ev["accuracy"]
    # and training can continue afterwards
    a.train(1)


@pytest.mark.parametrize("cfg,n,nv,mak,muf", [(1, 300, 60, 4, 3), (2, 200, 50, 8, 5), (3, 60, 24, 16, 7), (4, 120, 30, 8, 6)])
def test_train_and_eval_instances_in_one_launch(cfg, n, nv, mak, muf):
    """Section 1: training and inference at the same time.  One launch trains on the training set while the
    evaluation set's instances travel through the same graph forward-only, interleaved by the controller.  The
    event record (admissions marked as inference, the forward events of inference instances included) is replayed
    by the checker: parameters, the training instances' losses and every inference instance's loss -- taken with
    whatever parameters it met on the way -- must agree."""
    from paper_1705_09786_amd import runner
    if cfg == 3:
        model, dims = "tree", TREE_ODD
        data, valid = synth.make_tree(n, 21, dims, max_leaves=24), synth.make_tree(nv, 1021, dims, max_leaves=24)
        kw = dict(tiles={1: 2, 2: 3}, lookup_muf=11)
    else:
        model, dims, data = synth.workload(cfg, n=n)
        _, _, valid = synth.workload(cfg, n=nv, valid=True)
        kw = {}
    fp = synth.init_params(model, dims, 10 + cfg)
    ml, me = runner.max_len_of(model, data + valid)
    opt = dict(kind="sgd", lr=0.002 if model == "ggnn" else 0.03)
    tr = runner.Trainer(model, dims, fp, mak, ml, me, len(data), tiles=kw.get("tiles"))
    a = tr.amp
    a.set_watchdog(5.0)
    a.set_min_update_frequency(-1, muf)
    if "lookup_muf" in kw:
        a.set_min_update_frequency(0, kw["lookup_muf"])
    a.set_optimizer(-1, 0, lr=opt["lr"])
    a.set_event_log(16 * (2 * ml + 2) * max(1, dims.get("n_steps", 1)) * (len(data) + len(valid)) + 1024)
    tr.submit_all(data)
    tr.submit_all(valid, which=1)
    ev = a.train_eval(1)
    logs = a.get_event_log()
    adm = [(seq, local) for (_, kind, seq, local) in logs[0] if kind == "A"]
    assert len(adm) == len(data) + len(valid) and [s for s, _ in adm] == list(range(len(adm)))
    assert sum(1 for _, e in adm if e) == len(valid)
    check = 0
    for (_, kind, _, _) in logs[0]:
        check += 1 if kind == "A" else -1
        assert 0 <= check <= mak
    rt = oracle_runtime(model, dims, fp, muf, opt, lookup_muf=kw.get("lookup_muf"))
    it = ie = 0
    train_seqs, eval_seqs = [], []
    for seq, is_eval in adm:
        if is_eval:
            rt.mark_eval(seq, valid[ie])
            eval_seqs.append(seq)
            ie += 1
        else:
            rt.seq_inst[seq] = data[it]
            train_seqs.append(seq)
            it += 1
    # inference instances spread through the run, not bunched at either end
    assert eval_seqs[0] < len(adm) // 3 and eval_seqs[-1] > 2 * len(adm) // 3
    rt.replay(data, named_logs(model, dims, logs[1:]))
    g = dict(params=tr.params(), losses=a.get_instance_losses().astype(np.float64), init=[np.asarray(v, np.float32) for v in fp])
    compare(g, rt, len(data), opt=opt, ref_losses=[rt.loss[s] for s in train_seqs])
    ref_eval = float(np.mean([rt.loss[s] for s in eval_seqs]))
    assert ev["n_instances"] == len(valid)
    assert abs(ev["mean_loss"] - ref_eval) <= 1e-5 * max(1.0, abs(ref_eval)), (ev["mean_loss"], ref_eval)
    if model != "ggnn":
        ref_acc = sum(rt.correct[s] for s in eval_seqs) / sum(rt.npred[s] for s in eval_seqs)
        assert abs(ev["accuracy"] - ref_acc) < 1e-9
    # the ordinary calls still work on the same context afterwards
    a.train(1)
    assert a.eval()["n_instances"] == len(valid)


@pytest.mark.parametrize("cfg,dims,R,mak,muf,lmuf,opt,n", [
    (1, None, 4, 4, 3, None, SGD, 203),
    (3, TREE_ODD, 3, 8, 3, 5, SGD, 50),
    (4, GG_ODD, 2, 6, 4, 4, ADAM, 41),
    # the benchmark's replicated launch: 16 replicas of 5 leaf + 8 branch tiles on all 256 workgroups, two replicas
    # inside every XCD (releases without an L2 write-back)
    (3, synth.DEFAULT_DIMS["tree"], 16, 16, 5, 20, SGD, 192),
    # and the graph model's: 24 replicas of the unsplit 10-worker pipeline, three inside every XCD
    (4, synth.DEFAULT_DIMS["ggnn"], 24, 8, 4, 4, dict(kind="sgd", lr=0.01), 192),
])
def test_replicas_replay_parity(cfg, dims, R, mak, muf, lmuf, opt, n):
    """Every parameterized node replicated R times, instance i routed to replica i mod R, parameters averaged
    after each epoch (Section 5).  Two epochs as two training calls: each replica's record is replayed by a
    checker runtime of its own on its share of the instances, then the runtimes are averaged, twice."""
    from paper_1705_09786_amd import runner
    if cfg == 1:
        model, dims, data = synth.workload(1, n=n)
    elif cfg == 3:
        model, data = "tree", synth.make_tree(n, 27, dims, max_leaves=20)
    else:
        model, data = "ggnn", synth.make_ggnn(n, 28, dims)[0]
    fp = synth.init_params(model, dims, 12)
    tiles = None if cfg != 3 else {1: 5, 2: 8} if R == 16 else {1: 2, 2: 3}
    g = gpu_train(model, dims, fp, data, mak, muf, opt, lookup_muf=lmuf, replicas=R, tiles=tiles,
                  arena_bytes=(4 << 30) if R >= 16 else (1 << 30))
    a = g["trainer"].amp
    wpr = a.num_workers() // R
    if R >= 16:
        assert wpr == (16 if cfg == 3 else 10) and set(a.get_worker_placement()[r * wpr:(r + 1) * wpr] == [r % 8] * wpr for r in range(R)) == {True}
    rts = [oracle_runtime(model, dims, fp, muf, opt, lookup_muf=lmuf) for _ in range(R)]
    parts = oamp.replica_subsets(data, R)
    done = [0] * R
    losses_gpu = g["losses"]
    logs = g["logs"]
    for epoch in range(2):
        if epoch == 1:
            a.train(1)
            logs = a.get_event_log()
            losses_gpu = a.get_instance_losses().astype(np.float64)
        for r in range(R):
            check = logs[r * wpr]
            assert [e[2] for e in check if e[1] == "A"] == list(range(done[r], done[r] + len(parts[r])))
            rts[r].replay(parts[r], named_logs(model, dims, logs[r * wpr + 1:(r + 1) * wpr]), first_seq=done[r])
        oamp.average_replicas(rts)
        params = g["trainer"].params()
        for k, node in enumerate(rts[0].ppt):
            assert rel_err(params[k], oamp.C.pack_node(node.P)) <= 1e-5, (epoch, node.name)
            assert elementwise_err(params[k], oamp.C.pack_node(node.P))[0] <= elem_tol(opt), (epoch, node.name)
        ref = np.array([rts[i % R].loss[done[i % R] + i // R] for i in range(len(data))])
        le = np.abs(losses_gpu - ref) / np.maximum(np.abs(ref), 1.0)
        assert le.max() <= 1e-5, (epoch, int(le.argmax()), float(le.max()))
        for r in range(R):
            done[r] += len(parts[r])


@pytest.mark.parametrize("R,mak,muf,opt,n,sync", [(2, 8, 5, SGD, 160, 0), (3, 16, 7, RNN_ADAM, 240, 0),
                                                   (2, 8, 5, SGD, 160, 25), (3, 16, 3, SGD, 240, 16),
                                                   # the benchmark's `cell_copies` launch: eight copies, 64 in flight
                                                   (8, 64, 16, SGD, 480, 0), (8, 64, 4, SGD, 480, 60)])
def test_rnn_replicated_cell_replay_parity(R, mak, muf, opt, n, sync):
    """The RNN's heavy node alone replicated (Section 5): R copies of the cell between a Cond and a Phi that route
    on the instance, the output layer and the loss shared, the copies averaged at the end of each epoch.  Two
    epochs as two training calls: the checker replays every worker's record (the copies are nodes of their own in
    it), averages its copies, and must agree with the GPU on all parameters and losses.  With sync > 0 the
    controller also requests a synchronisation of the copies after every `sync` retirements while training runs
    (the paper's message-passing trigger of a whole-group synchronisation): the copies' records then hold the
    publish and load steps of every round, which the checker replays where they stand."""
    model, dims, data = synth.workload(2, n=n)
    fp = synth.init_params(model, dims, 13)
    g = gpu_train(model, dims, fp, data, mak, muf, opt, lookup_muf=muf, node_replicas={1: R}, group_sync=sync)
    tr = g["trainer"]
    a = tr.amp
    assert a.num_workers() == 3 + (R - 1) and a.num_nodes() == 3 + 2 * (R - 1)
    rt = oracle_runtime(model, dict(dims, node_replicas=R), fp, muf, opt, lookup_muf=muf)
    names = [p.name for p in rt.ppt]
    assert names[:3] == ["lookup", "cell", "out"] and len(names) == a.num_nodes()
    logs, losses = g["logs"], g["losses"]
    for epoch in range(2):
        if epoch == 1:
            a.train(1)
            logs = a.get_event_log()
            losses = a.get_instance_losses().astype(np.float64)
        first = epoch * n
        assert [e[2] for e in logs[0] if e[1] == "A"] == list(range(first, first + n))
        wl = [[(names[node], k, s, l) for (node, k, s, l) in w] for w in logs[1:]]
        for w in wl:   # a copy only ever sees its own instances
            for name, k, s, l in w:
                if k in ("F", "B") and name != "out":
                    assert s % R == (int(name.split(".r")[1]) if ".r" in name else 0), (name, k, s)
        assert sum(1 for w in wl if w) == 1 + R    # every copy worked
        rounds = [sorted(s for name, k, s, l in w if k == "S" and name.startswith("cell")) for w in wl if w and w[0][0] != "out"]
        if sync:
            # rounds are numbered from 1 in every training call, every copy publishes in every round it takes part
            # in, and at least half the requests that fell due were carried out (a round waits for the previous one)
            assert all(r == list(range(1, len(r) + 1)) for r in rounds) and min(len(r) for r in rounds) >= (n // sync) // 2
            rt.snapshots.clear()
        else:
            assert not any(rounds)
        rt.replay(data, wl, first_seq=first)
        oamp.average_node_replicas(rt)
        params = tr.params()
        for k, node in enumerate(rt.ppt):
            ref = oamp.C.pack_node(node.P)
            assert rel_err(params[k], ref) <= 1e-5, (epoch, node.name, rel_err(params[k], ref))
            assert elementwise_err(params[k], ref)[0] <= elem_tol(opt), (epoch, node.name)
        for r in range(1, R):   # after the averaging the copies hold the same values, bit for bit
            assert np.array_equal(params[1 + 2 * r], params[0]) and np.array_equal(params[2 + 2 * r], params[1])
        ref = np.array([rt.loss[first + i] for i in range(n)])
        le = np.abs(losses - ref) / np.maximum(np.abs(ref), 1.0)
        assert le.max() <= 1e-5, (epoch, int(le.argmax()), float(le.max()))
    tr.close()
