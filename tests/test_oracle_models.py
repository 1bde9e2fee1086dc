"""Pins for the CPU checker's whole-model code and AMP simulator (no GPU).

  * whole-model gradients: central finite differences of the instance loss;
  * the message-passing simulator at max_active_keys = 1 with one update per
    instance equals plain per-instance SGD (Section 3 and its footnote), and
    for the MLP with min_update_frequency = m equals minibatch-m SGD;
  * with learning rate 0 any schedule gives the losses of a plain forward;
  * sparse GGNN propagation equals the dense (N H) x (N H) formulation
    (Section 6, results);
  * invariants of Section 3 / 4 under asynchronous schedules;
  * the replay driver reproduces a recorded run and refuses illegal orders.
"""
import copy

import numpy as np
import pytest

from oracle import amp, direct
from paper_1705_09786_amd import synth

TINY = {
    "mlp": dict(d_in=5, hidden=4, n_class=3),
    "rnn": dict(vocab=6, emb=3, hidden=4, n_class=3),
    "tree": dict(vocab=11, emb=4, hidden=3, n_class=3),
    "ggnn": dict(n_node_types=4, hidden=3, n_edge_types=4, n_steps=2),
}


def tiny_data(model, n, seed=3):
    d = TINY[model]
    if model == "mlp":
        return synth.make_mlp(n, seed, d)
    if model == "rnn":
        return synth.make_rnn(n, seed, d, min_len=1, max_len=5)
    if model == "tree":
        return synth.make_tree(n, seed, d, min_leaves=2, max_leaves=5, teacher=False)
    return synth.make_ggnn(n, seed, d, min_nodes=3, max_nodes=6)[0]


def tiny_params(model, seed=11, scale=3.0):
    fp = synth.init_params(model, TINY[model], seed)
    rng = np.random.default_rng(seed)
    # larger weights and non-zero biases so that every term matters
    return [(scale * v + 0.1 * rng.standard_normal(v.shape)).astype(np.float32) for v in fp]


MODELS = ["mlp", "rnn", "tree", "ggnn"]


@pytest.mark.parametrize("model", MODELS)
def test_direct_gradients_by_finite_differences(model):
    dims = TINY[model]
    P = direct.unpack(model, dims, tiny_params(model))
    for inst in tiny_data(model, 3):
        res = direct.MODELS[model](P, inst, dims)
        eps = 1e-6
        for k, node in enumerate(P):
            for name, w in node.items():
                num = np.zeros_like(w)
                flat, nflat = w.reshape(-1), num.reshape(-1)
                for i in range(flat.size):
                    old = flat[i]
                    flat[i] = old + eps
                    lp = direct.MODELS[model](P, inst, dims, want_grad=False)["loss"]
                    flat[i] = old - eps
                    lm = direct.MODELS[model](P, inst, dims, want_grad=False)["loss"]
                    flat[i] = old
                    nflat[i] = (lp - lm) / (2 * eps)
                scale = max(np.abs(num).max(), 1e-8)
                assert np.abs(num - res["grads"][k][name]).max() / scale < 1e-6, (model, k, name)


def test_direct_counts_match_message_counts():
    """The number of gradient messages per node that the direct code assumes
    is the number of backward events the simulator produces."""
    for model in MODELS:
        dims = TINY[model]
        fp = tiny_params(model)
        P = direct.unpack(model, dims, fp)
        for inst in tiny_data(model, 3):
            rt = amp.Runtime(model, dims, fp)
            rt.set_muf(10 ** 9)
            rt.run([inst], mak=1)
            got = [sum(1 for e in rt.events if e[0] == n.name and e[1] == "B") for n in rt.ppt]
            assert got == direct.MODELS[model](P, inst, dims)["counts"], model


@pytest.mark.parametrize("model", MODELS)
def test_amp_mak1_update_at_retirement_equals_per_instance_sgd(model):
    dims = TINY[model]
    fp = tiny_params(model, scale=1.0)
    data = tiny_data(model, 6)
    lr = 0.05
    P = direct.unpack(model, dims, fp)
    ref_losses = direct.train(model, dims, P, data, lr)
    rt = amp.Runtime(model, dims, fp)
    rt.set_optimizer(kind="sgd", lr=lr)
    Pc = direct.unpack(model, dims, fp)
    losses = []
    for i, inst in enumerate(data):
        counts = direct.MODELS[model](Pc, inst, dims)["counts"]
        for node, c in zip(rt.ppt, counts):
            node.muf = max(c, 1)
        losses += rt.run([inst], mak=1, first_seq=i)
        for node, c in zip(rt.ppt, counts):
            assert node.count == 0 or c == 0
    assert np.allclose(losses, ref_losses, rtol=1e-12, atol=1e-13)
    for node, ref in zip(rt.ppt, P):
        for name in ref:
            assert np.allclose(node.P[name], ref[name], rtol=1e-11, atol=1e-13), (model, node.name, name)


@pytest.mark.parametrize("muf", [1, 4])
def test_amp_mlp_mak1_equals_minibatch_sgd(muf):
    dims = TINY["mlp"]
    fp = tiny_params("mlp", scale=1.0)
    data = tiny_data("mlp", 12)
    P = direct.unpack("mlp", dims, fp)
    ref = direct.train("mlp", dims, P, data, lr=0.1, batch=muf)
    rt = amp.Runtime("mlp", dims, fp)
    rt.set_optimizer(kind="sgd", lr=0.1)
    rt.set_muf(muf)
    losses = rt.run(data, mak=1)
    assert np.allclose(losses, ref, rtol=1e-12)
    for node, r in zip(rt.ppt, P):
        assert np.allclose(node.P["W"], r["W"], rtol=1e-11, atol=1e-13)
        assert np.allclose(node.P["b"], r["b"], rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("model", MODELS)
@pytest.mark.parametrize("mak", [1, 3, 8])
def test_lr_zero_any_schedule_gives_plain_forward_losses(model, mak):
    dims = TINY[model]
    fp = tiny_params(model)
    data = tiny_data(model, 9)
    P = direct.unpack(model, dims, fp)
    ref = [direct.MODELS[model](P, inst, dims, want_grad=False)["loss"] for inst in data]
    rt = amp.Runtime(model, dims, fp)
    rt.set_optimizer(kind="sgd", lr=0.0)
    rt.set_muf(3)
    losses = rt.run(data, mak=mak)
    assert np.allclose(losses, ref, rtol=1e-12, atol=1e-14)
    assert rt.max_active_seen == min(mak, len(data))


def test_ggnn_sparse_equals_dense_propagation():
    """One propagation step written as a dense (N H) x (N H) matrix acting on
    the stacked node states must give the same aggregated messages."""
    dims = TINY["ggnn"]
    H = dims["hidden"]
    fp = tiny_params("ggnn")
    P = direct.unpack("ggnn", dims, fp)
    for g in tiny_data("ggnn", 4):
        N = g["n_nodes"]
        h0 = P[0]["W"][g["node_type"]]
        big = np.zeros((N * H, N * H))
        bias = np.zeros(N * H)
        for e in range(len(g["src"])):
            s, t, c = g["src"][e], g["dst"][e], g["etype"][e]
            big[t * H:(t + 1) * H, s * H:(s + 1) * H] += P[1 + c]["W"]
            bias[t * H:(t + 1) * H] += P[1 + c]["b"]
        a_dense = (big @ h0.reshape(-1) + bias).reshape(N, H)
        # run the simulator for this instance and read the aggregated messages
        # that reached the GRU in step 0
        rt = amp.Runtime("ggnn", dims, fp)
        rt.set_muf(10 ** 9)
        seen = {}
        node = next(n for n in rt.nodes if n.name == "bcast_a")
        orig = node.forward

        def spy(rt_, port, msg, orig=orig):
            seen[msg.state] = msg.payload.copy()
            orig(rt_, port, msg)
        node.forward = spy
        rt.run([g], mak=1)
        assert np.allclose(seen[(0, 0)], a_dense, rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- control nodes
class FakeRT:
    def __init__(self):
        self.f, self.b = [], []

    def emit_fwd(self, node, port, msg):
        self.f.append((port, msg.payload, msg.state))

    def emit_bwd(self, node, port, msg):
        self.b.append((port, msg.payload, msg.state))


def test_isu_inverse_and_phi_origin():
    rt = FakeRT()
    isu = amp.Isu("i", lambda r, s: (s[0], s[1] + 1), lambda r, s: (s[0], s[1] - 1))
    isu.forward(rt, 0, amp.Msg(1.0, (7, 3)))
    assert rt.f[-1][2] == (7, 4)
    isu.backward(rt, 0, amp.Msg(2.0, rt.f[-1][2]))
    assert rt.b[-1][2] == (7, 3)
    phi = amp.Phi("p")
    phi.forward(rt, 1, amp.Msg("x", (7, 1)))
    phi.forward(rt, 0, amp.Msg("y", (7, 0)))
    phi.backward(rt, 0, amp.Msg("gy", (7, 0)))
    assert rt.b[-1][0] == 0
    phi.backward(rt, 0, amp.Msg("gx", (7, 1)))
    assert rt.b[-1][0] == 1 and not phi.origin


def test_flatmap_sums_and_restores_state():
    rt = FakeRT()
    fm = amp.Flatmap("f", lambda r, s: [(s[0], "e", k) for k in range(3)])
    fm.forward(rt, 0, amp.Msg(np.array([1.0, 2.0]), (5,)))
    assert [m[2] for m in rt.f] == [(5, "e", 0), (5, "e", 1), (5, "e", 2)]
    assert all(np.array_equal(m[1], [1.0, 2.0]) for m in rt.f)
    for k in (2, 0):
        fm.backward(rt, 0, amp.Msg(np.array([k, 1.0]), (5, "e", k)))
        assert not rt.b
    fm.backward(rt, 0, amp.Msg(np.array([1.0, 1.0]), (5, "e", 1)))
    assert rt.b[-1][2] == (5,) and np.array_equal(rt.b[-1][1], [3.0, 3.0])


def test_group_ungroup_concat_restore_states():
    rt = FakeRT()
    g = amp.Group("g", lambda r, s: (s[0], "all"), lambda r, k: 3, lambda r, s: s[1])
    for v in (2, 0, 1):
        g.forward(rt, 0, amp.Msg(np.array([float(v)]), (9, v)))
    assert len(rt.f) == 1 and rt.f[0][2] == (9, "all")
    assert np.array_equal(rt.f[0][1], [[0.0], [1.0], [2.0]])
    g.backward(rt, 0, amp.Msg(np.array([[10.0], [11.0], [12.0]]), (9, "all")))
    assert [(b[2], float(b[1][0])) for b in rt.b] == [((9, 0), 10.0), ((9, 1), 11.0), ((9, 2), 12.0)]
    rt = FakeRT()
    u = amp.Ungroup("u", lambda r, s: [(s[0], k) for k in range(2)])
    u.forward(rt, 0, amp.Msg(np.array([[1.0], [2.0]]), (4,)))
    assert [m[2] for m in rt.f] == [(4, 0), (4, 1)]
    u.backward(rt, 0, amp.Msg(np.array([7.0]), (4, 1)))
    u.backward(rt, 0, amp.Msg(np.array([6.0]), (4, 0)))
    assert rt.b[-1][2] == (4,) and np.array_equal(rt.b[-1][1], [[6.0], [7.0]])
    rt = FakeRT()
    kc = amp.KeyedConcat("c", 2, lambda s: (s[0], s[1]), lambda s: s[2])
    kc.forward(rt, 0, amp.Msg(np.array([3.0]), (1, 8, 1)))
    kc.forward(rt, 0, amp.Msg(np.array([2.0, 2.5]), (1, 8, 0)))
    assert rt.f[-1][2] == (1, 8) and np.array_equal(rt.f[-1][1], [2.0, 2.5, 3.0])
    kc.backward(rt, 0, amp.Msg(np.array([1.0, 2.0, 3.0]), (1, 8)))
    assert rt.b[0][2] == (1, 8, 0) and np.array_equal(rt.b[0][1], [1.0, 2.0])
    assert rt.b[1][2] == (1, 8, 1) and np.array_equal(rt.b[1][1], [3.0])


def test_bcast_sums_in_port_order():
    rt = FakeRT()
    b = amp.Bcast("b", 3)
    b.forward(rt, 0, amp.Msg(np.array([1.0]), (0,)))
    assert [m[0] for m in rt.f] == [0, 1, 2]
    b.backward(rt, 2, amp.Msg(np.array([4.0]), (0,)))
    b.backward(rt, 0, amp.Msg(np.array([1.0]), (0,)))
    assert not rt.b
    b.backward(rt, 1, amp.Msg(np.array([2.0]), (0,)))
    assert np.array_equal(rt.b[0][1], [7.0])


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("model", MODELS)
def test_invariants_under_asynchrony(model):
    dims = TINY[model]
    fp = tiny_params(model, scale=1.0)
    data = tiny_data(model, 20)
    mak, muf = 4, 3
    rt = amp.Runtime(model, dims, fp)
    rt.set_optimizer(kind="sgd", lr=0.05)
    rt.set_muf(muf)
    rt.run(data, mak=mak)           # asserts every forward was answered and caches are empty
    assert rt.max_active_seen == mak
    for n in rt.ppt:
        ev = [e for e in rt.events if e[0] == n.name]
        nf = sum(1 for e in ev if e[1] == "F")
        nb = sum(1 for e in ev if e[1] == "B")
        nu = sum(1 for e in ev if e[1] == "U")
        assert nf == nb
        assert sorted(e[2] for e in ev if e[1] == "F") == sorted(e[2] for e in ev if e[1] == "B")
        assert nu == nb // muf and n.count == nb - nu * muf
        cnt = 0
        for e in ev:
            if e[1] == "B":
                cnt += 1
            elif e[1] == "U":
                assert cnt >= muf
                cnt = 0
    # active count from the controller's admit / retire events never exceeds mak
    active = 0
    for e in rt.events:
        if e[0] == "controller":
            active += 1 if e[1] == "A" else -1
            assert 0 <= active <= mak


@pytest.mark.parametrize("mak", [1, 2, 4, 7])
def test_mlp_staleness_bounded_by_mak_minus_one(mak):
    """Section 3: staleness = number of updates at a node between the forward
    and the backward pass of a message.  For the MLP with an update after every
    gradient, only the other mak - 1 active instances can update in between."""
    dims = TINY["mlp"]
    rt = amp.Runtime("mlp", dims, tiny_params("mlp", scale=1.0))
    rt.set_optimizer(kind="sgd", lr=0.05)
    rt.run(tiny_data("mlp", 40), mak=mak)
    st = rt.staleness()
    worst = max(max(v) for v in st.values())
    assert worst <= mak - 1
    if mak == 1:
        assert worst == 0
    else:
        assert worst > 0


# ---------------------------------------------------------------- replay
def split_log(events, workers):
    logs = [[] for _ in workers]
    where = {name: w for w, names in enumerate(workers) for name in names}
    for name, kind, key in events:
        if name == "controller":
            continue
        seq, local = key if key is not None else (0, 0)
        logs[where[name]].append((name, kind, seq, local))
    return logs


@pytest.mark.parametrize("model", MODELS)
def test_replay_reproduces_a_recorded_run(model):
    dims = TINY[model]
    fp = tiny_params(model, scale=1.0)
    data = tiny_data(model, 15)
    rt = amp.Runtime(model, dims, fp)
    rt.set_optimizer(kind="adam", lr=0.01)
    rt.set_muf(2)
    losses = rt.run(data, mak=4)
    names = [n.name for n in rt.ppt]
    # workers: first two nodes share a worker, every other node has its own
    workers = [names[:2]] + [[n] for n in names[2:]]
    logs = split_log(rt.events, workers)
    rp = amp.Runtime(model, dims, fp)
    rp.set_optimizer(kind="adam", lr=0.01)
    rp.set_muf(2)
    rp.replay(data, logs)
    assert [rp.loss[s] for s in range(len(data))] == losses
    for a, b in zip(rt.ppt, rp.ppt):
        for k in a.P:
            assert np.array_equal(a.P[k], b.P[k])


def test_replay_refuses_illegal_logs():
    dims = TINY["mlp"]
    fp = tiny_params("mlp", scale=1.0)
    data = tiny_data("mlp", 6)
    rt = amp.Runtime("mlp", dims, fp)
    rt.set_muf(2)
    rt.run(data, mak=2)
    logs = split_log(rt.events, [["lin1"], ["lin2"], ["lin3"]])

    def fresh():
        r = amp.Runtime("mlp", dims, fp)
        r.set_muf(2)
        return r
    fresh().replay(data, copy.deepcopy(logs))
    # an update dropped
    bad = copy.deepcopy(logs)
    bad[1].remove(next(e for e in bad[1] if e[1] == "U"))
    with pytest.raises(RuntimeError):
        fresh().replay(data, bad)
    # an update before enough gradients were accumulated
    bad = copy.deepcopy(logs)
    i = next(k for k, e in enumerate(bad[2]) if e[1] == "U")
    bad[2].insert(i - 1, bad[2].pop(i))
    with pytest.raises(RuntimeError):
        fresh().replay(data, bad)
    # a backward event before its forward
    bad = copy.deepcopy(logs)
    i = next(k for k, e in enumerate(bad[0]) if e[1] == "B")
    bad[0].insert(0, bad[0].pop(i))
    with pytest.raises(RuntimeError):
        fresh().replay(data, bad)
    # a forward event lost
    bad = copy.deepcopy(logs)
    bad[2] = [e for e in bad[2] if not (e[1] in "FB" and e[2] == 5)]
    with pytest.raises(RuntimeError):
        fresh().replay(data, bad)


def test_replicas_with_one_update_per_epoch_equal_full_batch_sgd():
    """Section 5: replicas are data parallelism.  If every replica makes exactly one update per epoch, from the
    mean gradient of its (equally large) share, the average of the replicas is plain SGD on the mean gradient of
    the whole set -- computed here by the direct trainer, which knows nothing of messages or replicas."""
    model, dims, data = synth.workload(1, n=24)
    fp = synth.init_params(model, dims, 3)
    R, lr, epochs = 3, 0.1, 2
    rts = []
    for _ in range(R):
        rt = amp.Runtime(model, dims, fp)
        rt.set_muf(len(data) // R)
        rt.set_optimizer(kind="sgd", lr=lr)
        rts.append(rt)
    losses = amp.run_replicas(rts, data, mak=2, epochs=epochs)
    P = direct.unpack(model, dims, fp)
    ref = []
    for _ in range(epochs):
        ref += direct.train(model, dims, P, data, lr=lr, batch=len(data))
    assert np.allclose(losses, ref, rtol=1e-12, atol=1e-12)
    for rt in rts:
        for k, node in enumerate(rt.ppt):
            for name in node.P:
                assert np.allclose(node.P[name], P[k][name], rtol=1e-12, atol=1e-14), (k, name)


def test_replica_routing_and_average():
    data = list(range(10))
    assert amp.replica_subsets(data, 3) == [[0, 3, 6, 9], [1, 4, 7], [2, 5, 8]]
    model, dims, _ = synth.workload(1, n=1)
    rts = [amp.Runtime(model, dims, synth.init_params(model, dims, s)) for s in (1, 2, 3, 4)]
    before = [[{k: v.copy() for k, v in n.P.items()} for n in rt.ppt] for rt in rts]
    amp.average_replicas(rts)
    for k in range(len(rts[0].ppt)):
        for name in rts[0].ppt[k].P:
            want = (before[0][k][name] + before[1][k][name] + before[2][k][name] + before[3][k][name]) / 4.0
            for rt in rts:
                assert np.allclose(rt.ppt[k].P[name], want, rtol=0, atol=1e-15)


@pytest.mark.parametrize("mak,muf,lr", [(16, 7, 0.0005), (4, 3, 0.0002)])
def test_rnn_adam_parity_setting_is_well_conditioned(mak, muf, lr):
    """The GPU parity cases for the recurrent model under Adam compare two fp32/fp64 runs to 1e-5; that only
    makes sense where the training run does not amplify rounding differences.  A 1e-7 relative perturbation of
    the initial parameters must stay near 1e-7 at the settings the parity test uses (300 sequences; lr = 5e-4 at
    max_active_keys 16, min_update_frequency 7; lr = 2e-4 at max_active_keys 4, min_update_frequency 3)."""
    model, dims, data = synth.workload(2, n=300)
    fp = synth.init_params(model, dims, 6)
    rng = np.random.default_rng(0)
    fp2 = [(p * (1 + 1e-7 * rng.standard_normal(p.shape))).astype(np.float32) for p in fp]
    res = []
    for f in (fp, fp2):
        rt = amp.Runtime(model, dims, f)
        rt.set_muf(muf)
        rt.set_optimizer(kind="adam", lr=float(np.float32(lr)), beta1=float(np.float32(0.9)),
                         beta2=float(np.float32(0.999)), eps=float(np.float32(1e-6)))
        rt.set_optimizer("lookup", kind="sgd", lr=float(np.float32(lr)))
        rt.run(data, mak)
        res.append([amp.C.pack_node(n.P) for n in rt.ppt])
    for a, b in zip(*res):
        assert np.linalg.norm(a - b) / np.linalg.norm(a) < 1e-6


def test_mlp_momentum_parity_setting_is_well_conditioned():
    """The same for the MLP's momentum case (max_active_keys 8, min_update_frequency 5, momentum 0.9): at lr = 0.02
    the training run is unstable (losses spike to twice their initial value); at lr = 0.005, which the parity
    case uses, a 1e-7 perturbation stays at 1e-7."""
    model, dims, data = synth.workload(1)
    fp = synth.init_params(model, dims, 5)
    rng = np.random.default_rng(1)
    fp2 = [(p * (1 + 1e-7 * rng.standard_normal(p.shape))).astype(np.float32) for p in fp]
    res = []
    for f in (fp, fp2):
        rt = amp.Runtime(model, dims, f)
        rt.set_muf(5)
        rt.set_optimizer(kind="momentum", lr=float(np.float32(0.005)), momentum=float(np.float32(0.9)))
        rt.run(data, 8)
        res.append([amp.C.pack_node(n.P) for n in rt.ppt])
    for a, b in zip(*res):
        assert np.linalg.norm(a - b) / np.linalg.norm(a) < 1e-6


def _perturbation_response(model, dims, data, fp, mak, muf, opt, lookup_muf=None):
    """Trains twice on the checker's own schedule, the second time from initial parameters perturbed by 1e-7
    (relative, Gaussian): per node, (difference of the results in the 2-norm, largest element-wise difference), both
    relative -- the second to max(|element|, rms of the tensor)."""
    rng = np.random.default_rng(0)
    fp2 = [(p * (1 + 1e-7 * rng.standard_normal(p.shape))).astype(np.float32) for p in fp]
    res = []
    for f in (fp, fp2):
        rt = amp.Runtime(model, dims, f)
        rt.set_muf(muf)
        if lookup_muf is not None:
            rt.set_muf(lookup_muf, "lookup")
        rt.set_optimizer(**{k: (float(np.float32(v)) if isinstance(v, float) else v) for k, v in opt.items()})
        if model != "mlp":
            rt.set_optimizer("lookup", kind="sgd", lr=float(np.float32(opt["lr"])))
        rt.run(data, mak)
        res.append([amp.C.pack_node(n.P) for n in rt.ppt])
    out = []
    for a, b in zip(*res):
        scale = np.maximum(np.abs(a), np.sqrt(np.mean(a * a)))
        out.append((float(np.linalg.norm(a - b) / np.linalg.norm(a)), float((np.abs(a - b) / scale).max())))
    return out


_ADAM = dict(kind="adam", lr=0.0005, beta1=0.9, beta2=0.999, eps=1e-6)
_TREE_ODD = dict(vocab=97, emb=50, hidden=37, n_class=5)


@pytest.mark.parametrize("case", ["ggnn-adam", "ggnn-momentum", "tree-momentum", "tree-adam"])
def test_softened_parity_settings_are_well_conditioned(case):
    """The GPU replay cases for the graph model under Adam (lr 2e-4, eps 1e-6), the graph and tree models under
    momentum (lr 5e-4 / 5e-3) and the odd-size tree under Adam run at smaller steps than first tried.  What
    justifies a setting is that the training run itself does not amplify rounding: a 1e-7 perturbation of the
    initial parameters must come out below 3e-7 in every tensor's norm.  For contrast the graph model under Adam at
    the step first tried (2e-3) amplifies it more than three times."""
    if case.startswith("ggnn"):
        _, dims, data = synth.workload(4, n=150)
        fp = synth.init_params("ggnn", dims, 9)
        if case == "ggnn-adam":
            resp = _perturbation_response("ggnn", dims, data, fp, 32, 20, dict(_ADAM, lr=0.0002))
            worse = _perturbation_response("ggnn", dims, data, fp, 32, 20, dict(_ADAM, lr=0.002))
            assert max(n for n, _ in worse) > 3e-7
        else:
            resp = _perturbation_response("ggnn", dims, data, fp, 8, 3, dict(kind="momentum", lr=0.0005, momentum=0.9))
    else:
        data = synth.make_tree(64, 21, _TREE_ODD)
        fp = synth.init_params("tree", _TREE_ODD, 8)
        if case == "tree-momentum":
            resp = _perturbation_response("tree", _TREE_ODD, data, fp, 8, 4, dict(kind="momentum", lr=0.005, momentum=0.9), 5)
        else:
            resp = _perturbation_response("tree", _TREE_ODD, data, fp, 8, 3, _ADAM, 5)
    assert max(n for n, _ in resp) < 3e-7, resp


def test_adam_amplifies_single_elements_and_eps_sets_how_much():
    """Why the Adam replay cases use eps = 1e-6 and why their element-wise bound is wider than SGD's: Adam's step
    has slope up to lr / eps in an element whose gradient is near zero.  On the benchmark-size tree cell the same
    1e-7 perturbation leaves the tensors' norms within 2e-7 either way, but single elements move by more than 1e-5
    of the tensor's typical magnitude at eps = 1e-8, against a few 1e-6 at eps = 1e-6 and below 1e-6 (little more than the
    perturbation's own largest element) under SGD -- at 1e-8 no fp32 run could be held to 1e-5 element by element, or, on an
    unlucky run, in the norm."""
    from util import ETOL_ADAM
    dims = synth.DEFAULT_DIMS["tree"]
    data = synth.make_tree(40, 21, dims)
    fp = synth.init_params("tree", dims, 8)
    loose = _perturbation_response("tree", dims, data, fp, 64, 7, _ADAM, 333)
    tight = _perturbation_response("tree", dims, data, fp, 64, 7, dict(_ADAM, eps=1e-8), 333)
    sgd = _perturbation_response("tree", _TREE_ODD, synth.make_tree(64, 21, _TREE_ODD), synth.init_params("tree", _TREE_ODD, 8),
                                 8, 3, dict(kind="sgd", lr=0.05), 5)
    assert max(n for n, _ in loose + tight) < 3e-7
    assert max(e for _, e in sgd) < 1e-6
    assert 1e-6 < max(e for _, e in loose) < ETOL_ADAM / 5
    assert max(e for _, e in tight) > 1e-5


def test_relu_decision_hook():
    """The checker's ReLU lists its decisions on inputs within kink_tau of zero and records the ones named in
    `flip` the other way round for the backward pass; everything else is untouched."""
    class Catch:
        def __init__(self):
            self.f, self.b = [], []

        def emit_fwd(self, node, port, msg):
            self.f.append(msg.payload)

        def emit_bwd(self, node, port, msg):
            self.b.append(msg.payload)

    x = np.array([1e-9, -1e-9, 0.5, -0.5])
    dy = np.array([2.0, 3.0, 4.0, 5.0])
    for flip, want in ((set(), [2.0, 0.0, 4.0, 0.0]), ({((7,), 0)}, [0.0, 0.0, 4.0, 0.0]), ({((7,), 1)}, [2.0, 3.0, 4.0, 0.0])):
        node = amp.NPT("relu1", amp.C.relu_fwd, amp.C.relu_bwd)
        node.kink_tau, node.flip = 1e-6, flip
        rt = Catch()
        node.forward(rt, 0, amp.Msg(x, (7,)))
        node.backward(rt, 0, amp.Msg(dy, (7,)))
        assert node.kinks == [((7,), 0), ((7,), 1)]
        assert np.array_equal(rt.f[0], np.maximum(x, 0.0))
        assert np.array_equal(rt.b[0], np.array(want))
    plain = amp.NPT("relu1", amp.C.relu_fwd, amp.C.relu_bwd)
    rt = Catch()
    plain.forward(rt, 0, amp.Msg(x, (7,)))
    assert plain.kinks == []


def test_staleness_bounded_admission_in_the_checker():
    """The controller's own limit on the instances in flight (Appendix B, MNIST).  Bound 0 keeps one instance in
    flight once an update has happened and so repeats the max_active_keys = 1 run exactly; a bound nothing reaches
    lets the limit rise to max_active_keys; in between the limit settles below max_active_keys and the measured
    gradient staleness (Section 3) stays below the greedy controller's."""
    model, dims, data = synth.workload(2, n=60)
    fp = synth.init_params(model, dims, 6)

    def run(mak, bound):
        rt = amp.Runtime(model, dims, fp)
        rt.set_muf(1)
        rt.set_optimizer(kind="sgd", lr=0.05)
        losses = rt.run(data, mak, max_staleness=bound)
        worst = max(max(v) for v in rt.staleness().values() if v)
        return rt, losses, worst

    seq, seq_losses, _ = run(1, None)
    b0, b0_losses, _ = run(16, 0.0)
    assert b0.max_active_seen == 1 and b0_losses == seq_losses
    for a, b in zip(seq.ppt, b0.ppt):
        for k in a.P:
            assert np.array_equal(a.P[k], b.P[k])
    greedy, _, greedy_stale = run(16, None)
    free, _, _ = run(16, 1e9)
    assert greedy.max_active_seen == 16 and free.max_active_seen == 16 and free.limit >= 16
    mid, _, mid_stale = run(16, 40.0)
    assert 1 < mid.max_active_seen < 16
    assert mid_stale < greedy_stale


# ---------------------------------------------------------------- training and inference instances in one run
@pytest.mark.parametrize("model", ["mlp", "rnn", "tree", "ggnn"])
def test_inference_instances_leave_training_untouched(model):
    """Section 1: inference instances travel through the same graph as training instances, forward only.  With one
    instance in flight the interleaved run must leave exactly the parameters of the training-only run, the
    training losses must be the same, every inference instance's loss must be the plain forward loss under the
    parameters the training instances before it produced, and nothing may stay cached in any node."""
    dims = TINY[model]
    train, evals = tiny_data(model, 12, 5), tiny_data(model, 4, 6)
    fp = synth.init_params(model, dims, 3)

    def runtime():
        rt = amp.Runtime(model, dims, fp)
        rt.set_muf(2)
        rt.set_optimizer(kind="sgd", lr=0.05)
        return rt
    mixed = runtime()
    tl, el = mixed.run_mixed(train, evals, mak=1)
    plain = runtime()
    pl = plain.run(train, mak=1)
    assert tl == pl
    for a, b in zip(mixed.params(), plain.params()):
        assert np.array_equal(a, b)
    stride = len(train) // len(evals)
    for j, inst in enumerate(evals):
        prefix = runtime()
        prefix.run(train[:(j + 1) * stride], mak=1)
        P = direct.unpack(model, dims, prefix.params())
        ref = direct.MODELS[model](P, inst, dims, want_grad=False)["loss"]
        assert abs(el[j] - ref) <= 1e-12 * max(1.0, abs(ref)), (j, el[j], ref)
    # several in flight: every training forward is still answered, inference instances leave nothing behind
    busy = runtime()
    tl2, el2 = busy.run_mixed(train, evals, mak=5, epochs=2)
    assert len(tl2) == 2 * len(train) and len(el2) == len(evals)
    assert busy.max_active_seen <= 5
    kinds = [k for (n, k, _) in busy.events if n == "controller"]
    assert kinds.count("A") == kinds.count("R") == 2 * len(train) + len(evals)


# ---------------------------------------------------------------- replicas of one heavy node (Section 5)
def _fixed_len_rnn(n, length, seed=5):
    return synth.make_rnn(n, seed, TINY["rnn"], min_len=length, max_len=length)


def test_node_replicas_with_one_update_per_epoch_equal_full_batch_sgd():
    """Copies of the RNN's cell between a Cond and a Phi, the output layer shared.  If every copy makes exactly one
    update per epoch, from the mean of the gradient messages of its (equally long) share, and so does the shared
    layer from all of them, then after the end-of-epoch averaging the model is what plain full-batch SGD gives --
    computed by the direct trainer, which knows nothing of messages, Cond, Phi or copies."""
    R, n, T, lr, epochs = 3, 12, 3, 0.1, 2
    dims = dict(TINY["rnn"], node_replicas=R)
    fp = tiny_params("rnn", scale=1.0)
    data = _fixed_len_rnn(n, T)
    rt = amp.Runtime("rnn", dims, fp)
    assert [p.name for p in rt.ppt] == ["lookup", "cell", "out", "lookup.r1", "cell.r1", "lookup.r2", "cell.r2"]
    rt.set_optimizer(kind="sgd", lr=lr)
    rt.set_muf(n // R * T, "lookup")
    rt.set_muf(n // R * T, "cell")
    rt.set_muf(n, "out")
    P = direct.unpack("rnn", TINY["rnn"], fp)
    losses, ref = [], []
    for e in range(epochs):
        losses += rt.run(data, mak=4, first_seq=e * n)
        assert all(p.count == 0 for p in rt.ppt)          # everybody has just updated
        amp.average_node_replicas(rt)
        ref += direct.train("rnn", TINY["rnn"], P, data, lr=lr, batch=n)
    assert np.allclose(losses, ref, rtol=1e-12, atol=1e-12)
    for p in rt.ppt:
        k = ["lookup", "cell", "out"].index(p.name.split(".r")[0])
        for name in p.P:
            assert np.allclose(p.P[name], P[k][name], rtol=1e-11, atol=1e-13), (p.name, name)


def test_node_replicas_route_on_the_instance_and_stay_apart():
    """The Conds send admission a to copy a mod R, every step of it, and its gradients come back to that copy; with
    the shared layer frozen a copy therefore trains exactly as a model of its own on its share of the instances."""
    R, n = 2, 8
    dims = dict(TINY["rnn"], node_replicas=R)
    fp = tiny_params("rnn", scale=1.0)
    data = tiny_data("rnn", n)
    rt = amp.Runtime("rnn", dims, fp)
    rt.set_optimizer(kind="sgd", lr=0.05)
    rt.set_optimizer("out", kind="sgd", lr=0.0)
    rt.set_muf(2)
    rt.run(data, mak=1)
    for name, kind, key in rt.events:
        if name.split(".r")[0] in ("lookup", "cell") and kind in ("F", "B"):
            copy = int(name.split(".r")[1]) if ".r" in name else 0
            assert key[0] % R == copy, (name, kind, key)
    for r in range(R):
        alone = amp.Runtime("rnn", TINY["rnn"], fp)
        alone.set_optimizer(kind="sgd", lr=0.05)
        alone.set_optimizer("out", kind="sgd", lr=0.0)
        alone.set_muf(2)
        alone.run(data[r::R], mak=1)
        for base in ("lookup", "cell"):
            mine = next(p for p in rt.ppt if p.name == (base if r == 0 else "%s.r%d" % (base, r)))
            ref = next(p for p in alone.ppt if p.name == base)
            for name in ref.P:
                assert np.array_equal(mine.P[name], ref.P[name]), (r, base, name)


def test_one_copy_is_the_plain_graph():
    fp = tiny_params("rnn", scale=1.0)
    data = tiny_data("rnn", 6)
    a = amp.Runtime("rnn", TINY["rnn"], fp)
    b = amp.Runtime("rnn", dict(TINY["rnn"], node_replicas=1), fp)
    for rt in (a, b):
        rt.set_muf(3)
    assert a.run(data, mak=3) == b.run(data, mak=3)


# ---------------------------------------------------------------- asynchronous synchronisation of the copies
def _worker_logs(rt):
    """The recorded run as per-node logs in the form the replay driver takes."""
    logs = {}
    for name, kind, key in rt.events:
        if name != "controller":
            logs.setdefault(name, []).append((name, kind) + (key if key is not None else (0, 0)))
    return list(logs.values())


def test_group_synchronisation_by_hand():
    """A copy publishes its parameters when the request reaches it and carries on; once every copy has published,
    each moves to the mean of the published values and keeps what it learned since it published."""
    dims = dict(TINY["rnn"], node_replicas=2)
    rt = amp.Runtime("rnn", dims, tiny_params("rnn"))
    c0 = next(p for p in rt.ppt if p.name == "cell")
    c1 = next(p for p in rt.ppt if p.name == "cell.r1")
    a0, a1 = c0.P["W"].copy(), c0.P["W"] + 2.0
    c1.P["W"] = a1.copy()
    rt.sync_snapshot(c0, 1)
    assert not rt.sync_ready(c0, 1)
    rt.sync_snapshot(c1, 1)
    assert rt.sync_ready(c0, 1) and rt.sync_ready(c1, 1)
    c1.P["W"] = c1.P["W"] + 0.25                       # an update of copy 1 between its snapshot and its load
    rt.sync_load(c0, 1)
    rt.sync_load(c1, 1)
    assert np.allclose(c0.P["W"], (a0 + a1) / 2, rtol=0, atol=1e-15)
    assert np.allclose(c1.P["W"], (a0 + a1) / 2 + 0.25, rtol=0, atol=1e-15)
    assert np.array_equal(c0.P["b"], c1.P["b"])        # equal before, equal after
    look = next(p for p in rt.ppt if p.name == "lookup")
    assert not rt.sync_ready(look, 1)                  # the tables are a group of their own


def test_one_synchronisation_at_the_end_of_the_epoch_is_the_epoch_end_average():
    dims = dict(TINY["rnn"], node_replicas=3)
    fp = tiny_params("rnn", scale=1.0)
    data = tiny_data("rnn", 9)
    a = amp.Runtime("rnn", dims, fp)
    b = amp.Runtime("rnn", dims, fp)
    for rt in (a, b):
        rt.set_muf(2)
    a.sync_every = len(data)
    la, lb = a.run(data, mak=3), b.run(data, mak=3)
    amp.average_node_replicas(b)
    assert la == lb
    for pa, pb in zip(a.ppt, b.ppt):
        for name in pa.P:
            assert np.allclose(pa.P[name], pb.P[name], rtol=0, atol=1e-15), (pa.name, name)


def test_replay_of_a_run_with_synchronisation_rounds():
    """The replay driver takes the snapshots and loads where each copy's record has them; a load waits until every
    copy's snapshot of the round is there, whatever the order of the records; a load without a snapshot is refused."""
    dims = dict(TINY["rnn"], node_replicas=2)
    fp = tiny_params("rnn", scale=1.0)
    data = tiny_data("rnn", 8)

    def fresh():
        rt = amp.Runtime("rnn", dims, fp)
        rt.set_muf(3)
        return rt
    rec = fresh()
    rec.sync_every = 3
    rec.run(data, mak=3)
    logs = _worker_logs(rec)
    assert sum(1 for log in logs for e in log if e[1] == "S") == 2 * 4       # two rounds, four replicated nodes
    for order in (logs, logs[::-1]):
        rt = fresh().replay(data, order)
        for p, q in zip(rt.ppt, rec.ppt):
            for name in p.P:
                assert np.array_equal(p.P[name], q.P[name]), (p.name, name)
    # copy 1 of the cell loads later, after one more of its own updates: it keeps that update on top of the mean
    late = [list(log) for log in logs]
    w = next(log for log in late if log[0][0] == "cell.r1")
    i = next(k for k, e in enumerate(w) if e[1] == "L")
    j = next(k for k in range(i + 1, len(w)) if w[k][1] == "U")
    w.insert(j, w.pop(i))
    rt = fresh().replay(data, late)
    c1, r1 = next(p for p in rt.ppt if p.name == "cell.r1"), next(p for p in rec.ppt if p.name == "cell.r1")
    assert not np.array_equal(c1.P["W"], r1.P["W"])
    bad = [[e for e in log if not (e[0] == "cell" and e[1] == "S" and e[2] == 1)] for log in logs]
    with pytest.raises(RuntimeError):
        fresh().replay(data, bad)
