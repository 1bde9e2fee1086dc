"""Seeded synthetic workloads and initial parameters.

Stand-ins for the datasets the paper trains on (Section 6: MNIST, list
reduction, Stanford Sentiment Treebank, QM9), which are not available here.
Shapes and sizes follow the paper's experiment descriptions; the items
themselves are generated.  Everything is drawn from a counter-based Philox
stream, so the same (config, seed) always yields the same instances.

This module serves both the HIP path and the CPU checker as a source of
*inputs only*: it builds instance structures, labels and initial parameter
values.  The label rules for the tree and graph workloads are small
"teacher" networks written here in plain numpy; neither the HIP path nor the
checker imports them for anything but the labels they produce.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 1705

# PPT node names per model, in node-id order (the ids used at the C boundary).
NODE_NAMES = {
    "mlp": ["lin1", "lin2", "lin3"],
    "rnn": ["lookup", "cell", "out"],
    "tree": ["lookup", "leaf", "branch", "out"],
    "ggnn": ["lookup", "edge0", "edge1", "edge2", "edge3", "gz", "gr", "gh", "readout"],
}

DEFAULT_DIMS = {
    "mlp": dict(d_in=64, hidden=128, n_class=10),
    "rnn": dict(vocab=20, emb=128, hidden=128, n_class=10),
    "tree": dict(vocab=20000, emb=300, hidden=150, n_class=5),
    "tree_big": dict(vocab=20000, emb=1024, hidden=1024, n_class=5),
    "ggnn": dict(n_node_types=16, hidden=100, n_edge_types=4, n_steps=4),
}


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(int(seed)))


# --------------------------------------------------------------------------
# parameter shapes and initial values
# --------------------------------------------------------------------------
def param_shapes(model: str, dims: dict) -> list:
    """[(name, rows, cols, has_bias)] per PPT node, node-id order.

    A node's flat parameter vector is W (rows x cols, row-major) followed by
    b (rows) when has_bias.  Gate row blocks: leaf = [i; o; u], branch =
    [i; f_l; f_r; o; u], each block `hidden` rows.
    """
    if model == "mlp":
        d, h, c = dims["d_in"], dims["hidden"], dims["n_class"]
        return [("lin1", h, d, True), ("lin2", h, h, True), ("lin3", c, h, True)]
    if model == "rnn":
        v, e, h, c = dims["vocab"], dims["emb"], dims["hidden"], dims["n_class"]
        return [("lookup", v, e, False), ("cell", h, e + h, True), ("out", c, h, True)]
    if model == "tree":
        v, e, h, c = dims["vocab"], dims["emb"], dims["hidden"], dims["n_class"]
        return [("lookup", v, e, False), ("leaf", 3 * h, e, True),
                ("branch", 5 * h, 2 * h, True), ("out", c, h, True)]
    if model == "ggnn":
        t, h, ne = dims["n_node_types"], dims["hidden"], dims["n_edge_types"]
        out = [("lookup", t, h, False)]
        out += [("edge%d" % c, h, h, True) for c in range(ne)]
        out += [("gz", h, 2 * h, True), ("gr", h, 2 * h, True), ("gh", h, 2 * h, True),
                ("readout", 1, h, True)]
        return out
    raise ValueError(model)


def init_params(model: str, dims: dict, seed: int) -> list:
    """Initial parameters: one flat float32 vector per PPT node.

    Uniform(-a, a) with a = 1/sqrt(cols) for weights, zeros for biases,
    N(0, 0.1) rows for lookup tables.
    """
    rng = _rng(seed)
    out = []
    for name, rows, cols, has_bias in param_shapes(model, dims):
        if name == "lookup":
            w = (0.1 * rng.standard_normal((rows, cols))).astype(np.float32)
            out.append(w.reshape(-1))
            continue
        a = 1.0 / np.sqrt(cols)
        w = rng.uniform(-a, a, size=(rows, cols)).astype(np.float32)
        vec = [w.reshape(-1)]
        if has_bias:
            vec.append(np.zeros(rows, np.float32))
        out.append(np.concatenate(vec))
    return out


# --------------------------------------------------------------------------
# config 1: MLP, argmax of a fixed linear teacher
# --------------------------------------------------------------------------
def make_mlp(n: int, seed: int, dims: dict | None = None) -> list:
    dims = dims or DEFAULT_DIMS["mlp"]
    teacher = _rng(BASE_SEED * 7 + 1).standard_normal((dims["n_class"], dims["d_in"]))
    rng = _rng(seed)
    x = rng.standard_normal((n, dims["d_in"])).astype(np.float32)
    labels = np.argmax(x.astype(np.float64) @ teacher.T, axis=1).astype(np.int32)
    return [dict(x=x[i], label=int(labels[i])) for i in range(n)]


# --------------------------------------------------------------------------
# config 2: variable-length list reduction (sum of token values mod 10)
# --------------------------------------------------------------------------
def make_rnn(n: int, seed: int, dims: dict | None = None, min_len: int = 4, max_len: int = 32,
             reduction: str = "sum") -> list:
    """reduction "sum": label = sum of the token values mod n_class (the benchmark workload; a tanh RNN of this size
    does not learn it within hundreds of epochs).  reduction "max": label = largest token value scaled to n_class
    classes -- a reduction the RNN learns in a few epochs, for experiments that measure time to convergence."""
    dims = dims or DEFAULT_DIMS["rnn"]
    rng = _rng(seed)
    out = []
    for _ in range(n):
        t = int(rng.integers(min_len, max_len + 1))
        tok = rng.integers(0, dims["vocab"], size=t).astype(np.int32)
        if reduction == "sum":
            label = int(tok.sum() % dims["n_class"])
        elif reduction == "max":
            label = int(tok.max()) * dims["n_class"] // dims["vocab"]
        else:
            raise ValueError("reduction must be 'sum' or 'max'")
        out.append(dict(tokens=tok, label=label))
    return out


# --------------------------------------------------------------------------
# configs 3 and 5: random binary trees with a label at every node
# --------------------------------------------------------------------------
def _zipf_cdf(vocab: int, a: float = 1.1) -> np.ndarray:
    p = 1.0 / np.arange(1, vocab + 1, dtype=np.float64) ** a
    return np.cumsum(p / p.sum())


def _random_tree(rng, n_leaves: int):
    """Leaves are nodes 0..L-1 left to right; internal nodes follow in
    post-order (children before parents); the root is node 2L-2."""
    left = [-1] * n_leaves
    right = [-1] * n_leaves

    def build(lo: int, cnt: int) -> int:
        if cnt == 1:
            return lo
        k = int(rng.integers(1, cnt))
        a = build(lo, k)
        b = build(lo + k, cnt - k)
        left.append(a)
        right.append(b)
        return len(left) - 1

    root = build(0, n_leaves)
    assert root == 2 * n_leaves - 2
    return np.asarray(left, np.int32), np.asarray(right, np.int32)


def _sig(x):
    return 1.0 / (1.0 + np.exp(-x))


def _tree_teacher_labels(trees: list, vocab: int, n_class: int) -> None:
    """Label rule: a small fixed random tree network (hidden 32) run bottom-up;
    label = argmax of a linear map of each node's hidden vector."""
    rng = _rng(BASE_SEED * 7 + 3)
    ht = 32
    emb = rng.standard_normal((vocab, ht))
    wl = rng.standard_normal((3 * ht, ht)) / np.sqrt(ht) * 2.0
    wb = rng.standard_normal((5 * ht, 2 * ht)) / np.sqrt(2 * ht) * 2.0
    wo = rng.standard_normal((n_class, ht))
    for tr in trees:
        nl = tr["n_leaves"]
        nn = 2 * nl - 1
        h = np.zeros((nn, ht))
        c = np.zeros((nn, ht))
        g = emb[tr["tokens"]] @ wl.T
        c[:nl] = _sig(g[:, :ht]) * np.tanh(g[:, 2 * ht:])
        h[:nl] = _sig(g[:, ht:2 * ht]) * np.tanh(c[:nl])
        for p in range(nl, nn):
            a, b = tr["left"][p], tr["right"][p]
            g = wb @ np.concatenate([h[a], h[b]])
            i, fl, fr, o, u = (g[k * ht:(k + 1) * ht] for k in range(5))
            c[p] = _sig(i) * np.tanh(u) + _sig(fl) * c[a] + _sig(fr) * c[b]
            h[p] = _sig(o) * np.tanh(c[p])
        tr["labels"] = np.argmax(h @ wo.T, axis=1).astype(np.int32)


def make_tree(n: int, seed: int, dims: dict | None = None, min_leaves: int = 2,
              max_leaves: int = 60, teacher: bool = True) -> list:
    dims = dims or DEFAULT_DIMS["tree"]
    rng = _rng(seed)
    cdf = _zipf_cdf(dims["vocab"])
    out = []
    for _ in range(n):
        nl = int(rng.integers(min_leaves, max_leaves + 1))
        left, right = _random_tree(rng, nl)
        tok = np.searchsorted(cdf, rng.random(nl)).astype(np.int32)
        tok = np.minimum(tok, dims["vocab"] - 1)
        out.append(dict(n_leaves=nl, tokens=tok, left=left, right=right))
    if teacher:
        _tree_teacher_labels(out, dims["vocab"], dims["n_class"])
    else:
        for tr in out:
            tr["labels"] = rng.integers(0, dims["n_class"], size=2 * tr["n_leaves"] - 1).astype(np.int32)
    return out


# --------------------------------------------------------------------------
# config 4: molecule-like typed graphs with a scalar regression target
# --------------------------------------------------------------------------
EDGE_TYPE_P = (0.7, 0.2, 0.05, 0.05)


def _graph_teacher_targets(graphs: list, dims: dict) -> np.ndarray:
    """Label rule: a small fixed random gated graph network (hidden 16)."""
    rng = _rng(BASE_SEED * 7 + 4)
    ht = 16
    emb = rng.standard_normal((dims["n_node_types"], ht))
    we = rng.standard_normal((dims["n_edge_types"], ht, ht)) / np.sqrt(ht)
    wz, wr, wh = (rng.standard_normal((ht, 2 * ht)) / np.sqrt(2 * ht) for _ in range(3))
    wout = rng.standard_normal(ht)
    ys = np.zeros(len(graphs))
    for gi, g in enumerate(graphs):
        h = emb[g["node_type"]]
        for _ in range(dims["n_steps"]):
            a = np.zeros_like(h)
            m = np.einsum("eij,ej->ei", we[g["etype"]], h[g["src"]])
            np.add.at(a, g["dst"], m)
            ah = np.concatenate([a, h], axis=1)
            z = _sig(ah @ wz.T)
            r = _sig(ah @ wr.T)
            ht_ = np.tanh(np.concatenate([a, r * h], axis=1) @ wh.T)
            h = (1 - z) * h + z * ht_
        ys[gi] = h.sum(axis=0) @ wout
    return ys


def make_ggnn(n: int, seed: int, dims: dict | None = None, min_nodes: int = 9,
              max_nodes: int = 29, norm=None):
    """Returns (graphs, norm).  Each undirected bond j becomes directed edges
    2j (u->v) and 2j+1 (v->u) of the same type.  `norm` = (mean, std) used to
    standardise the teacher output; computed from this set when None."""
    dims = dims or DEFAULT_DIMS["ggnn"]
    rng = _rng(seed)
    out = []
    for _ in range(n):
        nn = int(rng.integers(min_nodes, max_nodes + 1))
        bonds = set()
        for v in range(1, nn):
            bonds.add((int(rng.integers(0, v)), v))
        extra = int(round(0.1 * nn)) + 1
        tries = 0
        while extra > 0 and tries < 100:
            u, v = sorted(int(t) for t in rng.integers(0, nn, size=2))
            tries += 1
            if u != v and (u, v) not in bonds:
                bonds.add((u, v))
                extra -= 1
        bonds = sorted(bonds)
        bt = rng.choice(dims["n_edge_types"], size=len(bonds), p=EDGE_TYPE_P[:dims["n_edge_types"]]
                        if dims["n_edge_types"] == 4 else None)
        src, dst, et = [], [], []
        for (u, v), t in zip(bonds, bt):
            src += [u, v]
            dst += [v, u]
            et += [int(t), int(t)]
        out.append(dict(n_nodes=nn,
                        node_type=rng.integers(0, dims["n_node_types"], size=nn).astype(np.int32),
                        src=np.asarray(src, np.int32), dst=np.asarray(dst, np.int32),
                        etype=np.asarray(et, np.int32)))
    ys = _graph_teacher_targets(out, dims)
    if norm is None:
        norm = (float(ys.mean()), float(ys.std() + 1e-12))
    for g, y in zip(out, ys):
        g["target"] = float(np.float32((y - norm[0]) / norm[1]))
    return out, norm


# --------------------------------------------------------------------------
# the five named workloads
# --------------------------------------------------------------------------
def workload(cfg: int, n: int | None = None, valid: bool = False):
    """(model, dims, instances) of benchmark workload cfg (1 MLP, 2 RNN, 3 Tree-LSTM, 4 GGNN, 5 Tree-LSTM with
    hidden = embedding = 1024)."""
    seed = BASE_SEED + cfg + (1000 if valid else 0)
    if cfg == 1:
        d = DEFAULT_DIMS["mlp"]
        return "mlp", d, make_mlp(n or (256 if valid else 1024), seed, d)
    if cfg == 2:
        d = DEFAULT_DIMS["rnn"]
        return "rnn", d, make_rnn(n or (1000 if valid else 10000), seed, d)
    if cfg == 3:
        d = DEFAULT_DIMS["tree"]
        return "tree", d, make_tree(n or (1101 if valid else 8544), seed, d)
    if cfg == 4:
        d = DEFAULT_DIMS["ggnn"]
        norm = None
        if valid:
            _, norm = make_ggnn(2000, BASE_SEED + cfg, d)
        return "ggnn", d, make_ggnn(n or (2000 if valid else 20000), seed, d, norm=norm)[0]
    if cfg == 5:
        d = DEFAULT_DIMS["tree_big"]
        return "tree", d, make_tree(n or (1101 if valid else 8544), seed, d)
    raise ValueError(cfg)
