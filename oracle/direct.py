"""CPU checker, part 2: whole-model forward and backpropagation per instance.

TEST INFRASTRUCTURE ONLY.  Plain float64 numpy with its own formulas: it does
not use the message-passing simulator or the cell functions next to it, so
that agreement between the two is a real cross-check.  No messages, no
queues: the instance's loss is written as an ordinary function of all
parameters and differentiated by hand (backpropagation through time for the
sequence model, through structure for trees, Section 2).

With max_active_keys = 1 and every node updating once per instance, AMP
training is plain per-instance gradient descent (Section 3 and its footnote);
`train` implements exactly that special case.
"""
from __future__ import annotations

import numpy as np


def _sg(x):
    return 1.0 / (1.0 + np.exp(-x))


def node_shapes(model, dims):
    """(name, rows, cols, has_bias) per PPT node, in node-id order."""
    if model == "mlp":
        d, h, c = dims["d_in"], dims["hidden"], dims["n_class"]
        return [("lin1", h, d, 1), ("lin2", h, h, 1), ("lin3", c, h, 1)]
    if model == "rnn":
        v, e, h, c = dims["vocab"], dims["emb"], dims["hidden"], dims["n_class"]
        return [("lookup", v, e, 0), ("cell", h, e + h, 1), ("out", c, h, 1)]
    if model == "tree":
        v, e, h, c = dims["vocab"], dims["emb"], dims["hidden"], dims["n_class"]
        return [("lookup", v, e, 0), ("leaf", 3 * h, e, 1), ("branch", 5 * h, 2 * h, 1), ("out", c, h, 1)]
    if model == "ggnn":
        t, h, ne = dims["n_node_types"], dims["hidden"], dims["n_edge_types"]
        return ([("lookup", t, h, 0)] + [("edge%d" % c, h, h, 1) for c in range(ne)] +
                [("gz", h, 2 * h, 1), ("gr", h, 2 * h, 1), ("gh", h, 2 * h, 1), ("readout", 1, h, 1)])
    raise ValueError(model)


def unpack(model, dims, flat):
    out = []
    for (name, r, c, hb), v in zip(node_shapes(model, dims), flat):
        v = np.asarray(v, np.float64)
        assert v.size == r * c + (r if hb else 0), (name, v.size)
        P = {"W": v[:r * c].reshape(r, c).copy()}
        if hb:
            P["b"] = v[r * c:].copy()
        out.append(P)
    return out


def _xent(z, label):
    z = z - z.max()
    lse = np.log(np.exp(z).sum())
    p = np.exp(z - lse)
    d = p.copy()
    d[label] -= 1.0
    return -(z[label] - lse), d, int(np.argmax(z))


def _zero_grads(P):
    return [{k: np.zeros_like(v) for k, v in p.items()} for p in P]


# ------------------------------------------------------------------ MLP
def mlp(P, inst, dims, want_grad=True):
    x = np.asarray(inst["x"], np.float64)
    a1 = P[0]["W"] @ x + P[0]["b"]
    r1 = np.where(a1 > 0, a1, 0.0)
    a2 = P[1]["W"] @ r1 + P[1]["b"]
    r2 = np.where(a2 > 0, a2, 0.0)
    z = P[2]["W"] @ r2 + P[2]["b"]
    loss, dz, pred = _xent(z, inst["label"])
    res = dict(loss=loss, correct=int(pred == inst["label"]), npred=1)
    if not want_grad:
        return res
    G = _zero_grads(P)
    G[2]["W"], G[2]["b"] = dz[:, None] * r2[None, :], dz
    d2 = (P[2]["W"].T @ dz) * (a2 > 0)
    G[1]["W"], G[1]["b"] = d2[:, None] * r1[None, :], d2
    d1 = (P[1]["W"].T @ d2) * (a1 > 0)
    G[0]["W"], G[0]["b"] = d1[:, None] * x[None, :], d1
    res.update(grads=G, counts=[1, 1, 1])
    return res


# ------------------------------------------------------------------ RNN
def rnn(P, inst, dims, want_grad=True):
    E, Wc, bc, Wo, bo = P[0]["W"], P[1]["W"], P[1]["b"], P[2]["W"], P[2]["b"]
    tok = inst["tokens"]
    T, H = len(tok), dims["hidden"]
    hs = np.zeros((T + 1, H))
    xs = []
    for t in range(T):
        xs.append(np.concatenate([E[tok[t]], hs[t]]))
        hs[t + 1] = np.tanh(Wc @ xs[t] + bc)
    z = Wo @ hs[T] + bo
    loss, dz, pred = _xent(z, inst["label"])
    res = dict(loss=loss, correct=int(pred == inst["label"]), npred=1)
    if not want_grad:
        return res
    G = _zero_grads(P)
    G[2]["W"], G[2]["b"] = np.outer(dz, hs[T]), dz
    dh = Wo.T @ dz
    ne = dims["emb"]
    for t in range(T - 1, -1, -1):
        dp = dh * (1.0 - hs[t + 1] ** 2)
        G[1]["W"] += np.outer(dp, xs[t])
        G[1]["b"] += dp
        dx = Wc.T @ dp
        G[0]["W"][tok[t]] += dx[:ne]
        dh = dx[ne:]
    res.update(grads=G, counts=[T, T, 1])
    return res


# ------------------------------------------------------------------ Tree-LSTM
def tree(P, inst, dims, want_grad=True):
    E, Wl, bl, Wb, bb, Wo, bo = (P[0]["W"], P[1]["W"], P[1]["b"], P[2]["W"], P[2]["b"],
                                 P[3]["W"], P[3]["b"])
    L, H = inst["n_leaves"], dims["hidden"]
    nn = 2 * L - 1
    left, right, lab = inst["left"], inst["right"], inst["labels"]
    h = np.zeros((nn, H))
    c = np.zeros((nn, H))
    gate = [None] * nn
    xin = [None] * nn
    for n in range(nn):
        if n < L:
            xin[n] = E[inst["tokens"][n]].copy()
            g = Wl @ xin[n] + bl
            i, o, u = _sg(g[:H]), _sg(g[H:2 * H]), np.tanh(g[2 * H:])
            c[n] = i * u
            gate[n] = (i, o, u)
        else:
            a, b = left[n], right[n]
            xin[n] = np.concatenate([h[a], h[b]])
            g = Wb @ xin[n] + bb
            i, fl, fr, o = _sg(g[:H]), _sg(g[H:2 * H]), _sg(g[2 * H:3 * H]), _sg(g[3 * H:4 * H])
            u = np.tanh(g[4 * H:])
            c[n] = i * u + fl * c[a] + fr * c[b]
            gate[n] = (i, fl, fr, o, u)
        o_ = gate[n][1] if n < L else gate[n][3]
        h[n] = o_ * np.tanh(c[n])
    loss, correct = 0.0, 0
    dzs = []
    for n in range(nn):
        l, dz, pred = _xent(Wo @ h[n] + bo, lab[n])
        loss += l
        correct += int(pred == lab[n])
        dzs.append(dz)
    res = dict(loss=loss, correct=correct, npred=nn)
    if not want_grad:
        return res
    G = _zero_grads(P)
    dh = np.zeros((nn, H))
    dc = np.zeros((nn, H))
    for n in range(nn):
        G[3]["W"] += np.outer(dzs[n], h[n])
        G[3]["b"] += dzs[n]
        dh[n] += Wo.T @ dzs[n]
    for n in range(nn - 1, -1, -1):
        tc = np.tanh(c[n])
        if n < L:
            i, o, u = gate[n]
            dct = dc[n] + dh[n] * o * (1 - tc * tc)
            dg = np.concatenate([dct * u * i * (1 - i), dh[n] * tc * o * (1 - o), dct * i * (1 - u * u)])
            G[1]["W"] += np.outer(dg, xin[n])
            G[1]["b"] += dg
            G[0]["W"][inst["tokens"][n]] += Wl.T @ dg
        else:
            a, b = left[n], right[n]
            i, fl, fr, o, u = gate[n]
            dct = dc[n] + dh[n] * o * (1 - tc * tc)
            dg = np.concatenate([dct * u * i * (1 - i), dct * c[a] * fl * (1 - fl),
                                 dct * c[b] * fr * (1 - fr), dh[n] * tc * o * (1 - o),
                                 dct * i * (1 - u * u)])
            G[2]["W"] += np.outer(dg, xin[n])
            G[2]["b"] += dg
            dx = Wb.T @ dg
            dh[a] += dx[:H]
            dh[b] += dx[H:]
            dc[a] += dct * fl
            dc[b] += dct * fr
    res.update(grads=G, counts=[L, L, L - 1, nn])
    return res


# ------------------------------------------------------------------ GGNN
def ggnn(P, inst, dims, want_grad=True):
    """h_v^0 = E[type_v]; per step: m_e = W_type(e) h_src(e) + b_type(e) for
    each directed edge, a_v = sum of m_e into v, GRU update with
    h' = (1-z) h + z h~; yhat = w . sum_v h_v + b; loss = (yhat - y)^2 / 2."""
    ne, S, H = dims["n_edge_types"], dims["n_steps"], dims["hidden"]
    E = P[0]["W"]
    We = [P[1 + c] for c in range(ne)]
    Pz, Pr, Ph, Po = P[1 + ne], P[2 + ne], P[3 + ne], P[4 + ne]
    N = inst["n_nodes"]
    src, dst, et = inst["src"], inst["dst"], inst["etype"]
    hs = [E[inst["node_type"]].copy()]
    tr = []
    for s in range(S):
        h = hs[-1]
        a = np.zeros((N, H))
        for e in range(len(src)):
            a[dst[e]] += We[et[e]]["W"] @ h[src[e]] + We[et[e]]["b"]
        ah = np.concatenate([a, h], axis=1)
        z = _sg(ah @ Pz["W"].T + Pz["b"])
        r = _sg(ah @ Pr["W"].T + Pr["b"])
        arh = np.concatenate([a, r * h], axis=1)
        ht = np.tanh(arh @ Ph["W"].T + Ph["b"])
        hs.append((1 - z) * h + z * ht)
        tr.append((a, ah, z, r, arh, ht))
    pooled = hs[-1].sum(axis=0)
    yhat = float(Po["W"][0] @ pooled + Po["b"][0])
    d = yhat - inst["target"]
    res = dict(loss=0.5 * d * d, correct=0, npred=1, yhat=yhat)
    if not want_grad:
        return res
    G = _zero_grads(P)
    G[4 + ne]["W"][0] = d * pooled
    G[4 + ne]["b"][0] = d
    dh = np.tile(d * Po["W"][0], (N, 1))
    cnt_e = [0] * ne
    for s in range(S - 1, -1, -1):
        h = hs[s]
        a, ah, z, r, arh, ht = tr[s]
        dz = dh * (ht - h)
        dht = dh * z
        dhp = dh * (1 - z)
        dph = dht * (1 - ht * ht)
        G[3 + ne]["W"] += dph.T @ arh
        G[3 + ne]["b"] += dph.sum(0)
        darh = dph @ Ph["W"]
        da = darh[:, :H].copy()
        drh = darh[:, H:]
        dhp += drh * r
        dr = drh * h
        dpz = dz * z * (1 - z)
        dpr = dr * r * (1 - r)
        G[1 + ne]["W"] += dpz.T @ ah
        G[1 + ne]["b"] += dpz.sum(0)
        G[2 + ne]["W"] += dpr.T @ ah
        G[2 + ne]["b"] += dpr.sum(0)
        dah = dpz @ Pz["W"] + dpr @ Pr["W"]
        da += dah[:, :H]
        dhp += dah[:, H:]
        seen = set()
        for e in range(len(src)):
            t = et[e]
            G[1 + t]["W"] += np.outer(da[dst[e]], h[src[e]])
            G[1 + t]["b"] += da[dst[e]]
            dhp[src[e]] += We[t]["W"].T @ da[dst[e]]
            seen.add(int(t))
        for t in seen:
            cnt_e[t] += 1
        dh = dhp
    np.add.at(G[0]["W"], inst["node_type"], dh)
    res.update(grads=G, counts=[1] + cnt_e + [S, S, S, 1])
    return res


MODELS = {"mlp": mlp, "rnn": rnn, "tree": tree, "ggnn": ggnn}


def evaluate(model, dims, P, instances):
    """Forward only: mean loss per instance and accuracy over predictions."""
    f = MODELS[model]
    loss = correct = npred = 0
    for inst in instances:
        r = f(P, inst, dims, want_grad=False)
        loss += r["loss"]
        correct += r["correct"]
        npred += r["npred"]
    return loss / max(len(instances), 1), correct / max(npred, 1)


def train(model, dims, P, instances, lr, batch=1):
    """Synchronous SGD, in place.  Each node steps with the mean of the
    gradient messages it would have received for the `batch` instances.
    Returns the per-instance losses."""
    f = MODELS[model]
    losses = []
    for b0 in range(0, len(instances), batch):
        acc, cnt = _zero_grads(P), [0] * len(P)
        for inst in instances[b0:b0 + batch]:
            r = f(P, inst, dims)
            losses.append(r["loss"])
            for k in range(len(P)):
                cnt[k] += r["counts"][k]
                for name in acc[k]:
                    acc[k][name] += r["grads"][k][name]
        for k in range(len(P)):
            if cnt[k]:
                for name in P[k]:
                    P[k][name] -= lr * acc[k][name] / cnt[k]
    return losses
