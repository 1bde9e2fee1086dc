"""CPU checker, part 1: the dense cells, their gradients and the optimizers.

TEST INFRASTRUCTURE ONLY.  Plain, slow, float64 numpy.  Shares no code with
the HIP path and is never imported by it.

Each cell is a pair of functions
    fwd(P, x)            -> (y, cache)
    bwd(P, cache, dy)    -> (dx, {param name: gradient})
where P is a dict of float64 arrays.  A payload is a vector, or a k-row matrix
when several messages were grouped into one (Section 4, aggregation); a
grouped payload yields one gradient, the sum over its rows.

The paper gives the structure of the cells (Sections 2, 6 and Appendix C) but
not their equations; the equations below are the standard ones for a linear
layer, a tanh RNN, the binary Tree-LSTM split into a leaf and a branch cell
(Section 6, Tree-LSTM paragraph) and the gated graph network's per-edge-type
linear message plus GRU update (Section 4 GNN description, Appendix C).
"""
from __future__ import annotations

import numpy as np


def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


# ---------------------------------------------------------------- linear PPT
def linear_fwd(P, x):
    """y = W x + b (rows of x are independent messages).  Section 4, PPT."""
    return x @ P["W"].T + P["b"], x


def linear_bwd(P, x, dy):
    """dx = W^T dy with the node's present W; dW = dy x^T; db = dy."""
    dx = dy @ P["W"]
    if x.ndim == 1:
        return dx, {"W": np.outer(dy, x), "b": dy.copy()}
    return dx, {"W": dy.T @ x, "b": dy.sum(axis=0)}


# ---------------------------------------------------------------- lookup PPT
def lookup_fwd(P, idx):
    """Row gather: the lookup table is a PPT whose parameter is the table
    (Section 4, RNN example).  idx is an int or an int vector."""
    return P["W"][idx].copy(), idx


class RowGradient:
    """Gradient of a table that is zero except in the listed rows (repeated
    indices add up): a dense gradient in sparse clothing, so that large
    tables do not cost a full-size array per message."""

    def __init__(self, shape, idx, rows):
        self.shape = shape
        self.idx = np.atleast_1d(np.asarray(idx))
        self.rows = np.atleast_2d(np.asarray(rows, np.float64))

    def add_to(self, dense):
        np.add.at(dense, self.idx, self.rows)

    def dense(self):
        g = np.zeros(self.shape)
        self.add_to(g)
        return g


def lookup_bwd(P, idx, dy):
    """The gradient of a gather is a scatter-add of the incoming rows."""
    return None, {"W": RowGradient(P["W"].shape, idx, dy)}


# ---------------------------------------------------------------- NPTs
def relu_fwd(x):
    return np.maximum(x, 0.0), x


def relu_bwd(x, dy):
    return dy * (x > 0)


def tanh_fwd(x):
    y = np.tanh(x)
    return y, y


def tanh_bwd(y, dy):
    return dy * (1.0 - y * y)


def sigmoid_fwd(x):
    y = sigmoid(x)
    return y, y


def sigmoid_bwd(y, dy):
    return dy * y * (1.0 - y)


# ---------------------------------------------------------------- losses
def softmax_xent(z, label):
    """loss = -log softmax(z)[label]; returns (loss, dz, predicted class)."""
    m = z.max()
    e = np.exp(z - m)
    s = e.sum()
    p = e / s
    loss = -(z[label] - m - np.log(s))
    dz = p.copy()
    dz[label] -= 1.0
    return float(loss), dz, int(np.argmax(z))


def squared_error(yhat, y):
    """loss = 0.5 (yhat - y)^2."""
    d = float(np.ravel(yhat)[0]) - y
    return 0.5 * d * d, np.asarray([d]), d


# ---------------------------------------------------------------- Tree-LSTM cells
def leaf_fwd(P, x):
    """Leaf cell: zero hidden and cell state below it, so there is no forget
    gate.  Rows of W: [i; o; u].  Output payload is [h; c]."""
    h3 = P["W"].shape[0]
    hd = h3 // 3
    g = P["W"] @ x + P["b"]
    i, o, u = sigmoid(g[:hd]), sigmoid(g[hd:2 * hd]), np.tanh(g[2 * hd:])
    c = i * u
    tc = np.tanh(c)
    h = o * tc
    return np.concatenate([h, c]), (x, i, o, u, tc)


def leaf_bwd(P, cache, dhc):
    x, i, o, u, tc = cache
    hd = i.shape[0]
    dh, dc = dhc[:hd], dhc[hd:]
    do = dh * tc
    dct = dc + dh * o * (1.0 - tc * tc)
    di = dct * u
    du = dct * i
    dg = np.concatenate([di * i * (1 - i), do * o * (1 - o), du * (1 - u * u)])
    return P["W"].T @ dg, {"W": np.outer(dg, x), "b": dg}


def branch_fwd(P, x):
    """Branch cell: zero input, two children.  x = [h_l; c_l; h_r; c_r].
    Rows of W: [i; f_l; f_r; o; u], columns [h_l; h_r]."""
    hd = P["W"].shape[0] // 5
    hl, cl, hr, cr = x[:hd], x[hd:2 * hd], x[2 * hd:3 * hd], x[3 * hd:]
    xin = np.concatenate([hl, hr])
    g = P["W"] @ xin + P["b"]
    i, fl, fr, o = (sigmoid(g[k * hd:(k + 1) * hd]) for k in range(4))
    u = np.tanh(g[4 * hd:])
    c = i * u + fl * cl + fr * cr
    tc = np.tanh(c)
    h = o * tc
    return np.concatenate([h, c]), (xin, cl, cr, i, fl, fr, o, u, tc)


def branch_bwd(P, cache, dhc):
    xin, cl, cr, i, fl, fr, o, u, tc = cache
    hd = i.shape[0]
    dh, dc = dhc[:hd], dhc[hd:]
    do = dh * tc
    dct = dc + dh * o * (1.0 - tc * tc)
    di, du = dct * u, dct * i
    dfl, dfr = dct * cl, dct * cr
    dg = np.concatenate([di * i * (1 - i), dfl * fl * (1 - fl), dfr * fr * (1 - fr),
                         do * o * (1 - o), du * (1 - u * u)])
    dxin = P["W"].T @ dg
    dx = np.concatenate([dxin[:hd], dct * fl, dxin[hd:], dct * fr])
    return dx, {"W": np.outer(dg, xin), "b": dg}


# ---------------------------------------------------------------- optimizers
class Optimizer:
    """Per-node optimizer state (Appendix A: (momentum-)SGD and Adam are
    runtime options; Appendix C: parameter, gradient buffer and two Adam
    slots per node).  `g` is the mean of the accumulated gradients."""

    def __init__(self, kind="sgd", lr=0.1, momentum=0.0, beta1=0.9, beta2=0.999, eps=1e-8):
        self.kind, self.lr, self.momentum = kind, lr, momentum
        self.beta1, self.beta2, self.eps = beta1, beta2, eps
        self.t = 0
        self.slots = {}

    def step(self, P, G):
        self.t += 1
        for k, g in G.items():
            if self.kind == "sgd":
                P[k] -= self.lr * g
            elif self.kind == "momentum":
                v = self.slots.setdefault(k, np.zeros_like(g))
                v *= self.momentum
                v += g
                P[k] -= self.lr * v
            elif self.kind == "adam":
                m, v = self.slots.setdefault(k, (np.zeros_like(g), np.zeros_like(g)))
                m *= self.beta1
                m += (1 - self.beta1) * g
                v *= self.beta2
                v += (1 - self.beta2) * g * g
                mh = m / (1 - self.beta1 ** self.t)
                vh = v / (1 - self.beta2 ** self.t)
                P[k] -= self.lr * mh / (np.sqrt(vh) + self.eps)
            else:
                raise ValueError(self.kind)


def unpack_node(flat, rows, cols, has_bias):
    """Flat float32 node vector [W row-major; b] -> float64 dict."""
    v = np.asarray(flat, np.float64)
    assert v.size == rows * cols + (rows if has_bias else 0)
    P = {"W": v[:rows * cols].reshape(rows, cols).copy()}
    if has_bias:
        P["b"] = v[rows * cols:].copy()
    return P


def pack_node(P):
    v = [P["W"].reshape(-1)]
    if "b" in P:
        v.append(P["b"])
    return np.concatenate(v)
