"""Pins for the CPU checker's cells, losses and optimizers (no GPU).

Each check compares the checker with something fixed outside it: central
finite differences of a scalar function, closed forms, or a library routine
(scipy's log-softmax, torch's optimizers on the CPU).
"""
import numpy as np
import pytest
import scipy.special
import torch

from oracle import cells as C

RNG = np.random.default_rng(7)


def fd_check(f, x, analytic, eps=1e-6, tol=1e-6):
    """f: array -> scalar.  Central differences against `analytic`."""
    x = np.array(x, dtype=np.float64)
    num = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + eps
        fp = f(x)
        x[i] = old - eps
        fm = f(x)
        x[i] = old
        num[i] = (fp - fm) / (2 * eps)
    err = np.abs(num - analytic).max() / max(np.abs(num).max(), 1e-12)
    assert err < tol, err


def check_cell(fwd, bwd, P, x, tol=1e-6):
    """Gradient of L = sum(r * fwd(x)) w.r.t. x and every parameter."""
    y, cache = fwd(P, x)
    r = RNG.standard_normal(y.shape)
    dx, g = bwd(P, cache, r)
    fd_check(lambda xx: float((r * fwd(P, xx)[0]).sum()), x, dx, tol=tol)
    for name in P:
        def f(w, name=name):
            Q = dict(P)
            Q[name] = w
            return float((r * fwd(Q, x)[0]).sum())
        fd_check(f, P[name], g[name], tol=tol)


def rand_P(rows, cols):
    return {"W": RNG.standard_normal((rows, cols)) * 0.5, "b": RNG.standard_normal(rows) * 0.5}


def test_linear_vector_and_grouped_rows():
    P = rand_P(3, 4)
    check_cell(C.linear_fwd, C.linear_bwd, P, RNG.standard_normal(4))
    check_cell(C.linear_fwd, C.linear_bwd, P, RNG.standard_normal((5, 4)))


def test_linear_forward_definition():
    P = rand_P(3, 4)
    x = RNG.standard_normal(4)
    y, _ = C.linear_fwd(P, x)
    for i in range(3):
        assert abs(y[i] - (sum(P["W"][i, j] * x[j] for j in range(4)) + P["b"][i])) < 1e-14


def test_leaf_and_branch_cells():
    H, D = 3, 4
    check_cell(C.leaf_fwd, C.leaf_bwd, rand_P(3 * H, D), RNG.standard_normal(D))
    check_cell(C.branch_fwd, C.branch_bwd, rand_P(5 * H, 2 * H), RNG.standard_normal(4 * H))


def fused_tree_lstm(W, b, x, hl, cl, hr, cr):
    """One binary Tree-LSTM cell over [x; h_l; h_r], gates [i; f_l; f_r; o; u]."""
    H = hl.shape[0]
    g = W @ np.concatenate([x, hl, hr]) + b
    i, fl, fr, o = (C.sigmoid(g[k * H:(k + 1) * H]) for k in range(4))
    u = np.tanh(g[4 * H:])
    c = i * u + fl * cl + fr * cr
    return o * np.tanh(c), c


def test_leaf_branch_split_equals_fused_cell():
    """Section 6 (Tree-LSTM paragraph): the leaf cell is the full cell with zero hidden states, the
    branch cell is the full cell with zero input; they share no weights."""
    H, D = 3, 4
    W = RNG.standard_normal((5 * H, D + 2 * H))
    b = RNG.standard_normal(5 * H)
    x = RNG.standard_normal(D)
    z = np.zeros(H)
    rows = np.r_[0:H, 3 * H:5 * H]            # i, o, u
    h, c = fused_tree_lstm(W, b, x, z, z, z, z)
    hc, _ = C.leaf_fwd({"W": W[rows][:, :D], "b": b[rows]}, x)
    assert np.allclose(hc, np.concatenate([h, c]), atol=1e-14)
    hl, cl, hr, cr = (RNG.standard_normal(H) for _ in range(4))
    h, c = fused_tree_lstm(W, b, np.zeros(D), hl, cl, hr, cr)
    hc, _ = C.branch_fwd({"W": W[:, D:], "b": b}, np.concatenate([hl, cl, hr, cr]))
    assert np.allclose(hc, np.concatenate([h, c]), atol=1e-14)


def test_lookup():
    P = {"W": RNG.standard_normal((5, 3))}
    y, cache = C.lookup_fwd(P, 2)
    assert np.array_equal(y, P["W"][2])
    _, g = C.lookup_bwd(P, cache, np.array([1., 2., 3.]))
    g = {"W": g["W"].dense()}
    assert np.array_equal(g["W"][2], [1, 2, 3]) and np.abs(g["W"]).sum() == 6
    idx = np.array([1, 1, 4])
    y, cache = C.lookup_fwd(P, idx)
    _, g = C.lookup_bwd(P, cache, np.ones((3, 3)))
    g = {"W": g["W"].dense()}
    assert np.array_equal(g["W"][1], [2, 2, 2]) and np.array_equal(g["W"][4], [1, 1, 1])


@pytest.mark.parametrize("fwd,bwd", [(C.relu_fwd, C.relu_bwd), (C.tanh_fwd, C.tanh_bwd),
                                     (C.sigmoid_fwd, C.sigmoid_bwd)])
def test_elementwise(fwd, bwd):
    x = RNG.standard_normal(6) + 0.05
    y, cache = fwd(x)
    r = RNG.standard_normal(6)
    fd_check(lambda xx: float((r * fwd(xx)[0]).sum()), x, bwd(cache, r))


def test_softmax_xent_against_scipy_and_fd():
    z = RNG.standard_normal(5) * 3
    loss, dz, pred = C.softmax_xent(z, 3)
    assert abs(loss + scipy.special.log_softmax(z)[3]) < 1e-12
    assert pred == int(np.argmax(z))
    fd_check(lambda zz: C.softmax_xent(zz, 3)[0], z, dz)
    assert abs(dz.sum()) < 1e-12
    big = np.array([1000.0, 0.0, -1000.0])
    assert np.isfinite(C.softmax_xent(big, 2)[0])


def test_squared_error():
    loss, d, _ = C.squared_error(np.array([1.5]), 0.5)
    assert loss == 0.5 and d[0] == 1.0


@pytest.mark.parametrize("kind,kw,topt", [
    ("sgd", dict(lr=0.1), lambda p: torch.optim.SGD(p, lr=0.1)),
    ("momentum", dict(lr=0.05, momentum=0.9), lambda p: torch.optim.SGD(p, lr=0.05, momentum=0.9)),
    ("adam", dict(lr=0.01), lambda p: torch.optim.Adam(p, lr=0.01)),
])
def test_optimizers_against_torch(kind, kw, topt):
    w0 = RNG.standard_normal((3, 4))
    P = {"W": w0.copy()}
    tw = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    o = topt([tw])
    mine = C.Optimizer(kind=kind, **kw)
    for _ in range(5):
        g = RNG.standard_normal((3, 4))
        mine.step(P, {"W": g})
        tw.grad = torch.tensor(g)
        o.step()
    assert np.allclose(P["W"], tw.detach().numpy(), rtol=1e-12, atol=1e-12)
