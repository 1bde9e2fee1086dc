"""Algorithmic flop and byte counts of the dense cells, per message visit.

Used by the benchmark to turn counted visits into roofline figures, and
checked against the closed-form estimate of Appendix C.
"""
from __future__ import annotations


def appendix_c(H, N, E, C, steps, device_flops=1e12, overhead=0.5, bytes_per_float=4):
    """The throughput estimate of Appendix C for a GGSNN pipelined over
    devices that each hold one linear node.

    Per time step the slower of the GRU stage (2 N H^2 multiply-adds for a
    2H x H node over N rows) and the per-edge-type stage (E H^2 / C) bounds
    the pipeline; a forward visit costs 2 flops per multiply-add, a backward
    visit three times a forward one.
    """
    stage = max(2 * N * H * H, E * H * H / C)
    fwdop = 2 * stage
    bwdop = 6 * stage
    ops = (fwdop + bwdop) * steps
    thr = overhead * device_flops / ops
    return dict(
        ops_per_sample=ops,
        throughput=thr,
        network_bits_per_s=8 * bytes_per_float * thr * max(N, E) * H,
        device_memory_bytes=4 * (2 * H * H) * bytes_per_float,
        min_devices=C + 3,
    )


def cell_weights(model: str, dims: dict) -> dict:
    """Number of weight-matrix elements |W| per dense node."""
    if model == "mlp":
        d, h, c = dims["d_in"], dims["hidden"], dims["n_class"]
        return {"lin1": h * d, "lin2": h * h, "lin3": c * h}
    if model == "rnn":
        e, h, c = dims["emb"], dims["hidden"], dims["n_class"]
        return {"cell": h * (e + h), "out": c * h}
    if model == "tree":
        e, h, c = dims["emb"], dims["hidden"], dims["n_class"]
        return {"leaf": 3 * h * e, "branch": 5 * h * 2 * h, "out": c * h}
    if model == "ggnn":
        h, ne = dims["hidden"], dims["n_edge_types"]
        w = {"edge%d" % k: h * h for k in range(ne)}
        w.update(gz=2 * h * h, gr=2 * h * h, gh=2 * h * h, readout=h)
        return w
    raise ValueError(model)


def visit_cost(n_weights: int, rows: int = 1) -> dict:
    """One forward plus one backward visit of `rows` grouped rows to a node
    with n_weights matrix elements whose weights stay on chip.

    Forward reads each weight once (4 B) for 2*rows flops; backward reads it
    once more for W^T delta and performs the outer-product accumulation:
    2*rows flops each.  The accumulation's own memory traffic depends on
    where the accumulator lives and is not counted here.
    """
    return dict(weight_bytes=2 * 4 * n_weights, flops=6 * rows * n_weights)
