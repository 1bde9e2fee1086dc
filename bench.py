#!/usr/bin/env python3
"""Benchmark of the AMP training hot path on one MI355X.

A step is one pass of the whole path (admission, lookup, cell forward and
backward, loss, local updates, retirement) over the full synthetic workload:
one amp_train epoch.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--mak 64]

The default workload is number 3 (binary Tree-LSTM, 8,544 random trees,
hidden 150, 300-d embeddings, max_active_keys 64), the configuration the
metric is quoted on; the metric's second workload, the gated graph network
(config 4), is measured in the same run and reported as the object `ggnn`.
--config 1, 2, 4, 5 select the MLP, RNN, GGNN and hidden-1024 Tree-LSTM
workloads as the headline instead.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_1705_09786_amd import costmodel, synth  # noqa: E402

CLOCK_HZ = 2.4e9
LDS_BYTES_PER_CLK_PER_CU = 128
N_CU = 256
FP32_MFMA_PEAK = 157.3e12          # whole chip, dense fp32 matrix
DEFAULTS = {
    # cfg: mak, muf, lookup muf, optimizer
    1: dict(mak=4, muf=1, lmuf=None, opt=("sgd", dict(lr=0.05))),
    2: dict(mak=16, muf=16, lmuf=16, opt=("sgd", dict(lr=0.05))),
    # 10 leaf + 17 branch tiles: the single model's best rate (39.5k trees/s on 30 workgroups): 15 leaf and 9 or 8
    # branch units per tile are 45 and 45 or 40 rows, three 16-row blocks almost full, where 8 + 16 tiles (57 and 50
    # rows, 37k trees/s) pad to four; the fewest tiles that fit LDS (5 + 8, 16 workgroups, 30k trees/s) use each CU
    # better and are what the replicated run packs two per XCD
    3: dict(mak=64, muf=50, lmuf=1000, opt=("sgd", dict(lr=0.05)), tiles={1: 10, 2: 17}, replica_tiles={1: 5, 2: 8},
            replica_workers=16),
    # the commonest edge type's linear split over four workgroups, the two GRU gates over two each, the candidate over
    # three (17 workgroups): 21.7k graphs/s against 12.7k unsplit and 18.7k with that linear over two; more tiles of
    # the GRU nodes add nothing (20.8-21.4k on 18-22 workgroups)
    # the replicated run keeps the nodes whole: 24 replicas of 10 workgroups beat 16 of 15
    4: dict(mak=32, muf=20, lmuf=20, opt=("adam", dict(lr=0.001)), tiles={1: 4, 5: 2, 6: 2, 7: 3}, replica_tiles=None,
            replica_workers=10),
    5: dict(mak=128, muf=50, lmuf=1000, opt=("sgd", dict(lr=0.02)), tiles={1: 16, 2: 64}),
}
NAMES = {1: "mlp_64-128-128-10_1024inst", 2: "rnn_h128_len4-32_10000seq",
         3: "treelstm_h150_e300_2-60leaves_8544trees", 4: "ggnn_h100_4steps_9-29nodes_20000graphs",
         5: "treelstm_h1024_e1024_2-60leaves_8544trees"}


def visits(model, data):
    """Message visits per node for one pass over `data` (forward = backward)."""
    if model == "mlp":
        n = len(data)
        return dict(lin1=n, lin2=n, lin3=n)
    if model == "rnn":
        return dict(cell=sum(len(d["tokens"]) for d in data), out=len(data))
    if model == "tree":
        nl = sum(d["n_leaves"] for d in data)
        return dict(leaf=nl, branch=nl - len(data), out=2 * nl - len(data))
    raise ValueError(model)


def ggnn_cost(dims, data):
    """(weight bytes, flops) of one pass: each node is visited once per step
    with k grouped rows (edges of its type, or all graph nodes)."""
    W = costmodel.cell_weights("ggnn", dims)
    S, ne = dims["n_steps"], dims["n_edge_types"]
    nbytes = nflops = 0
    for g in data:
        for c in range(ne):
            k = int((g["etype"] == c).sum())
            if k:
                vc = costmodel.visit_cost(W["edge%d" % c], rows=k)
                nbytes += S * vc["weight_bytes"]
                nflops += S * vc["flops"]
        for name in ("gz", "gr", "gh"):
            vc = costmodel.visit_cost(W[name], rows=g["n_nodes"])
            nbytes += S * vc["weight_bytes"]
            nflops += S * vc["flops"]
    return nbytes, nflops


def cpu_model_name():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(model, dims, fp, data, cfg, budget_s=30.0):
    """The CPU checker's own-schedule AMP driver, as it stands (interpreted Python over float64 numpy, never tuned
    for this), on a prefix of the same workload; one thread."""
    from threadpoolctl import threadpool_limits
    from oracle import amp as oamp
    n = min(len(data), 16)
    with threadpool_limits(limits=1):
        while True:
            rt = oamp.Runtime(model, dims, fp)
            rt.set_muf(cfg["muf"])
            if cfg["lmuf"]:
                rt.set_muf(cfg["lmuf"], "lookup")
            rt.set_optimizer(kind=cfg["opt"][0], **cfg["opt"][1])
            t0 = time.perf_counter()
            rt.run(data[:n], mak=cfg["mak"])
            dt = time.perf_counter() - t0
            if dt > budget_s / 4 or n >= len(data):
                break
            n = min(len(data), max(n * 2, int(n * budget_s / 2 / max(dt, 1e-3))))
    return dict(value=n / dt, unit="instances/s", cores=1, cpu_model=cpu_model_name(), kind="oracle",
                implementation="interpreted Python + float64 numpy message-passing simulator (the parity checker as it stands)",
                sample="first %d instances of the workload, 1 epoch, same mak/muf, %.1f s" % (n, dt))


def measured_traffic(config, mak, muf, n, tiles):
    """HBM bytes per launch of exactly this configuration, from the table kept with the rocprofv3 summaries
    (profiles/hbm_traffic.md: one row per profiled configuration, written when the profile is taken); None when
    this configuration has not been profiled with the present kernels."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.md")
    want = (str(config), str(mak), str(muf), str(n), "+".join(str(t) for _, t in sorted(tiles.items())) if tiles else "-")
    try:
        rows = [[c.strip() for c in line.strip().strip("|").split("|")] for line in open(path) if line.startswith("|")]
    except OSError:
        return None
    for r in rows:
        if len(r) >= 7 and tuple(r[:5]) == want:
            return dict(bytes=float(r[5]) + float(r[6]), fetch_bytes=float(r[5]), write_bytes=float(r[6]), source=r[7] if len(r) > 7 else None)
    return None


def run_config(config, steps, warmup, mak=None, muf=None, n=None):
    """Times `steps` training epochs of one workload (after `warmup` untimed ones) on one model copy and returns
    everything the JSON line says about it, plus what the caller needs for the replicated run."""
    import torch
    from paper_1705_09786_amd import binding as B
    from paper_1705_09786_amd import runner
    cfg = dict(DEFAULTS[config])
    if mak:
        cfg["mak"] = mak
    if muf:
        cfg["muf"] = muf
    model, dims, data = synth.workload(config, n=n)
    fp = synth.init_params(model, dims, 100 + config)
    ml, me = runner.max_len_of(model, data)
    tr = runner.Trainer(model, dims, fp, cfg["mak"], ml, me, len(data), arena_bytes=(20 if config == 5 else 4) << 30,
                        tiles=cfg.get("tiles"))
    a = tr.amp
    a.set_min_update_frequency(-1, cfg["muf"])
    if cfg["lmuf"]:
        a.set_min_update_frequency(0, cfg["lmuf"])
    kind = {"sgd": B.OPT_SGD, "momentum": B.OPT_MOMENTUM, "adam": B.OPT_ADAM}[cfg["opt"][0]]
    a.set_optimizer(-1, kind, **cfg["opt"][1])
    tr.submit_all(data)                       # inputs are resident in HBM from the first training call on
    for _ in range(warmup):
        a.train(1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    kern_s = []
    for _ in range(steps):
        a.train(1)
        kern_s.append(a.get_loss()["seconds"])     # HIP events around the kernel, on its stream
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    stats = a.get_loss()
    n_workers = a.num_workers()
    tr.close()

    n_inst = len(data)
    kern = float(np.mean(kern_s))
    # algorithmic work of one launch: every visit reads the node's weights once forward and once backward (the
    # paper's cost of a batch-1 visit) and performs 6 |W| flop per row
    if model == "ggnn":
        lds_bytes, flops = ggnn_cost(dims, data)
    else:
        W = costmodel.cell_weights(model, dims)
        v = visits(model, data)
        lds_bytes = sum(costmodel.visit_cost(W[k])["weight_bytes"] * v[k] for k in v)
        flops = sum(costmodel.visit_cost(W[k])["flops"] * v[k] for k in v)
    # What bounds the kernel that was timed: the workers batch waiting messages and run the products on the fp32
    # matrix cores (one pass over the weights per batch), so the bound is the fp32 matrix rate of the CUs the
    # pipeline occupies -- for every workload.  Beside it, `lds_equivalent`: the same run priced the way the paper
    # prices a batch-1 visit (weights loaded once per forward and once per backward visit, from LDS) against the
    # LDS bandwidth of the occupied CUs -- a statement about throughput in the paper's terms, not about what the
    # LDS pins carried (the profile's LDS-active share is far lower).
    mfma_chip = FP32_MFMA_PEAK / 1e12
    lds_chip = N_CU * LDS_BYTES_PER_CLK_PER_CU * CLOCK_HZ / 1e9
    ach_f, ach_b = flops / kern / 1e12, lds_bytes / kern / 1e9
    traffic = measured_traffic(config, cfg["mak"], cfg["muf"], n_inst, cfg.get("tiles"))
    roof = {"bound": "mfma", "achieved": ach_f, "peak": mfma_chip * n_workers / N_CU, "unit": "TFLOP/s",
            "frac": ach_f / (mfma_chip * n_workers / N_CU),
            "peak_basis": "published dense fp32 matrix rate (157.3 TFLOP/s) x occupied CUs / 256",
            "traffic": traffic["bytes"] if traffic else None,
            "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, separate runs; profiles/hbm_traffic.md)",
            "traffic_source": traffic["source"] if traffic else None,
            "kernel": "amp_persistent", "occupied_cus": n_workers, "peak_whole_chip": mfma_chip,
            "frac_whole_chip": ach_f / mfma_chip, "algorithmic_flops_per_launch": flops,
            "lds_equivalent": {"achieved": ach_b, "peak": lds_chip * n_workers / N_CU, "unit": "GB/s",
                               "frac": ach_b / (lds_chip * n_workers / N_CU), "frac_whole_chip": ach_b / lds_chip,
                               "algorithmic_bytes_per_launch": lds_bytes,
                               "meaning": "8 B per weight and forward+backward visit, as if every visit loaded the weights from LDS"}}
    res = {"value": n_inst * steps / wall, "unit": "instances/s", "steps": steps, "warmup": warmup,
           "ms_per_step": 1e3 * wall / steps,
           "config": {"workload": NAMES[config], "instances": n_inst, "max_active_keys": cfg["mak"],
                      "min_update_frequency": cfg["muf"], "lookup_min_update_frequency": cfg["lmuf"],
                      "optimizer": cfg["opt"][0], "workgroups": n_workers,
                      "tiles": ({"node %d" % k: t for k, t in sorted(cfg["tiles"].items())} if model == "ggnn" else
                                {"leaf": cfg["tiles"][1], "branch": cfg["tiles"][2]}) if cfg.get("tiles") else None},
           "kernel_ms_per_step": 1e3 * kern, "kernel_instances_per_s": n_inst / kern,
           "train_loss": stats["mean_loss"], "train_accuracy": stats["accuracy"], "roofline": roof}
    ctx = dict(cfg=cfg, model=model, dims=dims, data=data, fp=fp, ml=ml, me=me, kind=kind, n_workers=n_workers,
               flops=flops, lds_bytes=lds_bytes)
    return res, ctx


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--mak", type=int, default=None)
    ap.add_argument("--muf", type=int, default=None)
    ap.add_argument("--n", type=int, default=None, help="instances (default: the config's full set)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ggnn", action="store_true", help="skip the second headline workload (config 4) beside the first")
    ap.add_argument("--replicas", type=int, default=None,
                    help="replicas for the extra 'replicated' measurement (default: as many whole replicas as fit each 32-CU XCD; 1 = skip)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run one device-to-device copy of this many MiB (the kernel of "
                         "known traffic that rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1705_09786_amd import binding as B
    from paper_1705_09786_amd import runner

    if args.copy_calibration:
        n = args.copy_calibration << 20
        a = torch.empty(n, dtype=torch.uint8, device="cuda:0")
        b = torch.empty_like(a)
        a.zero_()
        torch.cuda.synchronize()
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n, "copies": 3}))
        return

    res, ctx = run_config(args.config, args.steps, args.warmup, args.mak, args.muf, args.n)
    cfg, model, dims, data, fp = ctx["cfg"], ctx["model"], ctx["dims"], ctx["data"], ctx["fp"]
    n = len(data)
    out = {"metric": "trained instances/sec", "value": res["value"], "unit": "instances/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": res["config"], "kernel_ms_per_step": res["kernel_ms_per_step"],
           "kernel_instances_per_s": res["kernel_instances_per_s"], "train_loss": res["train_loss"],
           "train_accuracy": res["train_accuracy"], "roofline": res["roofline"]}
    # Beside the headline (one copy of the model, as the configuration names it): the paper's own way to use more
    # of the machine -- every parameterized node replicated, instances dealt round-robin to the replicas, parameters
    # averaged at the end of each epoch (Section 5).  A different training procedure, so reported apart from `value`.
    rep_tiles = cfg.get("replica_tiles", cfg.get("tiles"))
    rep_workers = cfg.get("replica_workers", ctx["n_workers"])
    fit = 8 * (32 // rep_workers) if rep_workers <= 32 else 240 // rep_workers   # whole replicas per 32-CU XCD
    R = args.replicas if args.replicas is not None else min(128, fit, len(data) // (4 * cfg["mak"]))
    if R > 1:
        tr = runner.Trainer(model, dims, fp, cfg["mak"], ctx["ml"], ctx["me"], len(data),
                            arena_bytes=(48 if args.config == 5 else 24) << 30, tiles=rep_tiles, replicas=R)
        assert tr.amp.num_workers() == R * rep_workers
        a = tr.amp
        a.set_min_update_frequency(-1, cfg["muf"])
        if cfg["lmuf"]:
            a.set_min_update_frequency(0, cfg["lmuf"])
        a.set_optimizer(-1, ctx["kind"], **cfg["opt"][1])
        tr.submit_all(data)
        for _ in range(args.warmup):
            a.train(1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        a.train(args.steps)
        torch.cuda.synchronize()
        rwall = time.perf_counter() - t0
        rk = a.get_loss()["seconds"]
        out["replicated"] = {"replicas": R, "value": n * args.steps / rwall, "unit": "instances/s",
                             "kernel_instances_per_s": n * args.steps / rk, "workgroups": R * rep_workers,
                             "max_active_keys_per_replica": cfg["mak"], "parameter_averaging": "end of every epoch",
                             "mfma_frac_whole_chip": ctx["flops"] * args.steps / rk / FP32_MFMA_PEAK,
                             "lds_equivalent_frac_whole_chip": ctx["lds_bytes"] * args.steps / rk
                             / (N_CU * LDS_BYTES_PER_CLK_PER_CU * CLOCK_HZ),
                             "train_loss": a.get_loss()["mean_loss"]}
        tr.close()
    # The RNN is the paper's own example of a single heavy node (Section 5): copies of the cell alone between a Cond
    # and a Phi, the output layer shared, the copies averaged at the end of each epoch; the instances in flight
    # grow with the copies, as in the paper's table (2 copies at 4, 4 copies at 8 there).
    if args.config == 2 and (args.replicas is None or args.replicas > 1):
        copies = 8
        tr = runner.Trainer(model, dims, fp, 4 * cfg["mak"], ctx["ml"], ctx["me"], len(data), arena_bytes=4 << 30,
                            node_replicas={1: copies})
        a = tr.amp
        a.set_min_update_frequency(-1, cfg["muf"])
        a.set_optimizer(-1, ctx["kind"], **cfg["opt"][1])
        tr.submit_all(data)
        for _ in range(args.warmup):
            a.train(1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        a.train(args.steps)
        torch.cuda.synchronize()
        cwall = time.perf_counter() - t0
        out["cell_copies"] = {"copies": copies, "max_active_keys": 4 * cfg["mak"], "value": n * args.steps / cwall,
                              "unit": "instances/s", "kernel_instances_per_s": n * args.steps / a.get_loss()["seconds"],
                              "workgroups": a.num_workers(), "parameter_averaging": "end of every epoch, the copies only",
                              "train_loss": a.get_loss()["mean_loss"]}
        tr.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(model, dims, fp, data, cfg)
    # The metric names two workloads: the graph network (config 4) is measured in the same run, as an object of its
    # own with its own rate, kernel time, roofline and CPU baseline.  Its epochs are long (20,000 graphs), so it
    # takes at most 5 timed steps.
    if args.config == 3 and not args.no_ggnn:
        gsteps = max(1, min(args.steps, 5))
        gres, gctx = run_config(4, gsteps, min(args.warmup, 1))
        if not args.no_cpu_baseline:
            gres["cpu_baseline"] = cpu_baseline(gctx["model"], gctx["dims"], gctx["fp"], gctx["data"], gctx["cfg"], budget_s=20.0)
        gres["metric"] = "trained instances/sec"
        out["ggnn"] = gres
    # The published peaks above are what `roofline.peak` quotes; the rates this chip actually reaches on the two
    # access patterns (a worker-shaped workgroup streaming 16-byte LDS reads on every CU; a grid-wide streaming sum
    # over 2 GiB of HBM) are measured beside them.
    buf = torch.zeros(2 << 30, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    lds_cu, hbm = B.measure_peaks(buf.data_ptr(), buf.numel(), torch.cuda.current_stream().cuda_stream)
    del buf
    out["measured_peaks"] = {"lds_read_GBps_per_cu": lds_cu / 1e9, "lds_read_fraction_of_nominal": lds_cu / (
        LDS_BYTES_PER_CLK_PER_CU * CLOCK_HZ), "hbm_read_GBps": hbm / 1e9, "hbm_read_fraction_of_nominal": hbm / 8e12}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
