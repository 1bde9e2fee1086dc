"""Asynchrony sweep (Section 6, "Asynchrony", Figure 7): an 8-replica RNN on a
synthetic list-reduction task, trained for every (max_active_keys,
min_update_frequency) pair of a grid until it reaches 96 % validation
accuracy; reports the epochs (data) and the device time that took, and the
training rate.

    python -m paper_1705_09786_amd.sweep [--replicas 8] [--max-epochs 40] [--out sweep.json]
                                         [--admission bounded --max-staleness 8] [--maks 32,64] [--mufs 1,4]
                                         [--copies 8 [--group-sync 500]]

`--replicas R` replicates the whole pipeline (every node R times, max_active_keys per replica); `--copies R`
replicates the recurrent cell alone between a Cond and a Phi, as Section 5 does, with the output layer shared
and max_active_keys counting all instances in flight; `--group-sync k` adds a synchronisation round of the
copies after every k retirements.

With `--admission bounded` the controller keeps the number of instances in
flight below max_active_keys whenever they would see more than
`--max-staleness` updates per worker (Appendix B, MNIST: a better schedule
than the greedy one); the cells then also report the largest number in flight.

The paper's list-reduction dataset is not available; the stand-in is the
"max" reduction of `synth.make_rnn` (lists of 2..10 tokens, label = largest
token value scaled to 10 classes), which this RNN learns within a few epochs.
"""
from __future__ import annotations

import argparse
import json
import sys

from . import binding as B
from . import runner, synth

TARGET = 0.96
MAKS = (1, 2, 4, 8, 16, 32, 64)
MUFS = (1, 4, 16, 64, 256)


def run_one(data, valid, dims, fp, replicas, mak, muf, lr, max_epochs, bounded=None, copies=0, group_sync=0):
    ml, _ = runner.max_len_of("rnn", data + valid)
    tr = runner.Trainer("rnn", dims, fp, mak, ml, 0, len(data), arena_bytes=2 << 30, replicas=1 if copies else replicas,
                        node_replicas={1: copies} if copies else None)
    a = tr.amp
    if group_sync:
        a.set_group_sync(group_sync)
    a.set_min_update_frequency(-1, muf)
    a.set_optimizer(-1, B.OPT_ADAM, lr=lr)
    if bounded is not None:
        a.set_admission(B.ADMIT_BOUNDED, bounded)
    tr.submit_all(data)
    tr.submit_all(valid, which=1)
    seconds, reached, acc, in_flight = 0.0, None, 0.0, 0
    for ep in range(1, max_epochs + 1):
        a.train(1)
        seconds += a.get_loss()["seconds"]
        in_flight = max(in_flight, a.get_admission()["max_in_flight"])
        acc = a.eval()["accuracy"]
        if acc >= TARGET:
            reached = ep
            break
    tr.close()
    epochs = reached if reached is not None else max_epochs
    return dict(max_active_keys=mak, min_update_frequency=muf, converged=reached is not None, epochs=epochs,
                device_seconds=seconds, instances_per_s=len(data) * epochs / seconds, valid_accuracy=acc,
                max_in_flight=in_flight)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--replicas", type=int, default=8)
    ap.add_argument("--copies", type=int, default=0, help="copies of the recurrent cell alone instead of whole replicas")
    ap.add_argument("--group-sync", type=int, default=0, help="with --copies: a synchronisation round every this many retirements")
    ap.add_argument("--max-epochs", type=int, default=40)
    ap.add_argument("--lr", type=float, default=0.001)
    ap.add_argument("--instances", type=int, default=10000)
    ap.add_argument("--out", default=None, help="also write the table to this JSON file")
    ap.add_argument("--admission", choices=("greedy", "bounded"), default="greedy")
    ap.add_argument("--max-staleness", type=float, default=8.0, help="bound of the bounded admission (updates per worker)")
    ap.add_argument("--maks", default=None, help="comma-separated max_active_keys values (default: the full grid)")
    ap.add_argument("--mufs", default=None, help="comma-separated min_update_frequency values (default: the full grid)")
    args = ap.parse_args(argv)
    dims = synth.DEFAULT_DIMS["rnn"]
    data = synth.make_rnn(args.instances, synth.BASE_SEED + 20, dims, 2, 10, reduction="max")
    valid = synth.make_rnn(1000, synth.BASE_SEED + 1020, dims, 2, 10, reduction="max")
    fp = synth.init_params("rnn", dims, 102)
    rows = []
    maks = [int(v) for v in args.maks.split(",")] if args.maks else MAKS
    mufs = [int(v) for v in args.mufs.split(",")] if args.mufs else MUFS
    bounded = args.max_staleness if args.admission == "bounded" else None
    for mak in maks:
        for muf in mufs:
            r = run_one(data, valid, dims, fp, args.replicas, mak, muf, args.lr, args.max_epochs, bounded, args.copies,
                        args.group_sync)
            rows.append(r)
            print(json.dumps(r), flush=True)
    if args.out:
        with open(args.out, "w") as f:
            json.dump(dict(replicas=args.replicas, copies=args.copies, group_sync=args.group_sync, target_accuracy=TARGET,
                           lr=args.lr, admission=args.admission,
                           max_staleness=bounded, rows=rows), f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
