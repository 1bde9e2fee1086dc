"""Convergence at max_active_keys > 1, independent of the event record: the
HIP path on its own schedule and the CPU checker on its own schedule (one
worker, backward first) train from the same parameters on the same seeded
data with the same max_active_keys and min_update_frequency; the accuracy
each reaches on a held-out seeded validation set must agree within 0.5
points.  The two runs take different, equally legal asynchronous paths, so
nothing finer than the accuracy is compared."""
import numpy as np
import pytest

from oracle import amp as oamp
from oracle import direct
from paper_1705_09786_amd import runner, synth

from util import OPT_KIND, f32

pytestmark = pytest.mark.gpu


def gpu_accuracy(model, dims, fp, train, valid, mak, muf, lmuf, lr, epochs, tiles=None):
    ml, me = runner.max_len_of(model, train + valid)
    tr = runner.Trainer(model, dims, fp, mak, ml, me, max(len(train), len(valid)), tiles=tiles)
    a = tr.amp
    a.set_watchdog(10.0)
    a.set_min_update_frequency(-1, muf)
    if lmuf is not None:
        a.set_min_update_frequency(0, lmuf)
    a.set_optimizer(-1, OPT_KIND["sgd"], lr=lr)
    tr.submit_all(train)
    tr.submit_all(valid, which=1)
    a.train(epochs)
    ev = a.eval()
    return ev["accuracy"], tr.params()


def oracle_accuracy(model, dims, fp, train, valid, mak, muf, lmuf, lr, epochs):
    rt = oamp.Runtime(model, dims, fp)
    rt.set_muf(muf)
    if lmuf is not None:
        rt.set_muf(lmuf, "lookup")
    rt.set_optimizer(kind="sgd", lr=f32(lr))
    rt.run(train, mak=mak, epochs=epochs)
    P = direct.unpack(model, dims, [oamp.C.pack_node(n.P) for n in rt.ppt])
    return direct.evaluate(model, dims, P, valid)[1]


TREE_SMALL = dict(vocab=200, emb=32, hidden=48, n_class=5)


def workloads(name):
    """Settings under which the checker's own accuracy moves by less than 0.4 points when max_active_keys changes
    (measured on the CPU at max_active_keys 4..6 and 8..16), so that 0.5 points separates an implementation error
    from the spread between legal asynchronous schedules."""
    if name == "mlp":      # the pipelined MLP of config 1, eight passes' worth of its data
        model, dims, train = synth.workload(1, n=8192)
        _, _, valid = synth.workload(1, n=4000, valid=True)
        return model, dims, train, valid, dict(mak=4, muf=4, lmuf=None, lr=0.01, epochs=6, floor=0.8)
    # trees shaped like config 3 at a width the checker trains in half a minute; about 12,000 validation nodes
    train = synth.make_tree(1500, 51, TREE_SMALL, max_leaves=30)
    valid = synth.make_tree(400, 1051, TREE_SMALL, max_leaves=30)
    return "tree", TREE_SMALL, train, valid, dict(mak=16, muf=10, lmuf=10, lr=0.05, epochs=3, floor=0.8)


@pytest.mark.parametrize("name", ["mlp", "tree"])
def test_accuracy_matches_checker_own_schedule(name):
    model, dims, train, valid, c = workloads(name)
    fp = synth.init_params(model, dims, 44)
    args = (model, dims, fp, train, valid, c["mak"], c["muf"], c["lmuf"], c["lr"], c["epochs"])
    acc_gpu, _ = gpu_accuracy(*args)
    acc_ref = oracle_accuracy(*args)
    print("%s: accuracy HIP path %.4f, checker %.4f" % (name, acc_gpu, acc_ref))
    assert acc_ref >= c["floor"], "the reference run itself did not learn"
    assert abs(acc_gpu - acc_ref) <= 0.005, (acc_gpu, acc_ref)
