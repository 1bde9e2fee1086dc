"""Shared helpers of the GPU parity tests: run the HIP path through the C
boundary, replay its event record in the CPU checker, compare."""
import numpy as np

from oracle import amp as oamp
from oracle import direct
from paper_1705_09786_amd import binding as B
from paper_1705_09786_amd import runner, synth

# Tolerance (relative) for fp32 results against the float64 checker.  Parameters: per tensor in the 2-norm, and
# element by element as |gpu - ref| <= RTOL * max(|ref|, rms(ref)) (an element far below the tensor's typical
# magnitude is held to the typical magnitude: its own rounding history is that of the sums it took part in);
# lookup tables additionally row by row -- rows no instance touched must still hold their initial bits.
# Losses: per instance.
RTOL = 1e-5
# Element-wise bound under Adam.  Its step lr * m / (sqrt(v) + eps) responds to an element's gradient with slope up to
# lr / eps where the gradient is near zero, so single elements amplify rounding differences that the tensor's norm
# averages out: the checker's own element-wise response to a 1e-7 perturbation of the initial parameters is five times
# larger under Adam (eps = 1e-6) than under SGD, 26 times at eps = 1e-8 (pinned on the CPU in test_oracle_models.py).
# SGD and momentum are linear in the gradient and keep RTOL element by element.
ETOL_ADAM = 5e-5


def elem_tol(opt, tol=RTOL):
    return max(tol, ETOL_ADAM) if opt is not None and opt.get("kind") == "adam" else tol

OPT_KIND = {"sgd": B.OPT_SGD, "momentum": B.OPT_MOMENTUM, "adam": B.OPT_ADAM}


def f32(x):
    return float(np.float32(x))


def gpu_train(model, dims, fp, data, mak, muf, opt, epochs=1, log=True, tiles=None, watchdog=5.0,
              arena_bytes=1 << 30, lookup_muf=None, in_hbm=(), replicas=1, max_staleness=None, strict=False, graph=None,
              node_replicas=None, group_sync=0):
    ml, me = runner.max_len_of(model, data)
    tr = runner.Trainer(model, dims, fp, mak, ml, me, len(data), arena_bytes=arena_bytes, tiles=tiles, in_hbm=in_hbm,
                        replicas=replicas, strict=strict, graph=graph, node_replicas=node_replicas)
    a = tr.amp
    a.set_watchdog(watchdog)
    if max_staleness is not None:
        a.set_admission(B.ADMIT_BOUNDED, max_staleness)
    if group_sync:
        a.set_group_sync(group_sync)
    a.set_min_update_frequency(-1, muf)
    if lookup_muf is not None:
        a.set_min_update_frequency(0, lookup_muf)
    kw = dict(opt)
    kind = OPT_KIND[kw.pop("kind")]
    a.set_optimizer(-1, kind, **kw)
    if log:
        per_inst = 8 * (2 * ml + 2) * max(1, dims.get("n_steps", 1))
        a.set_event_log(per_inst * len(data) * epochs + 1024)
    tr.submit_all(data)
    a.train(epochs)
    out = dict(params=tr.params(), losses=a.get_instance_losses().astype(np.float64), stats=a.get_loss(),
               logs=a.get_event_log() if log else None, trainer=tr, admission=a.get_admission(),
               init=[np.asarray(v, np.float32) for v in fp])
    return out


def oracle_runtime(model, dims, fp, muf, opt, lookup_muf=None):
    names = [sh[0] for sh in synth.param_shapes(model, dims)]
    rt = oamp.Runtime(model, dims, fp)
    rt.set_muf(muf)
    if lookup_muf is not None:
        rt.set_muf(lookup_muf, "lookup")
    kw = {k: (f32(v) if isinstance(v, float) else v) for k, v in opt.items()}
    rt.set_optimizer(**kw)
    if "lookup" in names:
        rt.set_optimizer("lookup", kind="sgd", lr=kw["lr"])
    return rt


def named_logs(model, dims, logs):
    """Worker logs (controller's excluded) with node ids turned into node names."""
    names = [sh[0] for sh in synth.param_shapes(model, dims)]
    return [[(names[n], k, s, l) for (n, k, s, l) in w] for w in logs]


def oracle_replay(model, dims, fp, data, logs, muf, opt, lookup_muf=None, kink_tau=None, flips=()):
    names = [sh[0] for sh in synth.param_shapes(model, dims)]
    rt = oamp.Runtime(model, dims, fp)
    if kink_tau is not None:
        for node in rt.nodes:
            if isinstance(node, oamp.NPT) and node.name.startswith("relu"):
                node.kink_tau = kink_tau
                node.flip = {(state, i) for (name, state, i) in flips if name == node.name}
    rt.set_muf(muf)
    if lookup_muf is not None:
        rt.set_muf(lookup_muf, "lookup")
    kw = {k: (f32(v) if isinstance(v, float) else v) for k, v in opt.items()}
    rt.set_optimizer(**kw)
    if "lookup" in names:
        rt.set_optimizer("lookup", kind="sgd", lr=kw["lr"])
    wl = [[(names[n], k, s, l) for (n, k, s, l) in w] for w in logs[1:]]
    rt.replay(data, wl)
    return rt


def rel_err(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def elementwise_err(a, ref):
    """max over elements of |a - ref| / max(|ref|, rms(ref)), and the flat index where it is reached."""
    a, ref = np.asarray(a, np.float64).ravel(), np.asarray(ref, np.float64).ravel()
    scale = np.maximum(np.abs(ref), max(float(np.sqrt(np.mean(ref * ref))), 1e-30))
    e = np.abs(a - ref) / scale
    i = int(e.argmax())
    return float(e[i]), i


def lookup_tokens(model, instances):
    """Rows of the model's lookup table that the instances read."""
    key = "node_type" if model == "ggnn" else "tokens"
    return np.unique(np.concatenate([np.asarray(i[key], np.int64).ravel() for i in instances]))


def check_lookup_rows(name, table_gpu, table_ref, table_init, touched, tol=RTOL):
    """A lookup's gradient is a scatter-add into the rows its instances read: those rows are compared with the
    checker's row by row (a lost or misplaced scatter of one row shows here, where the whole table's norm hides
    it); every other row must be bit-equal to the initial table."""
    touched = np.asarray(touched, np.int64)
    untouched = np.setdiff1d(np.arange(table_init.shape[0]), touched)
    same = table_gpu[untouched].view(np.uint32) == table_init[untouched].view(np.uint32)
    assert same.all(), "%s: %d untouched rows changed, first %d" % (name, int((~same.all(axis=1)).sum()),
                                                                    int(untouched[np.flatnonzero(~same.all(axis=1))[0]]))
    rms = max(float(np.sqrt(np.mean(table_ref[touched] ** 2))), 1e-30)
    row_err = np.linalg.norm(table_gpu[touched].astype(np.float64) - table_ref[touched], axis=1) \
        / np.maximum(np.linalg.norm(table_ref[touched], axis=1), rms)
    worst = int(row_err.argmax())
    assert row_err[worst] <= tol, "%s: row %d off by %.3e" % (name, int(touched[worst]), float(row_err[worst]))
    return float(row_err[worst])


def compare(gpu, rt, n_adm, tol=RTOL, opt=None, ref_losses=None):
    """opt: the optimizer setting of the run (None = SGD-like), which fixes the element-wise bound.
    ref_losses: the checker's losses in the order of gpu["losses"], where that is not admissions 0 .. n_adm - 1."""
    etol = elem_tol(opt, tol)
    errs, elem = {}, {}
    for k, node in enumerate(rt.ppt):
        ref = oamp.C.pack_node(node.P)
        errs[node.name] = rel_err(gpu["params"][k], ref)
        elem[node.name] = elementwise_err(gpu["params"][k], ref)
    ref_loss = np.array([rt.loss[s] for s in range(n_adm)]) if ref_losses is None else np.asarray(ref_losses, np.float64)
    le = np.abs(gpu["losses"] - ref_loss) / np.maximum(np.abs(ref_loss), 1.0)
    off = np.flatnonzero(le > tol)
    # everything a failure needs in one message: every tensor's error and where the losses part ways
    report = dict(params=errs, elementwise=elem, loss_max=float(le.max()), first_loss_off=int(off[0]) if len(off) else None,
                  n_loss_off=len(off))
    assert max(errs.values()) <= tol, report
    assert max(e for e, _ in elem.values()) <= etol, report
    assert le.max() <= tol, report
    if rt.ppt[0].name == "lookup" and "init" in gpu:
        W = rt.ppt[0].P["W"]
        # rows touched: those of the instances that trained (inference instances read rows but never write them)
        check_lookup_rows("lookup", np.asarray(gpu["params"][0], np.float32).reshape(W.shape), W,
                          np.asarray(gpu["init"][0], np.float32).reshape(W.shape), lookup_tokens(rt.model, rt.instances), etol)
    return max(errs.values()), float(le.max())


def check_controller_log(logs, mak, n_adm):
    active = 0
    adm = []
    for (_, kind, seq, _) in logs[0]:
        if kind == "A":
            active += 1
            adm.append(seq)
        else:
            assert kind == "R"
            active -= 1
        assert 0 <= active <= mak
    assert adm == list(range(n_adm))
    assert active == 0


# |pre-activation| below which a ReLU decision may fall either way: a 128-term fp32 dot product of O(1) terms is
# good to about 1e-6 absolute, and the kernel sums in another order than the checker.
RELU_TAU = 3e-6


def compare_up_to_relu_decisions(model, dims, fp, data, gpu, muf, opt, max_flips=6):
    """Replay parity for a model with ReLUs.  A pre-activation within rounding of zero is a yes / no decision that
    fp32 on the GPU and fp64 in the checker may take differently; the whole gradient of that unit then differs and
    no tolerance covers it.  Both decisions are correct, so the check is: some assignment of the (few) decisions
    the checker itself marks as ambiguous (|x| < RELU_TAU) reproduces the GPU's result to the usual tolerance.  The
    search is greedy: replay, and while the results differ, reverse the ambiguous decision closest before the
    first instance whose loss differs."""
    flips = []
    report = None
    for _ in range(max_flips + 1):
        rt = oracle_replay(model, dims, fp, data, gpu["logs"], muf, opt, kink_tau=RELU_TAU, flips=flips)
        try:
            return compare(gpu, rt, len(data), opt=opt) + (len(flips),)
        except AssertionError as e:
            report = e.args[0]
        kinks = [(node.name, state, i) for node in rt.nodes if isinstance(node, oamp.NPT) for (state, i) in node.kinks]
        cands = [k for k in kinks if k not in flips]
        first = report["first_loss_off"] if report["first_loss_off"] is not None else len(data)
        before = [k for k in cands if k[1][0] <= first]
        if not before:
            break
        flips.append(max(before, key=lambda k: k[1][0]))
    raise AssertionError(dict(report, ambiguous_relu_decisions_reversed=flips))
