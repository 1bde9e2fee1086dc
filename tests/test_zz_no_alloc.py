"""amp_create_static: the entry point for callers that cannot allocate device memory.  The context works inside the
library's built-in device array instead of a caller's arena; everything it computes must be what a context created
with amp_create computes.  Two uses in a row share the array, the second smaller than the first and laid out
differently, so whatever the first left behind lies under the second.

With one instance in flight the recurrent model and the MLP are sequential programs, so the two kinds of context
must agree bit for bit; with several in flight each run takes its own order, and the built-in-arena run is held to
the checker's replay of its own event record, like every other parity case."""
import ctypes as ct

import numpy as np
import pytest

from paper_1705_09786_amd import binding as B
from paper_1705_09786_amd import runner, synth

from util import OPT_KIND, compare, compare_up_to_relu_decisions, oracle_replay

pytestmark = pytest.mark.gpu

SGD = dict(kind="sgd", lr=0.05)


def run_in(amp_ctx, model, dims, fp, data, mak, muf, opt, log=False):
    """Drives a context through the C boundary: build, finalize, parameters, instances, one epoch."""
    ml, me = runner.max_len_of(model, data)
    amp_ctx.build(model, dims)
    amp_ctx.finalize(mak, ml, me, len(data))
    for k, v in enumerate(fp):
        amp_ctx.set_params(k, v)
    amp_ctx.set_watchdog(5.0)
    amp_ctx.set_min_update_frequency(-1, muf)
    kw = dict(opt)
    amp_ctx.set_optimizer(-1, OPT_KIND[kw.pop("kind")], **kw)
    if log:
        amp_ctx.set_event_log(64 * (2 * ml + 2) * len(data) + 1024)
    for k, inst in enumerate(data):
        amp_ctx.submit(inst, key=k)
    amp_ctx.train(1)
    return dict(params=[amp_ctx.get_params(k) for k in range(amp_ctx.num_nodes())],
                losses=amp_ctx.get_instance_losses().astype(np.float64), stats=amp_ctx.get_loss(),
                logs=amp_ctx.get_event_log() if log else None, init=[np.asarray(v, np.float32) for v in fp])


def in_callers_arena(*args, **kw):
    import torch
    buf = torch.empty((256 << 20) + 256, dtype=torch.uint8, device="cuda:0")
    ptr = (buf.data_ptr() + 255) // 256 * 256
    a = B.Amp(ptr, 256 << 20, torch.cuda.current_stream().cuda_stream)
    try:
        return run_in(a, *args, **kw)
    finally:
        a.close()
        del buf


def in_builtin_arena(*args, **kw):
    import torch
    torch.cuda.set_device(0)
    a = B.Amp(None, stream=torch.cuda.current_stream().cuda_stream)
    try:
        return run_in(a, *args, **kw)
    finally:
        a.close()


def assert_same(x, y):
    assert np.array_equal(x["losses"], y["losses"])
    for p, q in zip(x["params"], y["params"]):
        assert np.array_equal(p.view(np.uint32), q.view(np.uint32))


def test_builtin_arena_matches_callers_arena_twice_in_a_row():
    # first use: the recurrent model of the benchmark, 300 sequences
    model, dims, data = synth.workload(2, n=300)
    fp = synth.init_params(model, dims, 6)
    assert_same(in_builtin_arena(model, dims, fp, data, 1, 3, SGD), in_callers_arena(model, dims, fp, data, 1, 3, SGD))
    # second use, smaller and laid out differently, on top of what the first left in the array
    model2, dims2, data2 = synth.workload(1, n=96)
    fp2 = synth.init_params(model2, dims2, 5)
    assert_same(in_builtin_arena(model2, dims2, fp2, data2, 1, 2, SGD), in_callers_arena(model2, dims2, fp2, data2, 1, 2, SGD))
    # several instances in flight: replay parity of the built-in-arena run itself, tree model (tiles, joins, lookup)
    tdims = dict(vocab=97, emb=50, hidden=37, n_class=5)
    tdata = synth.make_tree(40, 21, tdims, max_leaves=20)
    tfp = synth.init_params("tree", tdims, 8)
    g = in_builtin_arena("tree", tdims, tfp, tdata, 8, 3, SGD, log=True)
    rt = oracle_replay("tree", tdims, tfp, tdata, g["logs"], 3, SGD)
    compare(g, rt, len(tdata), opt=SGD)
    # and the MLP with four in flight
    g = in_builtin_arena(model2, dims2, fp2, data2, 4, 1, SGD, log=True)
    compare_up_to_relu_decisions(model2, dims2, fp2, data2, g, 1, SGD)


def test_builtin_arena_limits():
    import torch
    torch.cuda.set_device(0)
    a = B.Amp(None)
    try:
        # one context per GPU at a time
        h = ct.c_void_p()
        assert B.lib().amp_create_static(ct.byref(h), None) == B.AMP_ESTATE
        # the benchmark's Tree-LSTM (a 24 MB lookup table with three more arrays of its size) does not fit 64 MiB
        a.build("tree", synth.DEFAULT_DIMS["tree"])
        with pytest.raises(B.AmpError) as e:
            a.finalize(64, 60, 0, 8544)
        assert e.value.code == B.AMP_ENOMEM and "built-in arena" in str(e.value)
    finally:
        a.close()
    # after the first context is gone the array can be used again
    b = B.Amp(None)
    b.close()
