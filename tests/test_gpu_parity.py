"""GPU parity: the HIP path, called through the C boundary, against the CPU
checker replaying the order in which the GPU's workers executed their
events.  Parameters and per-instance losses must agree to 1e-5 (relative)."""
import numpy as np
import pytest

from oracle import direct
from paper_1705_09786_amd import synth

from util import check_controller_log, compare, gpu_train, oracle_replay

pytestmark = pytest.mark.gpu

SGD = dict(kind="sgd", lr=0.05)
ADAM = dict(kind="adam", lr=0.002, beta1=0.9, beta2=0.999, eps=1e-8)


@pytest.mark.parametrize("mak,muf,opt", [(1, 1, SGD), (4, 1, SGD), (4, 3, ADAM), (8, 5, dict(kind="momentum", lr=0.02, momentum=0.9))])
def test_mlp_replay_parity(mak, muf, opt):
    model, dims, data = synth.workload(1)
    fp = synth.init_params(model, dims, 5)
    g = gpu_train(model, dims, fp, data, mak, muf, opt)
    check_controller_log(g["logs"], mak, len(data))
    rt = oracle_replay(model, dims, fp, data, g["logs"], muf, opt)
    compare(g, rt, len(data))


def test_mlp_mak1_is_synchronous_sgd():
    """max_active_keys = 1 on the MLP is plain per-instance SGD (Section 5,
    Table 1 caption): compare with the checker's direct trainer, no log."""
    model, dims, data = synth.workload(1)
    fp = synth.init_params(model, dims, 5)
    g = gpu_train(model, dims, fp, data, 1, 1, SGD, log=False)
    P = direct.unpack(model, dims, fp)
    ref = direct.train(model, dims, P, data, lr=float(np.float32(0.05)))
    assert np.abs(g["losses"] - np.array(ref)).max() <= 1e-5 * max(1.0, np.abs(ref).max())
    for k in range(3):
        refv = np.concatenate([P[k]["W"].reshape(-1), P[k]["b"]])
        assert np.linalg.norm(g["params"][k] - refv) / np.linalg.norm(refv) <= 1e-5


@pytest.mark.parametrize("mak,muf,opt,n", [(1, 1, SGD, 200), (16, 1, SGD, 600), (16, 7, ADAM, 600)])
def test_rnn_replay_parity(mak, muf, opt, n):
    model, dims, data = synth.workload(2, n=n)
    fp = synth.init_params(model, dims, 6)
    g = gpu_train(model, dims, fp, data, mak, muf, opt)
    check_controller_log(g["logs"], mak, len(data))
    rt = oracle_replay(model, dims, fp, data, g["logs"], muf, opt)
    compare(g, rt, len(data))


def test_rnn_edge_lengths():
    """Length-1 sequences, the maximum length, and a ragged mix."""
    dims = synth.DEFAULT_DIMS["rnn"]
    data = synth.make_rnn(40, 3, dims, min_len=1, max_len=1) + synth.make_rnn(40, 4, dims, min_len=32, max_len=32) \
        + synth.make_rnn(40, 5, dims, min_len=1, max_len=32)
    fp = synth.init_params("rnn", dims, 6)
    g = gpu_train("rnn", dims, fp, data, 5, 2, SGD)
    rt = oracle_replay("rnn", dims, fp, data, g["logs"], 2, SGD)
    compare(g, rt, len(data))
