"""ctypes binding of include/amp.h: argument marshalling only.

Every function of the C boundary is exposed under its own name on `lib()`;
`Amp` is a small convenience wrapper (same calls, Python containers in and
out).  There is no fallback: if libamp.so is missing the import of the
library raises.
"""
from __future__ import annotations

import ctypes as ct
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libamp.so")
# the same sources built with -DAMP_STRICT_JOIN (explicitly ordered join completion), for attribution runs
LIB_STRICT_PATH = os.path.join(_HERE, "libamp_strict.so")

AMP_OK, AMP_EINVAL, AMP_ESTATE, AMP_ENOMEM, AMP_EFULL, AMP_EDEVICE, AMP_EUNSUPPORTED = 0, -1, -2, -3, -4, -5, -6
MODEL_MLP, MODEL_RNN, MODEL_TREE, MODEL_GGNN = 1, 2, 3, 4
ADMIT_GREEDY, ADMIT_BOUNDED = 0, 1
OPT_SGD, OPT_MOMENTUM, OPT_ADAM = 0, 1, 2
EV_NAMES = "FBUARSL"

_f32p = ct.POINTER(ct.c_float)
_i32p = ct.POINTER(ct.c_int32)


class ModelDims(ct.Structure):
    _fields_ = [(n, ct.c_int32) for n in ("d_in", "hidden", "n_class", "vocab", "emb",
                                          "n_node_types", "n_edge_types", "n_steps")]


class Instance(ct.Structure):
    _fields_ = [("n_x", ct.c_int32), ("x", _f32p),
                ("n_tokens", ct.c_int32), ("tokens", _i32p),
                ("n_labels", ct.c_int32), ("labels", _i32p),
                ("n_nodes", ct.c_int32), ("left", _i32p), ("right", _i32p),
                ("n_edges", ct.c_int32), ("src", _i32p), ("dst", _i32p), ("etype", _i32p),
                ("target", ct.c_float)]


class NodeDesc(ct.Structure):
    _fields_ = [(n, ct.c_int32) for n in ("rows", "cols", "n_in", "n_out", "aux")]


NODE_KINDS = ("controller", "lookup", "linear", "rnn_tanh", "gru", "leaf_lstm", "branch_lstm", "ggnn_edge_linear",
              "sum_readout", "softmax_xent", "squared_err", "cond", "phi", "isu", "concat", "split", "bcast", "group",
              "ungroup", "flatmap", "sum", "sink")
ACT_NONE, ACT_RELU = 0, 1


class OptParams(ct.Structure):
    _fields_ = [(n, ct.c_float) for n in ("lr", "momentum", "beta1", "beta2", "eps")]


class Event(ct.Structure):
    _fields_ = [("worker", ct.c_uint16), ("node", ct.c_uint8), ("kind", ct.c_uint8),
                ("seq", ct.c_uint32), ("local", ct.c_uint32)]


class EvalResult(ct.Structure):
    _fields_ = [("mean_loss", ct.c_double), ("accuracy", ct.c_double), ("n_instances", ct.c_uint64),
                ("n_predictions", ct.c_uint64), ("seconds", ct.c_double)]


_ctxp = ct.c_void_p
SIGNATURES = {
    "amp_create": (ct.c_int, [ct.POINTER(_ctxp), ct.c_void_p, ct.c_size_t, ct.c_void_p]),
    "amp_create_static": (ct.c_int, [ct.POINTER(_ctxp), ct.c_void_p]),
    "amp_destroy": (None, [_ctxp]),
    "amp_add_node": (ct.c_int, [_ctxp, ct.c_int, ct.POINTER(NodeDesc), ct.POINTER(ct.c_int)]),
    "amp_connect": (ct.c_int, [_ctxp, ct.c_int, ct.c_int, ct.c_int, ct.c_int]),
    "amp_validate_graph": (ct.c_int, [_ctxp]),
    "amp_get_node_index": (ct.c_int, [_ctxp, ct.c_int, ct.POINTER(ct.c_int)]),
    "amp_build_mlp": (ct.c_int, [_ctxp, ct.POINTER(ModelDims)]),
    "amp_build_rnn": (ct.c_int, [_ctxp, ct.POINTER(ModelDims)]),
    "amp_build_treelstm": (ct.c_int, [_ctxp, ct.POINTER(ModelDims)]),
    "amp_build_ggnn": (ct.c_int, [_ctxp, ct.POINTER(ModelDims)]),
    "amp_set_tiles": (ct.c_int, [_ctxp, ct.c_int, ct.c_int]),
    "amp_set_weights_in_hbm": (ct.c_int, [_ctxp, ct.c_int, ct.c_int]),
    "amp_set_replicas": (ct.c_int, [_ctxp, ct.c_int]),
    "amp_set_node_replicas": (ct.c_int, [_ctxp, ct.c_int, ct.c_int]),
    "amp_set_group_sync": (ct.c_int, [_ctxp, ct.c_int]),
    "amp_finalize": (ct.c_int, [_ctxp, ct.c_int, ct.c_int, ct.c_int, ct.c_size_t]),
    "amp_set_max_active_keys": (ct.c_int, [_ctxp, ct.c_int]),
    "amp_set_min_update_frequency": (ct.c_int, [_ctxp, ct.c_int, ct.c_int]),
    "amp_set_optimizer": (ct.c_int, [_ctxp, ct.c_int, ct.c_int, ct.POINTER(OptParams)]),
    "amp_set_gradient_mean": (ct.c_int, [_ctxp, ct.c_int]),
    "amp_num_nodes": (ct.c_int, [_ctxp]),
    "amp_num_workers": (ct.c_int, [_ctxp]),
    "amp_param_count": (ct.c_int, [_ctxp, ct.c_int, ct.POINTER(ct.c_size_t)]),
    "amp_set_params": (ct.c_int, [_ctxp, ct.c_int, _f32p, ct.c_size_t]),
    "amp_get_params": (ct.c_int, [_ctxp, ct.c_int, _f32p, ct.c_size_t, ct.POINTER(ct.c_size_t)]),
    "amp_submit": (ct.c_int, [_ctxp, ct.c_int, ct.c_uint64, ct.POINTER(Instance)]),
    "amp_clear_instances": (ct.c_int, [_ctxp, ct.c_int]),
    "amp_set_event_log": (ct.c_int, [_ctxp, ct.c_size_t]),
    "amp_set_watchdog": (ct.c_int, [_ctxp, ct.c_double]),
    "amp_set_probe": (ct.c_int, [_ctxp, ct.c_uint, ct.c_size_t]),
    "amp_get_probe": (ct.c_int, [_ctxp, _f32p, ct.c_size_t, ct.POINTER(ct.c_size_t), ct.POINTER(ct.c_size_t)]),
    "amp_set_admission": (ct.c_int, [_ctxp, ct.c_int, ct.c_double]),
    "amp_get_admission": (ct.c_int, [_ctxp, ct.POINTER(ct.c_int), ct.POINTER(ct.c_int)]),
    "amp_train": (ct.c_int, [_ctxp, ct.c_int]),
    "amp_eval": (ct.c_int, [_ctxp, ct.POINTER(EvalResult)]),
    "amp_train_eval": (ct.c_int, [_ctxp, ct.c_int, ct.POINTER(EvalResult)]),
    "amp_get_loss": (ct.c_int, [_ctxp, ct.POINTER(ct.c_double), ct.POINTER(ct.c_double),
                                ct.POINTER(ct.c_uint64), ct.POINTER(ct.c_double)]),
    "amp_get_instance_losses": (ct.c_int, [_ctxp, _f32p, ct.c_size_t, ct.POINTER(ct.c_size_t)]),
    "amp_get_event_log": (ct.c_int, [_ctxp, ct.POINTER(Event), ct.c_size_t, ct.POINTER(ct.c_size_t)]),
    "amp_get_staleness_hist": (ct.c_int, [_ctxp, ct.POINTER(ct.c_uint64), ct.c_size_t]),
    "amp_get_worker_stats": (ct.c_int, [_ctxp, ct.POINTER(ct.c_double), ct.POINTER(ct.c_uint64), _i32p,
                                        ct.c_size_t, ct.POINTER(ct.c_size_t), ct.POINTER(ct.c_uint64),
                                        ct.POINTER(ct.c_double)]),
    "amp_get_worker_placement": (ct.c_int, [_ctxp, _i32p, ct.c_size_t, ct.POINTER(ct.c_size_t)]),
    "amp_last_error": (ct.c_char_p, [_ctxp]),
    "amp_measure_peaks": (ct.c_int, [ct.c_void_p, ct.c_size_t, ct.c_void_p, ct.POINTER(ct.c_double),
                                     ct.POINTER(ct.c_double)]),
}

_libs = {}


def lib(strict: bool = False):
    """The loaded C library (raises if it has not been built); strict = the build with ordered joins."""
    if strict not in _libs:
        path = LIB_STRICT_PATH if strict else LIB_PATH
        if not os.path.exists(path):
            raise RuntimeError("%s is not built: run `python -m paper_1705_09786_amd.build`" % os.path.basename(path))
        l = ct.CDLL(path)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _libs[strict] = l
    return _libs[strict]


def measure_peaks(dev_ptr: int, nbytes: int, stream: int = 0):
    """(LDS bytes/s per CU, HBM read bytes/s) measured on the current device; dev_ptr = device buffer of nbytes."""
    a, b = ct.c_double(), ct.c_double()
    rc = lib().amp_measure_peaks(ct.c_void_p(dev_ptr), nbytes, ct.c_void_p(stream), ct.byref(a), ct.byref(b))
    if rc != 0:
        raise RuntimeError("amp_measure_peaks failed with code %d" % rc)
    return a.value, b.value


class AmpError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("amp error %d: %s" % (code, msg))
        self.code = code


def _ip(a):
    return a.ctypes.data_as(_i32p)


def to_c_instance(model: int, inst: dict):
    """dict (as produced by synth) -> (Instance, list of arrays kept alive)."""
    ci = Instance()
    keep = []

    def i32(v):
        a = np.ascontiguousarray(v, dtype=np.int32)
        keep.append(a)
        return a
    if model == MODEL_MLP:
        x = np.ascontiguousarray(inst["x"], dtype=np.float32)
        keep.append(x)
        ci.n_x, ci.x = x.size, x.ctypes.data_as(_f32p)
        lab = i32([inst["label"]])
        ci.n_labels, ci.labels = 1, _ip(lab)
    elif model == MODEL_RNN:
        tok = i32(inst["tokens"])
        lab = i32([inst["label"]])
        ci.n_tokens, ci.tokens, ci.n_labels, ci.labels = tok.size, _ip(tok), 1, _ip(lab)
    elif model == MODEL_TREE:
        tok, lab, le, ri = i32(inst["tokens"]), i32(inst["labels"]), i32(inst["left"]), i32(inst["right"])
        ci.n_tokens, ci.tokens, ci.n_labels, ci.labels = tok.size, _ip(tok), lab.size, _ip(lab)
        ci.n_nodes, ci.left, ci.right = le.size, _ip(le), _ip(ri)
    elif model == MODEL_GGNN:
        tok, s, d, t = i32(inst["node_type"]), i32(inst["src"]), i32(inst["dst"]), i32(inst["etype"])
        ci.n_tokens, ci.tokens, ci.n_nodes = tok.size, _ip(tok), tok.size
        ci.n_edges, ci.src, ci.dst, ci.etype = s.size, _ip(s), _ip(d), _ip(t)
        ci.target = float(inst["target"])
    return ci, keep


MODEL_IDS = {"mlp": MODEL_MLP, "rnn": MODEL_RNN, "tree": MODEL_TREE, "ggnn": MODEL_GGNN}
_BUILDERS = {MODEL_MLP: "amp_build_mlp", MODEL_RNN: "amp_build_rnn", MODEL_TREE: "amp_build_treelstm",
             MODEL_GGNN: "amp_build_ggnn"}


class Amp:
    """One context of the C library.  `arena` is a device pointer (int) to
    `arena_bytes` bytes owned by the caller; `stream` a hipStream_t (int)."""

    def __init__(self, arena: int | None, arena_bytes: int = 0, stream: int = 0, strict: bool = False):
        """arena None: the library's built-in device arena (amp_create_static)."""
        self.L = lib(strict)
        self.h = _ctxp()
        if arena is None:
            rc = self.L.amp_create_static(ct.byref(self.h), ct.c_void_p(stream))
        else:
            rc = self.L.amp_create(ct.byref(self.h), ct.c_void_p(arena), arena_bytes, ct.c_void_p(stream))
        if rc:
            raise AmpError(rc, "amp_create_static failed" if arena is None else "amp_create failed")
        self.model = 0

    def close(self):
        if self.h:
            self.L.amp_destroy(self.h)
            self.h = _ctxp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _chk(self, rc):
        if rc:
            raise AmpError(rc, self.L.amp_last_error(self.h).decode())

    def build(self, model: str, dims: dict):
        self.model = MODEL_IDS[model]
        d = ModelDims(**{k: int(v) for k, v in dims.items()})
        self._chk(getattr(self.L, _BUILDERS[self.model])(self.h, ct.byref(d)))

    def add_node(self, kind: str, rows=0, cols=0, n_in=1, n_out=1, aux=0) -> int:
        d = NodeDesc(rows, cols, n_in, n_out, aux)
        nid = ct.c_int(-1)
        self._chk(self.L.amp_add_node(self.h, NODE_KINDS.index(kind), ct.byref(d), ct.byref(nid)))
        return nid.value

    def connect(self, src, src_port, dst, dst_port):
        self._chk(self.L.amp_connect(self.h, src, src_port, dst, dst_port))

    def validate_graph(self, model: str | None = None):
        """Validates and lowers a graph made with add_node / connect; `model` names what the caller expects it to
        be, so that submit() knows how to marshal instances."""
        self._chk(self.L.amp_validate_graph(self.h))
        if model is not None:
            self.model = MODEL_IDS[model]

    def get_node_index(self, graph_node):
        v = ct.c_int(-2)
        self._chk(self.L.amp_get_node_index(self.h, graph_node, ct.byref(v)))
        return v.value

    def set_tiles(self, node, n):
        self._chk(self.L.amp_set_tiles(self.h, node, n))

    def set_replicas(self, n):
        self._chk(self.L.amp_set_replicas(self.h, n))

    def set_node_replicas(self, node, n):
        self._chk(self.L.amp_set_node_replicas(self.h, node, n))

    def set_group_sync(self, every_retirements):
        self._chk(self.L.amp_set_group_sync(self.h, every_retirements))

    def set_weights_in_hbm(self, node, on=True):
        self._chk(self.L.amp_set_weights_in_hbm(self.h, node, int(on)))

    def finalize(self, max_active_keys, max_instance_len, max_edges, max_instances):
        self._chk(self.L.amp_finalize(self.h, max_active_keys, max_instance_len, max_edges, max_instances))

    def set_max_active_keys(self, mak):
        self._chk(self.L.amp_set_max_active_keys(self.h, mak))

    def set_min_update_frequency(self, node, muf):
        self._chk(self.L.amp_set_min_update_frequency(self.h, node, muf))

    def set_optimizer(self, node, kind, lr=0.1, momentum=0.9, beta1=0.9, beta2=0.999, eps=1e-8):
        p = OptParams(lr, momentum, beta1, beta2, eps)
        self._chk(self.L.amp_set_optimizer(self.h, node, kind, ct.byref(p)))

    def set_gradient_mean(self, mean):
        self._chk(self.L.amp_set_gradient_mean(self.h, int(mean)))

    def num_nodes(self):
        return self.L.amp_num_nodes(self.h)

    def num_workers(self):
        return self.L.amp_num_workers(self.h)

    def set_params(self, node, vec):
        v = np.ascontiguousarray(vec, dtype=np.float32)
        self._chk(self.L.amp_set_params(self.h, node, v.ctypes.data_as(_f32p), v.size))

    def get_params(self, node):
        n = ct.c_size_t()
        self._chk(self.L.amp_param_count(self.h, node, ct.byref(n)))
        out = np.empty(n.value, np.float32)
        self._chk(self.L.amp_get_params(self.h, node, out.ctypes.data_as(_f32p), out.size, ct.byref(n)))
        return out

    def submit(self, inst: dict, which=0, key=0):
        ci, keep = to_c_instance(self.model, inst)
        self._chk(self.L.amp_submit(self.h, which, key, ct.byref(ci)))

    def clear_instances(self, which=0):
        self._chk(self.L.amp_clear_instances(self.h, which))

    def set_event_log(self, n):
        self._chk(self.L.amp_set_event_log(self.h, n))

    def set_admission(self, policy, max_staleness=0.0):
        self._chk(self.L.amp_set_admission(self.h, policy, max_staleness))

    def get_admission(self):
        a, b = ct.c_int(0), ct.c_int(0)
        self._chk(self.L.amp_get_admission(self.h, ct.byref(a), ct.byref(b)))
        return dict(max_in_flight=a.value, final_limit=b.value)

    def set_probe(self, period, max_entries=0):
        self._chk(self.L.amp_set_probe(self.h, period, max_entries))

    def get_probe(self):
        """(header int32 array [n][4] = kind, admission number, tree node, 0; payload float32 array [n][w - 4])."""
        n, w = ct.c_size_t(), ct.c_size_t()
        self._chk(self.L.amp_get_probe(self.h, None, 0, ct.byref(n), ct.byref(w)))
        buf = np.zeros(max(n.value * w.value, 1), np.float32)
        self._chk(self.L.amp_get_probe(self.h, buf.ctypes.data_as(_f32p), buf.size, ct.byref(n), ct.byref(w)))
        e = buf[:n.value * w.value].reshape(n.value, max(w.value, 4))
        return e[:, :4].copy().view(np.int32), e[:, 4:].copy()

    def set_watchdog(self, seconds):
        self._chk(self.L.amp_set_watchdog(self.h, seconds))

    def train(self, epochs=1):
        self._chk(self.L.amp_train(self.h, epochs))

    def eval(self):
        r = EvalResult()
        self._chk(self.L.amp_eval(self.h, ct.byref(r)))
        return dict(mean_loss=r.mean_loss, accuracy=r.accuracy, n_instances=r.n_instances,
                    n_predictions=r.n_predictions, seconds=r.seconds)

    def train_eval(self, epochs=1):
        """Training and evaluation instances mixed in one launch; returns the evaluation results."""
        r = EvalResult()
        self._chk(self.L.amp_train_eval(self.h, epochs, ct.byref(r)))
        return dict(mean_loss=r.mean_loss, accuracy=r.accuracy, n_instances=r.n_instances,
                    n_predictions=r.n_predictions, seconds=r.seconds)

    def get_loss(self):
        ml, acc, n, sec = ct.c_double(), ct.c_double(), ct.c_uint64(), ct.c_double()
        self._chk(self.L.amp_get_loss(self.h, ct.byref(ml), ct.byref(acc), ct.byref(n), ct.byref(sec)))
        return dict(mean_loss=ml.value, accuracy=acc.value, n_instances=n.value, seconds=sec.value)

    def get_instance_losses(self):
        n = ct.c_size_t()
        self.L.amp_get_instance_losses(self.h, ct.cast(ct.c_void_p(1), _f32p), 0, ct.byref(n))
        out = np.empty(max(n.value, 1), np.float32)
        self._chk(self.L.amp_get_instance_losses(self.h, out.ctypes.data_as(_f32p), out.size, ct.byref(n)))
        return out[:n.value]

    def get_event_log(self):
        """List per worker of (node id, kind letter, seq, local)."""
        n = ct.c_size_t()
        self._chk(self.L.amp_get_event_log(self.h, None, 0, ct.byref(n)))
        buf = (Event * max(n.value, 1))()
        self._chk(self.L.amp_get_event_log(self.h, buf, n.value, ct.byref(n)))
        logs = [[] for _ in range(self.num_workers())]
        for e in buf[:n.value]:
            logs[e.worker].append((e.node, EV_NAMES[e.kind], e.seq, e.local))
        return logs

    def get_event_array(self):
        """The same record as one numpy structured array (fields worker, node, kind, seq, local), for long runs."""
        import numpy as np
        n = ct.c_size_t()
        self._chk(self.L.amp_get_event_log(self.h, None, 0, ct.byref(n)))
        buf = (Event * max(n.value, 1))()
        self._chk(self.L.amp_get_event_log(self.h, buf, n.value, ct.byref(n)))
        dt = np.dtype([("worker", np.uint16), ("node", np.uint8), ("kind", np.uint8), ("seq", np.uint32),
                       ("local", np.uint32)])
        return np.frombuffer(buf, dtype=dt, count=n.value).copy()

    def get_worker_stats(self):
        """List per worker of dict(node, wait_fraction, messages)."""
        nw = self.num_workers()
        wf, ms, nd = (ct.c_double * nw)(), (ct.c_uint64 * nw)(), (ct.c_int32 * nw)()
        bt, ph = (ct.c_uint64 * nw)(), (ct.c_double * (8 * nw))()
        n = ct.c_size_t()
        self._chk(self.L.amp_get_worker_stats(self.h, wf, ms, nd, nw, ct.byref(n), bt, ph))
        return [dict(node=nd[i], wait_fraction=wf[i], messages=ms[i], batches=bt[i],
                     phases=[ph[8 * i + j] for j in range(8)]) for i in range(min(nw, n.value))]

    def get_worker_placement(self):
        """The XCC (die) every worker's workgroup ran on, in worker order."""
        nw = self.num_workers()
        x = (ct.c_int32 * nw)()
        n = ct.c_size_t()
        self._chk(self.L.amp_get_worker_placement(self.h, x, nw, ct.byref(n)))
        return list(x[:n.value])

    def get_staleness_hist(self, nbins=16):
        bins = (ct.c_uint64 * nbins)()
        self._chk(self.L.amp_get_staleness_hist(self.h, bins, nbins))
        return list(bins)
