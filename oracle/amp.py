"""CPU checker, part 3: message-passing simulator of asynchronous
model-parallel (AMP) training over the paper's static IR.

TEST INFRASTRUCTURE ONLY.  Plain float64 numpy and Python loops.  Shares no
code with the HIP path and is never imported by it.

What is simulated (citations are to the paper):
  * messages = payload + state; forward messages travel with the graph's
    edges, backward messages against them; every forward message a node
    emits is answered by exactly one backward message with the same state
    (Section 4, Overview) -- checked at run time;
  * the IR node kinds of Section 4: parameterized and non-parameterized
    payload transforms, Cond, Phi, Isu, Concat, Bcast, Group, Ungroup,
    Flatmap, and a loss layer that starts backpropagation;
  * the AMP rule of Section 3: a parameterized node adds each gradient to a
    local accumulator and, once the number accumulated since its last update
    reaches min_update_frequency, applies its optimizer by itself and clears
    the accumulator; the controller keeps at most max_active_keys instances
    in flight.

Inference instances (Section 1: training and inference at the same time) are
forward-only: the controller marks them at admission, parameterized nodes
apply their present parameters without a gradient ever coming back, the loss
layer scores them and does not start backpropagation, and the instance
retires once all its predictions are scored; whatever the nodes cached for
it on the way is dropped then.

Two drivers:
  * run():    one worker hosts every node; backward messages are served
              before forward ones, first-in first-out within each class
              (Appendix A); the controller admits a new instance whenever
              fewer than max_active_keys are active.
  * replay(): executes the parameterized nodes' forward / backward / update
              events in an order recorded elsewhere (one ordered list per
              worker), and refuses orders that are not legal AMP executions.

Readings of points the paper leaves open:
the backward pass uses the node's present parameters (only the activation is
recorded); "exceeds the threshold" means count >= min_update_frequency; the
applied gradient is the mean of the accumulated ones; one backward message is
one gradient whatever its row count; Bcast sums its successors' gradients in
port order.
"""
from __future__ import annotations

from collections import deque

import numpy as np

from . import cells as C


class Msg:
    __slots__ = ("payload", "state")

    def __init__(self, payload, state):
        self.payload, self.state = payload, state


# ============================================================== IR node kinds
class Node:
    is_ppt = False

    def __init__(self, name):
        self.name = name
        self.succ = {}   # out port -> (node, in port)
        self.pred = {}   # in port  -> (node, out port)

    def forward(self, rt, port, msg):
        raise NotImplementedError(self.name)

    def backward(self, rt, port, msg):
        raise NotImplementedError(self.name)


class PPT(Node):
    """Parameterized payload transform: applies `fwd`, records the activation
    keyed on the message state, and on the backward message produces the input
    gradient and a new parameter gradient (Section 4)."""
    is_ppt = True

    def __init__(self, name, fwd, bwd, P, logkey=None):
        super().__init__(name)
        self.fwd, self.bwd, self.P = fwd, bwd, P
        self.logkey = logkey or (lambda s: (s[0], s[1] if len(s) > 1 else 0))
        self.stash = {}
        self.acc = None
        self.count = 0
        self.muf = 1
        self.mean = True
        self.opt = C.Optimizer()
        self.n_updates = 0
        self.staleness = []

    def forward(self, rt, port, msg):
        y, cache = self.fwd(self.P, msg.payload)
        assert msg.state not in self.stash, (self.name, msg.state)
        self.stash[msg.state] = (cache, self.n_updates)
        rt.log(self, "F", msg.state)
        if rt.probe is not None:
            rt.probe(self.name, "F", msg.state, y)
        rt.emit_fwd(self, 0, Msg(y, msg.state))

    def backward(self, rt, port, msg):
        cache, version = self.stash.pop(msg.state)
        self.staleness.append(self.n_updates - version)
        dx, g = self.bwd(self.P, cache, msg.payload)
        if self.acc is None:
            self.acc = {k: np.zeros_like(v) for k, v in self.P.items()}
        for k in g:
            if isinstance(g[k], C.RowGradient):
                g[k].add_to(self.acc[k])
            else:
                self.acc[k] += g[k]
        self.count += 1
        rt.log(self, "B", msg.state)
        if rt.probe is not None:
            rt.probe(self.name, "B", msg.state, dx)
        rt.emit_bwd(self, 0, Msg(dx, msg.state))
        if rt.auto_update and self.count >= self.muf:
            self.update(rt)

    def update(self, rt):
        if self.count < self.muf or self.count == 0:
            raise RuntimeError("update at %s with %d < min_update_frequency %d"
                               % (self.name, self.count, self.muf))
        scale = 1.0 / self.count if self.mean else 1.0
        self.opt.step(self.P, {k: v * scale for k, v in self.acc.items()})
        for v in self.acc.values():
            v[...] = 0.0
        self.count = 0
        self.n_updates += 1
        rt.log(self, "U", None)


class NPT(Node):
    """Non-parameterized payload transform with one input (ReLU, tanh, ...)."""

    def __init__(self, name, fwd, bwd):
        super().__init__(name)
        self.fwd, self.bwd = fwd, bwd
        self.stash = {}
        # A transform with a kink at zero (ReLU) takes a yes / no decision on every input element, and an input
        # within rounding of zero can fall either way in another precision or summation order.  With kink_tau set,
        # every decision on an input with |x| < kink_tau is listed in `kinks` as (state, element), and the ones
        # named in `flip` are recorded the other way round for the backward pass (the output, within kink_tau
        # of zero either way, is left as it is).  Parity tests use this to accept either decision.
        self.kink_tau = None
        self.kinks = []
        self.flip = set()

    def forward(self, rt, port, msg):
        y, cache = self.fwd(msg.payload)
        if self.kink_tau is not None:
            x = np.asarray(msg.payload)
            for i in np.flatnonzero(np.abs(x) < self.kink_tau):
                self.kinks.append((msg.state, int(i)))
                if (msg.state, int(i)) in self.flip:
                    cache = np.array(cache, copy=True)
                    cache[i] = self.kink_tau if x[i] <= 0 else -self.kink_tau
        self.stash[msg.state] = cache
        rt.emit_fwd(self, 0, Msg(y, msg.state))

    def backward(self, rt, port, msg):
        rt.emit_bwd(self, 0, Msg(self.bwd(self.stash.pop(msg.state), msg.payload), msg.state))


class Join(Node):
    """n-input transform: waits until one message per input port has arrived
    for a state, then applies fn; Concat is the case fn = concatenation."""

    def __init__(self, name, n_in, fn, vjp):
        super().__init__(name)
        self.n_in, self.fn, self.vjp = n_in, fn, vjp
        self.pend, self.stash = {}, {}

    def forward(self, rt, port, msg):
        slot = self.pend.setdefault(msg.state, {})
        assert port not in slot
        slot[port] = msg.payload
        if len(slot) == self.n_in:
            del self.pend[msg.state]
            y, cache = self.fn(*[slot[i] for i in range(self.n_in)])
            self.stash[msg.state] = cache
            rt.emit_fwd(self, 0, Msg(y, msg.state))

    def backward(self, rt, port, msg):
        grads = self.vjp(self.stash.pop(msg.state), msg.payload)
        for i in range(self.n_in):
            rt.emit_bwd(self, i, Msg(grads[i], msg.state))


def concat_join(name, n_in=2):
    def fn(*xs):
        return np.concatenate(xs, axis=-1), [x.shape[-1] for x in xs]

    def vjp(sizes, dy):
        return np.split(dy, np.cumsum(sizes)[:-1], axis=-1)
    return Join(name, n_in, fn, vjp)


class KeyedConcat(Node):
    """Concat whose parts arrive on one edge and are told apart by their
    state: key_fn gives the state of the joined message, part_fn the position
    of a part.  Keys on the new state to cache the original states, which are
    restored on the way back (Section 4, aggregation)."""

    def __init__(self, name, n_parts, key_fn, part_fn):
        super().__init__(name)
        self.n, self.key_fn, self.part_fn = n_parts, key_fn, part_fn
        self.pend, self.cache = {}, {}

    def forward(self, rt, port, msg):
        key = self.key_fn(msg.state)
        slot = self.pend.setdefault(key, {})
        slot[self.part_fn(msg.state)] = msg
        if len(slot) == self.n:
            del self.pend[key]
            parts = [slot[i] for i in range(self.n)]
            self.cache[key] = [(m.state, m.payload.shape[-1]) for m in parts]
            rt.emit_fwd(self, 0, Msg(np.concatenate([m.payload for m in parts], axis=-1), key))

    def backward(self, rt, port, msg):
        off = 0
        for state, size in self.cache.pop(msg.state):
            rt.emit_bwd(self, 0, Msg(msg.payload[..., off:off + size], state))
            off += size


class Loss(Node):
    """Loss layer: port 0 = prediction, port 1 = label pumped by the
    controller.  Emits the loss and starts backpropagation (Section 4)."""

    def __init__(self, name, kind):
        super().__init__(name)
        self.kind = kind
        self.pend = {}

    def forward(self, rt, port, msg):
        slot = self.pend.setdefault(msg.state, {})
        slot[port] = msg.payload
        if len(slot) < 2:
            return
        del self.pend[msg.state]
        if self.kind == "xent":
            loss, dz, pred = C.softmax_xent(slot[0], int(slot[1]))
            rt.record(msg.state[0], loss, int(pred == int(slot[1])), 1)
        else:
            loss, dz, _ = C.squared_error(slot[0], float(slot[1]))
            rt.record(msg.state[0], loss, 0, 1, yhat=float(np.ravel(slot[0])[0]))
        if rt.is_eval(msg.state[0]):
            rt.eval_scored(msg.state[0])    # an inference instance: scored, nothing turns round
            return
        rt.emit_bwd(self, 0, Msg(dz, msg.state))
        rt.emit_bwd(self, 1, Msg(None, msg.state))


class Cond(Node):
    """Routes on the state only; backward is a pass-through."""

    def __init__(self, name, f):
        super().__init__(name)
        self.f = f

    def forward(self, rt, port, msg):
        rt.emit_fwd(self, self.f(rt, msg.state), msg)

    def backward(self, rt, port, msg):
        rt.emit_bwd(self, 0, msg)


class Phi(Node):
    """Join of alternative paths: forwards what arrives and records the
    origin so that the gradient returns to it."""

    def __init__(self, name):
        super().__init__(name)
        self.origin = {}

    def forward(self, rt, port, msg):
        assert msg.state not in self.origin
        self.origin[msg.state] = port
        rt.emit_fwd(self, 0, msg)

    def backward(self, rt, port, msg):
        rt.emit_bwd(self, self.origin.pop(msg.state), msg)


class Isu(Node):
    """Invertible state update: f forward, f^-1 backward."""

    def __init__(self, name, f, finv):
        super().__init__(name)
        self.f, self.finv = f, finv

    def forward(self, rt, port, msg):
        rt.emit_fwd(self, 0, Msg(msg.payload, self.f(rt, msg.state)))

    def backward(self, rt, port, msg):
        rt.emit_bwd(self, 0, Msg(msg.payload, self.finv(rt, msg.state)))


class Bcast(Node):
    """Replicates a message to all successors; the gradients that come back
    for a state are summed in port order."""

    def __init__(self, name, n_out):
        super().__init__(name)
        self.n_out = n_out
        self.pend = {}

    def forward(self, rt, port, msg):
        for k in range(self.n_out):
            rt.emit_fwd(self, k, Msg(msg.payload, msg.state))

    def backward(self, rt, port, msg):
        slot = self.pend.setdefault(msg.state, {})
        assert port not in slot
        slot[port] = msg.payload
        if len(slot) == self.n_out:
            del self.pend[msg.state]
            total = np.array(slot[0], dtype=np.float64, copy=True)
            for k in range(1, self.n_out):
                total = total + slot[k]
            rt.emit_bwd(self, 0, Msg(total, msg.state))


class Group(Node):
    """Gathers the messages whose states map to one key into a single message
    whose payload stacks theirs as rows (ordered by order_fn); caches the
    original states and restores them, with the gradient rows, on the way
    back."""

    def __init__(self, name, key_fn, expect_fn, order_fn):
        super().__init__(name)
        self.key_fn, self.expect_fn, self.order_fn = key_fn, expect_fn, order_fn
        self.pend, self.cache = {}, {}

    def forward(self, rt, port, msg):
        key = self.key_fn(rt, msg.state)
        buf = self.pend.setdefault(key, [])
        buf.append(msg)
        if len(buf) == self.expect_fn(rt, key):
            del self.pend[key]
            buf.sort(key=lambda m: self.order_fn(rt, m.state))
            self.cache[key] = [m.state for m in buf]
            rt.emit_fwd(self, 0, Msg(np.stack([m.payload for m in buf]), key))

    def backward(self, rt, port, msg):
        for i, state in enumerate(self.cache.pop(msg.state)):
            rt.emit_bwd(self, 0, Msg(msg.payload[i], state))


class Ungroup(Node):
    """One message with k rows -> k messages with states states_fn(state);
    the k gradients are stacked back in the same order."""

    def __init__(self, name, states_fn):
        super().__init__(name)
        self.states_fn = states_fn
        self.parent, self.pend = {}, {}

    def forward(self, rt, port, msg):
        states = self.states_fn(rt, msg.state)
        assert len(states) == len(msg.payload)
        self.pend[msg.state] = [None] * len(states)
        for i, st in enumerate(states):
            self.parent[st] = (msg.state, i)
        for i, st in enumerate(states):
            rt.emit_fwd(self, 0, Msg(msg.payload[i], st))

    def backward(self, rt, port, msg):
        pst, i = self.parent.pop(msg.state)
        rows = self.pend[pst]
        rows[i] = msg.payload
        if all(r is not None for r in rows):
            del self.pend[pst]
            rt.emit_bwd(self, 0, Msg(np.stack(rows), pst))


class Flatmap(Node):
    """One message in, a sequence out: the payload is replicated and the new
    states come from a state-generation function.  Keys on the outgoing states
    and caches the incoming state and the number of messages expected, so as
    to sum all gradients and restore the original state (Section 4)."""

    def __init__(self, name, gen_fn):
        super().__init__(name)
        self.gen_fn = gen_fn
        self.parent, self.pend = {}, {}

    def forward(self, rt, port, msg):
        states = self.gen_fn(rt, msg.state)
        if not states:
            if not rt.is_eval(msg.state[0]):
                rt.emit_bwd(self, 0, Msg(np.zeros_like(msg.payload), msg.state))
            return
        self.pend[msg.state] = [None] * len(states)
        for i, st in enumerate(states):
            self.parent[st] = (msg.state, i)
        for st in states:
            rt.emit_fwd(self, 0, Msg(msg.payload, st))

    def backward(self, rt, port, msg):
        pst, i = self.parent.pop(msg.state)
        parts = self.pend[pst]
        parts[i] = msg.payload
        if all(p is not None for p in parts):
            del self.pend[pst]
            total = np.array(parts[0], dtype=np.float64, copy=True)
            for p in parts[1:]:
                total = total + p
            rt.emit_bwd(self, 0, Msg(total, pst))


class Sink(Node):
    """End of a path that carries no loss: answers with a zero gradient."""

    def forward(self, rt, port, msg):
        if not rt.is_eval(msg.state[0]):
            rt.emit_bwd(self, 0, Msg(np.zeros_like(msg.payload), msg.state))


class Controller(Node):
    """Pumps instances and other data into the graph, receives the backward
    messages that answer them, and throttles asynchrony (Section 4)."""

    def __init__(self):
        super().__init__("controller")

    def backward(self, rt, port, msg):
        rt.source_answered(msg.state[0])


# ============================================================== the runtime
class Runtime:
    def __init__(self, model, dims, flat_params):
        self.model, self.dims = model, dims
        self.ctrl = Controller()
        self.nodes = [self.ctrl]
        self.ppt = []
        BUILDERS[model](self, dims, flat_params)
        self.auto_update = True
        self.instances = None
        self.open_fwd = set()
        self.queue_b, self.queue_f = deque(), deque()
        self.parked = None
        self.events = []            # (node name, kind, (seq, local)) in execution order
        self.active = 0
        self.max_active_seen = 0
        self.pending_sources = {}
        self.retired = []
        self.loss, self.correct, self.npred, self.yhat = {}, {}, {}, {}
        self.max_staleness, self.limit, self.updates_at = None, 1, {}
        self.probe = None           # optional callback(node name, "F" | "B", state, output payload) at every PPT event
        self.eval_seqs = set()      # admission numbers of forward-only (inference) instances
        self.seq_inst = {}          # admission number -> instance, where it is not instances[seq % len]
        self.eval_pending = {}      # predictions an inference instance in flight still waits for
        self.sync_every = None      # own schedule: a synchronisation of every replicated node's copies after this many retirements
        self.snapshots = {}         # (node name, round) -> its parameters when the round's request reached it

    # ---- graph construction helpers
    def add(self, node):
        self.nodes.append(node)
        if node.is_ppt:
            self.ppt.append(node)
        return node

    @staticmethod
    def connect(src, sport, dst, dport):
        assert sport not in src.succ, (src.name, sport)
        assert dport not in dst.pred, (dst.name, dport)
        src.succ[sport] = (dst, dport)
        dst.pred[dport] = (src, sport)

    def chain(self, *nodes):
        for a, b in zip(nodes[:-1], nodes[1:]):
            self.connect(a, 0, b, 0)

    # ---- configuration
    def set_muf(self, muf, node=None):
        """node: a node's name (its copies "<name>.r<k>" included), or None for every node."""
        for n in self.ppt:
            if node is None or n.name == node or n.name.startswith(node + ".r"):
                n.muf = int(muf)

    def set_optimizer(self, node=None, **kw):
        for n in self.ppt:
            if node is None or n.name == node or n.name.startswith(node + ".r"):
                n.opt = C.Optimizer(**kw)

    def params(self):
        return [C.pack_node(n.P) for n in self.ppt]

    # ---- asynchronous synchronisation of a replicated node's copies (Section 5, last sentence)
    def replica_group(self, node):
        """A node and its copies "<name>.r<k>", in copy order."""
        base = node.name.split(".r")[0]
        return [n for n in self.ppt if n.name.split(".r")[0] == base]

    def sync_snapshot(self, node, rnd):
        """The request of round `rnd` reaches `node`: it publishes its parameters as they stand and carries on."""
        self.snapshots[(node.name, rnd)] = {k: v.copy() for k, v in node.P.items()}
        self.events.append((node.name, "S", (rnd, 0)))

    def sync_ready(self, node, rnd):
        return all((n.name, rnd) in self.snapshots for n in self.replica_group(node))

    def sync_load(self, node, rnd):
        """Every copy has published: `node` moves to the mean of the published values (summed in copy order) and
        keeps what it has learned since it published its own."""
        group = self.replica_group(node)
        own = self.snapshots[(node.name, rnd)]
        for k in node.P:
            mean = sum(self.snapshots[(n.name, rnd)][k] for n in group) / float(len(group))
            node.P[k] = mean + (node.P[k] - own[k])
        self.events.append((node.name, "L", (rnd, 0)))

    # ---- message plumbing
    def inst(self, seq):
        if seq in self.seq_inst:
            return self.seq_inst[seq]
        return self.instances[seq % len(self.instances)]

    def is_eval(self, seq):
        return seq in self.eval_seqs

    def mark_eval(self, seq, inst):
        """Admission number `seq` will be an inference instance: `inst`, forward only."""
        self.eval_seqs.add(seq)
        self.seq_inst[seq] = inst

    def eval_scored(self, seq):
        self.eval_pending[seq] -= 1
        if self.eval_pending[seq] == 0:
            del self.eval_pending[seq]
            self.active -= 1
            self.retired.append(seq)
            self.events.append(("controller", "R", (seq, 0)))
            # what the nodes cached for the instance on its way forward is never asked for again
            for n in self.nodes:
                for attr in ("stash", "pend", "cache", "origin", "parent"):
                    d = getattr(n, attr, None)
                    if d:
                        for key in [k for k in d if isinstance(k, tuple) and k[0] == seq]:
                            del d[key]
            self.open_fwd = {t for t in self.open_fwd if t[2][0] != seq}
            self.pending_sources.pop(seq, None)

    def emit_fwd(self, node, port, msg):
        tag = (id(node), port, msg.state)
        assert tag not in self.open_fwd, ("duplicate forward", node.name, port, msg.state)
        self.open_fwd.add(tag)
        dst, dport = node.succ[port]
        self._enqueue("F", dst, dport, msg)

    def emit_bwd(self, node, port, msg):
        src, sport = node.pred[port]
        tag = (id(src), sport, msg.state)
        if tag not in self.open_fwd:
            raise RuntimeError("backward message with no matching forward: %s -> %s %r"
                               % (node.name, src.name, msg.state))
        self.open_fwd.discard(tag)
        self._enqueue("B", src, sport, msg)

    def _enqueue(self, kind, node, port, msg):
        if self.parked is not None and node.is_ppt:
            key = (node.name, kind, node.logkey(msg.state))
            assert key not in self.parked, key
            self.parked[key] = (port, msg)
        elif kind == "B":
            self.queue_b.append((kind, node, port, msg))
        else:
            self.queue_f.append((kind, node, port, msg))

    def _dispatch(self, item):
        kind, node, port, msg = item
        if kind == "F":
            node.forward(self, port, msg)
        else:
            node.backward(self, port, msg)

    def _drain(self):
        while self.queue_b or self.queue_f:
            self._dispatch(self.queue_b.popleft() if self.queue_b else self.queue_f.popleft())

    def log(self, node, kind, state):
        self.events.append((node.name, kind, node.logkey(state) if state is not None else None))

    def record(self, seq, loss, correct, npred, yhat=None):
        self.loss[seq] = self.loss.get(seq, 0.0) + loss
        self.correct[seq] = self.correct.get(seq, 0) + correct
        self.npred[seq] = self.npred.get(seq, 0) + npred
        if yhat is not None:
            self.yhat[seq] = yhat

    # ---- controller
    def admit(self, seq):
        msgs = PUMPS[self.model](self, seq, self.inst(seq))
        self.pending_sources[seq] = len(msgs)
        if self.is_eval(seq):
            # one prediction per instance; one per tree node for the tree model
            self.eval_pending[seq] = 2 * self.inst(seq)["n_leaves"] - 1 if self.model == "tree" else 1
        self.active += 1
        self.max_active_seen = max(self.max_active_seen, self.active)
        self.events.append(("controller", "A", (seq, 0)))
        for port, msg in msgs:
            self.emit_fwd(self.ctrl, port, msg)

    def source_answered(self, seq):
        self.pending_sources[seq] -= 1
        if self.pending_sources[seq] == 0:
            del self.pending_sources[seq]
            self.active -= 1
            self.retired.append(seq)
            self.events.append(("controller", "R", (seq, 0)))
            if self.sync_every and self.parked is None and len(self.retired) % self.sync_every == 0:
                # the controller's request reaches every copy at once on this single-worker schedule: snapshot and
                # load follow each other directly, so the copies simply take their mean
                rnd = len(self.retired) // self.sync_every
                copies = [n for n in self.ppt if len(self.replica_group(n)) > 1]
                for n in copies:
                    self.sync_snapshot(n, rnd)
                for n in copies:
                    self.sync_load(n, rnd)
            if self.max_staleness is not None:
                # staleness-bounded admission: the limit on the instances in flight moves by one with every
                # retirement, up if the instance saw at most max_staleness updates per parameterized node
                # during its life, down otherwise
                seen = (sum(n.n_updates for n in self.ppt) - self.updates_at.pop(seq)) / float(len(self.ppt))
                if seen > self.max_staleness:
                    self.limit = max(1, self.limit - 1)
                else:
                    self.limit += 1

    # ---- driver 1: own schedule
    def run_mixed(self, train, evals, mak, epochs=1, first_seq=0):
        """Training and inference instances in one run (Section 1): `epochs` passes over `train`, and every
        instance of `evals` once, forward only, interleaved -- after every (training admissions // inference
        instances) training admissions the controller admits one inference instance.  Returns (losses of the
        training admissions, losses of the inference instances), each in its own admission order."""
        n_tr, n_ev = len(train) * epochs, len(evals)
        stride = max(1, n_tr // n_ev)
        order, it, ie = [], 0, 0
        while it < n_tr or ie < n_ev:
            for _ in range(stride):
                if it < n_tr:
                    order.append(("t", it))
                    it += 1
            if ie < n_ev:
                order.append(("e", ie))
                ie += 1
        for a, (kind, i) in enumerate(order):
            if kind == "e":
                self.mark_eval(first_seq + a, evals[i])
            else:
                self.seq_inst[first_seq + a] = train[i % len(train)]
        self.run(train, mak, first_seq=first_seq, n_admissions=len(order))
        tl = [self.loss[first_seq + a] for a, (kind, _) in enumerate(order) if kind == "t"]
        el = [self.loss[first_seq + a] for a, (kind, _) in enumerate(order) if kind == "e"]
        return tl, el

    def run(self, instances, mak, epochs=1, first_seq=0, max_staleness=None, n_admissions=None):
        """Train on `instances` in order, `epochs` times; returns the list of
        per-instance losses in admission order.  The controller is the greedy
        one (a new instance whenever fewer than mak are in flight) unless
        max_staleness is given: then the number in flight has a limit of its
        own in 1..mak, starting at 1 (Appendix B, MNIST, asks for a schedule
        that keeps gradients from going stale at a high max_active_keys)."""
        self.instances = instances
        self.parked = None
        self.auto_update = True
        self.max_staleness = max_staleness
        self.limit = 1
        self.updates_at = {}
        total = first_seq + (len(instances) * epochs if n_admissions is None else n_admissions)
        nxt = first_seq
        while True:
            while self.active < (mak if max_staleness is None else min(mak, self.limit)) and nxt < total:
                if max_staleness is not None:
                    self.updates_at[nxt] = sum(n.n_updates for n in self.ppt)
                self.admit(nxt)
                nxt += 1
            assert self.active <= mak
            if self.queue_b:
                self._dispatch(self.queue_b.popleft())
            elif self.queue_f:
                self._dispatch(self.queue_f.popleft())
            else:
                break
        self.check_quiescent()
        return [self.loss[s] for s in range(first_seq, total)]

    def check_quiescent(self):
        assert self.active == 0 and not self.pending_sources
        assert not self.open_fwd, "forward messages left unanswered: %d" % len(self.open_fwd)
        for n in self.nodes:
            for attr in ("stash", "pend", "cache", "origin", "parent"):
                assert not getattr(n, attr, None), (n.name, attr)

    # ---- driver 2: replay of a recorded order
    def replay(self, instances, worker_logs, first_seq=0):
        """worker_logs: one list per worker of (node name, kind, seq, local),
        kind in {"F", "B", "U"}, in the order that worker executed them.
        Cross-worker order follows from data dependencies."""
        self.instances = instances
        self.parked = {}
        self.auto_update = False
        by_name = {n.name: n for n in self.ppt}
        admitted = set()
        must_update = set()
        pos = [0] * len(worker_logs)
        progress = True
        while progress:
            progress = False
            for w, log in enumerate(worker_logs):
                while pos[w] < len(log):
                    name, kind, seq, local = log[pos[w]]
                    node = by_name[name]
                    if kind == "U":
                        node.update(self)
                        must_update.discard(name)
                    elif kind == "S":
                        self.sync_snapshot(node, seq)
                    elif kind == "L":
                        if (name, seq) not in self.snapshots:
                            raise RuntimeError("%s loads round %d without having published" % (name, seq))
                        if not self.sync_ready(node, seq):
                            break          # another copy's snapshot is still to come
                        self.sync_load(node, seq)
                    else:
                        if name in must_update:
                            raise RuntimeError("%s reached min_update_frequency but the log has no update" % name)
                        key = (name, kind, (seq, local))
                        if key not in self.parked and kind == "F" and seq not in admitted:
                            admitted.add(seq)
                            self.admit(seq)
                            self._drain()
                        if key not in self.parked:
                            break
                        port, msg = self.parked.pop(key)
                        self._dispatch((kind, node, port, msg))
                        self._drain()
                        if kind == "B" and node.count >= node.muf:
                            must_update.add(name)
                    pos[w] += 1
                    progress = True
        for w, log in enumerate(worker_logs):
            if pos[w] != len(log):
                raise RuntimeError("worker %d: event %r has no input (log position %d of %d)"
                                   % (w, log[pos[w]], pos[w], len(log)))
        if self.parked:
            raise RuntimeError("messages never consumed by the log: %r" % list(self.parked)[:4])
        if must_update:
            raise RuntimeError("missing updates at %r" % sorted(must_update))
        self.check_quiescent()
        return self

    def staleness(self):
        return {n.name: list(n.staleness) for n in self.ppt}


# ============================================================== model graphs
def _lin(rt, name, flat, rows, cols, logkey=None):
    return rt.add(PPT(name, C.linear_fwd, C.linear_bwd, C.unpack_node(flat, rows, cols, True), logkey))


def _lookup(rt, flat, rows, cols, logkey=None, name="lookup"):
    return rt.add(PPT(name, C.lookup_fwd, C.lookup_bwd, C.unpack_node(flat, rows, cols, False), logkey))


def build_mlp(rt, d, fp):
    """Controller -> Linear -> ReLU -> Linear -> ReLU -> Linear -> loss
    (Section 6, MLP paragraph)."""
    l1 = _lin(rt, "lin1", fp[0], d["hidden"], d["d_in"])
    l2 = _lin(rt, "lin2", fp[1], d["hidden"], d["hidden"])
    l3 = _lin(rt, "lin3", fp[2], d["n_class"], d["hidden"])
    r1 = rt.add(NPT("relu1", C.relu_fwd, C.relu_bwd))
    r2 = rt.add(NPT("relu2", C.relu_fwd, C.relu_bwd))
    loss = rt.add(Loss("loss", "xent"))
    rt.connect(rt.ctrl, 0, l1, 0)
    rt.chain(l1, r1, l2, r2, l3, loss)
    rt.connect(rt.ctrl, 1, loss, 1)


def pump_mlp(rt, seq, inst):
    return [(0, Msg(np.asarray(inst["x"], np.float64), (seq,))), (1, Msg(inst["label"], (seq,)))]


def build_rnn(rt, d, fp):
    """The variable-length RNN of Figure 2: lookup -> Concat(embedding, h) ->
    Linear-1 -> activation -> Isu(t+1) -> Cond(end?) -> back to Phi, or on to
    Linear-2 and the loss.  State = (instance, position); the length is read
    from the instance."""
    if d.get("node_replicas", 1) > 1:
        return build_rnn_replicated(rt, d, fp, d["node_replicas"])
    look = _lookup(rt, fp[0], d["vocab"], d["emb"])
    cell = _lin(rt, "cell", fp[1], d["hidden"], d["emb"] + d["hidden"])
    out = _lin(rt, "out", fp[2], d["n_class"], d["hidden"], logkey=lambda s: (s[0], 0))
    phi = rt.add(Phi("phi"))
    cat = rt.add(concat_join("concat"))
    act = rt.add(NPT("tanh", C.tanh_fwd, C.tanh_bwd))
    isu = rt.add(Isu("isu", lambda rt_, s: (s[0], s[1] + 1), lambda rt_, s: (s[0], s[1] - 1)))
    cond = rt.add(Cond("cond", lambda rt_, s: 1 if s[1] == len(rt_.inst(s[0])["tokens"]) else 0))
    loss = rt.add(Loss("loss", "xent"))
    rt.connect(rt.ctrl, 0, look, 0)
    rt.connect(rt.ctrl, 1, phi, 0)
    rt.connect(rt.ctrl, 2, loss, 1)
    rt.connect(look, 0, cat, 0)
    rt.connect(phi, 0, cat, 1)
    rt.chain(cat, cell, act, isu, cond)
    rt.connect(cond, 0, phi, 1)
    rt.connect(cond, 1, out, 0)
    rt.connect(out, 0, loss, 0)


def build_rnn_replicated(rt, d, fp, R):
    """The RNN with its heavy node replicated (Section 5): R copies of Linear-1
    between a Cond and a Phi, the rest of the loop shared.  Each copy comes
    with a copy of the embedding table in front of it (the two are hosted
    together), also between a Cond and a Phi.  Both Conds route on the
    instance: admission number mod R.  Parameterized nodes in the order
    lookup, cell, out, then (lookup.r<k>, cell.r<k>) for k = 1 .. R - 1; every
    copy starts from the same values."""
    looks, cells = [None] * R, [None] * R
    looks[0] = _lookup(rt, fp[0], d["vocab"], d["emb"])
    cells[0] = _lin(rt, "cell", fp[1], d["hidden"], d["emb"] + d["hidden"])
    out = _lin(rt, "out", fp[2], d["n_class"], d["hidden"], logkey=lambda s: (s[0], 0))
    for r in range(1, R):
        looks[r] = _lookup(rt, fp[0], d["vocab"], d["emb"], name="lookup.r%d" % r)
        cells[r] = _lin(rt, "cell.r%d" % r, fp[1], d["hidden"], d["emb"] + d["hidden"])
    route = lambda rt_, s: s[0] % R
    cond_t, phi_t = rt.add(Cond("cond_tok", route)), rt.add(Phi("phi_tok"))
    cond_c, phi_c = rt.add(Cond("cond_cell", route)), rt.add(Phi("phi_cell"))
    phi = rt.add(Phi("phi"))
    cat = rt.add(concat_join("concat"))
    act = rt.add(NPT("tanh", C.tanh_fwd, C.tanh_bwd))
    isu = rt.add(Isu("isu", lambda rt_, s: (s[0], s[1] + 1), lambda rt_, s: (s[0], s[1] - 1)))
    cond = rt.add(Cond("cond", lambda rt_, s: 1 if s[1] == len(rt_.inst(s[0])["tokens"]) else 0))
    loss = rt.add(Loss("loss", "xent"))
    rt.connect(rt.ctrl, 0, cond_t, 0)
    rt.connect(rt.ctrl, 1, phi, 0)
    rt.connect(rt.ctrl, 2, loss, 1)
    for r in range(R):
        rt.connect(cond_t, r, looks[r], 0)
        rt.connect(looks[r], 0, phi_t, r)
        rt.connect(cond_c, r, cells[r], 0)
        rt.connect(cells[r], 0, phi_c, r)
    rt.connect(phi_t, 0, cat, 0)
    rt.connect(phi, 0, cat, 1)
    rt.chain(cat, cond_c)
    rt.chain(phi_c, act, isu, cond)
    rt.connect(cond, 0, phi, 1)
    rt.connect(cond, 1, out, 0)
    rt.connect(out, 0, loss, 0)


def average_node_replicas(rt):
    """End-of-epoch synchronisation of a replicated node (Section 5): the
    parameters of a node and of its copies "<name>.r<k>" become their mean,
    summed in copy order.  Accumulators, counts and optimizer slots stay with
    their copy."""
    groups = {}
    for n in rt.ppt:
        groups.setdefault(n.name.split(".r")[0], []).append(n)
    for nodes in groups.values():
        if len(nodes) > 1:
            for name in nodes[0].P:
                mean = sum(n.P[name] for n in nodes) / float(len(nodes))
                for n in nodes:
                    n.P[name] = mean.copy()


def pump_rnn(rt, seq, inst):
    T = len(inst["tokens"])
    msgs = [(0, Msg(int(inst["tokens"][t]), (seq, t))) for t in range(T)]
    msgs.append((1, Msg(np.zeros(rt.dims["hidden"]), (seq, 0))))
    msgs.append((2, Msg(inst["label"], (seq, T))))
    return msgs


def _parent_tables(inst):
    if "_parent" not in inst:
        nn = 2 * inst["n_leaves"] - 1
        par = np.full(nn, -1, np.int64)
        side = np.zeros(nn, np.int64)
        for p in range(inst["n_leaves"], nn):
            par[inst["left"][p]], side[inst["left"][p]] = p, 0
            par[inst["right"][p]], side[inst["right"][p]] = p, 1
        inst["_parent"], inst["_side"] = par, side
    return inst["_parent"], inst["_side"]


def build_tree(rt, d, fp):
    """Binary Tree-LSTM with separate leaf and branch cells and a label at
    every node (Section 6, Tree-LSTM paragraph).  State = (instance, tree node).  A node's [h; c]
    is broadcast to the output layer and towards its parent, where the two
    children are concatenated, keyed on (instance, parent)."""
    H = d["hidden"]
    look = _lookup(rt, fp[0], d["vocab"], d["emb"])
    leaf = rt.add(PPT("leaf", C.leaf_fwd, C.leaf_bwd, C.unpack_node(fp[1], 3 * H, d["emb"], True)))
    branch = rt.add(PPT("branch", C.branch_fwd, C.branch_bwd, C.unpack_node(fp[2], 5 * H, 2 * H, True)))
    out = _lin(rt, "out", fp[3], d["n_class"], H)
    phi = rt.add(Phi("phi"))
    bc = rt.add(Bcast("bcast", 2))
    take_h = rt.add(NPT("take_h", lambda x: (x[:H].copy(), x.shape[0]),
                        lambda n, dy: np.concatenate([dy, np.zeros(n - H)])))
    loss = rt.add(Loss("loss", "xent"))
    cond = rt.add(Cond("is_root", lambda rt_, s: 0 if s[1] == 2 * rt_.inst(s[0])["n_leaves"] - 2 else 1))
    sink = rt.add(Sink("root_sink"))

    def up(rt_, s):
        par, side = _parent_tables(rt_.inst(s[0]))
        return (s[0], int(par[s[1]]), int(side[s[1]]))

    def down(rt_, s):
        inst = rt_.inst(s[0])
        return (s[0], int(inst["left"][s[1]] if s[2] == 0 else inst["right"][s[1]]))

    isu = rt.add(Isu("to_parent", up, down))
    cat = rt.add(KeyedConcat("children", 2, lambda s: (s[0], s[1]), lambda s: s[2]))
    rt.connect(rt.ctrl, 0, look, 0)
    rt.connect(rt.ctrl, 1, loss, 1)
    rt.connect(look, 0, leaf, 0)
    rt.connect(leaf, 0, phi, 0)
    rt.connect(branch, 0, phi, 1)
    rt.connect(phi, 0, bc, 0)
    rt.connect(bc, 0, take_h, 0)
    rt.chain(take_h, out, loss)
    rt.connect(bc, 1, cond, 0)
    rt.connect(cond, 0, sink, 0)
    rt.connect(cond, 1, isu, 0)
    rt.chain(isu, cat, branch)


def pump_tree(rt, seq, inst):
    L = inst["n_leaves"]
    msgs = [(0, Msg(int(inst["tokens"][n]), (seq, n))) for n in range(L)]
    msgs += [(1, Msg(int(inst["labels"][n]), (seq, n))) for n in range(2 * L - 1)]
    return msgs


def build_ggnn(rt, d, fp):
    """Gated graph network of Figure 4(a).  The lookup emits one matrix per
    instance (a row per graph node); it is broadcast, ungrouped into node
    messages, flat-mapped over each node's outgoing edges, grouped by edge
    type for one linear layer per type, ungrouped, regrouped by target node
    and summed, regrouped over all nodes and sent, with the previous hidden
    states, to the GRU cell; an outer loop (Phi / Isu / Cond) repeats this
    n_steps times before the regression layer.  The GRU is three linear nodes
    (update and reset gates side by side, then the candidate; Appendix C) and
    non-parameterized glue.  States: (instance, step) for matrices,
    (instance, step, 'v', node) for nodes, (instance, step, 'e', edge) for
    edges, (instance, step, 't', type) for per-type groups."""
    H, ne, S = d["hidden"], d["n_edge_types"], d["n_steps"]
    look = _lookup(rt, fp[0], d["n_node_types"], H, logkey=lambda s: (s[0], 0))
    phi_h = rt.add(Phi("phi_h"))
    bc_h = rt.add(Bcast("bcast_h", 4))
    ung_nodes = rt.add(Ungroup("ungroup_nodes", lambda rt_, s: [(s[0], s[1], "v", v)
                                                               for v in range(rt_.inst(s[0])["n_nodes"])]))

    def out_edges(rt_, s):
        g = rt_.inst(s[0])
        return [(s[0], s[1], "e", int(e)) for e in np.nonzero(g["src"] == s[3])[0]]

    fmap = rt.add(Flatmap("flatmap_edges", out_edges))
    by_type = rt.add(Cond("edge_type", lambda rt_, s: int(rt_.inst(s[0])["etype"][s[3]])))
    phi_e = rt.add(Phi("phi_e"))
    rt.connect(rt.ctrl, 0, look, 0)
    rt.connect(look, 0, phi_h, 0)
    rt.chain(phi_h, bc_h)
    rt.connect(bc_h, 0, ung_nodes, 0)
    rt.chain(ung_nodes, fmap, by_type)
    for c in range(ne):
        grp = rt.add(Group("group_type%d" % c,
                           lambda rt_, s, c=c: (s[0], s[1], "t", c),
                           lambda rt_, k, c=c: int((rt_.inst(k[0])["etype"] == c).sum()),
                           lambda rt_, s: s[3]))
        lin = _lin(rt, "edge%d" % c, fp[1 + c], H, H)
        ung = rt.add(Ungroup("ungroup_type%d" % c,
                             lambda rt_, s, c=c: [(s[0], s[1], "e", int(e))
                                                  for e in np.nonzero(rt_.inst(s[0])["etype"] == c)[0]]))
        rt.connect(by_type, c, grp, 0)
        rt.chain(grp, lin, ung)
        rt.connect(ung, 0, phi_e, c)
    by_dst = rt.add(Group("group_target",
                          lambda rt_, s: (s[0], s[1], "v", int(rt_.inst(s[0])["dst"][s[3]])),
                          lambda rt_, k: int((rt_.inst(k[0])["dst"] == k[3]).sum()),
                          lambda rt_, s: s[3]))
    rowsum = rt.add(NPT("sum_messages", lambda x: (x.sum(axis=0), x.shape[0]),
                        lambda k, dy: np.tile(dy, (k, 1))))
    allnodes = rt.add(Group("group_nodes",
                            lambda rt_, s: (s[0], s[1]),
                            lambda rt_, k: int(len(np.unique(rt_.inst(k[0])["dst"]))),
                            lambda rt_, s: s[3]))
    rt.chain(phi_e, by_dst, rowsum, allnodes)
    # GRU cell: z = sig(Wz [a; h]), r = sig(Wr [a; h]), h~ = tanh(Wh [a; r*h]), h' = (1 - z) h + z h~
    bc_a = rt.add(Bcast("bcast_a", 2))
    cat_ah = rt.add(concat_join("concat_ah"))
    bc_ah = rt.add(Bcast("bcast_ah", 2))
    gz = _lin(rt, "gz", fp[1 + ne], H, 2 * H)
    gr = _lin(rt, "gr", fp[2 + ne], H, 2 * H)
    gh = _lin(rt, "gh", fp[3 + ne], H, 2 * H)
    sz = rt.add(NPT("sig_z", C.sigmoid_fwd, C.sigmoid_bwd))
    sr = rt.add(NPT("sig_r", C.sigmoid_fwd, C.sigmoid_bwd))
    th = rt.add(NPT("tanh_h", C.tanh_fwd, C.tanh_bwd))
    mul = rt.add(Join("r_times_h", 2, lambda r, h: (r * h, (r, h)), lambda c, dy: [dy * c[1], dy * c[0]]))
    cat_arh = rt.add(concat_join("concat_arh"))
    blend = rt.add(Join("blend", 3, lambda z, h, ht: ((1 - z) * h + z * ht, (z, h, ht)),
                        lambda c, dy: [dy * (c[2] - c[1]), dy * (1 - c[0]), dy * c[0]]))
    rt.chain(allnodes, bc_a)
    rt.connect(bc_a, 0, cat_ah, 0)
    rt.connect(bc_a, 1, cat_arh, 0)
    rt.connect(bc_h, 1, cat_ah, 1)
    rt.connect(bc_h, 2, mul, 1)
    rt.connect(bc_h, 3, blend, 1)
    rt.chain(cat_ah, bc_ah)
    rt.connect(bc_ah, 0, gz, 0)
    rt.connect(bc_ah, 1, gr, 0)
    rt.chain(gz, sz)
    rt.connect(sz, 0, blend, 0)
    rt.chain(gr, sr)
    rt.connect(sr, 0, mul, 0)
    rt.connect(mul, 0, cat_arh, 1)
    rt.chain(cat_arh, gh, th)
    rt.connect(th, 0, blend, 2)
    isu = rt.add(Isu("next_step", lambda rt_, s: (s[0], s[1] + 1), lambda rt_, s: (s[0], s[1] - 1)))
    done = rt.add(Cond("steps_done", lambda rt_, s: 1 if s[1] == S else 0))
    pool = rt.add(NPT("sum_nodes", lambda x: (x.sum(axis=0), x.shape[0]), lambda k, dy: np.tile(dy, (k, 1))))
    ro = _lin(rt, "readout", fp[4 + ne], 1, H, logkey=lambda s: (s[0], 0))
    loss = rt.add(Loss("loss", "sqerr"))
    rt.chain(blend, isu, done)
    rt.connect(done, 0, phi_h, 1)
    rt.connect(done, 1, pool, 0)
    rt.chain(pool, ro, loss)
    rt.connect(rt.ctrl, 1, loss, 1)


def pump_ggnn(rt, seq, inst):
    return [(0, Msg(np.asarray(inst["node_type"], np.int64), (seq, 0))),
            (1, Msg(inst["target"], (seq, rt.dims["n_steps"])))]


BUILDERS = {"mlp": build_mlp, "rnn": build_rnn, "tree": build_tree, "ggnn": build_ggnn}
PUMPS = {"mlp": pump_mlp, "rnn": pump_rnn, "tree": pump_tree, "ggnn": pump_ggnn}


# ---------------------------------------------------------------------------
# replicas (Section 5, "Interaction with data parallelism and replicas")
# ---------------------------------------------------------------------------
def average_replicas(runtimes):
    """End-of-epoch replica synchronisation: the parameters of every replicated
    node become the mean over its replicas.  Accumulators, counts and
    optimizer slots stay with their replica."""
    for nodes in zip(*[rt.ppt for rt in runtimes]):
        for name in nodes[0].P:
            mean = sum(n.P[name] for n in nodes) / float(len(nodes))
            for n in nodes:
                n.P[name] = mean.copy()


def replica_subsets(instances, n_replicas):
    """The Cond in front of the replicas routes on the instance number:
    instance i (in submit order) goes to replica i mod n_replicas."""
    return [instances[r::n_replicas] for r in range(n_replicas)]


def run_replicas(runtimes, instances, mak, epochs=1):
    """Own-schedule training with every parameterized node replicated: the
    replicas train side by side on their share of the instances, each with
    `mak` instances in flight, and are averaged after every epoch.  Returns
    the per-instance losses in submit order, epoch by epoch."""
    R = len(runtimes)
    parts = replica_subsets(instances, R)
    done = [0] * R
    out = []
    for _ in range(epochs):
        per = []
        for r, rt in enumerate(runtimes):
            per.append(rt.run(parts[r], mak=mak, epochs=1, first_seq=done[r]))
            done[r] += len(parts[r])
        average_replicas(runtimes)
        out += [per[i % R][i // R] for i in range(len(instances))]
    return out
