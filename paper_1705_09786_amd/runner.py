"""Convenience layer over the binding: device arena from PyTorch, one call to
set a model up from synthetic-workload containers.  Marshalling only."""
from __future__ import annotations

import numpy as np

from . import binding as B


def max_len_of(model: str, instances) -> tuple:
    if model == "mlp":
        return 1, 0
    if model == "rnn":
        return max(len(i["tokens"]) for i in instances), 0
    if model == "tree":
        return max(i["n_leaves"] for i in instances), 0
    return max(i["n_nodes"] for i in instances), max(len(i["src"]) for i in instances)


class Trainer:
    """Owns a torch uint8 tensor as device arena and an Amp context in it."""

    def __init__(self, model: str, dims: dict, params, max_active_keys: int, max_len: int, max_edges: int,
                 max_instances: int, arena_bytes: int = 1 << 30, tiles: dict | None = None, device: str = "cuda:0",
                 in_hbm=(), replicas: int = 1, strict: bool = False, graph=None, node_replicas: dict | None = None):
        """graph: a callable that describes the model with add_node / connect on the context it is given, in place
        of the canned builder for `model`.  node_replicas: {node: copies} of single heavy nodes (Section 5)."""
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the AMP path has no CPU fallback")
        self.torch = torch
        self.arena = torch.empty(arena_bytes + 256, dtype=torch.uint8, device=device)
        ptr = (self.arena.data_ptr() + 255) // 256 * 256
        stream = torch.cuda.current_stream(self.arena.device).cuda_stream
        self.amp = B.Amp(ptr, arena_bytes, stream, strict=strict)
        self.model, self.dims = model, dims
        if graph is not None:
            graph(self.amp)
            self.amp.validate_graph(model)
        else:
            self.amp.build(model, dims)
        for node, n in (tiles or {}).items():
            self.amp.set_tiles(node, n)
        if replicas != 1:
            self.amp.set_replicas(replicas)
        for node, n in (node_replicas or {}).items():
            self.amp.set_node_replicas(node, n)
        for node in in_hbm:
            self.amp.set_weights_in_hbm(node, True)
        self.amp.finalize(max_active_keys, max_len, max_edges, max_instances)
        for k, v in enumerate(params):
            self.amp.set_params(k, v)

    def submit_all(self, instances, which=0):
        for k, inst in enumerate(instances):
            self.amp.submit(inst, which=which, key=k)

    def params(self):
        return [self.amp.get_params(k) for k in range(self.amp.num_nodes())]

    def close(self):
        self.amp.close()
        self.arena = None
