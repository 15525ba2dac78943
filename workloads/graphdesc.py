"""Neutral description of a computation graph G (paper Sec. 4.1: a DAG whose
nodes are tensor operators with attributes).

A description is plain data.  Nodes are appended in topological order and the
node id is the insertion index.  `kind` is "input", "const" or one of
OP_KINDS.  Shapes are recorded only for inputs and constants; operator output
shapes are for the consumer (oracle or library) to infer.
"""
from __future__ import annotations

import numpy as np

# Primitive operator kinds, in the order of the C enum (value = index).
OP_KINDS = (
    "conv2d",             # (x[N,C,H,W], w[O,C/G,kh,kw]) stride, pad, groups
    "conv2d_transpose",   # (x[N,C,H,W], w[C,O,kh,kw])   stride, pad
    "dense",              # (x[M,K], w[U,K])             y = x w^T
    "batch_matmul",       # (a[B,M,K], b[B,N,K] | b[B,K,N]) transpose_b
    "bias_add",           # (x, b[C]) axis (1 = channel of NCHW, -1 = last)
    "add",                # (x, y) same shape
    "mul_scalar",         # (x) scalar
    "relu", "gelu", "tanh",
    "softmax",            # last axis
    "layer_norm",         # (x, gamma[L], beta[L]) eps, last axis
    "max_pool2d",         # (x) kernel, stride, pad
    "global_avg_pool2d",  # (x[N,C,H,W]) -> [N,C]
    "take",               # (table[V,H], ids[L] int32) -> [L,H]
    "reshape",            # (x) dims
    "transpose",          # (x) dims = permutation
    "avg_pool2d",         # (x) kernel, stride, pad; padding is not counted
    "concat",             # (x0, x1, ...) axis; 2 to 8 operands
    "conv3d",             # (x[N,C,D,H,W], w[O,C,kd,kh,kw]) stride, pad: 3 entries each (d, h, w)
    "max_pool3d",         # (x[N,C,D,H,W]) kernel, stride, pad: 3 entries each
    "global_avg_pool3d",  # (x[N,C,D,H,W]) -> [N,C]
)


class GraphDesc:
    def __init__(self, name: str):
        self.name = name
        self.nodes: list[dict] = []
        self.tensors: dict[int, np.ndarray] = {}   # const node -> value
        self.feeds: dict[int, np.ndarray] = {}     # input node -> value
        self.outputs: list[int] = []

    # ---- construction -------------------------------------------------
    def _push(self, node: dict) -> int:
        self.nodes.append(node)
        return len(self.nodes) - 1

    def input(self, value: np.ndarray, name: str = "") -> int:
        value = np.ascontiguousarray(value)
        assert value.dtype in (np.float32, np.int32)
        nid = self._push(dict(kind="input", inputs=[], attrs={},
                              shape=tuple(value.shape),
                              dtype=str(value.dtype), name=name))
        self.feeds[nid] = value
        return nid

    def const(self, value: np.ndarray, name: str = "") -> int:
        value = np.ascontiguousarray(value)
        assert value.dtype in (np.float32, np.int32)
        nid = self._push(dict(kind="const", inputs=[], attrs={},
                              shape=tuple(value.shape),
                              dtype=str(value.dtype), name=name))
        self.tensors[nid] = value
        return nid

    def op(self, kind: str, inputs, name: str = "", **attrs) -> int:
        assert kind in OP_KINDS, kind
        inputs = [int(i) for i in inputs]
        assert all(0 <= i < len(self.nodes) for i in inputs)
        return self._push(dict(kind=kind, inputs=inputs, attrs=dict(attrs),
                               name=name))

    def mark_output(self, nid: int) -> None:
        self.outputs.append(int(nid))

    # ---- inspection ---------------------------------------------------
    def op_nodes(self) -> list[int]:
        return [i for i, n in enumerate(self.nodes)
                if n["kind"] not in ("input", "const")]

    def __len__(self) -> int:
        return len(self.nodes)
