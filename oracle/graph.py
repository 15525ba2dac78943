"""Oracle computation graph: evaluation of G, alone or under a placement.

TEST INFRASTRUCTURE ONLY (parity anchor; never imported by the product path).

Paper Sec. 4.1: G is a DAG of tensor operators; a placement P(G) is a set of
disjoint matched subgraphs (g_i, b_i) whose union is G.  A placement changes
who runs each subgraph, never what is computed, so executing G under any
placement is: run the groups in a topological order of the quotient graph,
each group being its primitive operators run in sequence.  Only a group's
sink value is visible outside the group.
"""
from __future__ import annotations

import heapq

import numpy as np

from . import ops


class Graph:
    def __init__(self, desc):
        self.desc = desc
        self.nodes = desc.nodes
        n = len(self.nodes)
        self.is_op = [nd["kind"] not in ("input", "const") for nd in self.nodes]
        self.consumers = [[] for _ in range(n)]
        for i, nd in enumerate(self.nodes):
            for j in nd["inputs"]:
                if j >= i:
                    raise ValueError("nodes must be in topological order")
                self.consumers[j].append(i)
        self.outputs = list(desc.outputs)
        # depth = longest operator path from a virtual root feeding every
        # graph input / constant (priority-queue key of Alg. 1)
        self.depth = [0] * n
        for i, nd in enumerate(self.nodes):
            if self.is_op[i]:
                self.depth[i] = 1 + max([self.depth[j] for j in nd["inputs"]
                                         if self.is_op[j]], default=0)
        self.op_ids = [i for i in range(n) if self.is_op[i]]
        self.order = sorted(self.op_ids, key=lambda i: (self.depth[i], i))
        self.rank = {v: r for r, v in enumerate(self.order)}

    # ---- one primitive operator ------------------------------------------
    def eval_op(self, nid, vals):
        nd = self.nodes[nid]
        a = nd["attrs"]
        x = [vals[j] for j in nd["inputs"]]
        k = nd["kind"]
        if k == "conv2d":
            return ops.conv2d(x[0], x[1], a["stride"], a["pad"], a.get("groups", 1))
        if k == "conv3d":
            return ops.conv3d(x[0], x[1], a["stride"], a["pad"])
        if k == "max_pool3d":
            return ops.max_pool3d(x[0], a["kernel"], a["stride"], a["pad"])
        if k == "global_avg_pool3d":
            return ops.global_avg_pool3d(x[0])
        if k == "conv2d_transpose":
            return ops.conv2d_transpose(x[0], x[1], a["stride"], a["pad"])
        if k == "dense":
            return ops.dense(x[0], x[1])
        if k == "batch_matmul":
            return ops.batch_matmul(x[0], x[1], a.get("transpose_b", True))
        if k == "bias_add":
            return ops.bias_add(x[0], x[1], a.get("axis", 1))
        if k == "add":
            return ops.add(x[0], x[1])
        if k == "mul_scalar":
            return ops.mul_scalar(x[0], a["scalar"])
        if k == "relu":
            return ops.relu(x[0])
        if k == "gelu":
            return ops.gelu(x[0])
        if k == "tanh":
            return ops.tanh(x[0])
        if k == "softmax":
            return ops.softmax(x[0])
        if k == "layer_norm":
            return ops.layer_norm(x[0], x[1], x[2], a.get("eps", 1e-12))
        if k == "max_pool2d":
            return ops.max_pool2d(x[0], a["kernel"], a["stride"], a["pad"])
        if k == "avg_pool2d":
            return ops.avg_pool2d(x[0], a["kernel"], a["stride"], a["pad"])
        if k == "concat":
            return ops.concat(x, a.get("axis", 1))
        if k == "global_avg_pool2d":
            return ops.global_avg_pool2d(x[0])
        if k == "take":
            return ops.take(x[0], x[1])
        if k == "reshape":
            return ops.reshape(x[0], a["dims"])
        if k == "transpose":
            return ops.transpose(x[0], a["dims"])
        raise ValueError(f"unknown op kind {k}")

    def _leaves(self, feeds):
        vals = {}
        for i, nd in enumerate(self.nodes):
            if nd["kind"] == "const":
                vals[i] = self.desc.tensors[i]
            elif nd["kind"] == "input":
                vals[i] = (feeds or self.desc.feeds)[i]
        return vals

    # ---- G with no placement: every operator in node order -------------------
    def run(self, feeds=None, keep_all=False):
        vals = self._leaves(feeds)
        for i in self.op_ids:
            vals[i] = self.eval_op(i, vals)
        if keep_all:
            return vals
        return [vals[o] for o in self.outputs]

    def run_timed(self, feeds=None):
        """As run(keep_all=True), also returning the wall-clock seconds every
        operator took: {node id: seconds}."""
        import time
        vals = self._leaves(feeds)
        secs = {}
        for i in self.op_ids:
            t0 = time.perf_counter()
            vals[i] = self.eval_op(i, vals)
            secs[i] = time.perf_counter() - t0
        return vals, secs

    # ---- G under a placement -----------------------------------------------
    def check_placement(self, groups):
        """groups: list of node-id lists.  Raises unless they are disjoint and
        cover every operator node (Sec. 4.1 definition of P(G))."""
        seen = {}
        for gi, g in enumerate(groups):
            for v in g:
                if not self.is_op[v]:
                    raise ValueError(f"node {v} is not an operator")
                if v in seen:
                    raise ValueError(f"overlap at node {v}")
                seen[v] = gi
        if len(seen) != len(self.op_ids):
            raise ValueError("not a cover")
        return seen

    def run_placement(self, groups, feeds=None):
        owner = self.check_placement(groups)
        ng = len(groups)
        sinks = []
        for g in groups:
            gs = set(g)
            # the sink: the one node of the group none of whose consumers is inside
            s = [v for v in g if not any(c in gs for c in self.consumers[v])]
            if len(s) != 1:
                raise ValueError("group without a unique sink")
            sinks.append(s[0])
        # quotient graph and Kahn's algorithm (ties: lower sink rank first)
        preds = [set() for _ in range(ng)]
        for gi, g in enumerate(groups):
            for v in g:
                for j in self.nodes[v]["inputs"]:
                    if self.is_op[j] and owner[j] != gi:
                        preds[gi].add(owner[j])
        succs = [set() for _ in range(ng)]
        for gi in range(ng):
            for p in preds[gi]:
                succs[p].add(gi)
        indeg = [len(p) for p in preds]
        heap = [(self.rank[sinks[gi]], gi) for gi in range(ng) if indeg[gi] == 0]
        heapq.heapify(heap)
        visible = self._leaves(feeds)
        done = 0
        while heap:
            _, gi = heapq.heappop(heap)
            local = {}
            for v in sorted(groups[gi]):
                env = {}
                for j in self.nodes[v]["inputs"]:
                    if j in local:
                        env[j] = local[j]
                    elif j in visible:
                        env[j] = visible[j]
                    else:
                        raise ValueError(
                            f"node {v} reads {j}, which no executed group exposes")
                local[v] = self.eval_op(v, env)
            visible[sinks[gi]] = local[sinks[gi]]
            done += 1
            for s in succs[gi]:
                indeg[s] -= 1
                if indeg[s] == 0:
                    heapq.heappush(heap, (self.rank[sinks[s]], s))
        if done != ng:
            raise ValueError("quotient graph has a cycle")
        return [visible[o] for o in self.outputs]


def norm_err(got, ref) -> float:
    """max |got - ref| / max |ref| over one tensor."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    den = float(np.max(np.abs(ref))) if ref.size else 0.0
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(got - ref))) / (den if den > 0 else 1.0)
