"""Marshals a graph description and a pattern registry into the C-ABI calls.

PyTorch is used here for device memory and the current HIP stream only; every
step of the path (matching, profiling, search, compilation, execution) runs in
libcollage_mi.so.  With device=None the session is host-only: no torch, no
device pointers; matching, search and plan validation still work.
"""
from __future__ import annotations

import numpy as np

from . import binding as B


class Session:
    def __init__(self, desc, registry, device=0, rules=()):
        """registry: (backend name, pattern) pairs, registered in order.  rules:
        (backend name, op_class dict, max_ops, grow_from_elemwise) tuples; the
        library's pattern generator adds their patterns for this graph after
        the listed ones (see full_registry())."""
        self.desc = desc
        self.registry = list(registry)
        self.device = device
        self.ctx = B.clg_create(-1 if device is None else device)
        self.graph = B.clg_graph_create(self.ctx)
        self._torch = None
        self._keep = []          # device tensors the graph borrows
        self.const_tensors = {}  # constant node -> its device tensor
        self.matches = None
        self._plans = []         # plans compiled from the graph: it cannot go before they do
        if device is not None:
            import torch
            self._torch = torch
            torch.cuda.set_device(device)
        # registry B, in order
        self.pattern_ids = []
        for backend, pat in self.registry:
            bid = B.clg_register_backend(self.ctx, backend)
            self.pattern_ids.append(B.clg_register_pattern(self.ctx, bid, pat))
        # graph G
        self.input_nodes = []
        for nid, nd in enumerate(desc.nodes):
            kind = nd["kind"]
            if kind == "input":
                dt = B.I32 if nd["dtype"] == "int32" else B.F32
                got = B.clg_graph_input(self.graph, dt, nd["shape"])
                self.input_nodes.append(nid)
            elif kind == "const":
                arr = desc.tensors[nid]
                dt = B.I32 if arr.dtype == np.int32 else B.F32
                ptr = 0
                if self._torch is not None:
                    t = self._torch.from_numpy(arr).to(f"cuda:{device}")
                    self._keep.append(t)
                    self.const_tensors[nid] = t
                    ptr = t.data_ptr()
                got = B.clg_graph_const(self.graph, dt, arr.shape, ptr)
            else:
                a = nd["attrs"]
                got = B.clg_graph_op(self.graph, kind, nd["inputs"], B.make_attrs(**a))
            assert got == nid
        for o in desc.outputs:
            B.clg_graph_mark_output(self.graph, o)
        self.out_shapes = [B.clg_graph_node_shape(self.graph, o)[1] for o in desc.outputs]
        self.generated = 0
        for backend, op_class, max_ops, grow in rules:
            bid = B.clg_register_backend(self.ctx, backend)
            self.generated += B.clg_generate_patterns(self.ctx, self.graph, bid, B.make_rule(op_class, max_ops, grow))
        self._backend_names = {}
        for backend in [b for b, _ in self.registry] + [r[0] for r in rules]:
            self._backend_names[B.clg_register_backend(self.ctx, backend)] = backend

    def full_registry(self):
        """The whole registry B in registration order, generated patterns included,
        as (backend name, pattern) pairs read back from the library."""
        out = []
        for pid in range(B.clg_num_patterns(self.ctx)):
            be, pat = B.clg_get_pattern(self.ctx, pid)
            out.append((self._backend_names[be], pat))
        return out

    # ---- steps of the path -----------------------------------------------------
    def match(self):
        self.matches = B.clg_match_all(self.ctx, self.graph)
        return self.matches

    def profile(self, opts=None):
        if self.matches is None:
            self.match()
        return B.clg_profile_all(self.ctx, self.graph, len(self.matches), opts)

    def search(self, costs, eps=0):
        return B.clg_search_dp(self.ctx, self.graph, costs, eps)

    def compile(self, match_ids):
        plan = Plan(self, B.clg_compile(self.ctx, self.graph, list(match_ids)))
        self._plans.append(plan)
        return plan

    def close(self):
        for plan in self._plans:
            plan.destroy()
        self._plans = []
        if self.graph is not None:
            B.clg_graph_destroy(self.graph)
            B.clg_destroy(self.ctx)
            self.graph = self.ctx = None
            self._keep = []


class Plan:
    def __init__(self, session, handle):
        self.s = session
        self.h = handle
        self.ws_bytes = B.clg_plan_workspace_bytes(handle)
        self.n_kernels = B.clg_plan_num_kernels(handle)
        self._ws = None
        self._in = None
        self._out = None

    def kernels(self):
        return [B.clg_plan_kernel_info(self.h, i) for i in range(self.n_kernels)]

    @property
    def n_launches(self):
        """Launches of one execution under the current digits: the kernel list without the concatenations
        planned as aliases, the handed-over members of a region counted once."""
        return B.clg_plan_num_launches(self.h)

    def constants_not_read(self):
        """{constant node: bytes of the plan's packed copies} for the constants whose device buffer no execution
        of this plan reads (the kernels read the packed copies)."""
        out = {}
        for nid, nd in enumerate(self.s.desc.nodes):
            if nd["kind"] == "const":
                reads, packed = B.clg_plan_reads_constant(self.h, nid)
                if not reads and packed:
                    out[nid] = packed
        return out

    def regions(self):
        """Region index of every kernel (-1: in none)."""
        return [B.clg_plan_region_of(self.h, i) for i in range(self.n_kernels)]

    def set_lanes(self, lanes):
        B.clg_plan_set_lanes(self.h, lanes)
        return self

    def set_handover(self, digits, lanes=2):
        B.clg_plan_set_handover(self.h, digits, lanes)
        return self

    def measure(self, warmup=5, batches=5, reps=20):
        """Nanoseconds of one execution of the whole sequence (smallest batch mean)."""
        return B.clg_plan_measure(self.h, *self._args(), warmup=warmup, batches=batches, reps=reps)

    def search_graph_level(self, opts, rand, lanes=2, warmup=3, batches=3, reps=20):
        """Sec. 4.3 on this plan: (best digits, best ns, seed ns, evaluations, history); leaves the plan set to best."""
        return B.clg_search_graph_level(self.h, *self._args(), lanes, opts, rand, warmup=warmup, batches=batches, reps=reps)

    @property
    def n_lanes(self):
        return B.clg_plan_num_lanes(self.h)

    def bind(self, feeds=None):
        """Allocates workspace, inputs and outputs on the device (torch)."""
        s = self.s
        torch = s._torch
        if torch is None:
            raise RuntimeError("host-only session cannot execute")
        dev = f"cuda:{s.device}"
        feeds = feeds or s.desc.feeds
        self._in = [torch.from_numpy(np.ascontiguousarray(feeds[n])).to(dev) for n in s.input_nodes]
        self._out = [torch.empty(shp, dtype=torch.float32, device=dev) for shp in s.out_shapes]
        self._ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=dev)
        assert self._ws.data_ptr() % 256 == 0
        return self

    def _args(self):
        if self._ws is None:
            self.bind()
        stream = self.s._torch.cuda.current_stream().cuda_stream
        return ([t.data_ptr() for t in self._in], [t.data_ptr() for t in self._out],
                self._ws.data_ptr(), self._ws.numel(), stream)

    def execute(self):
        """One asynchronous pass over the kernel sequence."""
        B.clg_execute(self.h, *self._args())

    def execute_static(self):
        """One asynchronous pass with the intermediates in the library's fixed device array."""
        ins, outs, _, _, stream = self._args()
        B.clg_execute_static(self.h, ins, outs, stream)

    def execute_timed(self):
        return B.clg_execute_timed(self.h, *self._args())

    def run(self, feeds=None):
        """Execute once and return the outputs as numpy arrays."""
        if feeds is not None or self._ws is None:
            self.bind(feeds)
        self.execute()
        self.s._torch.cuda.synchronize()
        return [t.cpu().numpy() for t in self._out]

    def destroy(self):
        if self.h is not None:
            B.clg_plan_destroy(self.h)
            self.h = None
