"""Helpers of the GPU parity tests: one fused group run alone as one kernel and
compared with the oracle by two metrics, and the cutting of one match out of a
whole-model graph.  No test lives here.

Metrics (fp32, per fused operator):
 * tensor-normalised: max|gpu - ref| / max|ref| <= 1e-4;
 * element-wise: |gpu - ref| <= 1e-4 * rms(ref) + 1e-4 * |ref| for every
   element (an absolute floor scaled to the tensor's typical magnitude, so
   that elements near zero are held to the accuracy of the sums they come
   from, plus the same relative bar).
"""
import numpy as np

import workloads as wl
import paper_2111_00655_amd as clg
from oracle.graph import Graph, norm_err

OP_TOL = 1e-4


def elementwise_ok(got, ref, tol=OP_TOL):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    bad = np.abs(got - ref) > tol * rms + tol * np.abs(ref)
    return not bool(bad.any()), int(bad.sum())


def check_outputs(got, ref, tol=OP_TOL, what=""):
    for a, b in zip(got, ref):
        assert a.shape == b.shape, (what, a.shape, b.shape)
        e = norm_err(a, b)
        assert e <= tol, (what, "normalised error", e)
        ok, n_bad = elementwise_ok(a, b, tol)
        assert ok, (what, "elements outside atol = tol * rms(ref)", n_bad)


def run_group(desc, backend, pattern, ref=None, tol=OP_TOL, what=""):
    """The operators of `desc` form exactly one match of `pattern`: run it as one kernel of
    `backend`.  Returns (kernel name, oracle outputs) so that the oracle's result can be reused
    for the same graph under another backend; None as the name when the backend refuses the match."""
    s = clg.Session(desc, [(backend, pattern)], device=0)
    ms = s.match()
    full = [i for i, m in enumerate(ms) if m.n_nodes == len(desc.op_nodes())]
    assert len(full) == 1, (what, [(m.pattern, m.n_nodes) for m in ms])
    if ref is None:
        ref = Graph(desc).run()
    try:
        plan = s.compile(full)
    except clg.ClgError as e:
        assert e.status == "NO_KERNEL", (what, str(e))
        s.close()
        return None, ref
    assert plan.n_kernels == 1
    got = plan.run()
    again = plan.run()
    name = plan.kernels()[0]["name"]
    s.close()
    assert all(np.array_equal(a, b) for a, b in zip(got, again)), (what, name, "not deterministic")
    check_outputs(got, ref, tol, (what, backend, name))
    return name, ref


def cut_out(desc, shape_of, nodes, seed):
    """A graph holding only the operators `nodes` (ascending ids) of `desc`.  Constants keep their values,
    graph inputs their feeds; a value produced by an operator outside the group becomes an input with
    seeded N(0, 1) contents of its shape (shape_of(node id) -> dims).  The group's last node is the output."""
    r = np.random.default_rng([seed, len(nodes), nodes[0]])
    d = wl.GraphDesc(f"{desc.name}_group_{nodes[0]}")
    new = {}
    for v in nodes:
        nd = desc.nodes[v]
        ins = []
        for u in nd["inputs"]:
            if u not in new:
                src = desc.nodes[u]
                if src["kind"] == "const":
                    new[u] = d.const(desc.tensors[u])
                elif src["kind"] == "input":
                    new[u] = d.input(desc.feeds[u])
                else:
                    new[u] = d.input(r.standard_normal(shape_of(u)).astype(np.float32))
            ins.append(new[u])
        new[v] = d.op(nd["kind"], ins, **nd["attrs"])
    d.mark_output(new[nodes[-1]])
    return d
