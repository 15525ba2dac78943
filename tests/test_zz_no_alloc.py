"""The entry point that allocates nothing (clg_execute_static): same kernels as
clg_execute, with the plan's intermediates and split-K partial sums in the
library's fixed device array.  Its outputs must equal clg_execute's bit for bit
(the same kernels on the same data), on two calls in a row, the second on a
smaller graph that reuses the front of the array the first one filled.
"""
import numpy as np
import pytest

import workloads as wl
import paper_2111_00655_amd as clg
from paper_2111_00655_amd import binding as B
from oracle.graph import Graph, norm_err

pytestmark = pytest.mark.gpu


def _f32(r, *shape, scale=1.0):
    return (r.standard_normal(shape) * scale).astype(np.float32)


def _split_k_graph():
    """Long reductions over few output pixels: the LDS-tiled kernels split K across workgroups and add
    the partial tiles from scratch memory in a second kernel."""
    r = np.random.default_rng([7, 1])
    d = wl.GraphDesc("split_k_chain")
    x = d.input(_f32(r, 1, 512, 7, 7))
    y = d.op("conv2d", [x, d.const(_f32(r, 64, 512, 1, 1, scale=512 ** -0.5))], stride=(1, 1), pad=(0, 0), groups=1)
    y = d.op("relu", [d.op("bias_add", [y, d.const(_f32(r, 64))], axis=1)])
    z = d.op("conv2d", [y, d.const(_f32(r, 96, 64, 3, 3, scale=576 ** -0.5))], stride=(1, 1), pad=(1, 1), groups=1)
    z = d.op("relu", [d.op("bias_add", [z, d.const(_f32(r, 96))], axis=1)])
    p = d.op("global_avg_pool2d", [z])
    o = d.op("dense", [p, d.const(_f32(r, 10, 96, scale=0.1))])
    d.mark_output(d.op("softmax", [d.op("bias_add", [o, d.const(_f32(r, 10))], axis=-1)]))
    d.mark_output(z)
    return d


def _plan(desc, variants):
    reg = wl.default_registry(variants)
    s = clg.Session(desc, reg, device=0)
    s.match()
    costs = s.profile(B.ProfileOpts(warmup=2, batches=2, min_batch_us=30, max_launches=30))
    _, ids = s.search(costs, 0)
    return s, s.compile(ids).bind()


def _both_ways(plan):
    import torch
    want = plan.run()                                   # clg_execute with a caller's workspace
    for t in plan._out:
        t.fill_(float("nan"))
    plan._ws.fill_(255)                                 # the caller's workspace plays no part below
    plan.execute_static()
    torch.cuda.synchronize()
    got = [t.cpu().numpy() for t in plan._out]
    return want, got


def test_static_workspace_gives_the_bits_of_clg_execute_on_two_calls_in_a_row():
    big_desc = _split_k_graph()
    s1, big = _plan(big_desc, ("igemm_s8",))
    assert any("_k" in k["name"] for k in big.kernels()), [k["name"] for k in big.kernels()]     # scratch partials in use
    small_desc = wl.tiny_cnn(0, image=8)
    s2, small = _plan(small_desc, ("igemm_s8", "igemm_r16"))
    assert 0 < small.ws_bytes < big.ws_bytes <= B.STATIC_WORKSPACE_BYTES
    for plan, desc in ((big, big_desc), (small, small_desc), (big, big_desc)):
        want, got = _both_ways(plan)
        assert all(np.array_equal(a, b) for a, b in zip(want, got))
        assert max(norm_err(a, b) for a, b in zip(got, Graph(desc).run())) <= 1e-3
    s1.close()
    s2.close()


def test_static_workspace_refuses_what_does_not_fit():
    r = np.random.default_rng(3)
    d = wl.GraphDesc("too_big")
    x = d.input(_f32(r, 1, 48, 512, 512))               # 48 MiB per intermediate
    d.mark_output(d.op("tanh", [d.op("relu", [x])]))
    s = clg.Session(d, wl.default_registry(), device=0)
    ms = s.match()
    single = {}
    for i, m in enumerate(ms):
        if m.n_nodes == 1:
            single.setdefault(m.sink, i)
    plan = s.compile(sorted(single.values())).bind()
    assert plan.ws_bytes > B.STATIC_WORKSPACE_BYTES
    with pytest.raises(clg.ClgError, match="static") as e:
        plan.execute_static()
    assert e.value.status == "WORKSPACE_TOO_SMALL"
    got = plan.run()                                    # the ordinary entry point still runs it
    assert norm_err(got[0], Graph(d).run()[0]) <= 1e-6
    s.close()
