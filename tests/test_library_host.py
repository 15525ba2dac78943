"""CPU-only tests of the C-ABI library: it loads, exports every symbol the
header declares, and its host logic (graph building, matching, search, plan
validation, cost-log files, error codes) agrees with the oracle.  No compute
call is made: contexts are host-only (device = -1).
"""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads as wl
from workloads.patterns import P, W
import paper_2111_00655_amd as clg
from paper_2111_00655_amd import binding as B
from oracle.graph import Graph
from oracle.match import enumerate_matches
from oracle import search

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "collage_mi.h")).read()
    declared = set(re.findall(r"\b(clg_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 30
    so = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(so, name), name
    assert declared == set(B.SYMBOLS), declared ^ set(B.SYMBOLS)
    assert clg.clg_version() == 102


def test_struct_layouts_match_the_header_sizes():
    # sizes implied by the header's field lists on LP64
    assert ctypes.sizeof(B.Attrs) == 4 * 10 + 8 * 6 + 16 + 4 * 4
    assert ctypes.sizeof(B.Match) == 4 * 5 + 4 * 16 * 2
    assert ctypes.sizeof(B.PatternNode) == 4 * (3 + 8) + 4 + 24 * 4        # op, n_args, args[8], n_constraints, pad
    assert ctypes.sizeof(B.KernelInfo) == 64 + 8 + 16


def _small_models():
    return [wl.tiny_cnn(0, image=8),
            wl.resnet50(0, image=32, width=8, blocks=(1, 2, 1, 1), classes=10),
            wl.resnext50(0, image=32, width=8, blocks=(1, 1), groups=4, classes=10),
            wl.bert_base(0, layers=2, seq=8, hidden=32, heads=4, ffn=64, vocab=50, max_pos=16),
            wl.dcgan(0, batch=2, latent=8, base=16),
            wl.nasnet_a(0, image=24, stem=4, filters=4, cells=1, classes=5),
            wl.resnet3d_50(0, frames=4, image=16, width=8, blocks=(1, 1), classes=5)]


def _same_matches(lib_ms, orc_ms):
    assert len(lib_ms) == len(orc_ms)
    for a, b in zip(lib_ms, orc_ms):
        assert (a.pattern, a.first, a.sink) == (b.pattern, b.first, b.sink)
        assert tuple(a.nodes[:a.n_nodes]) == b.nodes
        assert tuple(a.binding[:a.n_nodes]) == b.binding


@pytest.mark.parametrize("idx", range(7))
def test_matches_and_placements_bit_exact_vs_oracle(idx):
    d = _small_models()[idx]
    reg = wl.default_registry(("igemm", "igemm_s", "igemm_r16"))
    s = clg.Session(d, reg, device=None)
    g = Graph(d)
    oms = enumerate_matches(g, reg)
    _same_matches(s.match(), oms)
    sizes = [len(m.nodes) for m in oms]
    for seed in range(8):
        costs = wl.synthetic_costs(len(oms), seed, sizes, ties=(seed % 2 == 1))
        for eps in (0, 333):
            assert s.search(costs, eps) == search.dp(g, reg, oms, costs, eps)
    st = {}
    search.dp(g, reg, oms, costs, 0, st)
    assert clg.clg_search_stats(s.graph) == st
    s.close()


@pytest.mark.parametrize("seed", range(30))
def test_search_equals_exhaustive_on_random_dags(seed):
    # the abstract two-backend registry has no kernels: register it under real
    # family names, structure checks permitting, else compare on the subset
    d = wl.random_dag(seed, n_ops=6 + seed % 9)
    reg = []
    for be, p in wl.small_registry():
        reg.append(("igemm" if p[0] != "add" and _anchor(p) == "conv2d" else "eltwise", p))
    ctx = clg.clg_create(-1)
    ok = []
    for be, p in reg:
        try:
            clg.clg_register_pattern(ctx, clg.clg_register_backend(ctx, be), p)
            ok.append((be, p))
        except clg.ClgError as e:
            assert e.status == "NO_KERNEL"
    clg.clg_destroy(ctx)
    assert len(ok) >= 12
    s = clg.Session(d, ok, device=None)
    g = Graph(d)
    oms = enumerate_matches(g, ok)
    _same_matches(s.match(), oms)
    for cs in range(4):
        costs = wl.synthetic_costs(len(oms), 31 * seed + cs, ties=(cs % 2 == 1))
        best, _ = search.exhaustive(g, oms, costs, 20)
        assert s.search(costs, 20) == best
    s.close()


@pytest.mark.parametrize("seed", range(40))
def test_every_searched_or_enumerated_placement_compiles_on_random_dags(seed):
    """Search-then-compile contract (Sec. 4.1 / 4.2): whatever cover the search returns, and any other
    cover of the match list, must lower to a kernel sequence in which every operand has been produced."""
    d = wl.random_dag(seed, n_ops=6 + seed % 9)
    reg = []
    for be, p in wl.small_registry():
        reg.append(("igemm" if p[0] != "add" and _anchor(p) == "conv2d" else "eltwise", p))
    ctx = clg.clg_create(-1)
    ok = []
    for be, p in reg:
        try:
            clg.clg_register_pattern(ctx, clg.clg_register_backend(ctx, be), p)
            ok.append((be, p))
        except clg.ClgError as e:
            assert e.status == "NO_KERNEL"
    clg.clg_destroy(ctx)
    s = clg.Session(d, ok, device=None)
    g = Graph(d)
    oms = enumerate_matches(g, ok)
    _same_matches(s.match(), oms)
    for cs in range(6):
        costs = wl.synthetic_costs(len(oms), 77 * seed + cs, ties=(cs % 2 == 1))
        _, ids = s.search(costs, 0)
        plan = s.compile(ids)
        assert plan.n_kernels == len(ids)
        plan.destroy()
    covers = list(search.all_placements(g, oms))
    pick = np.random.default_rng(seed).permutation(len(covers))[:8]
    for pi in pick:
        s.compile(covers[pi]).destroy()
    s.close()


def _anchor(p):
    while True:
        subs = [a for a in p[1] if a != W]
        if not subs:
            return p[0]
        p = subs[0]


def test_infinite_costs_are_never_chosen_and_uncoverable_is_reported():
    d = wl.tiny_cnn(0, image=8)
    reg = wl.default_registry()
    s = clg.Session(d, reg, device=None)
    ms = s.match()
    costs = np.full(len(ms), 1000, np.int64)
    direct = [i for i, m in enumerate(ms) if reg[m.pattern][0] == "direct" and reg[m.pattern][1][0] != "global_avg_pool2d"]
    costs[direct] = B.COST_INF
    total, ids = s.search(costs, 0)
    assert not set(ids) & set(direct)
    g, oms = Graph(d), enumerate_matches(Graph(d), reg)
    assert (total, ids) == search.dp(g, reg, oms, costs, 0)
    costs[:] = B.COST_INF
    with pytest.raises(clg.ClgError) as e:
        s.search(costs, 0)
    assert e.value.status == "NOT_A_COVER"
    assert search.dp(g, reg, oms, costs, 0) is None            # the oracle agrees: no placement
    # random tables with dead entries: library and oracle agree on the optimum or on there being none
    r = np.random.default_rng(3)
    for trial in range(20):
        costs = r.integers(100, 5000, len(ms)).astype(np.int64)
        costs[r.random(len(ms)) < 0.4] = B.COST_INF
        want = search.dp(g, reg, oms, costs, 11)
        if want is None:
            with pytest.raises(clg.ClgError) as e:
                s.search(costs, 11)
            assert e.value.status == "NOT_A_COVER"
        else:
            assert s.search(costs, 11) == want
    costs = np.full(len(ms), 1000, np.int64)
    with pytest.raises(clg.ClgError) as e:
        s.search(-np.ones(len(ms), np.int64), 0)
    assert e.value.status == "INVALID_ARG"
    with pytest.raises(clg.ClgError) as e:
        s.search(np.ones(3, np.int64), 0)
    assert e.value.status == "INVALID_ARG"
    s.close()


def test_compile_validates_the_placement():
    d = wl.tiny_cnn(0, image=8)
    reg = wl.default_registry()
    s = clg.Session(d, reg, device=None)
    ms = s.match()
    costs = wl.synthetic_costs(len(ms), 0)
    _, ids = s.search(costs, 0)
    plan = s.compile(ids)
    assert plan.n_kernels == len(ids) and plan.ws_bytes > 0
    names = [k["name"] for k in plan.kernels()]
    assert len(names) == len(ids)
    plan.destroy()
    for bad, status in ((ids[:-1], "NOT_A_COVER"), (ids + (ids[0],), "OVERLAP"), (ids + (len(ms),), "UNKNOWN_ID")):
        with pytest.raises(clg.ClgError) as e:
            s.compile(bad)
        assert e.value.status == status
    # host-only context cannot execute
    plan = s.compile(ids)
    with pytest.raises(clg.ClgError) as e:
        B.clg_execute(plan.h, [1], [1, 1], 256, plan.ws_bytes)
    assert e.value.status == "HIP_ERROR"
    with pytest.raises(clg.ClgError) as e:
        B.clg_execute_static(plan.h, [1], [1, 1])
    assert e.value.status == "HIP_ERROR"
    with pytest.raises(clg.ClgError) as e:
        B.clg_profile_match(s.ctx, s.graph, 0)
    assert e.value.status == "HIP_ERROR"
    s.close()


def test_workspace_plan_never_overlaps_live_values():
    # replay the plan's schedule on the host: a value's buffer must not be
    # handed to another value before its last reader has run
    d = wl.resnet50(0, image=32, width=8, blocks=(2, 2), classes=10)
    reg = wl.default_registry()
    s = clg.Session(d, reg, device=None)
    ms = s.match()
    g = Graph(d)
    oms = enumerate_matches(g, reg)
    _, ids = s.search(wl.synthetic_costs(len(ms), 1, [len(m.nodes) for m in oms]), 0)
    plan = s.compile(ids)
    assert plan.ws_bytes % 256 == 0
    # peak must be at least the largest single intermediate and at most their sum
    inter = [4 * int(np.prod(B.clg_graph_node_shape(s.graph, ms[i].sink)[1])) for i in ids
             if ms[i].sink not in d.outputs]
    assert max(inter) <= plan.ws_bytes <= sum((b + 255) // 256 * 256 for b in inter) + 2 ** 20
    s.close()


def test_graph_building_errors():
    ctx = clg.clg_create(-1)
    g = clg.clg_graph_create(ctx)
    x = clg.clg_graph_input(g, B.F32, (1, 3, 8, 8))
    w = clg.clg_graph_const(g, B.F32, (4, 2, 3, 3), 0)
    with pytest.raises(clg.ClgError) as e:
        clg.clg_graph_op(g, "conv2d", [x, w], B.make_attrs(stride=(1, 1), pad=(1, 1), groups=1))
    assert e.value.status == "SHAPE_MISMATCH" and "conv2d" in str(e.value)
    with pytest.raises(clg.ClgError) as e:
        clg.clg_graph_op(g, "relu", [7])
    assert e.value.status == "UNKNOWN_ID"
    with pytest.raises(clg.ClgError) as e:
        clg.clg_graph_op(g, "relu", [x, x])
    assert e.value.status == "INVALID_ARG"
    with pytest.raises(clg.ClgError) as e:
        clg.clg_graph_mark_output(g, x)
    assert e.value.status == "INVALID_ARG"
    with pytest.raises(clg.ClgError) as e:
        clg.clg_graph_input(g, B.F32, (0, 3))
    assert e.value.status == "INVALID_ARG"
    # the size limit: 2^29 elements fit, one more row does not, and absurd extents do not wrap around
    big = clg.clg_graph_input(g, B.F32, (1 << 14, 1 << 15))
    assert clg.clg_graph_node_shape(g, big)[1] == (1 << 14, 1 << 15)
    for dims in ((1 << 14, (1 << 15) + 1), (1 << 62, 4), (1 << 40, 1 << 40, 1 << 40)):
        with pytest.raises(clg.ClgError) as e:
            clg.clg_graph_input(g, B.F32, dims)
        assert e.value.status == "INVALID_ARG"
    with pytest.raises(clg.ClgError) as e:
        clg.clg_graph_op(g, "concat", [big, big], B.make_attrs(axis=0))
    assert e.value.status == "SHAPE_MISMATCH"
    r = clg.clg_graph_op(g, "relu", [x])
    assert clg.clg_graph_node_shape(g, r) == (B.F32, (1, 3, 8, 8))
    t = clg.clg_graph_op(g, "transpose", [r], B.make_attrs(dims=(0, 2, 3, 1)))
    assert clg.clg_graph_node_shape(g, t)[1] == (1, 8, 8, 3)
    with pytest.raises(clg.ClgError):
        clg.clg_graph_op(g, "transpose", [r], B.make_attrs(dims=(0, 2, 2, 1)))
    with pytest.raises(clg.ClgError):
        clg.clg_graph_op(g, "reshape", [r], B.make_attrs(dims=(5, 5)))
    assert clg.clg_graph_num_nodes(g) == 5
    clg.clg_graph_destroy(g)
    clg.clg_destroy(ctx)


def test_output_shapes_agree_with_the_oracle_on_every_model():
    for d in _small_models():
        s = clg.Session(d, [], device=None)
        vals = Graph(d).run(keep_all=True)
        for nid, v in vals.items():
            assert B.clg_graph_node_shape(s.graph, nid)[1] == tuple(v.shape), d.nodes[nid]
        s.close()


def test_registration_errors():
    ctx = clg.clg_create(-1)
    with pytest.raises(clg.ClgError) as e:
        clg.clg_register_backend(ctx, "cudnn")
    assert e.value.status == "UNKNOWN_ID"
    ig = clg.clg_register_backend(ctx, "igemm")
    assert clg.clg_register_backend(ctx, "igemm") == ig
    rw = clg.clg_register_backend(ctx, "rowwise")
    for be, pat in ((ig, P("softmax", W)), (rw, P("relu", W)), (ig, P("add", P("relu", W), P("relu", W))),
                    (rw, P("relu", P("softmax", W))), (ig, P("relu", P("max_pool2d", W)))):
        with pytest.raises(clg.ClgError) as e:
            clg.clg_register_pattern(ctx, be, pat)
        assert e.value.status == "NO_KERNEL"
    with pytest.raises(clg.ClgError) as e:
        clg.clg_register_pattern(ctx, 9, P("relu", W))
    assert e.value.status == "UNKNOWN_ID"
    bad = B.flatten_pattern(P("relu", W))
    bad[1].args[0] = 1                      # argument refers to itself
    with pytest.raises(clg.ClgError) as e:
        clg.clg_register_pattern(ctx, ig, bad)
    assert e.value.status == "INVALID_ARG"
    assert clg.clg_num_patterns(ctx) == 0
    clg.clg_register_pattern(ctx, ig, P("relu", P("bias_add", P("conv2d", W, W, groups=(1, 1)), W)))
    assert clg.clg_num_patterns(ctx) == 1
    clg.clg_destroy(ctx)


def test_cost_log_round_trip(tmp_path):
    ctx = clg.clg_create(-1)
    p = tmp_path / "log.tsv"
    p.write_text("# comment\nigemm|conv2d+bias_add|s1x1|[1,3,8,8]\t1234\nrowwise|softmax|x\t77\n")
    clg.clg_cost_log_load(ctx, str(p))
    assert clg.clg_cost_log_size(ctx) == 2
    q = tmp_path / "out.tsv"
    clg.clg_cost_log_save(ctx, str(q))
    lines = [l for l in q.read_text().splitlines() if not l.startswith("#")]
    assert sorted(lines) == ["igemm|conv2d+bias_add|s1x1|[1,3,8,8]\t1234", "rowwise|softmax|x\t77"]
    with pytest.raises(clg.ClgError) as e:
        clg.clg_cost_log_load(ctx, str(tmp_path / "missing.tsv"))
    assert e.value.status == "IO_ERROR"
    (tmp_path / "bad.tsv").write_text("no tab here\n")
    with pytest.raises(clg.ClgError) as e:
        clg.clg_cost_log_load(ctx, str(tmp_path / "bad.tsv"))
    assert e.value.status == "IO_ERROR"
    clg.clg_destroy(ctx)


def test_match_keys_identify_shape_and_fused_kind():
    d = wl.resnet50(0, image=32, width=8, blocks=(2,), classes=10)
    reg = wl.default_registry()
    s = clg.Session(d, reg, device=None)
    ms = s.match()
    keys = {}
    for i, m in enumerate(ms):
        try:
            keys.setdefault(clg.clg_match_key(s.ctx, s.graph, i), []).append(i)
        except clg.ClgError as e:
            assert e.status == "NO_KERNEL"
    # two matches share a key only if backend, pattern and all shapes agree
    for k, ids in keys.items():
        pats = {ms[i].pattern for i in ids}
        assert len(pats) == 1
        assert k.split("|")[0] == reg[ms[ids[0]].pattern][0]
    assert any(len(v) > 1 for v in keys.values())      # repeated blocks share entries
    s.close()


def test_concat_of_kernel_results_is_planned_without_a_copy():
    """Host-only: the plan lists an aliasable concat as an entry that launches nothing and keeps one buffer for
    the result and its pieces; a concat with a graph input among its operands stays a copy."""
    r = np.random.default_rng(3)
    for with_input in (False, True):
        d = wl.GraphDesc("cat")
        x = d.input(r.standard_normal((1, 8, 4, 4)).astype(np.float32))
        parts = [d.op("relu", [x]), d.op("tanh", [x])] + ([x] if with_input else [d.op("gelu", [x])])
        d.mark_output(d.op("relu", [d.op("concat", parts, axis=1)]))
        s = clg.Session(d, wl.default_registry(), device=None)
        ms = s.match()
        _, ids = s.search([1000 * m.n_nodes for m in ms], 0)
        plan = s.compile(ids)
        names = [k["name"] for k in plan.kernels()]
        assert ("concat3" if with_input else "concat3_alias") in names, names
        assert plan.n_launches == plan.n_kernels - (0 if with_input else 1)
        ws = B.clg_plan_workspace_bytes(plan.h)
        # aliased: the three pieces live inside the result's 3 x 512 bytes; copied: two pieces + the result
        assert ws == (1536 if not with_input else 1024 + 1536), ws
        s.close()


def test_a_graph_with_plans_can_neither_go_nor_change():
    d = wl.tiny_cnn(0, image=8)
    s = clg.Session(d, wl.default_registry(), device=None)
    ms = s.match()
    _, ids = s.search(wl.synthetic_costs(len(ms), 0), 0)
    h1 = B.clg_compile(s.ctx, s.graph, list(ids))
    h2 = B.clg_compile(s.ctx, s.graph, list(ids))
    for call in (lambda: B.clg_graph_destroy(s.graph), lambda: B.clg_graph_op(s.graph, "relu", [d.outputs[0]]),
                 lambda: B.clg_graph_input(s.graph, B.F32, (1, 2)), lambda: B.clg_graph_mark_output(s.graph, ms[0].sink)):
        with pytest.raises(clg.ClgError, match="plan") as e:
            call()
        assert e.value.status == "INVALID_ARG"
    B.clg_plan_destroy(h1)
    with pytest.raises(clg.ClgError, match="1 compiled plan"):
        B.clg_graph_destroy(s.graph)
    with pytest.raises(clg.ClgError):                          # a failed compile leaves no claim on the graph
        B.clg_compile(s.ctx, s.graph, list(ids[:-1]))
    B.clg_plan_destroy(h2)
    n = B.clg_graph_num_nodes(s.graph)
    assert B.clg_graph_op(s.graph, "relu", [d.outputs[0]]) == n        # open again
    s.close()


def test_which_constants_a_plan_still_reads():
    d = wl.tiny_cnn(0, image=8)
    reg = wl.default_registry(("igemm_s8", "igemm_r16"))
    s = clg.Session(d, reg, device=None)
    ms = s.match()
    costs = []
    for i, m in enumerate(ms):
        try:
            clg.clg_match_key(s.ctx, s.graph, i)
            costs.append((10 if reg[m.pattern][0] == "igemm_r16" else 1000) * m.n_nodes)
        except clg.ClgError:
            costs.append(B.COST_INF)
    _, ids = s.search(costs, 0)
    plan = s.compile(ids)
    kinds = {}
    for nid, nd in enumerate(d.nodes):
        if nd["kind"] == "const":
            kinds[nid] = B.clg_plan_reads_constant(plan.h, nid)
    weights = [nid for nid in kinds if len(d.nodes[nid]["shape"]) >= 2]
    small = [nid for nid in kinds if len(d.nodes[nid]["shape"]) == 1]
    assert weights and small
    for nid in weights:                      # convolution / dense weights: the register-fed kernels read packed copies
        reads, packed = kinds[nid]
        assert not reads and packed >= 4 * int(np.prod(d.nodes[nid]["shape"])), (nid, kinds[nid])
    for nid in small:                        # biases are read in place
        assert kinds[nid] == (True, 0)
    assert set(plan.constants_not_read()) == set(weights)
    with pytest.raises(clg.ClgError) as e:
        B.clg_plan_reads_constant(plan.h, d.outputs[0])
    assert e.value.status == "UNKNOWN_ID"
    s.close()
