"""Pins of the oracle's graph execution, matcher and placement search (CPU).

What fixes them with no implementation to compare against:
 * every placement of a graph computes the same network output (a placement
   changes who runs a subgraph, not what it computes: paper Sec. 4.1);
 * the DP of Alg. 1 returns the plain optimum of Eq. 1, found independently by
   enumerating every placement, and on tiny graphs by trying every subset of
   the match list;
 * closed form on a chain: the classic segmentation recurrence;
 * C_opt(empty) = 0 (Eq. 3); adding patterns never worsens the optimum
   (Sec. 5.4 ablation); the sizes N, P, F, S stay inside the bounds of Sec. 4.2.
"""
import os

import numpy as np
import pytest

import workloads as wl
from workloads.patterns import P, W
from oracle.graph import Graph
from oracle.match import enumerate_matches
from oracle import search

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def pat_name(p):
    if p == W:
        return None
    inner = [pat_name(a) for a in p[1]]
    inner = [i for i in inner if i]
    return p[0] + ("(" + ",".join(inner) + ")" if inner else "")


# ------------------------------------------------------------------ matcher
def test_tiny_cnn_match_counts_hand_derived():
    g = Graph(wl.tiny_cnn(0, image=8))
    reg = wl.default_registry()
    ms = enumerate_matches(g, reg)
    got = {}
    for m in ms:
        key = (m.backend, pat_name(reg[m.pattern][1]))
        got[key] = got.get(key, 0) + 1
    want = {}
    for line in open(os.path.join(GOLD, "tiny_cnn_matches.txt")):
        if line.startswith("#") or not line.strip():
            continue
        be, name, cnt = line.split()
        want[(be, name)] = int(cnt)
    assert got == want
    assert len(ms) == 37


def test_match_legality_and_ids():
    d = wl.tiny_cnn(0, image=8)
    g = Graph(d)
    reg = wl.default_registry()
    ms = enumerate_matches(g, reg)
    keys = [(g.rank[m.first], m.pattern) for m in ms]
    assert keys == sorted(keys) and len(set(keys)) == len(keys)
    relu2 = [i for i, n in enumerate(d.nodes) if n["name"] == "l2.relu"][0]
    logits = d.outputs[0]
    for m in ms:
        assert m.first == min(m.nodes, key=lambda v: g.rank[v])
        for v in m.nodes:
            if v != m.sink:
                assert v not in (relu2, logits)            # two consumers / graph output
                assert all(c in m.nodes for c in g.consumers[v])
        kinds = [d.nodes[v]["kind"] for v in m.binding]
        assert kinds[-1] == reg[m.pattern][1][0]           # sink-rooted pattern text


def test_add_is_commutative_for_matching():
    # residual given as the FIRST operand of add: relu(add(bias(conv), *)) must still match
    d = wl.GraphDesc("swap")
    x = d.input(np.zeros((1, 2, 4, 4), np.float32))
    w = d.const(np.zeros((2, 2, 3, 3), np.float32))
    b = d.const(np.zeros(2, np.float32))
    c = d.op("conv2d", [x, w], stride=(1, 1), pad=(1, 1), groups=1)
    cb = d.op("bias_add", [c, b], axis=1)
    r0 = d.op("relu", [x])
    a = d.op("add", [r0, cb])
    r = d.op("relu", [a])
    d.mark_output(r)
    g = Graph(d)
    reg = [("k", P("relu", P("add", P("bias_add", P("conv2d", W, W), W), W)))]
    ms = enumerate_matches(g, reg)
    assert len(ms) == 1 and ms[0].nodes == (c, cb, a, r) and ms[0].first == c


def test_a_wildcard_never_binds_a_value_inside_the_match():
    # y = conv(x); a = add(bias(y), y): relu(add(bias_add(conv2d(*,*),*),*)) would need y both as the
    # conv inside the kernel and as an outside operand of the add; y has no consumer outside, so no
    # kernel ever writes it: the four-operator match is illegal, the shorter ones stay
    d = wl.GraphDesc("self_wild")
    x = d.input(np.zeros((1, 2, 4, 4), np.float32))
    w = d.const(np.zeros((2, 2, 3, 3), np.float32))
    b = d.const(np.zeros(2, np.float32))
    y = d.op("conv2d", [x, w], stride=(1, 1), pad=(1, 1), groups=1)
    yb = d.op("bias_add", [y, b], axis=1)
    a = d.op("add", [yb, y])
    r = d.op("relu", [a])
    d.mark_output(r)
    g = Graph(d)
    full = P("relu", P("add", P("bias_add", P("conv2d", W, W), W), W))
    assert enumerate_matches(g, [("k", full)]) == []
    ms = enumerate_matches(g, [("k", P("relu", P("add", W, W))), ("k", P("bias_add", W, W)), ("k", P("conv2d", W, W))])
    assert sorted(m.nodes for m in ms) == [(y,), (yb,), (a, r)]
    # with a second consumer outside the would-be match the single-exit rule already forbids it
    d.mark_output(d.op("tanh", [y]))
    assert enumerate_matches(Graph(d), [("k", full)]) == []


def test_both_branches_of_a_projection_block_match():
    # add(bias(convA), bias(convB)): one match per entry convolution
    d = wl.resnet50(0, image=32, width=8, blocks=(1,), classes=4)
    g = Graph(d)
    reg = [("k", P("relu", P("add", P("bias_add", P("conv2d", W, W), W), W)))]
    ms = enumerate_matches(g, reg)
    names = sorted(d.nodes[m.first]["name"] for m in ms)
    assert names == ["s0b0.c3.conv", "s0b0.proj.conv"]


def test_attr_constraints():
    d = wl.resnext50(0, image=32, width=8, blocks=(1, 1), groups=4, classes=4)
    g = Graph(d)
    n_conv = sum(1 for n in d.nodes if n["kind"] == "conv2d")
    n_grouped = sum(1 for n in d.nodes if n["kind"] == "conv2d" and n["attrs"]["groups"] > 1)
    assert n_grouped == 2
    ms = enumerate_matches(g, [("a", P("conv2d", W, W, groups=(1, 1))),
                               ("b", P("conv2d", W, W)),
                               ("c", P("conv2d", W, W, kernel_h=(3, 3), stride_h=(2, 2)))])
    cnt = [sum(1 for m in ms if m.pattern == i) for i in range(3)]
    assert cnt == [n_conv - n_grouped, n_conv, 1]


# ------------------------------------------------------- graph execution
def test_every_placement_gives_the_same_output_bitwise():
    d = wl.tiny_cnn(0, image=8)
    g = Graph(d)
    ms = enumerate_matches(g, wl.default_registry())
    ref = g.run()
    n = 0
    for ids in search.all_placements(g, ms):
        out = g.run_placement([ms[i].nodes for i in ids])
        assert all(np.array_equal(a, b) for a, b in zip(out, ref))
        n += 1
    assert n == 2048


def test_run_placement_rejects_invalid_placements():
    d = wl.tiny_cnn(0, image=8)
    g = Graph(d)
    singles = [[v] for v in g.op_ids]
    g.run_placement(singles)
    with pytest.raises(ValueError):
        g.run_placement(singles[:-1])                  # not a cover
    with pytest.raises(ValueError):
        g.run_placement(singles + [[g.op_ids[0]]])     # overlap
    # a group whose inner value is needed outside exposes only its sink
    relu2 = [i for i, n in enumerate(d.nodes) if n["name"] == "l2.relu"][0]
    conv3 = [i for i, n in enumerate(d.nodes) if n["name"] == "l3.conv"][0]
    bad = [[v] for v in g.op_ids if v not in (relu2, conv3)] + [[relu2, conv3]]
    with pytest.raises(ValueError):
        g.run_placement(bad)


def test_small_models_run_and_are_finite():
    for d in (wl.resnet50(0, image=32, width=8, blocks=(1, 1, 1, 1), classes=10),
              wl.resnext50(0, image=32, width=8, blocks=(1, 1), groups=4, classes=10),
              wl.bert_base(0, layers=1, seq=8, hidden=32, heads=4, ffn=64, vocab=50, max_pos=16),
              wl.dcgan(0, batch=2, latent=8, base=16)):
        out = Graph(d).run()
        assert all(np.all(np.isfinite(o)) for o in out)
    assert Graph(wl.dcgan(0, batch=2, latent=8, base=16)).run()[0].shape == (2, 3, 64, 64)


# ------------------------------------------------------------------ search
def _setup(desc, reg):
    g = Graph(desc)
    return g, enumerate_matches(g, reg)


@pytest.mark.parametrize("seed", range(12))
def test_dp_equals_exhaustive_on_tiny_cnn(seed):
    reg = wl.default_registry()
    g, ms = _setup(wl.tiny_cnn(0, image=8), reg)
    sizes = [len(m.nodes) for m in ms]
    costs = wl.synthetic_costs(len(ms), seed, sizes, ties=(seed % 3 == 0))
    for eps in (0, 700):
        best, count = search.exhaustive(g, ms, costs, eps)
        assert count == 2048
        assert search.dp(g, reg, ms, costs, eps) == best
        total, ids = best
        assert total == sum(int(costs[i]) + eps for i in ids)
        assert sorted(v for i in ids for v in ms[i].nodes) == g.op_ids


@pytest.mark.parametrize("seed", range(40))
def test_dp_equals_exhaustive_on_random_dags(seed):
    reg = wl.small_registry()
    g, ms = _setup(wl.random_dag(seed, n_ops=6 + seed % 8), reg)
    for cs in range(4):
        costs = wl.synthetic_costs(len(ms), 100 * seed + cs, [len(m.nodes) for m in ms],
                                   ties=(cs % 2 == 1))
        best, _ = search.exhaustive(g, ms, costs, 50)
        assert best is not None
        assert search.dp(g, reg, ms, costs, 50) == best


@pytest.mark.parametrize("seed", range(8))
def test_exhaustive_equals_subset_brute_force(seed):
    reg = wl.small_registry()
    g, ms = _setup(wl.random_dag(seed + 100, n_ops=5), reg)
    assert len(ms) <= 22
    for cs in range(3):
        costs = wl.synthetic_costs(len(ms), seed * 7 + cs, ties=(cs == 2))
        bf = search.brute_force_subsets(g, ms, costs, 10)
        assert search.exhaustive(g, ms, costs, 10)[0] == bf
        assert search.dp(g, reg, ms, costs, 10) == bf


def test_chain_closed_form_segment_dp():
    # chain of n relu ops; patterns = runs of 1, 2, 3 relus; cost depends on (start, len)
    n = 9
    d = wl.GraphDesc("chain")
    v = d.input(np.zeros((1, 4), np.float32))
    for _ in range(n):
        v = d.op("relu", [v])
    d.mark_output(v)
    reg = [("k", P("relu", W)), ("k", P("relu", P("relu", W))),
           ("k", P("relu", P("relu", P("relu", W))))]
    g, ms = _setup(d, reg)
    assert len(ms) == n + (n - 1) + (n - 2)
    for seed in range(6):
        costs = wl.synthetic_costs(len(ms), seed)
        eps = 40
        cost_of = {(g.rank[m.first], len(m.nodes)): int(costs[i]) for i, m in enumerate(ms)}
        f = [0] + [None] * n                      # f[i] = best cost of the first i ops
        for i in range(1, n + 1):
            f[i] = min(f[i - L] + cost_of[(i - L, L)] + eps for L in (1, 2, 3) if i - L >= 0)
        assert search.dp(g, reg, ms, costs, eps)[0] == f[n]


def test_empty_graph_costs_zero():
    d = wl.GraphDesc("empty")
    d.input(np.zeros((1,), np.float32))
    g = Graph(d)
    assert search.dp(g, [], [], [], 5) == (0, ())
    assert search.exhaustive(g, [], [], 5)[0] == (0, ())


def test_uncoverable_graph_has_no_placement():
    reg = [("k", P("conv2d", W, W))]
    g, ms = _setup(wl.tiny_cnn(0, image=8), reg)
    assert search.dp(g, reg, ms, np.ones(len(ms), np.int64), 0) is None
    assert search.exhaustive(g, ms, np.ones(len(ms), np.int64), 0)[0] is None


def test_expensive_fusions_leave_all_single_ops():
    reg = wl.default_registry()
    g, ms = _setup(wl.tiny_cnn(0, image=8), reg)
    costs = np.array([10 if len(m.nodes) == 1 else 10 ** 12 for m in ms], np.int64)
    total, ids = search.dp(g, reg, ms, costs, 0)
    assert all(len(ms[i].nodes) == 1 for i in ids) and len(ids) == len(g.op_ids)
    assert total == 10 * len(g.op_ids)
    # canonical tie-break: equal-cost single-op alternatives resolve to the lowest match id
    for i in ids:
        same = [j for j, m in enumerate(ms) if m.nodes == ms[i].nodes]
        assert i == min(same)


def test_large_eps_prefers_fewest_kernels():
    reg = wl.default_registry()
    g, ms = _setup(wl.tiny_cnn(0, image=8), reg)
    costs = np.full(len(ms), 5, np.int64)
    _, ids = search.dp(g, reg, ms, costs, 10 ** 6)
    fewest = min(len(p) for p in search.all_placements(g, ms))
    assert len(ids) == fewest == 6


def test_optimum_is_monotone_under_registry_growth():
    full = wl.default_registry()
    d = wl.tiny_cnn(0, image=8)
    g = Graph(d)
    ms_full = enumerate_matches(g, full)
    costs_full = wl.synthetic_costs(len(ms_full), 3, [len(m.nodes) for m in ms_full])
    by_key = {(m.pattern, m.first): int(costs_full[i]) for i, m in enumerate(ms_full)}
    prev = None
    # grow the registry: singles first, then everything; same cost for the same (pattern, node)
    single_idx = [i for i, (_, p) in enumerate(full) if wl.pattern_ops(p) == 1]
    for keep in (single_idx, list(range(len(full)))):
        reg = [full[i] for i in keep]
        ms = enumerate_matches(g, reg)
        costs = np.array([by_key[(keep[m.pattern], m.first)] for m in ms], np.int64)
        total = search.dp(g, reg, ms, costs, 100)[0]
        assert prev is None or total <= prev
        prev = total


def test_problem_sizes_stay_inside_the_papers_bounds():
    reg = wl.default_registry()
    for d in (wl.resnet50(0, image=32), wl.resnext50(0, image=32),
              wl.bert_base(0, seq=8, hidden=24, heads=12, ffn=48, vocab=64, max_pos=16),
              wl.dcgan(0, batch=1, latent=4, base=8)):
        g, ms = _setup(d, reg)
        st = {}
        costs = wl.synthetic_costs(len(ms), 0, [len(m.nodes) for m in ms])
        assert search.dp(g, reg, ms, costs, 100, st) is not None
        assert st["N"] < 1000 and st["P"] < 20 and st["F"] < 10 and st["S"] < 200


def test_interleaved_branches_need_non_prefix_states():
    # two branches off x, interleaved in the total order:
    #   a1=relu(x) b1=tanh(x) a2=relu(a1) b2=mul(b1) out=add(a2,b2)
    # relu(relu(*)) at a1 swallows a2, which lies AFTER b1 in the order, so the
    # stored sub-placement {a1,a2} is not a prefix of the order; the search
    # must still find the placement {a1,a2} {b1,b2} {out}.
    d = wl.GraphDesc("interleaved")
    x = d.input(np.zeros((1, 4), np.float32))
    a1 = d.op("relu", [x])
    b1 = d.op("tanh", [x])
    a2 = d.op("relu", [a1])
    b2 = d.op("mul_scalar", [b1], scalar=0.5)
    out = d.op("add", [a2, b2])
    d.mark_output(out)
    reg = [("k", P("relu", W)), ("k", P("tanh", W)), ("k", P("mul_scalar", W)), ("k", P("add", W, W)),
           ("k", P("relu", P("relu", W))), ("k", P("mul_scalar", P("tanh", W)))]
    g, ms = _setup(d, reg)
    costs = np.array([100 if len(m.nodes) == 1 else 1 for m in ms], np.int64)
    total, ids = search.dp(g, reg, ms, costs, 0)
    assert total == 102
    assert sorted(ms[i].nodes for i in ids) == [(a1, a2), (b1, b2), (out,)]
    assert (total, ids) == search.brute_force_subsets(g, ms, costs, 0)


def test_unusable_matches_are_no_candidates():
    """Costs of COST_INF or more mark matches no backend can run: the optimum is taken over the
    placements without them (DP == exhaustive == subset brute force), and when every cover needs
    one there is no placement at all."""
    d = wl.tiny_cnn(0, image=8)
    g = Graph(d)
    reg = wl.small_registry()
    ms = enumerate_matches(g, reg)
    r = np.random.default_rng(17)
    for trial in range(12):
        costs = r.integers(100, 2000, len(ms)).astype(object)
        dead = r.random(len(ms)) < 0.35
        for i in np.flatnonzero(dead):
            costs[i] = search.COST_INF + int(r.integers(0, 3))
        best, _ = search.exhaustive(g, ms, costs, 7)
        assert search.dp(g, reg, ms, costs, 7) == best
        if len(ms) <= 22:
            assert search.brute_force_subsets(g, ms, costs, 7) == best
        if best is not None:
            assert all(costs[i] < search.COST_INF for i in best[1]) and best[0] < search.COST_INF
    costs = [search.COST_INF] * len(ms)
    assert search.dp(g, reg, ms, costs, 0) is None and search.exhaustive(g, ms, costs, 0)[0] is None
    # one operator whose every match is dead: no cover, however cheap the rest
    costs = [10] * len(ms)
    victim = g.op_ids[3]
    for i, m in enumerate(ms):
        if victim in m.nodes:
            costs[i] = search.COST_INF
    assert search.dp(g, reg, ms, costs, 0) is None
