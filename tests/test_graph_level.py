"""Graph-level placement (paper Sec. 4.3): the evolutionary search over digit strings.

The oracle's search is pinned by a generation worked by hand and by what must hold for any
fitness; the library's search must then equal the oracle's draw for draw."""
import itertools
import os

import numpy as np
import pytest

from oracle import evolve as oe

HERE = os.path.dirname(__file__)


def worked_example():
    out = {}
    for line in open(os.path.join(HERE, "golden", "evolve_worked_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        out[k] = v
    return out


def example_cost(b):
    return 10 - 3 * b[0] - 2 * b[2] + 4 * b[0] * b[2] + b[1]


EXAMPLE_OPTS = dict(population=2, generations=1, tournament=2, p_init=0.5, p_mutate=0.5, p_flip=0.5, p_cross=1.0)


def u32(fracs):
    return [int(float(f) * 4294967296.0) for f in fracs]


def random_cost_table(n, seed):
    """A cost per string with pairwise terms, so that it is not a sum over digits."""
    r = np.random.default_rng(seed)
    lin = r.uniform(-1, 1, n)
    pair = np.triu(r.uniform(-1, 1, (n, n)), 1)

    def cost(b):
        v = np.asarray(b, dtype=np.float64)
        return float(10 + lin @ v + v @ pair @ v)
    return cost


def draws(seed, count=20000):
    return np.random.default_rng(seed).integers(0, 2 ** 32, count, dtype=np.uint64).tolist()


# ---- the oracle against facts that do not come from it ---------------------------------------------
def test_oracle_reproduces_the_generation_worked_by_hand():
    ex = worked_example()
    best, cost, evals, hist = oe.evolve(4, example_cost, u32(ex["draws"]), **EXAMPLE_OPTS)
    assert best == [int(x) for x in ex["best"]]
    assert cost == float(ex["best_cost"][0])
    assert evals == int(ex["evaluations"][0])
    assert hist == [float(x) for x in ex["history"]]
    # the hand derivation also says this is the minimum over all strings
    assert cost == min(example_cost(b) for b in itertools.product((0, 1), repeat=4))


def test_oracle_uses_exactly_the_draws_of_the_worked_example():
    ex = worked_example()
    r = u32(ex["draws"])
    with pytest.raises(ValueError):
        oe.evolve(4, example_cost, r[:-1], **EXAMPLE_OPTS)
    oe.evolve(4, example_cost, r, **EXAMPLE_OPTS)


@pytest.mark.parametrize("seed", range(6))
def test_oracle_invariants_for_any_cost(seed):
    n = 7
    cost = random_cost_table(n, seed)
    seen = []

    def f(b):
        seen.append(tuple(b))
        return cost(b)
    best, c, evals, hist = oe.evolve(n, f, draws(seed), population=6, generations=12, tournament=3,
                                     p_init=0.3, p_mutate=0.6, p_flip=0.2, p_cross=0.7)
    assert len(seen) == len(set(seen)) == evals               # a string is measured once
    assert seen[0] == (0,) * n                                # the operator-level placement is a seed
    assert c == cost(best) == min(cost(b) for b in seen)      # best ever evaluated
    assert c <= cost([0] * n)                                 # never worse than the seed
    assert all(a >= b for a, b in zip(hist, hist[1:])) and hist[-1] == c and len(hist) == 13


def test_oracle_finds_the_exhaustive_minimum_on_small_strings():
    n = 6
    for seed in range(4):
        cost = random_cost_table(n, 100 + seed)
        _, c, evals, _ = oe.evolve(n, cost, draws(seed, 200000), population=16, generations=80, tournament=3,
                                   p_init=0.5, p_mutate=0.8, p_flip=0.25, p_cross=0.7)
        assert c == min(cost(b) for b in itertools.product((0, 1), repeat=n))
        assert evals <= 2 ** n


def test_oracle_second_seed_is_all_ones():
    # with seed_ones the strings measured first are all zeros, then all ones; the random members come after and
    # use (population - 2) * n draws; without mutation and crossover nothing else is ever measured
    n = 5
    seen = []

    def f(b):
        seen.append(tuple(b))
        return float(10 - sum(b))                              # all ones is the optimum
    d = draws(4, (4 - 2) * n + 3 * 4 * 3 + 3 * 4 + 3 * 2)      # initial strings + 3 generations of mutation / selection / crossover draws
    best, c, evals, hist = oe.evolve(n, f, d, population=4, generations=3, tournament=3, p_init=0.5, p_mutate=0.0, p_cross=0.0,
                                     seed_ones=True)
    assert seen[0] == (0,) * n and seen[1] == (1,) * n and len(seen) <= 4
    assert best == [1] * n and c == 5.0 and hist[0] == 5.0
    with pytest.raises(ValueError):                            # one draw fewer is one too few
        oe.evolve(n, f, d[:-1], population=4, generations=3, tournament=3, p_init=0.5, p_mutate=0.0, p_cross=0.0, seed_ones=True)


def test_oracle_without_mutation_and_crossover_only_selects():
    n = 8
    cost = random_cost_table(n, 5)
    seen = []

    def f(b):
        seen.append(tuple(b))
        return cost(b)
    _, c, evals, hist = oe.evolve(n, f, draws(3), population=8, generations=5, p_init=0.5, p_mutate=0.0, p_cross=0.0)
    assert evals == len(set(seen)) <= 8 and hist == [c] * 6


def test_oracle_crossover_keeps_every_position_s_digits():
    # p_mutate = 0: whatever crossover does, the multiset of digits at each position of the two
    # strings is unchanged, so with a population of 2 and both strings surviving selection
    # (tournament of 1 = a copy of a random member) position-wise sums never exceed the initial ones
    n = 10
    seen = []

    def f(b):
        seen.append(tuple(b))
        return float(sum(b))
    oe.evolve(n, f, draws(11), population=2, generations=20, tournament=1, p_init=0.5, p_mutate=0.0, p_cross=1.0)
    first = seen[1]                                           # the random member; the seed is all zeros
    for s in seen:
        assert all(x <= y for x, y in zip(s, first))          # a 1 can only come from the random member


def test_oracle_patience_stops_early():
    calls = []

    def f(b):
        calls.append(1)
        return 1.0                                            # nothing ever improves
    _, _, _, hist = oe.evolve(5, f, draws(1), population=4, generations=50, patience=3)
    assert len(hist) == 4


# ---- the library's search equals the oracle's, draw for draw --------------------------------------------
from paper_2111_00655_amd import binding as B  # noqa: E402


def test_library_reproduces_the_generation_worked_by_hand():
    ex = worked_example()
    best, cost, evals, hist = B.clg_evolve(4, B.make_es_opts(patience=0, **EXAMPLE_OPTS), u32(ex["draws"]), example_cost)
    assert best == [int(x) for x in ex["best"]] and cost == 7.0 and evals == 5 and hist == [8.0, 7.0]


@pytest.mark.parametrize("seed", range(8))
def test_library_equals_oracle(seed):
    r = np.random.default_rng(1000 + seed)
    n = int(r.integers(1, 40))
    opts = dict(population=int(r.integers(2, 12)), generations=int(r.integers(0, 15)), tournament=int(r.integers(1, 5)),
                patience=int(r.integers(0, 4)), p_init=float(r.uniform(0, 1)), p_mutate=float(r.uniform(0, 1)),
                p_flip=float(r.uniform(0, 0.5)), p_cross=float(r.uniform(0, 1)), seed_ones=bool(seed % 2))
    cost = random_cost_table(n, seed)
    rand = draws(seed, 40000)
    want = oe.evolve(n, cost, rand, **opts)
    got = B.clg_evolve(n, B.make_es_opts(**opts), rand, cost)
    assert got[0] == want[0] and got[1] == want[1] and got[2] == want[2] and got[3] == want[3]


def test_library_measures_a_string_once_and_in_the_oracle_s_order():
    n = 9
    cost = random_cost_table(n, 2)
    a, b = [], []
    opts = dict(population=6, generations=8, tournament=2, p_init=0.4, p_mutate=0.7, p_flip=0.3, p_cross=0.6)
    oe.evolve(n, lambda d: (a.append(tuple(d)), cost(d))[1], draws(9), **opts)
    B.clg_evolve(n, B.make_es_opts(**opts), draws(9), lambda d: (b.append(tuple(d)), cost(d))[1])
    assert a == b and len(set(b)) == len(b)


def test_library_search_errors():
    ok = B.make_es_opts(population=4, generations=3)
    with pytest.raises(B.ClgError, match="draws"):
        B.clg_evolve(8, ok, [1, 2, 3], lambda d: 1.0)
    with pytest.raises(B.ClgError, match="population"):
        B.clg_evolve(8, B.make_es_opts(population=1), draws(0), lambda d: 1.0)
    with pytest.raises(B.ClgError, match="probability"):
        B.clg_evolve(8, B.make_es_opts(p_flip=1.5), draws(0), lambda d: 1.0)
    with pytest.raises(B.ClgError, match="NaN"):
        B.clg_evolve(8, ok, draws(0), lambda d: float("nan"))
    with pytest.raises(ZeroDivisionError):
        B.clg_evolve(8, ok, draws(0), lambda d: 1 / 0)
    # draws that run dry in the middle of a generation: like the oracle, the library measures no string
    # that was built from missing draws
    for k in range(24, 80, 3):
        a, b = [], []
        with pytest.raises(ValueError, match="exhausted"):
            oe.evolve(8, lambda d: (a.append(tuple(d)), 1.0 + sum(d))[1], draws(3, k), population=4, generations=3)
        with pytest.raises(B.ClgError, match="draws"):
            B.clg_evolve(8, ok, draws(3, k), lambda d: (b.append(tuple(d)), 1.0 + sum(d))[1])
        assert a == b, k
    # no digits: the seed is the only string
    best, cost, evals, hist = B.clg_evolve(0, ok, draws(0), lambda d: 3.0)
    assert best == [] and cost == 3.0 and evals == 1 and hist == [3.0] * 4


# ---- the plan's digits (host-only: the schedule is computed without a device) ----------------------------
def test_handover_digits_on_a_plan():
    import workloads as wl
    import paper_2111_00655_amd as clg
    d = wl.resnet50(0, image=32, width=8, blocks=(2, 2), classes=10)
    s = clg.Session(d, wl.default_registry(("igemm_s8",)), device=None)
    ms = s.match()
    _, ids = s.search(wl.synthetic_costs(len(ms), 0), 0)
    plan = s.compile(ids)
    n = plan.n_kernels
    plan.set_handover([0] * n, lanes=3)
    assert plan.n_lanes == 1                                  # all zeros: the operator-level plan as it is
    plan.set_handover([1] * n, lanes=3)
    assert plan.n_lanes > 1                                   # the projection shortcut can leave the main path
    with pytest.raises(clg.ClgError, match="digits"):
        plan.set_handover([0] * (n - 1))
    with pytest.raises(clg.ClgError, match="digit"):
        plan.set_handover([2] + [0] * (n - 1))
    with pytest.raises(clg.ClgError, match="lanes"):
        plan.set_handover([0] * n, lanes=5)
    with pytest.raises(clg.ClgError) as e:                    # no device: nothing to time
        B.clg_plan_measure(plan.h, [256], [256, 256], 256, plan.ws_bytes)
    assert e.value.status == "HIP_ERROR"
    plan.set_lanes(3)                                         # the plain lane option hands every kernel over
    assert plan.n_lanes > 1
    plan.destroy()
    s.close()


# ---- regions: sibling kernels that may share a launch (host-only: found and planned without a device) ------
def _plan_on_register_fed_kernels(d):
    import workloads as wl
    import paper_2111_00655_amd as clg
    reg = wl.default_registry(("igemm_s8", "igemm_r16"), attention=True)
    s = clg.Session(d, reg, device=None)
    ms = s.match()
    costs = []
    for i, m in enumerate(ms):
        try:
            clg.clg_match_key(s.ctx, s.graph, i)
            costs.append((10 if reg[m.pattern][0] == "igemm_r16" else 1000) * m.n_nodes)
        except clg.ClgError:
            costs.append(B.COST_INF)                   # the backend cannot run this match
    _, ids = s.search(costs, 0)
    return s, ms, s.compile(ids)


def test_regions_of_an_attention_layer_and_of_residual_blocks():
    import workloads as wl
    # BERT: the query, key and value projections of a layer read the same activations and are one region
    d = wl.bert_base(0, layers=2, seq=32, hidden=128, heads=2, ffn=256, vocab=50, max_pos=32)
    s, ms, plan = _plan_on_register_fed_kernels(d)
    n = plan.n_kernels
    rg = plan.regions()
    assert len(rg) == n and max(rg) == 1                       # one region per layer
    for r in (0, 1):
        members = [i for i in range(n) if rg[i] == r]
        assert len(members) == 3 and members == list(range(members[0], members[0] + 3))      # adjacent in the plan
        names = {d.nodes[ms[plan.kernels()[i]["match"]].first]["name"].split(".")[1] for i in members}
        assert names == {"q", "k", "v"}
    base, ws = plan.n_launches, plan.ws_bytes
    assert base == n
    plan.set_handover([1] * n, lanes=1)
    assert plan.n_launches == n - 4 and plan.n_lanes == 1      # two launches saved per layer
    assert B.clg_plan_workspace_bytes(plan.h) == ws            # the workspace does not depend on the digits
    one = [0] * n
    one[[i for i in range(n) if rg[i] == 0][0]] = 1
    plan.set_handover(one, lanes=1)
    assert plan.n_launches == n                                # a lone handed-over member changes nothing
    two = list(one)
    two[[i for i in range(n) if rg[i] == 0][2]] = 1
    plan.set_handover(two, lanes=1)
    assert plan.n_launches == n - 1                            # the gain needs a sibling: not a sum over digits
    plan.set_handover([1] * n, lanes=2)
    assert plan.n_launches == n                                # the lane scheduler fuses nothing
    plan.set_lanes(1)
    assert plan.n_launches == n
    s.close()
    # ResNet: projection shortcut + first 1x1 convolution of each stage's first block
    d = wl.resnet50(0, image=64, width=16, blocks=(2, 1, 1), classes=10)
    s, ms, plan = _plan_on_register_fed_kernels(d)
    rg = plan.regions()
    assert max(rg) == 2
    for r in range(3):
        firsts = sorted(d.nodes[ms[plan.kernels()[i]["match"]].first]["name"] for i in range(plan.n_kernels) if rg[i] == r)
        assert firsts == [f"s{r}b0.c1.conv", f"s{r}b0.proj.conv"]
    s.close()


def test_region_members_never_depend_on_each_other():
    """Whatever the graph: a region's members are adjacent, and none reads a value produced at or after the
    region's first kernel (checked on the plan's own kernel list through the match list)."""
    import workloads as wl
    for d in (wl.nasnet_a(0, image=24, stem=4, filters=4, cells=1, classes=5),
              wl.resnet3d_50(0, frames=4, image=16, width=8, blocks=(1, 1), classes=5),
              wl.resnext50(0, image=32, width=8, blocks=(1, 1), groups=4, classes=10)):
        s, ms, plan = _plan_on_register_fed_kernels(d)
        ks, rg = plan.kernels(), plan.regions()
        produced = {}
        for i, k in enumerate(ks):
            produced[ms[k["match"]].sink] = i
        for r in set(rg) - {-1}:
            members = [i for i in range(len(ks)) if rg[i] == r]
            assert 2 <= len(members) <= 8 and members == list(range(members[0], members[-1] + 1))
            for i in members:
                m = ms[ks[i]["match"]]
                inside = set(m.nodes[:m.n_nodes])
                for v in m.nodes[:m.n_nodes]:
                    for u in d.nodes[v]["inputs"]:
                        if u not in inside and u in produced:
                            assert produced[u] < members[0], (d.name, r, i)
        s.close()


@pytest.mark.parametrize("seed", range(12))
def test_regions_on_random_graphs_compile_and_keep_their_invariants(seed):
    """Host-only twin of the GPU test on random graphs of sibling kernels: the plan compiles (every operand produced
    before its reader, after members were moved next to each other), members are adjacent and independent, launches
    drop by members - 1 per region under all ones, and the workspace does not depend on the digits."""
    from test_gpu_parity import _random_sibling_graph
    d = _random_sibling_graph(seed)
    s, ms, plan = _plan_on_register_fed_kernels(d)
    ks, rg = plan.kernels(), plan.regions()
    produced = {ms[k["match"]].sink: i for i, k in enumerate(ks)}
    saved = 0
    for r in set(rg) - {-1}:
        members = [i for i in range(len(ks)) if rg[i] == r]
        assert 2 <= len(members) <= 8 and members == list(range(members[0], members[-1] + 1))
        saved += len(members) - 1
        for i in members:
            m = ms[ks[i]["match"]]
            inside = set(m.nodes[:m.n_nodes])
            for v in m.nodes[:m.n_nodes]:
                for u in d.nodes[v]["inputs"]:
                    if u not in inside and u in produced:
                        assert produced[u] < members[0], (seed, r, i)
    ws = plan.ws_bytes
    plan.set_handover([1] * len(ks), lanes=1)
    assert plan.n_launches == len(ks) - saved and B.clg_plan_workspace_bytes(plan.h) == ws
    s.close()
