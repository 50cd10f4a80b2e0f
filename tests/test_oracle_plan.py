"""Pins for the CPU checker's planner (oracle/plan_oracle.py).

The planner is a heuristic, so it is pinned step by step: the paper's worked example
and closed forms, brute force on tiny inputs, hand-computed cases and invariants.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import plan_oracle as po
from paper_2603_28768_amd import synth


def _read_kv(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, val = line.split("=")
        out[key.strip()] = [int(v) for v in val.split()]
    return out


# ----------------------------------------------------------------- Alg. 3

def test_alg3_paper_worked_example(golden_dir):
    ex = _read_kv(os.path.join(golden_dir, "alg3_worked_example.txt"))
    D, L, E = ex["D"][0], ex["L"][0], ex["E"][0]
    x = ex["x"]
    assert sum(x) == ex["total_replicas"][0] == ex["R"][0] * D      # r = R * D
    assert L * D == ex["uniform_replicas"][0]                        # uniform minimum
    A = po.capacity_assignment(D, [E + xl for xl in x])
    for l in range(L):
        base = (E + x[l]) // D
        if (E + x[l]) % D == 0:
            assert A[l] == [base] * D
            extras = list(range(D)) if x[l] else []
        else:
            extras = [g for g in range(D) if A[l][g] == base + 1]
        assert extras == ex[f"extras_layer{l}"], (l, A[l])
    per_dev = [sum(A[l][g] for l in range(L)) - L * E // D for g in range(D)]
    assert per_dev == ex["replicas_per_device"]


def test_alg3_endpoint_spacing_would_contradict_the_example():
    # the helper's one-line description ("including endpoints") gives devices {0,3} for
    # four tied devices and two extras; the worked example says {0,2}
    K, q = [0, 1, 2, 3], 2
    endpoint = [K[round(i * (len(K) - 1) / (q - 1))] for i in range(q)]
    assert endpoint == [0, 3]
    assert po.interleave_select(K, q) == [0, 2]


@pytest.mark.parametrize("seed", range(6))
def test_alg3_invariants(seed):
    g = np.random.default_rng(seed)
    D = int(g.integers(2, 9))
    L = int(g.integers(1, 12))
    E = D * int(g.integers(1, 5))
    x = [int(v) for v in g.integers(0, 2 * D, size=L)]
    short = (-sum(x)) % D                       # make the total a multiple of D (r = R*D)
    x[0] += short
    A = po.capacity_assignment(D, [E + v for v in x])
    running = [0] * D
    for l in range(L):
        assert sum(A[l]) == E + x[l]
        assert max(A[l]) - min(A[l]) <= 1       # per-layer capacity difference <= 1
        running = [running[g] + A[l][g] for g in range(D)]
        assert max(running) - min(running) <= 1  # extras always go to the emptiest devices
    assert max(running) == min(running)          # equal memory on every device at the end


def test_closed_forms(golden_dir):
    for line in open(os.path.join(golden_dir, "closed_forms.txt")):
        if line.startswith("#") or not line.strip():
            continue
        L, D, R, saving = line.split()
        L, D, R, saving = int(L), int(D), int(R), float(saving)
        assert (L * D) / (R * D) == saving
    # and the planner reports them: uniform loads, budget R*D
    L, D, E, R = 6, 4, 8, 3
    W = [[[5] * E for _ in range(L)]]
    plan = po.make_plan(W, D, None, R * D)
    assert plan["total_replicas"] == R * D
    assert plan["replication_factor"] == R
    assert plan["memory_saving_vs_uniform"] == L / R
    import math
    assert int(math.log2(64)) + 1 == 7           # K candidate counts 1,2,4,...,64


# --------------------------------------------------------- copies per expert

@pytest.mark.parametrize("seed", range(8))
def test_expert_copies_minimise_the_largest_quotient(seed):
    g = np.random.default_rng(100 + seed)
    E = int(g.integers(2, 6))
    D = int(g.integers(2, 5))
    ws = [int(v) for v in g.integers(0, 50, size=E)]
    n = int(g.integers(0, min(6, E * (D - 1)) + 1))
    c = po.expert_copies(ws, n, D)
    assert sum(c) == E + n and all(1 <= v <= D for v in c)
    from fractions import Fraction
    best = None
    for cand in itertools.product(range(1, D + 1), repeat=E):
        if sum(cand) != E + n:
            continue
        m = max(Fraction(ws[e], cand[e]) for e in range(E))
        best = m if best is None or m < best else best
    assert max(Fraction(ws[e], c[e]) for e in range(E)) == best


def test_expert_copies_ties_and_cap():
    assert po.expert_copies([4, 4, 4], 2, 4) == [2, 2, 1]       # lowest id first on ties
    assert po.expert_copies([100, 1], 2, 2) == [2, 2]           # capped at D copies
    with pytest.raises(ValueError):
        po.expert_copies([1, 1], 3, 2)


# ----------------------------------------------------------------- placement

def test_placement_hand_computed():
    # E=4, D=2, loads 10,1,1,1, no replicas: capacities 2,2
    held, load = po.placement([10, 1, 1, 1], [1, 1, 1, 1], [2, 2])
    assert load == [11, 2] and held == [[(0, 0), (3, 0)], [(1, 0), (2, 0)]]
    assert po.est_max_rank_load([10, 1, 1, 1], 0, 2) == 11
    # one replica: copies 2,1,1,1 -> items 5,5,1,1,1; capacities 3,2
    held, load = po.placement([10, 1, 1, 1], [2, 1, 1, 1], [3, 2])
    assert load == [7, 6]
    assert held == [[(0, 0), (1, 0), (3, 0)], [(0, 1), (2, 0)]]
    assert po.est_max_rank_load([10, 1, 1, 1], 1, 2) == 7
    # floor split: 11 over 2 copies weighs 5 each (Alg. 1 floors the per-copy load)
    _, load = po.placement([11], [2], [1, 1])
    assert load == [5, 5]


@pytest.mark.parametrize("seed", range(10))
def test_placement_invariants_and_brute_force_bound(seed):
    g = np.random.default_rng(200 + seed)
    D = int(g.integers(2, 4))
    E = int(g.integers(D, 6))
    n = int(g.integers(0, 3))
    ws = [int(v) for v in g.integers(0, 40, size=E)]
    c = po.expert_copies(ws, n, D)
    cap = po.canonical_capacities(E + n, D)
    held, load = po.placement(ws, c, cap)
    assert [len(h) for h in held] == cap                        # every rank exactly full
    for g_ in range(D):
        assert load[g_] == sum(ws[e] // c[e] for e, _ in held[g_])
        es = [e for e, _ in held[g_]]
        assert len(es) == len(set(es))                          # copies on distinct ranks
    items = [(ws[e] // c[e], e) for e in range(E) for _ in range(c[e])]
    best = None
    for assign in itertools.product(range(D), repeat=len(items)):
        cnt = [assign.count(r) for r in range(D)]
        if cnt != cap:
            continue
        m = max(sum(items[i][0] for i in range(len(items)) if assign[i] == r) for r in range(D))
        best = m if best is None or m < best else best
    assert best <= max(load)                                    # greedy never beats optimum
    assert max(load) <= best + max(w for w, _ in items)         # and is within one item of it


def test_placement_constructed_optimal_cases():
    # one dominant expert: the optimum is the dominant expert's rank
    _, load = po.placement([100, 1, 1, 1, 1, 1], [1] * 6, [2, 2, 2])
    assert max(load) == 101
    # equal loads: perfectly balanced
    _, load = po.placement([7] * 8, [1] * 8, [2] * 4)
    assert load == [14] * 4


def test_placement_drops_distinctness_only_when_forced():
    # two copies of one expert, a single rank: must share it
    held, _ = po.placement([10], [2], [2])
    assert held == [[(0, 0), (0, 1)]]


def test_est_load_is_insensitive_to_which_ranks_hold_the_extra_capacity():
    g = np.random.default_rng(7)
    for _ in range(20):
        D, E, n = 4, 8, int(g.integers(1, 4))
        ws = [int(v) for v in g.integers(1, 100, size=E)]
        c = po.expert_copies(ws, n, D)
        cap = po.canonical_capacities(E + n, D)
        base = max(po.placement(ws, c, cap)[1])
        for perm in itertools.permutations(range(D)):
            assert max(po.placement(ws, c, [cap[i] for i in perm])[1]) == base


# ------------------------------------------------------- cross-layer allocation

def _gain_table(Ws, D, C):
    return {r: [po.est_max_rank_load(ws, 0, D) - po.est_max_rank_load(ws, r, D) for ws in Ws]
            for r in range(1, C + 1)}


@pytest.mark.parametrize("seed", range(6))
def test_mckp_dp_equals_exhaustive_enumeration(seed):
    g = np.random.default_rng(300 + seed)
    L, C = int(g.integers(1, 4)), int(g.integers(0, 5))
    keys = sorted(set(int(v) for v in g.integers(1, 5, size=3)))
    T = {r: [float(v) for v in g.integers(-3, 10, size=L)] for r in keys}
    best = None
    for x in itertools.product([0] + keys, repeat=L):
        if sum(x) != C:
            continue
        val = sum(T[r][l] for l, r in enumerate(x) if r)
        best = val if best is None or val > best else best
    if best is None:
        with pytest.raises(ValueError):
            po.mckp_allocation(T, C)
        return
    x = po.mckp_allocation(T, C)
    assert sum(x) == C and all(v == 0 or v in keys for v in x)
    assert sum(T[r][l] for l, r in enumerate(x) if r) == best


def _zipf_layer(E, s, total, seed):
    pop = synth.popularity(E, s, 99, seed)
    return [int(round(p * total)) for p in pop]


@pytest.mark.parametrize("seed", range(5))
def test_greedy_against_the_exact_dp(seed):
    g = np.random.default_rng(400 + seed)
    L, D, E, C = 3, 4, 8, int(g.integers(1, 6))
    Ws = [_zipf_layer(E, float(g.uniform(0.6, 1.6)), 4000, seed * 10 + l) for l in range(L)]
    x, order = po.greedy_allocation(Ws, D, None, C)
    assert sum(x) == C and len(order) == C
    T = _gain_table(Ws, D, C)
    xdp = po.mckp_allocation(T, C)
    gain = lambda xs: sum(T[r][l] for l, r in enumerate(xs) if r)
    assert gain(x) <= gain(xdp)                                  # DP is exact
    M = [[po.est_max_rank_load(ws, n, D) for n in range(C + 2)] for ws in Ws]
    convex = all(M[l][n] - M[l][n + 1] >= M[l][n + 1] - M[l][n + 2] >= 0
                 for l in range(L) for n in range(C))
    if convex:
        assert gain(x) == gain(xdp)                              # greedy optimal when convex


def test_greedy_on_a_convex_table_is_optimal():
    # loads built so that each layer's M(n) is convex: one hot expert of size h on D=2
    # ranks with unit-load cold experts. M(0)=h+1, M(1)=floor(h/2)+... check via DP equality
    Ws = [[40, 1, 1, 1], [24, 1, 1, 1], [8, 1, 1, 1]]
    D, C = 4, 3
    x, _ = po.greedy_allocation(Ws, D, None, C)
    T = _gain_table(Ws, D, C)
    xdp = po.mckp_allocation(T, C)
    gain = lambda xs: sum(T[r][l] for l, r in enumerate(xs) if r)
    assert gain(x) == gain(xdp)
    assert x[0] >= x[1] >= x[2]


def test_greedy_budget_in_bytes_and_prefix_property():
    Ws = [_zipf_layer(16, 1.4, 10000, 1), _zipf_layer(16, 0.8, 10000, 2), _zipf_layer(16, 1.1, 10000, 3)]
    by = [3, 2, 5]
    budget = 17
    x, order = po.greedy_allocation(Ws, 4, by, budget)
    spent = sum(xi * b for xi, b in zip(x, by))
    assert spent <= budget and order[-1][1] == spent
    assert all(spent + b > budget for b in by)                   # nothing more fits
    # unit bytes: the plan for budget b is a prefix of the plan for budget b+1
    prev = []
    for b in range(0, 9):
        _, order = po.greedy_allocation(Ws, 4, None, b)
        layers = [l for l, _ in order]
        assert layers[:len(prev)] == prev and len(layers) == b
        prev = layers


def test_skewed_layers_get_the_replicas():
    # Observation 4 / the workflow example: balanced layers get few, skewed layers many
    E, D = 32, 8
    Ws = [_zipf_layer(E, 0.6, 100000, 1), _zipf_layer(E, 1.6, 100000, 2),
          _zipf_layer(E, 0.6, 100000, 3), _zipf_layer(E, 1.6, 100000, 4)]
    x, order = po.greedy_allocation(Ws, D, None, 4)
    assert x == [0, 2, 0, 2]                                     # low-skew layers get none
    x8, order8 = po.greedy_allocation(Ws, D, None, 8)
    assert [l for l, _ in order8[:4]] == [l for l, _ in order]   # skewed layers are served first


# ------------------------------------------------------------------ whole plan

@pytest.mark.parametrize("seed", range(4))
def test_make_plan_structure(seed):
    g = np.random.default_rng(500 + seed)
    L, D = int(g.integers(1, 5)), int(g.integers(2, 5))
    E = D * int(g.integers(1, 4))
    B = 3
    W = g.integers(0, 200, size=(B, L, E)).tolist()
    budget = D * int(g.integers(0, 3))
    plan = po.make_plan(W, D, None, budget)
    assert sum(plan["x"]) == budget
    Ws = po.aggregate_load(W)
    assert Ws == np.asarray(W).sum(0).tolist()
    for l, lay in enumerate(plan["layers"]):
        S = E + lay["n_replicas"]
        assert len(lay["slot_expert"]) == S
        assert np.bincount(lay["slot_expert"], minlength=E).tolist() == lay["copies"]
        off = lay["rank_slot_off"]
        assert off[0] == 0 and off[-1] == S
        assert [off[g_ + 1] - off[g_] for g_ in range(D)] == lay["capacity"]
        for g_ in range(D):
            seg = lay["slot_expert"][off[g_]:off[g_ + 1]]
            assert seg == sorted(seg)
            assert lay["rank_load"][g_] == sum(Ws[l][e] // lay["copies"][e] for e in seg)
        assert 0 < lay["est_balancedness"] <= 1
        assert lay["est_max_rank_load"] == max(lay["rank_load"])


def test_balancedness_is_one_for_equal_loads_and_is_avg_over_max():
    plan = po.make_plan([[[3] * 8]], 4, None, 0)
    assert plan["layers"][0]["est_balancedness"] == 1.0
    plan = po.make_plan([[[10, 1, 1, 1]]], 2, None, 0)
    assert plan["layers"][0]["rank_load"] == [11, 2]
    assert plan["layers"][0]["est_balancedness"] == (13 / 2) / 11


def test_realized_rows_and_heaviest_rank():
    assert po.realized_rank_rows([3, 1, 4, 1, 5], [0, 2, 3, 5]) == [4, 4, 6]
    assert po.heaviest_rank([4, 6, 6]) == 1


# ------------------------------------------------- Alg. 1 replay, step 2, paper pipeline

def _read_alg1_cases(path):
    out = []
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, batches, base, scores = [f.strip() for f in line.split("|")]
        W = [[[int(v) for v in b.split()]] for b in batches.split(";")]
        out.append((name, W, float(Fraction(base)), [float(Fraction(v)) for v in scores.split()]))
    return out


def test_alg1_hand_worked_cases(golden_dir):
    for name, W, base, scores in _read_alg1_cases(os.path.join(golden_dir, "alg1_hand_cases.txt")):
        counts, b, T = po.replication_benefit(W, 4)
        assert counts == [1, 2, 4], name
        assert b == [base], name
        assert [T[r][0] for r in counts] == [s - base for s in scores], name


def test_alg1_base_is_per_layer():
    # the gain of a layer must not depend on which other layers are planned with it
    g = np.random.default_rng(77)
    W = g.integers(0, 300, size=(3, 4, 10)).tolist()
    counts, base, T = po.replication_benefit(W, 4)
    for l in range(4):
        Wl = [[W[b][l]] for b in range(3)]
        c1, b1, T1 = po.replication_benefit(Wl, 4)
        assert b1[0] == base[l]
        assert all(T1[r][0] == T[r][l] for r in counts)


def test_alg1_single_batch_base_is_the_placement_estimate():
    # with one batch the replay of r = 0 scores exactly the planner's own estimate
    g = np.random.default_rng(78)
    W = g.integers(0, 1000, size=(1, 3, 12)).tolist()
    _, base, _ = po.replication_benefit(W, 4)
    ref = po.make_plan(W, 4, None, 0)
    assert base == [lay["est_balancedness"] for lay in ref["layers"]]


def test_alg1_scores_lie_in_unit_interval_and_counts_follow_D():
    g = np.random.default_rng(79)
    for D in (1, 2, 3, 4, 8, 16):
        W = g.integers(0, 500, size=(2, 2, 16)).tolist()
        counts, base, T = po.replication_benefit(W, D)
        assert counts == [r for r in (1, 2, 4, 8, 16) if r <= D and D > 1]
        for l in range(2):
            assert 1.0 / D <= base[l] <= 1.0
            for r in counts:
                assert 1.0 / D - 1e-12 <= base[l] + T[r][l] <= 1.0 + 1e-12


@pytest.mark.parametrize("seed", range(6))
def test_step2_and_value_table_against_enumeration(seed):
    g = np.random.default_rng(500 + seed)
    L, D = int(g.integers(1, 4)), int(g.choice([2, 4]))
    keys = [r for r in (1, 2, 4) if r <= D]
    T = {r: [float(v) for v in g.integers(-2, 12, size=L)] for r in keys}
    R_max = L                                     # at most D replicas per layer
    # exhaustive: best value for every exact total
    best = {}
    for x in itertools.product([0] + keys, repeat=L):
        val = sum(T[r][l] for l, r in enumerate(x) if r)
        c = sum(x)
        best[c] = val if c not in best or val > best[c] else best[c]
    tab = po.mckp_table(T, R_max * D)
    for c in range(R_max * D + 1):
        assert tab[c] == best.get(c)
    want, want_v = 0, None
    for R in range(1, R_max + 1):
        if R * D in best:
            per = best[R * D] / (R * D)
            if want == 0 or per > want_v:
                want, want_v = R, per
    assert po.choose_replication_factor(T, D, R_max) == want


def test_paper_pipeline_totals_and_fallback():
    g = np.random.default_rng(80)
    W = g.integers(0, 400, size=(2, 3, 8)).tolist()
    D = 4
    reachable = {sum(x) for x in itertools.product((0, 1, 2, 4), repeat=3)}
    for budget in range(0, 14):
        p = po.make_plan_paper(W, D, budget)
        assert p["total_replicas"] == max(c for c in reachable if c <= budget)
        assert all(v in (0, 1, 2, 4) for v in p["x"])
        assert p["total_gain"] == sum(p["benefit"][r][l] for l, r in enumerate(p["x"]) if r)
        for l, lay in enumerate(p["layers"]):
            assert sum(lay["copies"]) == 8 + p["x"][l] == len(lay["slot_expert"])
    # one layer: totals 3 is not a candidate count -> falls back to 2
    W1 = [[[50, 30, 5, 5]]]
    assert po.make_plan_paper(W1, 4, 3)["x"] == [2]
    # automatic mode spends a multiple of D
    for budget in (4, 8, 12):
        p = po.make_plan_paper(W, D, budget, auto_R=True)
        assert p["total_replicas"] % D == 0 and 0 < p["total_replicas"] <= budget


def test_paper_pipeline_puts_replicas_on_the_skewed_layer():
    # Sec. 4.2.1's example: the skewed layer takes the replicas, the balanced one none
    skew = [400, 10, 10, 10, 10, 10, 10, 10]
    flat = [50, 50, 50, 50, 50, 50, 50, 50]
    p = po.make_plan_paper([[skew, flat]], 4, 4)
    assert p["x"] == [4, 0]


def test_uniform_comparison_plans():
    g = np.random.default_rng(81)
    W = g.integers(0, 400, size=(2, 3, 8)).tolist()
    base = po.make_plan_uniform(W, 4, 0)
    assert base["x"] == [0, 0, 0] and base["total_replicas"] == 0
    same = po.make_plan(W, 4, None, 0)
    assert [l["slot_expert"] for l in base["layers"]] == [l["slot_expert"] for l in same["layers"]]
    uni = po.make_plan_uniform(W, 4, 4)
    assert uni["total_replicas"] == 3 * 4 and uni["memory_saving_vs_uniform"] == 1.0
    for lay in uni["layers"]:
        assert all(lay["rank_slot_off"][g + 1] - lay["rank_slot_off"][g] == 3 for g in range(4))
        # replication can only lower the estimated maximum rank load
    for l in range(3):
        assert uni["layers"][l]["est_max_rank_load"] <= base["layers"][l]["est_max_rank_load"]
