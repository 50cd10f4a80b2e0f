"""Host logic of the library: craft_plan and its accessors against the CPU checker's
independently written planner (bit-exact), plus argument checking.  No GPU needed."""
import ctypes

import numpy as np
import pytest

import oracle
from oracle import plan_oracle as po
from paper_2603_28768_amd import binding, synth


def _same(plan: binding.Plan, ref: dict):
    assert plan.greedy_order().tolist() == [l for l, _ in ref["order"]]
    s = plan.summary()
    assert s["total_replicas"] == ref["total_replicas"]
    assert s["replication_factor"] == ref["replication_factor"]
    assert s["memory_saving_vs_uniform"] == ref["memory_saving_vs_uniform"]
    for l, want in enumerate(ref["layers"]):
        got = plan.layer(l)
        assert got["n_replicas"] == want["n_replicas"]
        assert got["copies"].tolist() == want["copies"]
        assert got["slot_expert"].tolist() == want["slot_expert"]
        assert got["rank_slot_off"].tolist() == want["rank_slot_off"]
        assert got["rank_load"].tolist() == want["rank_load"]
        assert got["est_max_rank_load"] == want["est_max_rank_load"]
        assert got["est_balancedness"] == want["est_balancedness"]     # same double expression


@pytest.mark.parametrize("seed", range(12))
def test_plan_matches_checker_on_random_loads(seed):
    g = np.random.default_rng(seed)
    L, D = int(g.integers(1, 7)), int(g.integers(1, 9))
    E = int(g.integers(max(1, D // 2), 40))
    B = int(g.integers(1, 4))
    hi = int(g.choice([2, 50, 100000]))
    W = g.integers(0, hi, size=(B, L, E))
    budget = int(g.integers(0, 3 * D + 1))
    budget = min(budget, L * E * (D - 1))
    _same(binding.Plan(W, D, budget), po.make_plan(W.tolist(), D, None, budget))


@pytest.mark.parametrize("seed", range(4))
def test_plan_matches_checker_with_byte_costs(seed):
    g = np.random.default_rng(50 + seed)
    L, D, E = 4, 4, 12
    W = g.integers(0, 5000, size=(2, L, E))
    by = [int(v) for v in g.integers(1, 9, size=L)]
    budget = int(g.integers(5, 60))
    _same(binding.Plan(W, D, budget, by), po.make_plan(W.tolist(), D, by, budget))


@pytest.mark.parametrize("name", ["tiny", "qwen3", "dsv3"])
def test_plan_matches_checker_on_the_synthetic_configs(name):
    cfg = synth.CONFIGS[name]
    pop = synth.layer_popularity(cfg)
    W = np.zeros((cfg.profile_batches, 1, cfg.E), dtype=np.int64)
    for b in range(cfg.profile_batches):
        ids, _ = oracle.route(synth.router_logits(cfg, pop, "profile", b), cfg.k)
        W[b, 0] = oracle.expert_load(ids[None], cfg.E, cfg.T)[0, 0]
    plan = binding.Plan(W, cfg.D, cfg.replica_slots, gpus_per_node=cfg.gpus_per_node)
    ref = po.make_plan(W.tolist(), cfg.D, None, cfg.replica_slots)
    _same(plan, ref)
    assert plan.summary()["total_replicas"] == cfg.replica_slots


def test_multilayer_stack_shape_plan_and_prefix_sweep():
    # 58 layers x 256 experts, exponents in [0.6, 1.6], budgets 0..64: one incremental run
    L, E, D = 58, 256, 32
    s = synth.trace_layer_exponents(L, 5)
    W = np.stack([np.round(synth.popularity(E, s[l], 5, l) * 8 * 4096 * 16) for l in range(L)])
    W = W.astype(np.int64)[None]
    plan = binding.Plan(W, D, 64)
    ref = po.make_plan(W.tolist(), D, None, 64)
    _same(plan, ref)
    order = plan.greedy_order()
    small = binding.Plan(W, D, 32)
    assert small.greedy_order().tolist() == order[:32].tolist()      # prefix property
    x = np.array([plan.layer(l)["n_replicas"] for l in range(L)])
    assert x[s > 1.3].sum() > x[s < 0.9].sum()                        # skewed layers are served


def test_rank_rows_match_the_checker_dispatch():
    cfg = synth.CONFIGS["tiny"]
    pop = synth.layer_popularity(cfg)
    ids, _ = oracle.route(synth.router_logits(cfg, pop, "eval"), cfg.k)
    counts = oracle.expert_load(ids[None], cfg.E, cfg.T)
    plan = binding.Plan(counts, cfg.D, cfg.replica_slots)
    lay = plan.layer(0)
    _, _, cnt, _ = oracle.dispatch(ids, cfg.E, lay["slot_expert"])
    want = po.realized_rank_rows(cnt.tolist(), lay["rank_slot_off"].tolist())
    rows, top = plan.rank_rows(0, counts[0, 0])
    assert rows.tolist() == want and top == po.heaviest_rank(want)
    assert rows.sum() == cfg.T * cfg.k


def test_argument_checks():
    lib = binding.lib()
    W = np.ones((1, 1, 4), dtype=np.int64)
    with pytest.raises(binding.CraftError):
        binding.Plan(W, 0, 0)
    with pytest.raises(binding.CraftError):
        binding.Plan(W, 2, -1)
    with pytest.raises(binding.CraftError):
        binding.Plan(-W, 2, 0)
    with pytest.raises(binding.CraftError):
        binding.Plan(W, 2, 1, bytes_per_replica=[0])
    assert lib.craft_plan(None, None) == -1
    p = binding.Plan(W, 2, 1)
    assert lib.craft_plan_layer_info(p._h, 1, None, None, None, None) == -1
    n = ctypes.c_size_t()
    assert lib.craft_plan_tables_bytes(p._h, 0, 2, n) == -1
    assert lib.craft_plan_tables_bytes(p._h, 0, 1, n) == 0 and n.value > 0
    # device entry points reject bad sizes before touching the GPU
    assert lib.craft_route_topk(None, 4, 8, 9, 1, None, None, None) == -1
    assert lib.craft_route_topk(None, 4, 2000, 2, 1, None, None, None) == -1
    assert lib.craft_expert_load(None, 1, 4, 2, 5000, 4, None, None) == -1
    assert lib.craft_expert_load(None, 1, 4, 2, 8, 0, None, None) == -1
    a = binding.FwdArgs()
    a.dtype, a.T, a.H, a.I, a.k = 1, 8, 12, 16, 2          # H not a multiple of 8 for bf16
    assert lib.craft_moe_rank_forward_workspace(p._h, 0, 0, ctypes.byref(a), n) == -1
    a.H = 16
    assert lib.craft_moe_rank_forward_workspace(p._h, 0, 0, ctypes.byref(a), n) == 0
    assert lib.craft_moe_rank_forward(p._h, 0, 0, ctypes.byref(a), None) == -1   # no workspace


def test_budget_beyond_every_expert_on_every_rank_stops():
    W = np.array([[[5, 3]]], dtype=np.int64)
    p = binding.Plan(W, 2, 100)                 # at most E*(D-1) = 2 replicas exist
    assert p.summary()["total_replicas"] == 2
    assert p.layer(0)["copies"].tolist() == [2, 2]


# ------------------------------------------- the paper's own pipeline and the comparison plans

def _same_paper(plan: binding.Plan, ref: dict):
    b = plan.benefit()
    assert b["counts"].tolist() == ref["benefit_counts"]
    assert b["base"].tolist() == ref["benefit_base"]                  # same double expressions
    for i, r in enumerate(ref["benefit_counts"]):
        assert b["gain"][i].tolist() == ref["benefit"][r]
    assert b["total_gain"] == ref["total_gain"]
    _same(plan, ref)


@pytest.mark.parametrize("seed", range(12))
def test_paper_pipeline_matches_checker_on_random_loads(seed):
    g = np.random.default_rng(900 + seed)
    L, D = int(g.integers(1, 7)), int(g.choice([1, 2, 3, 4, 8, 16]))
    E = int(g.integers(1, 30))
    B = int(g.integers(1, 6))
    W = (g.zipf(1.4, size=(B, L, E)) % int(g.choice([3, 200, 50000]))).astype(np.int64)
    budget = int(g.integers(0, L * D + 4))
    for auto in (False, True):
        plan = binding.Plan(W, D, budget, objective=1, auto_r=auto)
        ref = po.make_plan_paper(W.tolist(), D, budget, auto)
        _same_paper(plan, ref)
        if auto and ref["benefit_counts"]:
            R = po.choose_replication_factor(ref["benefit"], D, min(budget, L * max(ref["benefit_counts"])) // D)
            assert plan.benefit()["auto_R"] == R and plan.summary()["total_replicas"] <= R * D


def test_paper_pipeline_counts_bytes_as_replicas():
    g = np.random.default_rng(950)
    W = g.integers(0, 900, size=(3, 4, 10))
    plan = binding.Plan(W, 4, 7 * 1000 + 999, bytes_per_replica=[1000] * 4, objective=1)
    _same_paper(plan, po.make_plan_paper(W.tolist(), 4, 7))
    with pytest.raises(binding.CraftError):
        binding.Plan(W, 4, 7000, bytes_per_replica=[1000, 1000, 1000, 999], objective=1)
    with pytest.raises(binding.CraftError):
        binding.Plan(W, 4, 7, objective=3)
    assert binding.Plan(W, 4, 7).benefit()["counts"].size == 0       # objective 0 keeps no matrix


@pytest.mark.parametrize("seed", range(6))
def test_uniform_comparison_plans_match_checker(seed):
    g = np.random.default_rng(970 + seed)
    L, D, E = int(g.integers(1, 6)), int(g.choice([1, 2, 4, 8])), int(g.integers(1, 24))
    W = g.integers(0, 3000, size=(2, L, E))
    for n in (0, 1, D, 3 * D):
        plan = binding.Plan(W, D, n * L + int(g.integers(0, L)), objective=2)
        _same(plan, po.make_plan_uniform(W.tolist(), D, min(n, E * (D - 1))))


def test_stack_shape_three_planners_side_by_side():
    # 58 layers x 256 experts on 32 ranks, four profiling batches drawn around each layer's
    # popularity.  At the same replica total: the paper's pipeline, the unit greedy and
    # uniform spreading; and uniform replication at its own minimum L * D.
    L, E, D, B = 58, 256, 32, 4
    s = synth.trace_layer_exponents(L, 5)
    g = np.random.default_rng(5)
    W = np.stack([[g.multinomial(8 * 4096, synth.popularity(E, s[l], 5, l)) for l in range(L)]
                  for _ in range(B)]).astype(np.int64)
    total = 8 * D                                                       # R = 8
    paper = binding.Plan(W, D, total, objective=1)
    _same_paper(paper, po.make_plan_paper(W.tolist(), D, total))
    greedy = binding.Plan(W, D, total)
    spread = binding.Plan(W, D, total, objective=2)
    uniform = binding.Plan(W, D, L * D, objective=2)
    base = binding.Plan(W, D, 0, objective=2)

    def mean_bal(p):
        return float(np.mean([p.layer(l)["est_balancedness"] for l in range(L)]))

    assert paper.summary()["total_replicas"] == total == greedy.summary()["total_replicas"]
    assert uniform.summary()["memory_saving_vs_uniform"] == 1.0
    assert paper.summary()["memory_saving_vs_uniform"] == L / 8            # Sec. 5.2: L / R
    # benefit-driven allocation beats spreading the same replicas evenly (Sec. 3.2); uniform
    # replication with L / R times the memory is the upper end of the curve
    b0, bp, bg, bs, bu = (mean_bal(p) for p in (base, paper, greedy, spread, uniform))
    assert bu > bp > bs > b0 and bg > bs
    # skewed layers take the replicas
    x = np.array([paper.layer(l)["n_replicas"] for l in range(L)])
    assert x[s > 1.3].sum() > x[s < 0.9].sum()
    # automatic mode lands on a multiple of D no larger than the budget
    auto = binding.Plan(W, D, 16 * D, objective=1, auto_r=True)
    R = auto.benefit()["auto_R"]
    assert 1 <= R <= 16 and auto.summary()["total_replicas"] == R * D


def test_ffn_tile_heights_query():
    # host-side choice of the grouped-GEMM row-tile height and of riders; no device work
    lib = binding.lib()
    g = np.random.default_rng(3)
    W = g.multinomial(8 * 4096, synth.popularity(128, 1.0, 2, 0), size=(4, 1)).astype(np.int64)
    plan = binding.Plan(W, 8, 8)
    a = binding.FwdArgs()
    a.dtype, a.T, a.H, a.I, a.k = 1, 4096, 4096, 1536, 8
    gu, dn, rgu, rdn = (ctypes.c_int32() for _ in range(4))

    def query(rank=0):
        return lib.craft_moe_rank_forward_tiles(plan._h, 0, rank, ctypes.byref(a), gu, dn, rgu, rdn)

    assert query() == 0
    assert (gu.value, dn.value, rgu.value, rdn.value) == (128, 128, 0, 0)   # row-major bf16 weights: fixed
    a.w_gateup_packed = a.w_down_packed = 0x1000               # packed: chosen from the plan's loads
    for rank in range(8):
        assert query(rank) == 0
        assert gu.value % 32 == 0 and 128 <= gu.value <= 256
        assert dn.value % 32 == 0 and 128 <= dn.value <= 256
        assert rgu.value in (0, 1) and rdn.value in (0, 1)
        assert not (rgu.value and gu.value > 224) and not (rdn.value and dn.value > 224)
        first = (gu.value, dn.value, rgu.value, rdn.value)
        assert query(rank) == 0
        assert (gu.value, dn.value, rgu.value, rdn.value) == first          # kept with the plan
    # the caller's knobs win; the tallest tile has no room for a rider
    a.tile_rows_gateup, a.tile_rows_down, a.riders_gateup, a.riders_down = 192, 256, -1, 1
    assert query() == 0
    assert (gu.value, dn.value, rgu.value, rdn.value) == (192, 256, 0, 0)
    a.riders_gateup, a.tile_rows_down = 1, 224
    assert query() == 0
    assert (gu.value, dn.value, rgu.value, rdn.value) == (192, 224, 1, 1)
    a.riders_down = 2
    assert query() == -1
    a.tile_rows_gateup = a.tile_rows_down = a.riders_gateup = a.riders_down = 0
    assert lib.craft_moe_rank_forward_tiles(plan._h, 0, 0, ctypes.byref(a), gu, None, None, None) == 0
    a.dtype = 0
    a.w_gateup_packed = a.w_down_packed = None
    assert query() == 0
    assert (gu.value, dn.value, rgu.value, rdn.value) == (32, 32, 0, 0)
    assert query(9) == -1


def test_gate_workspace_query_and_forward_workspace_with_own_gate():
    # host-side sizes only; no device work
    lib = binding.lib()
    n = ctypes.c_size_t()
    assert lib.craft_router_logits_workspace(binding.CRAFT_F32, 4096, 4096, 128, ctypes.byref(n)) == 0
    assert n.value == 0                                        # the fp32 gate is never split
    assert lib.craft_router_logits_workspace(binding.CRAFT_BF16, 4096, 4096, 128, ctypes.byref(n)) == 0
    assert n.value % (4096 * 128 * 4) == 0 and 1 < n.value // (4096 * 128 * 4) <= 8   # whole partial score matrices
    assert lib.craft_router_logits_workspace(binding.CRAFT_BF16, 1 << 20, 4096, 128, ctypes.byref(n)) == 0
    assert n.value == 0                                        # enough tiles of tokens: nothing to split
    assert lib.craft_router_logits_workspace(binding.CRAFT_BF16, 0, 4096, 128, ctypes.byref(n)) == 0 and n.value == 0
    assert lib.craft_router_logits_workspace(binding.CRAFT_BF16, 16, 4100, 128, ctypes.byref(n)) == -1   # H % 8
    assert lib.craft_router_logits_workspace(binding.CRAFT_BF16, 16, 4096, 1025, ctypes.byref(n)) == -1  # E limit
    assert lib.craft_router_logits_workspace(7, 16, 4096, 128, ctypes.byref(n)) == -1
    # a forward that runs the gate itself needs room for the scores and the gate's workspace
    g = np.random.default_rng(4)
    W = g.multinomial(8 * 4096, synth.popularity(128, 1.0, 2, 0), size=(4, 1)).astype(np.int64)
    plan = binding.Plan(W, 8, 8)
    a = binding.FwdArgs()
    a.dtype, a.T, a.H, a.I, a.k = 1, 4096, 4096, 1536, 8
    a.logits = 0x1000                                          # scores handed in
    given, own = ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.craft_moe_rank_forward_workspace(plan._h, 0, 0, ctypes.byref(a), ctypes.byref(given)) == 0
    a.logits = None
    assert lib.craft_moe_rank_forward_workspace(plan._h, 0, 0, ctypes.byref(a), ctypes.byref(own)) == 0
    assert lib.craft_router_logits_workspace(binding.CRAFT_BF16, 4096, 4096, 128, ctypes.byref(n)) == 0
    assert own.value - given.value >= 4096 * 128 * 4 + n.value


def test_static_scratch_forward_refuses_what_does_not_fit():
    # host-side size check of craft_moe_rank_forward_static: no device is touched before it
    lib = binding.lib()
    g = np.random.default_rng(4)
    W = g.multinomial(8 * 4096, synth.popularity(128, 1.0, 2, 0), size=(4, 1)).astype(np.int64)
    plan = binding.Plan(W, 8, 8)
    a = binding.FwdArgs()
    a.dtype, a.T, a.H, a.I, a.k = 1, 4096, 4096, 1536, 8
    a.logits = 0x1000
    need = ctypes.c_size_t()
    assert lib.craft_moe_rank_forward_workspace(plan._h, 0, 0, ctypes.byref(a), ctypes.byref(need)) == 0
    assert need.value > (64 << 20)
    assert lib.craft_moe_rank_forward_static(plan._h, 0, 0, ctypes.byref(a), None) == -5
    assert b"limit" in lib.craft_status_str(-5)
    a.k = 0                                                    # bad arguments are still bad arguments
    assert lib.craft_moe_rank_forward_static(plan._h, 0, 0, ctypes.byref(a), None) == -1
