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
