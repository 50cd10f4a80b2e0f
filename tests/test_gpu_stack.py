"""GPU parity for the planner-plus-multi-layer-stack workload: routing traces of 58 MoE
layers x 256 experts with per-layer Zipf exponents drawn from [0.6, 1.6]; the GPU computes
the load histogram, the host plans replicas for budgets up to 256, and DeepSeek-V3-shaped
layers at a long prefill batch run the heaviest rank's share under their own layer's plan."""
import numpy as np
import pytest

import oracle
from oracle import plan_oracle as po
from paper_2603_28768_amd import binding, synth

from cases import Case
from test_gpu_parity import _check_rank

pytestmark = pytest.mark.gpu

L, E, K, D = 58, 256, 8, 32
STACK_INDEX = 5


def _trace(T):
    s = synth.trace_layer_exponents(L, STACK_INDEX)
    return s, np.stack([synth.routing_trace_layer(E, K, T, s[l], STACK_INDEX, l) for l in range(L)])


@pytest.fixture(scope="module")
def stack(torch_cuda):
    """Trace -> GPU histogram -> plan at budget 256 (every smaller budget is a prefix)."""
    torch = torch_cuda
    T, bt = 32768, 4096
    s, ids = _trace(T)
    print("stack trace", ids.shape, flush=True)
    counts = binding.expert_load(torch.from_numpy(ids).cuda(), E, bt)
    torch.cuda.synchronize()
    W = counts.cpu().numpy()
    assert np.array_equal(W, oracle.expert_load(ids, E, bt))            # bit-exact counts
    assert np.all(W.sum(-1) == bt * K)
    plan = binding.Plan(W, D, 256)
    return dict(s=s, W=W, plan=plan)


def test_stack_plan_matches_checker_and_sweeps_by_prefix(stack):
    W, plan = stack["W"], stack["plan"]
    ref = po.make_plan(W.tolist(), D, None, 256)
    order = plan.greedy_order()
    assert order.tolist() == [l for l, _ in ref["order"]]
    for l in range(L):
        got, want = plan.layer(l), ref["layers"][l]
        assert got["n_replicas"] == want["n_replicas"]
        assert got["slot_expert"].tolist() == want["slot_expert"]
        assert got["rank_slot_off"].tolist() == want["rank_slot_off"]
    summ = plan.summary()
    assert summ["total_replicas"] == 256 and summ["replication_factor"] == 8.0
    assert summ["memory_saving_vs_uniform"] == L * D / 256              # L / R = 58 / 8 = 7.25
    for b in (0, 32, 64, 128):                                           # R = 0, 1, 2, 4
        small = binding.Plan(W, D, b)
        assert small.greedy_order().tolist() == order[:b].tolist()
    # skewed layers receive the replicas (Observation 4 of the paper)
    x = np.array([plan.layer(l)["n_replicas"] for l in range(L)])
    s = stack["s"]
    assert x[s > 1.3].mean() > x[s < 0.9].mean()


def test_full_length_trace_layer(torch_cuda):
    # one layer at the full 2^20 tokens: cells split over several workgroups (atomic merge)
    torch = torch_cuda
    T = 1 << 20
    ids = synth.routing_trace_layer(E, K, T, 1.2, STACK_INDEX, 0)[None]
    for bt in (4096, T):
        print("full-length trace, batch_tokens", bt, flush=True)
        got = binding.expert_load(torch.from_numpy(ids).cuda(), E, bt).cpu().numpy()
        assert np.array_equal(got, oracle.expert_load(ids, E, bt))


@pytest.mark.parametrize("which", ["most_skewed", "least_skewed", "lower_third", "upper_third"])
def test_stack_layer_forward_under_its_own_plan(torch_cuda, stack, which):
    s, plan = stack["s"], stack["plan"]
    by_s = np.argsort(s)
    layer = int({"most_skewed": by_s[-1], "least_skewed": by_s[0],
                 "lower_third": by_s[L // 3], "upper_third": by_s[2 * L // 3]}[which])
    cfg = synth.scaled(synth.CONFIGS["dsv3_long"], zipf_s=float(s[layer]))
    pop = synth.popularity(E, s[layer], STACK_INDEX, layer)              # the trace's popularity
    print(f"stack layer {layer}: s={s[layer]:.2f} replicas={plan.layer(layer)['n_replicas']}", flush=True)
    case = Case(cfg, plan=plan, layer=layer, pop=pop)
    g = case.heaviest
    print(f"  rows: max={max(case.rows)} mean={np.mean(case.rows):.0f} slots={len(case.rank_slots(g))}", flush=True)
    # every token of the 32768 (the checker needs some ten seconds for the rank's rows)
    _check_rank(torch_cuda, case, g, packed=True, cover=True)


# ------------------------------------- the paper's own planner and the comparison plans

@pytest.fixture(scope="module")
def other_plans(stack):
    """From the GPU histogram of the trace: the paper's pipeline (Alg. 1 replay, Alg. 2) at
    R = 8 and with the replication factor chosen automatically (Sec. 4.2.1 step 2), placement
    only and uniform replication (the setups of Sec. 5.1), each equal to the checker's plan."""
    from test_plan_host import _same, _same_paper
    W = stack["W"]
    Wl = W.tolist()
    plans = {}
    plans["paper_R8"] = binding.Plan(W, D, 8 * D, objective=1)
    _same_paper(plans["paper_R8"], po.make_plan_paper(Wl, D, 8 * D))
    plans["paper_auto"] = binding.Plan(W, D, 8 * D, objective=1, auto_r=True)
    ref = po.make_plan_paper(Wl, D, 8 * D, True)
    _same_paper(plans["paper_auto"], ref)
    R = po.choose_replication_factor(ref["benefit"], D, 8)
    assert plans["paper_auto"].benefit()["auto_R"] == R and ref["total_replicas"] <= R * D
    plans["placement_only"] = binding.Plan(W, D, 0, objective=2)
    _same(plans["placement_only"], po.make_plan_uniform(Wl, D, 0))
    plans["uniform"] = binding.Plan(W, D, L * D, objective=2)
    _same(plans["uniform"], po.make_plan_uniform(Wl, D, D))
    return plans


def test_paper_planner_and_comparison_plans_from_the_gpu_histogram(stack, other_plans):
    def mean_bal(p):
        return float(np.mean([p.layer(l)["est_balancedness"] for l in range(L)]))
    bal = {k: mean_bal(p) for k, p in other_plans.items()}
    bal["greedy_R8"] = mean_bal(stack["plan"])
    print("  mean estimated balancedness:", {k: round(v, 4) for k, v in bal.items()}, flush=True)
    assert other_plans["paper_R8"].summary()["total_replicas"] == 8 * D
    assert other_plans["paper_R8"].summary()["memory_saving_vs_uniform"] == L / 8     # Sec. 5.2
    assert other_plans["uniform"].summary()["memory_saving_vs_uniform"] == 1.0
    # replication beats placement alone, and uniform replication with L / R times the memory
    # is the upper end (Sec. 3.2)
    assert bal["uniform"] > bal["paper_R8"] > bal["placement_only"]
    assert bal["greedy_R8"] > bal["placement_only"]


@pytest.mark.parametrize("which", ["paper_R8", "paper_auto", "placement_only", "uniform"])
def test_layer_forward_under_the_paper_planner_and_comparison_plans(torch_cuda, stack, other_plans, which):
    # a DeepSeek-V3-shaped layer (T = 8192) of the stack, the most skewed one, under each of
    # those plans: heaviest rank's share, every token against the checker
    plan, s = other_plans[which], stack["s"]
    layer = int(np.argsort(s)[-1])
    cfg = synth.scaled(synth.CONFIGS["dsv3_long"], T=8192, zipf_s=float(s[layer]))
    pop = synth.popularity(E, s[layer], STACK_INDEX, layer)
    case = Case(cfg, plan=plan, layer=layer, pop=pop)
    g = case.heaviest
    print(f"  {which}: layer {layer} replicas={plan.layer(layer)['n_replicas']} rows max={max(case.rows)} "
          f"mean={np.mean(case.rows):.0f} slots={len(case.rank_slots(g))}", flush=True)
    _check_rank(torch_cuda, case, g, packed=True, cover=True)
