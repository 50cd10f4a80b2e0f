"""Periodic rebalancing (Sec. 4.3): load window, re-plan, weight relocation diff.

CPU part: the checker's diff against the multiset identity, the library's diff against the
checker, and a workload-shift scenario planned from the host side.  GPU part: the load window
accumulated on the device from the forwards' own counts, the re-plan made from it, and a
forward under the new plan, all against the CPU checker."""
from collections import Counter

import numpy as np
import pytest

import oracle
from oracle import plan_oracle as po
from paper_2603_28768_amd import binding, synth
from cases import Case


def _plans(seed, L=3, E=20, D=4, budget=9):
    g = np.random.default_rng(seed)
    Wa = (g.zipf(1.3, size=(2, L, E)) % 500).astype(np.int64)
    Wb = (g.zipf(1.3, size=(2, L, E)) % 500).astype(np.int64)
    return (Wa, Wb, binding.Plan(Wa, D, budget), binding.Plan(Wb, D, budget),
            po.make_plan(Wa.tolist(), D, None, budget), po.make_plan(Wb.tolist(), D, None, budget))


@pytest.mark.parametrize("seed", range(6))
def test_checker_diff_is_the_multiset_difference(seed):
    _, _, _, _, ra, rb = _plans(seed)
    for l in range(3):
        for g in range(4):
            a, b = ra["layers"][l], rb["layers"][l]
            old = a["slot_expert"][a["rank_slot_off"][g]:a["rank_slot_off"][g + 1]]
            new = b["slot_expert"][b["rank_slot_off"][g]:b["rank_slot_off"][g + 1]]
            reuse, nf, nd = po.plan_diff(a, b, g)
            co, cn = Counter(old), Counter(new)
            assert nf == sum((cn - co).values()) and nd == sum((co - cn).values())
            kept = [r for r in reuse if r >= 0]
            assert len(set(kept)) == len(kept)                         # an old slot is reused once
            assert all(old[r] == new[j] for j, r in enumerate(reuse) if r >= 0)
            assert len(old) - nd + nf == len(new)
    same, nf, nd = po.plan_diff(ra["layers"][0], ra["layers"][0], 1)
    assert nf == 0 and nd == 0 and same == list(range(len(same)))


@pytest.mark.parametrize("seed", range(6))
def test_library_diff_matches_checker(seed):
    _, _, pa, pb, ra, rb = _plans(100 + seed)
    for l in range(3):
        for g in range(4):
            got = pa.diff(pb, l, g)
            reuse, nf, nd = po.plan_diff(ra["layers"][l], rb["layers"][l], g)
            assert got["reuse"].tolist() == reuse and got["n_fetch"] == nf and got["n_drop"] == nd
    lib = binding.lib()
    other = binding.Plan(np.ones((1, 3, 20), np.int64), 2, 0)
    assert lib.craft_plan_diff(pa._h, other._h, 0, 0, None, None, None) == -1     # D differs
    assert lib.craft_plan_diff(pa._h, pb._h, 3, 0, None, None, None) == -1
    assert lib.craft_plan_diff(pa._h, pb._h, 0, 4, None, None, None) == -1
    assert lib.craft_load_accumulate(None, -1, None, None) == -1
    assert lib.craft_load_accumulate(None, 0, None, None) == 0


def _routed_counts(cfg, pop, tag, batch):
    ids, _ = oracle.route(synth.router_logits(cfg, pop, tag, batch), cfg.k)
    return np.bincount(ids.reshape(-1), minlength=cfg.E).astype(np.int64)


def test_workload_shift_replan_restores_balance():
    # the popular experts change; a plan made from a window of post-shift batches balances
    # the following batches better than the stale plan, and moves only part of the weights
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=1024, E=64, D=8, replica_slots=8, profile_batches=4)
    pop0 = synth.layer_popularity(cfg)
    pop1 = np.roll(pop0, 17)
    W0 = np.stack([_routed_counts(cfg, pop0, "profile", b) for b in range(4)])[:, None, :]
    W1 = np.stack([_routed_counts(cfg, pop1, "window", b) for b in range(4)])[:, None, :]
    stale = binding.Plan(W0, cfg.D, cfg.replica_slots)
    fresh = binding.Plan(W1, cfg.D, cfg.replica_slots)

    def balancedness(plan, counts):
        rows, _ = plan.rank_rows(0, counts)
        return rows.mean() / rows.max()

    later = [_routed_counts(cfg, pop1, "later", b) for b in range(4)]
    b_stale = np.mean([balancedness(stale, c) for c in later])
    b_fresh = np.mean([balancedness(fresh, c) for c in later])
    assert b_fresh > b_stale + 0.1
    moved = sum(stale.diff(fresh, 0, g)["n_fetch"] for g in range(cfg.D))
    assert 0 < moved < cfg.E + cfg.replica_slots
    # an unchanged workload needs no relocation
    again = binding.Plan(W0, cfg.D, cfg.replica_slots)
    assert sum(stale.diff(again, 0, g)["n_fetch"] for g in range(cfg.D)) == 0


@pytest.mark.gpu
def test_window_accumulated_on_device_and_replan(torch_cuda):
    torch = torch_cuda
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=512, H=256, I=128, E=32, D=4, replica_slots=4,
                       profile_batches=2)
    case = Case(cfg)
    rank = case.heaviest
    fwd, x, _ = case.gpu_rank(rank, packed=True)
    pop1 = np.roll(case.pop, 11)                                     # the workload shifts
    window = torch.zeros(cfg.E, dtype=torch.int64, device="cuda:0")
    want = np.zeros(cfg.E, np.int64)
    W1 = []
    for b in range(3):
        logits = synth.router_logits(cfg, pop1, "window", b)
        fwd(x, torch.from_numpy(logits).to("cuda:0"))
        binding.load_accumulate(fwd.debug["counts"], window)
        ids, _ = oracle.route(logits, cfg.k)
        W1.append(np.bincount(ids.reshape(-1), minlength=cfg.E))
        want += W1[-1]
    torch.cuda.synchronize()
    assert np.array_equal(window.cpu().numpy(), want)
    # re-plan from the device window (one batch: the window itself), as a rebalancing would
    fresh = binding.Plan(window.cpu().numpy()[None, None, :], cfg.D, cfg.replica_slots)
    ref = po.make_plan([[want.tolist()]], cfg.D, None, cfg.replica_slots)
    assert fresh.layer(0)["slot_expert"].tolist() == ref["layers"][0]["slot_expert"]
    d = case.plan.diff(fresh, 0, rank)
    reuse, nf, nd = po.plan_diff(po.make_plan(case.W.tolist(), cfg.D, None, cfg.replica_slots)["layers"][0],
                                 ref["layers"][0], rank)
    assert d["reuse"].tolist() == reuse and d["n_fetch"] == nf and d["n_drop"] == nd
    # the swap on this rank: slots that keep an expert it already holds take over the resident
    # buffers, only the rest is fetched (here: packed afresh); then a forward under the new plan
    after = Case(cfg, plan=fresh, pop=pop1)
    old_slots, new_slots = case.rank_slots(rank), after.rank_slots(rank)
    (og, ou, od), opacked = fwd._weights, fwd._packed[0]
    wg, wu, wd, pk, fetched = [], [], [], [], 0
    for j, e in enumerate(new_slots):
        r = int(d["reuse"][j])
        if r >= 0:
            assert old_slots[r] == e
            g_, u_, d_, p_ = og[r], ou[r], od[r], opacked[r]
        else:
            fetched += 1
            g_, u_, d_ = (binding.to_device(m, cfg.dtype) for m in synth.expert_weights(cfg, e))
            p_ = binding.pack_weights(g_, u_, d_)
        wg.append(g_); wu.append(u_); wd.append(d_); pk.append(p_)
    assert fetched == d["n_fetch"]
    assert sorted(r for r in d["reuse"].tolist() if r >= 0) == sorted(set(r for r in d["reuse"].tolist() if r >= 0))
    swapped = binding.RankForward(fresh, 0, rank, cfg.dtype, cfg.T, cfg.H, cfg.I, cfg.k, wg, wu, wd,
                                  want_debug_outputs=True, packed=pk)
    xs = binding.to_device(after.x, cfg.dtype)
    out = swapped(xs, torch.from_numpy(after.logits).to("cuda:0")).float().cpu().numpy().astype(np.float64)
    r = after.oracle_rank(rank)
    assert swapped.result() == (r["rows"], 0)
    assert np.abs(out - r["out"]).max() <= 1e-2 * np.abs(r["out"]).max()
    # and on the rank that is now the heaviest, with all weights placed afresh
    f2, x2, l2 = after.gpu_rank(after.heaviest, packed=True)
    out = f2(x2, l2).float().cpu().numpy().astype(np.float64)
    rows, ovf = f2.result()
    r = after.oracle_rank(after.heaviest)
    assert rows == r["rows"] and ovf == 0
    assert np.array_equal(f2.debug["dest"].cpu().numpy().reshape(-1), r["dest"])
    assert np.abs(out - r["out"]).max() <= 1e-2 * np.abs(r["out"]).max()


@pytest.mark.gpu
def test_weights_relocated_on_a_side_stream_while_the_old_plan_serves(torch_cuda):
    # Sec. 4.3 step 3 asks for the relocation not to stall serving: the experts the new plan
    # brings to this rank are copied from pinned host memory and packed on a second stream
    # while forwards under the old plan keep running on the first; the serving stream waits
    # for one event, then runs under the new plan with the second set of buffers.
    torch = torch_cuda
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=768, H=512, I=256, E=48, D=4, replica_slots=6,
                       profile_batches=2)
    case = Case(cfg)
    rank = case.heaviest
    fwd, x, logits = case.gpu_rank(rank, packed=True)
    ref_old = case.oracle_rank(rank)
    pop1 = np.roll(case.pop, 17)                                     # the workload shifts
    ids, _ = oracle.route(synth.router_logits(cfg, pop1, "window", 0), cfg.k)
    want = np.bincount(ids.reshape(-1), minlength=cfg.E).astype(np.int64)
    fresh = binding.Plan(want[None, None, :], cfg.D, cfg.replica_slots)
    d = case.plan.diff(fresh, 0, rank)
    after = Case(cfg, plan=fresh, pop=pop1)
    old_slots, new_slots = case.rank_slots(rank), after.rank_slots(rank)
    assert d["n_fetch"] > 0 and (d["reuse"] >= 0).any()
    # the experts to fetch wait in pinned host memory, as the paper's CPU-resident weights do
    host = {}
    for j, e in enumerate(new_slots):
        if d["reuse"][j] < 0 and e not in host:
            host[e] = [torch.from_numpy(np.ascontiguousarray(m, dtype=np.float32)).to(torch.bfloat16).pin_memory()
                       for m in synth.expert_weights(cfg, e)]
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    (og, ou, od), opacked = fwd._weights, fwd._packed[0]
    wg, wu, wd, pk = [None] * len(new_slots), [None] * len(new_slots), [None] * len(new_slots), [None] * len(new_slots)
    outs = [fwd(x, logits).clone()]
    side.wait_stream(main)
    for j, e in enumerate(new_slots):
        if d["reuse"][j] >= 0:
            continue
        with torch.cuda.stream(side):
            dev = [m.to("cuda:0", non_blocking=True) for m in host[e]]
        wg[j], wu[j], wd[j] = dev
        pk[j] = binding.pack_weights(*dev, stream=side)
        outs.append(fwd(x, logits, stream=main).clone())              # serving goes on meanwhile
    arrived = side.record_event()
    for j, e in enumerate(new_slots):
        r = int(d["reuse"][j])
        if r >= 0:
            assert old_slots[r] == e
            wg[j], wu[j], wd[j], pk[j] = og[r], ou[r], od[r], opacked[r]
    main.wait_event(arrived)
    swapped = binding.RankForward(fresh, 0, rank, cfg.dtype, cfg.T, cfg.H, cfg.I, cfg.k, wg, wu, wd,
                                  want_debug_outputs=True, packed=pk)
    xs = binding.to_device(after.x, cfg.dtype)
    out_new = swapped(xs, torch.from_numpy(after.logits).to("cuda:0")).float().cpu().numpy().astype(np.float64)
    torch.cuda.synchronize()
    # every forward under the old plan gave the same bits, and they are the checker's answer
    first = outs[0].float().cpu().numpy().astype(np.float64)
    assert len(outs) == 1 + d["n_fetch"]
    for o in outs[1:]:
        assert torch.equal(o, outs[0])
    assert np.abs(first - ref_old["out"]).max() <= 1e-2 * np.abs(ref_old["out"]).max()
    r = after.oracle_rank(rank)
    assert swapped.result() == (r["rows"], 0)
    assert np.array_equal(swapped.debug["dest"].cpu().numpy().reshape(-1), r["dest"])
    assert np.abs(out_new - r["out"]).max() <= 1e-2 * np.abs(r["out"]).max()
