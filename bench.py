#!/usr/bin/env python3
"""Throughput of one expert-parallel rank's MoE layer under a CRAFT replication plan.

A step is one pass of the hot path over one batch: craft_moe_rank_forward (route, load
counts, replica-aware dispatch, grouped SwiGLU FFN, combine) on the heaviest simulated rank
of every executed layer of the workload, inputs and weights resident in HBM.  The default
workload is the largest one: the multi-layer stack (routing traces of 58 layers x 256 experts
-> GPU histogram -> plan at 256 replicas -> four DeepSeek-V3-shaped layers at T = 32768, each
under its own layer's plan); the single-layer workloads are behind --config.  The plan is
made once before the timed region, through the library (craft_expert_load -> craft_plan), as
the paper does at initialisation (Sec. 5.4: planning has no inference-time cost).

Prints one JSON line: tokens/s through an MoE layer, plus
  roofline      for the dominant kernel (grouped gate/up GEMM): algorithmic bytes and flops
                per launch over its HIP-event duration measured inside the timed region; the
                per-slot bounds of the expert FFN; the other kernels' fractions; this
                machine's own copy and MFMA-loop rates
  cpu_baseline  the CPU checker timed on this host on a bounded sample of the same work
"""
from __future__ import annotations

import argparse
import hashlib
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
FP32_VALU_PEAK_TFLOPS = 157.3


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def setup(cfg, dev="cuda:0", packed=True, e4m3=False, plan=None, layer=0, pop=None, plan_ms=0.0,
          keep_host_weights=True):
    """Profiling -> plan -> evaluation batch -> heaviest rank, all through the library.
    With `plan` (a multi-layer plan made elsewhere): the evaluation batch of its layer `layer`,
    whose experts have popularity `pop`."""
    import torch
    from paper_2603_28768_amd import binding, synth

    if plan is None:
        pop = synth.layer_popularity(cfg)
        prof = np.concatenate([synth.router_logits(cfg, pop, "profile", b)
                               for b in range(cfg.profile_batches)])
        ids, _ = binding.route_topk(torch.from_numpy(prof).to(dev), cfg.k)
        W = binding.expert_load(ids.reshape(1, -1, cfg.k), cfg.E, cfg.T)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        plan = binding.Plan(W.cpu().numpy(), cfg.D, cfg.replica_slots, gpus_per_node=cfg.gpus_per_node)
        plan_ms = (time.perf_counter() - t0) * 1e3

    logits = synth.router_logits(cfg, pop, "eval", layer=layer)
    x = synth.activations(cfg, layer=layer)
    d_logits = torch.from_numpy(logits).to(dev)
    eids, _ = binding.route_topk(d_logits, cfg.k)
    counts = binding.expert_load(eids.reshape(1, -1, cfg.k), cfg.E, cfg.T)[0, 0].cpu().numpy()
    rows, rank = plan.rank_rows(layer, counts)
    lay = plan.layer(layer)
    slots = [int(e) for e in lay["slot_expert"][lay["rank_slot_off"][rank]:lay["rank_slot_off"][rank + 1]]]
    host_w, dev_w = {}, {}
    for e in slots:
        if e not in dev_w:
            hw = synth.expert_weights(cfg, e, layer)
            dev_w[e] = tuple(binding.to_device(m, cfg.dtype, dev) for m in hw)
            if keep_host_weights:
                host_w[e] = hw
    # model loading: weights are re-ordered once for the weight-streaming kernels
    packed = packed and cfg.dtype == "bf16"
    pack = binding.pack_weights_e4m3 if e4m3 else binding.pack_weights
    pk = {e: pack(*dev_w[e]) for e in dev_w} if packed else None
    fwd = binding.RankForward(plan, layer, rank, cfg.dtype, cfg.T, cfg.H, cfg.I, cfg.k,
                              [dev_w[e][0] for e in slots], [dev_w[e][1] for e in slots],
                              [dev_w[e][2] for e in slots],
                              packed=[pk[e] for e in slots] if packed else None,
                              weight_format=binding.CRAFT_W_E4M3 if (packed and e4m3) else 0)
    d_x = binding.to_device(x, cfg.dtype, dev)
    # rows per local slot (for the algorithmic byte count): copy q of expert e gets the
    # tokens i < n with i mod c == q
    seen, slot_rows = {}, []
    for p, e in enumerate(lay["slot_expert"]):
        q = seen.get(int(e), 0)
        seen[int(e)] = q + 1
        n, c = int(counts[e]), int(lay["copies"][e])
        if lay["rank_slot_off"][rank] <= p < lay["rank_slot_off"][rank + 1]:
            slot_rows.append((n - q + c - 1) // c if n > q else 0)
    return dict(cfg=cfg, layer=layer, plan=plan, plan_ms=plan_ms, lay=lay, rank=rank, rows=rows, slots=slots,
                slot_rows=slot_rows, fwd=fwd, x=d_x, logits=d_logits, host_x=x,
                host_logits=logits, host_w=host_w)


def setup_stack(dev="cuda:0", packed=True, e4m3=False):
    """The multi-layer stack: routing traces of 58 layers x 256 experts (32768 tokens per layer,
    profiling batches of 4096) -> craft_expert_load on the GPU -> craft_plan at 256 replicas over
    32 ranks; then the four executed layers (largest, smallest and the two tercile Zipf
    exponents), DeepSeek-V3-shaped at T = 32768, each under its own layer's plan.  Host weights
    are kept for the first layer only (the CPU baseline's sample)."""
    import torch
    from paper_2603_28768_amd import binding, synth
    L, E, K, D, idx = 58, 256, 8, 32, 5
    s = synth.trace_layer_exponents(L, idx)
    ids = np.stack([synth.routing_trace_layer(E, K, 32768, s[l], idx, l) for l in range(L)])
    W = binding.expert_load(torch.from_numpy(ids).to(dev), E, 4096)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plan = binding.Plan(W.cpu().numpy(), D, 256)
    plan_ms = (time.perf_counter() - t0) * 1e3
    by_s = np.argsort(s)
    states = []
    for n, layer in enumerate(int(l) for l in (by_s[-1], by_s[0], by_s[L // 3], by_s[2 * L // 3])):
        cfg = synth.scaled(synth.CONFIGS["dsv3_long"], zipf_s=round(float(s[layer]), 3))
        pop = synth.popularity(E, s[layer], idx, layer)
        st = setup(cfg, dev, packed, e4m3, plan=plan, layer=layer, pop=pop, plan_ms=plan_ms,
                   keep_host_weights=(n == 0))
        if n > 0:
            st["host_x"] = st["host_logits"] = None
        log(f"stack layer {layer}: Zipf s={s[layer]:.2f}, {plan.layer(layer)['n_replicas']} replicas, heaviest rank "
            f"{st['rank']}: {len(st['slots'])} slots, {int(st['rows'][st['rank']])} rows (mean {np.mean(st['rows']):.0f})")
        states.append(st)
    return states


def lay_slots(st):
    return st["lay"]["slot_expert"]


def cpu_baseline(cfg, st, budget_s=15.0):
    """The CPU checker on this host: routing, dispatch and combine on the whole batch, the
    FFN on a sample of the rank's rows sized to about `budget_s` seconds, scaled to all rows."""
    import oracle
    lay, rank, k = st["lay"], st["rank"], cfg.k
    t = time.perf_counter()
    ids, w = oracle.route(st["host_logits"], k)
    t_route = time.perf_counter() - t
    t = time.perf_counter()
    dest, src, cnt, off = oracle.dispatch(ids, cfg.E, lay["slot_expert"])
    t_disp = time.perf_counter() - t
    p_lo, p_hi = lay["rank_slot_off"][rank], lay["rank_slot_off"][rank + 1]
    lo, hi = int(off[p_lo]), int(off[p_hi])
    M = hi - lo
    x = st["host_x"]
    threads = oracle.num_threads()
    # calibrate on a few rows, then take an evenly spaced sample of every slot
    p0 = next(p for p in range(p_lo, p_hi) if cnt[p] > 0)
    Wg, Wu, Wd = st["host_w"][int(lay["slot_expert"][p0])]
    probe = x[src[off[p0]:off[p0] + min(cnt[p0], threads)] // k]
    t = time.perf_counter()
    oracle.ffn_rows(probe, Wg, Wu, Wd)
    per_row = (time.perf_counter() - t) / len(probe)
    stride = max(1, int(np.ceil(M * per_row / budget_s)))
    Y = np.zeros((M, cfg.H))
    done, t_ffn = 0, 0.0
    for p in range(p_lo, p_hi):
        rows = np.arange(int(off[p]), int(off[p + 1]), stride)
        if rows.size == 0:
            continue
        Wg, Wu, Wd = st["host_w"][int(lay["slot_expert"][p])]
        xr = x[src[rows] // k]
        t = time.perf_counter()
        Y[rows - lo] = oracle.ffn_rows(xr, Wg, Wu, Wd)
        t_ffn += time.perf_counter() - t
        done += rows.size
    t = time.perf_counter()
    oracle.combine(Y, lo, dest, w, cfg.T, k)
    t_comb = time.perf_counter() - t
    est = t_route + t_disp + t_ffn * (M / max(done, 1)) + t_comb
    return dict(value=cfg.T / est, unit="tokens/s", cores=threads, kind="oracle",
                sample=f"route+dispatch+combine on all {cfg.T} tokens; FFN on every "
                       f"{stride}-th row of each slot ({done} of {M} rows, {t_ffn:.1f} s), "
                       f"scaled to all rows; fp64 accumulation",
                est_seconds_per_step=est)


def bench_trace_load(args):
    """Secondary workload: craft_expert_load over the multi-layer stack's routing trace
    (58 layers x 2^20 tokens x top-8 of 256 experts, int32, 1.95 GB), resident in HBM.
    The trace is drawn on the device (Gumbel top-k over each layer's Zipf popularity)."""
    import torch
    from paper_2603_28768_amd import binding, synth
    L, E, k, T, bt = 58, 256, 8, 1 << 20, 4096
    s = synth.trace_layer_exponents(L, 5)
    g = torch.Generator(device="cuda").manual_seed(synth.BASE_SEED + 5)
    ids = torch.empty((L, T, k), dtype=torch.int32, device="cuda")
    for l in range(L):
        logp = torch.from_numpy(np.log(synth.popularity(E, s[l], 5, l))).float().cuda()
        for c in range(0, T, 1 << 18):
            u = torch.rand((1 << 18, E), generator=g, device="cuda").clamp_(1e-20, 1.0)
            gum = logp - torch.log(-torch.log(u))
            ids[l, c:c + (1 << 18)] = torch.topk(gum, k, dim=1).indices.to(torch.int32)
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        counts = binding.expert_load(ids, E, bt)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    t0 = time.perf_counter()
    ev[0].record()
    for _ in range(args.steps):
        counts = binding.expert_load(ids, E, bt)
    ev[1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = ev[0].elapsed_time(ev[1]) / args.steps         # kernels run on torch's current stream
    assert int(counts.sum()) == L * T * k
    nbytes = ids.numel() * 4 + counts.numel() * 8
    gbs = nbytes / (ms * 1e-3) / 1e9
    out = dict(metric="expert-load histogram assignments/s on 1 GPU", value=ids.numel() / (dt / args.steps),
               unit="assignments/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=dt / args.steps * 1e3, higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="int32", data="synthetic",
               config=dict(workload=f"routing trace {L} layers x {T} tokens x top-{k} of {E} experts, "
                                    f"Zipf s in [0.6,1.6], batches of {bt} tokens"),
               roofline=dict(bound="hbm", achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s",
                             frac=gbs / HBM_PEAK_GBS, traffic=None, kernel="expert_load_kernel",
                             avg_ms=ms, algorithmic_bytes=nbytes))
    print(json.dumps(out), flush=True)


def bench_gate(args, name):
    """Secondary workload: craft_router_logits (the linear gating network) at the shape of a
    layer configuration, activations and gate weights resident in HBM."""
    import torch
    from paper_2603_28768_amd import binding, synth
    cfg = synth.CONFIGS[name]
    g = torch.Generator(device="cuda").manual_seed(synth.BASE_SEED + 11)
    x = torch.randn((cfg.T, cfg.H), generator=g, device="cuda").to(torch.bfloat16)
    w = (torch.randn((cfg.E, cfg.H), generator=g, device="cuda") / math.sqrt(cfg.H)).to(torch.bfloat16)
    ws = binding.router_logits_workspace(x, w)           # partial scores of the split contraction
    for _ in range(args.warmup):
        logits = binding.router_logits(x, w, ws)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    t0 = time.perf_counter()
    ev[0].record()
    for _ in range(args.steps):
        logits = binding.router_logits(x, w, ws)
    ev[1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = ev[0].elapsed_time(ev[1]) / args.steps         # the kernel runs on torch's current stream
    assert bool(torch.isfinite(logits).all())
    nbytes = x.numel() * 2 + w.numel() * 2 + logits.numel() * 4
    flops = 2.0 * cfg.T * cfg.H * cfg.E
    gbs = nbytes / (ms * 1e-3) / 1e9
    out = dict(metric="gating-network tokens/s on 1 GPU", value=cfg.T / (dt / args.steps), unit="tokens/s",
               n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=dt / args.steps * 1e3,
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="bf16", data="synthetic",
               config=dict(workload=f"linear gate at the {name} shape: T={cfg.T} H={cfg.H} E={cfg.E}"),
               roofline=dict(bound="hbm", achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s",
                             frac=gbs / HBM_PEAK_GBS, traffic=None, kernel="router_logits_bf16_kernel",
                             avg_ms=ms, algorithmic_bytes=nbytes, algorithmic_flops=flops,
                             achieved_tflops=flops / (ms * 1e-3) / 1e12))
    print(json.dumps(out), flush=True)


def copy_calibration(args):
    """A plain 256 MiB device-to-device copy (the library's craft_probe_copy): the known-size
    kernel against which the FETCH_SIZE / WRITE_SIZE counters are scaled."""
    import torch
    from paper_2603_28768_amd import binding
    n = 256 << 20
    a = torch.ones(n, dtype=torch.uint8, device="cuda")
    b = torch.empty_like(a)
    for _ in range(3):
        binding.probe_copy(a, b)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for _ in range(args.steps):
        binding.probe_copy(a, b)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / args.steps
    print(json.dumps(dict(metric="device copy GB/s (read+write)", value=2 * n / (ms * 1e-3) / 1e9,
                          unit="GB/s", bytes_read=n, bytes_written=n, ms_per_step=ms)), flush=True)


# HBM traffic of the gate/up kernel per launch from rocprofv3 counters (profiles/
# rank_forward_<workload>_hbm_traffic.txt): FETCH_SIZE and WRITE_SIZE in KiB per dispatch (mean
# over the workload's launches), scaled by what the same counters read for a plain 256 MiB copy
# (x2.0 and x1.0).  A figure belongs to the kernel as it was when the counters were taken: it
# is reported only while the sources that shape that kernel still hash to the recorded value.
TRAFFIC_SOURCES = ["ffn_packed.hip", "ffn_common.h", "kernels.h", "dispatch.hip", "forward.cpp"]
_SHA = "c6e7b191b0bbc814dfb8e6b622d42f906ad8151d31b6f5a521d7ceaf97410647"
TRAFFIC = {
    "qwen3": dict(fetch_kib=286706.9, write_kib=13510.0, fetch_scale=2.0, write_scale=1.0, mfma_util=0.42, mfma_busy_of_peak_clock=0.38, l2_to_cu_mb=1296.4, l2_hit=0.551, sources_sha256=_SHA),
    "dsv3": dict(fetch_kib=195037.7, write_kib=10241.0, fetch_scale=2.0, write_scale=1.0, mfma_util=0.555, mfma_busy_of_peak_clock=0.477, l2_to_cu_mb=1545.1, l2_hit=0.74, sources_sha256=_SHA),
    "kimi": dict(fetch_kib=163133.8, write_kib=10827.0, fetch_scale=2.0, write_scale=1.0, mfma_util=0.504, mfma_busy_of_peak_clock=0.44, l2_to_cu_mb=1413.5, l2_hit=0.762, sources_sha256=_SHA),
    "stack": dict(fetch_kib=1050833.3, write_kib=75816.1, fetch_scale=2.0, write_scale=1.0, mfma_util=0.719, mfma_busy_of_peak_clock=0.55, l2_to_cu_mb=8925.2, l2_hit=0.749, sources_sha256=_SHA),
}


def kernel_sources_sha256():
    h = hashlib.sha256()
    csrc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2603_28768_amd", "csrc")
    for name in TRAFFIC_SOURCES:
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(cfg_name, packed):
    t = TRAFFIC.get(cfg_name)
    if t is None or not packed or t["sources_sha256"] != kernel_sources_sha256():
        return None
    return (t["fetch_kib"] * t["fetch_scale"] + t["write_kib"] * t["write_scale"]) * 1024.0


def measured_counters(cfg_name, packed):
    """The gate/up kernel's matrix-core and L2 counters from profiles/rank_forward_<workload>_
    mfma_l2_counters.txt, under the same condition as the traffic figure."""
    t = TRAFFIC.get(cfg_name)
    if t is None or not packed or t["sources_sha256"] != kernel_sources_sha256() or "mfma_util" not in t:
        return None
    return dict(mfma_util=t["mfma_util"], mfma_busy_of_peak_clock=t["mfma_busy_of_peak_clock"],
                l2_to_cu_bytes=t["l2_to_cu_mb"] * 1e6, l2_hit=t["l2_hit"],
                what="rocprofv3 counters of the gate/up kernel per launch: MfmaUtil = SQ_VALU_MFMA_BUSY_CYCLES / "
                     "(GRBM_GUI_ACTIVE per XCD x 1024 SIMDs); the same busy cycles over the cycles of the launch "
                     "at 2.4 GHz; TCP_TCC_READ_REQ x 128 B; TCC_HIT / TCC_REQ")


def machine_rates(steps=10):
    """This machine's own ceilings, measured with the library's probes on the current stream: a
    plain 256 MiB copy (bytes read + written per second) and a register-only bf16 MFMA loop."""
    import torch
    from paper_2603_28768_amd import binding
    n = 256 << 20
    a = torch.ones(n, dtype=torch.uint8, device="cuda")
    b = torch.empty_like(a)
    sink = torch.empty(8 * 1024 * 256, dtype=torch.float32, device="cuda")
    isink = torch.empty(8 * 1024 * 256, dtype=torch.int32, device="cuda")
    small = torch.ones(2 << 20, dtype=torch.uint8, device="cuda")     # fits every XCD's L2
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(10)]
    for _ in range(3):
        binding.probe_copy(a, b)
        binding.probe_mfma_bf16(2000, sink)
        binding.probe_read(small, 2, isink)
    torch.cuda.synchronize()
    ev[4].record()
    l2_bytes = 0.0
    for _ in range(steps):
        l2_bytes += binding.probe_read(small, 8, isink)
    ev[5].record()
    ev[0].record()
    for _ in range(steps):
        binding.probe_copy(a, b)
    ev[1].record()
    ev[2].record()
    flops = 0.0
    for _ in range(steps):
        flops += binding.probe_mfma_bf16(20000, sink)
    ev[3].record()
    # the same matrix work on operands with random signs and mantissas, in the shape the FFN
    # uses (16x16x32) and in the other one: what the power the matrix pipelines draw leaves
    rnd = []
    for n_ev, shape in ((6, 1), (8, 0)):
        binding.probe_mfma_operands(shape, 2, 2000, sink)
        ev[n_ev].record()
        fl = sum(binding.probe_mfma_operands(shape, 2, 30000, sink) for _ in range(2))
        ev[n_ev + 1].record()
        rnd.append(fl)
    torch.cuda.synchronize()
    assert bool((b == 1).all())
    return dict(copy_gbs=2.0 * n * steps / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9,
                mfma_bf16_tflops=flops / (ev[2].elapsed_time(ev[3]) * 1e-3) / 1e12,
                mfma_bf16_random_operands_16x16x32_tflops=rnd[0] / (ev[6].elapsed_time(ev[7]) * 1e-3) / 1e12,
                mfma_bf16_random_operands_32x32x16_tflops=rnd[1] / (ev[8].elapsed_time(ev[9]) * 1e-3) / 1e12,
                l2_read_gbs=l2_bytes / (ev[4].elapsed_time(ev[5]) * 1e-3) / 1e9)


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def ffn_work(st, wes):
    """Algorithmic work of one state's expert FFN: per GEMM (bytes, flops), and the two bounds of
    the pair over the rank's slots p with c_p rows: sum_p max(flops_p / MFMA peak, bytes_p / HBM
    peak) (nothing overlaps between slots) and max(sum flops / peak, sum bytes / peak)."""
    cfg = st["cfg"]
    es = 2 if cfg.dtype == "bf16" else 4
    H, I = cfg.H, cfg.I
    M = int(st["rows"][st["rank"]])
    live = sum(1 for r in st["slot_rows"] if r > 0)
    flop_peak = (MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else FP32_VALU_PEAK_TFLOPS) * 1e12
    gu = (live * 2 * H * I * wes + M * H * es + M * I * es, 4.0 * H * I * M)
    dn = (live * H * I * wes + M * I * es + M * H * es, 2.0 * H * I * M)
    no_overlap = 0.0
    for c in st["slot_rows"]:
        if c > 0:
            no_overlap += max(6.0 * H * I * c / flop_peak,
                              (3 * H * I * wes + c * (2 * H + 2 * I) * es) / (HBM_PEAK_GBS * 1e9))
    perfect = max((gu[1] + dn[1]) / flop_peak, (gu[0] + dn[0]) / (HBM_PEAK_GBS * 1e9))
    return dict(M=M, live=live, gateup=gu, down=dn, no_overlap_s=no_overlap, perfect_overlap_s=perfect)


def kernel_work(st, wes):
    """Algorithmic (bytes, flops) per launch of every kernel of one state's forward."""
    cfg = st["cfg"]
    es = 2 if cfg.dtype == "bf16" else 4
    f = ffn_work(st, wes)
    A, S = cfg.T * cfg.k, len(lay_slots(st))
    NB = (cfg.T + 31) // 32
    M = f["M"]
    return dict(route=(cfg.T * cfg.E * 4 + A * 9 + NB * cfg.E * 4, 0.0),
                scan=(2 * NB * cfg.E * 4 + S * 16, 0.0),
                dispatch=(A * 9 + A * 8, 0.0),
                gateup=f["gateup"], down=f["down"],
                combine=(M * cfg.H * es + cfg.T * cfg.H * es + A * 8, 0.0))


def plan_curves(args):
    """Balancedness against replica budget on the stack-shaped loads (58 layers x 256
    experts, 32 ranks, per-layer Zipf exponents in [0.6, 1.6]) for the three allocation rules
    of craft_plan: the paper's pipeline (Alg. 1 + Alg. 2), the unit greedy and even spreading
    (R = L is uniform replication).  Host only; prints one JSON line."""
    from paper_2603_28768_amd import binding, synth
    L, E, D, B = 58, 256, 32, 4
    s = synth.trace_layer_exponents(L, 5)
    g = np.random.default_rng(5)
    W = np.stack([[g.multinomial(8 * 4096, synth.popularity(E, s[l], 5, l)) for l in range(L)]
                  for _ in range(B)]).astype(np.int64)

    def mean_bal(p):
        return float(np.mean([p.layer(l)["est_balancedness"] for l in range(L)]))

    rows = []
    for R in (0, 1, 2, 4, 8, 16, 32, 58):
        row = {"R": R}
        for name, obj in (("paper", 1), ("greedy", 0), ("spread", 2)):
            t0 = time.perf_counter()
            p = binding.Plan(W, D, R * D, objective=obj)
            row[name] = round(mean_bal(p), 4)
            row[name + "_ms"] = round((time.perf_counter() - t0) * 1e3, 2)
        rows.append(row)
        log(str(row))
    auto = binding.Plan(W, D, L * D, objective=1, auto_r=True).benefit()["auto_R"]
    print(json.dumps({"metric": "mean estimated balancedness vs replication factor", "L": L, "E": E,
                      "D": D, "profiling_batches": B, "curves": rows, "auto_R": int(auto)}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="stack",
                    help="stack (default: plan over 58 layers, four T=32768 layers executed) | "
                         "tiny | qwen3 | dsv3 | kimi | dsv3_long | trace_load (histogram only) | "
                         "gate_qwen3 | gate_dsv3 | gate_kimi (gating network only) | "
                         "copy_calib (plain copy for counter calibration) | "
                         "plan_curves (host only: balancedness vs budget for the three planners)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--unpacked", action="store_true",
                    help="run the FFN on row-major weights (LDS-staged kernels) instead of packed ones")
    ap.add_argument("--weights", default="bf16", choices=["bf16", "e4m3"],
                    help="storage of the packed expert weights: bf16, or E4M3 codes with a scale per row")
    ap.add_argument("--tile-rows", type=int, nargs=2, default=[0, 0], metavar=("GATEUP", "DOWN"),
                    help="row-tile heights of the two packed GEMMs (128..256 in steps of 32; 0 = the library's choice)")
    ap.add_argument("--riders", type=int, nargs=2, default=[0, 0], metavar=("GATEUP", "DOWN"),
                    help="cold slots riding on busy tiles: 1 on, -1 off, 0 = the library's choice")
    ap.add_argument("--timing-level", type=int, default=1,
                    help="inside the timed region: 1 = HIP events around the gate/up GEMM only, "
                         "2 = around every kernel (a second, untimed pass always brackets every kernel)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py measures one GPU's share (the heaviest simulated rank); "
            "--gpus above 1 is not supported: there are no collectives here")
        sys.exit(2)

    import torch                        # before the library: both must share one HIP runtime
    from paper_2603_28768_amd import binding, synth
    binding.lib()                       # fail loudly if the HIP library is missing
    if args.config == "plan_curves":
        return plan_curves(args)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.config == "trace_load":
        return bench_trace_load(args)
    if args.config == "copy_calib":
        return copy_calibration(args)
    if args.config.startswith("gate_"):
        return bench_gate(args, args.config[5:])
    e4m3 = args.weights == "e4m3"
    packed = not args.unpacked
    if args.config == "stack":
        states = setup_stack(packed=packed, e4m3=e4m3)
    else:
        cfg = synth.CONFIGS[args.config]
        if e4m3:
            assert cfg.dtype == "bf16" and packed, "E4M3 weights go with the packed bf16 path"
        states = [setup(cfg, packed=packed, e4m3=e4m3)]
    cfg = states[0]["cfg"]
    packed = packed and cfg.dtype == "bf16"
    for st in states:
        fa = st["fwd"].args
        fa.tile_rows_gateup, fa.tile_rows_down = args.tile_rows
        fa.riders_gateup, fa.riders_down = args.riders
    for st in states:
        c = st["cfg"]
        log(f"config {c.name} layer {st['layer']}: T={c.T} H={c.H} I={c.I} E={c.E} k={c.k} D={c.D}; "
            f"heaviest rank {st['rank']} holds {len(st['slots'])} slots, {int(st['rows'][st['rank']])} rows "
            f"(mean {np.mean(st['rows']):.0f}); plan {st['plan_ms']:.2f} ms; tiles {st['fwd'].tile_choice()}")

    def one_step():
        for st in states:
            st["fwd"](st["x"], st["logits"])

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    binding.timing_enable(args.timing_level, args.steps * len(states))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    times = binding.timing_read()
    binding.timing_enable(0, 0)
    for st in states:
        rows, ovf = st["fwd"].result()
        assert ovf == 0 and rows == int(st["rows"][st["rank"]]), (rows, ovf)
    # a second, short pass with every kernel bracketed by events (outside the timed region: the
    # events between kernels cost a few microseconds each)
    side_steps = max(3, min(20, args.steps))
    binding.timing_enable(2, side_steps * len(states))
    for _ in range(side_steps):
        one_step()
    torch.cuda.synchronize()
    all_times = binding.timing_read()
    binding.timing_enable(0, 0)
    rates = machine_rates()

    ms_step = dt / args.steps * 1e3
    wes = 1 if e4m3 else (2 if cfg.dtype == "bf16" else 4)        # bytes per stored weight
    work = [ffn_work(st, wes) for st in states]
    n_l = len(states)
    tokens = sum(st["cfg"].T for st in states)
    M_all = sum(w["M"] for w in work)
    # dominant kernel: the grouped gate/up GEMM; work per launch = mean over the executed layers
    gu_ms = times["gateup"]["ms"] / max(times["gateup"]["launches"], 1)
    gu_bytes = sum(w["gateup"][0] for w in work) / n_l
    gu_flops = sum(w["gateup"][1] for w in work) / n_l
    gbs = gu_bytes / (gu_ms * 1e-3) / 1e9
    tfs = gu_flops / (gu_ms * 1e-3) / 1e12
    flop_peak = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else FP32_VALU_PEAK_TFLOPS
    traffic = measured_traffic(args.config, packed and not e4m3)             # bytes per launch
    t_hbm, t_mfma = gu_bytes / (HBM_PEAK_GBS * 1e9), gu_flops / (flop_peak * 1e12)
    if t_hbm >= t_mfma:
        roof = dict(bound="hbm", achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=gbs / HBM_PEAK_GBS, traffic=traffic)
    else:
        roof = dict(bound="mfma" if cfg.dtype == "bf16" else "alu", achieved=tfs, peak=flop_peak,
                    unit="TFLOP/s", frac=tfs / flop_peak, traffic=traffic)
    roof.update(counters=measured_counters(args.config, packed and not e4m3))
    roof.update(kernel="grouped gate/up GEMM + SwiGLU", avg_ms=gu_ms,
                launches=times["gateup"]["launches"], algorithmic_bytes=gu_bytes,
                algorithmic_flops=gu_flops, hbm_frac=gbs / HBM_PEAK_GBS, flop_frac=tfs / flop_peak,
                achieved_gbs=gbs, achieved_tflops=tfs)
    # every kernel of the forward from the second pass: mean duration per launch, algorithmic
    # bytes (and flops) per launch, fractions of the published peaks
    kms = {k: v["ms"] / max(v["launches"], 1) for k, v in all_times.items() if v["launches"]}
    per = [kernel_work(st, wes) for st in states]
    kernels = {}
    for name in ("route", "scan", "dispatch", "gateup", "down", "combine"):
        if name not in kms:
            continue
        b = sum(p_[name][0] for p_ in per) / n_l
        f = sum(p_[name][1] for p_ in per) / n_l
        d = dict(ms=kms[name], algorithmic_bytes=b, gbs=b / (kms[name] * 1e-3) / 1e9)
        d["hbm_frac"] = d["gbs"] / HBM_PEAK_GBS
        if f:
            d["tflops"] = f / (kms[name] * 1e-3) / 1e12
            d["flop_frac"] = d["tflops"] / flop_peak
        kernels[name] = d
    ffn_ms = kms.get("gateup", 0.0) + kms.get("down", 0.0)
    no_ov = sum(w["no_overlap_s"] for w in work) / n_l * 1e3
    perfect = sum(w["perfect_overlap_s"] for w in work) / n_l * 1e3
    roof.update(kernels=kernels,
                ffn_bounds=dict(what="gate/up + down of one layer's rank share against the published peaks: "
                                     "sum over slots of max(6HI c_p / MFMA peak, (3HI + c_p(2H+2I)) es / HBM peak), "
                                     "and max(sum flops / peak, sum bytes / peak)",
                                no_overlap_ms=no_ov, perfect_overlap_ms=perfect, measured_ms=ffn_ms,
                                frac_of_no_overlap=no_ov / ffn_ms if ffn_ms else None,
                                frac_of_perfect_overlap=perfect / ffn_ms if ffn_ms else None),
                machine=dict(copy_gbs=rates["copy_gbs"], mfma_bf16_tflops=rates["mfma_bf16_tflops"],
                             mfma_bf16_random_operands_16x16x32_tflops=rates["mfma_bf16_random_operands_16x16x32_tflops"],
                             mfma_bf16_random_operands_32x32x16_tflops=rates["mfma_bf16_random_operands_32x32x16_tflops"],
                             l2_read_gbs=rates["l2_read_gbs"],
                             frac_of_measured_copy=gbs / rates["copy_gbs"],
                             frac_of_measured_mfma=tfs / rates["mfma_bf16_tflops"],
                             frac_of_measured_mfma_random_operands=tfs / rates["mfma_bf16_random_operands_16x16x32_tflops"],
                             what="craft_probe_copy of 256 MiB (bytes read + written per second), "
                                  "craft_probe_mfma_bf16 (register-only v_mfma_f32_32x32x16_bf16 loop on small integers), "
                                  "craft_probe_mfma_operands (register-only loops of either MFMA shape on operands with "
                                  "random signs and mantissas: the rate the chip's power limit leaves on data like the "
                                  "FFN's; the FFN uses 16x16x32) and "
                                  "craft_probe_read (every workgroup re-reading a 2 MiB buffer out of L2) on this GPU"))

    if len(states) == 1:
        workload = (f"{cfg.name}: T={cfg.T} H={cfg.H} E={cfg.E} top-{cfg.k} I={cfg.I} Zipf s={cfg.zipf_s}, "
                    f"{cfg.D} simulated ranks, {cfg.replica_slots} replica slots; heaviest rank's share")
    else:
        workload = (f"stack: routing traces of 58 layers x 256 experts (Zipf s in [0.6,1.6]) -> GPU histogram -> "
                    f"plan at 256 replicas over {cfg.D} simulated ranks; {n_l} executed layers "
                    f"(T={cfg.T} H={cfg.H} E={cfg.E} top-{cfg.k} I={cfg.I}) each under its own layer's plan; "
                    f"heaviest rank's share of every layer; a step is all {n_l} layers, tokens/s counts "
                    f"T per layer")
    out = dict(metric="MoE rank-forward tokens/s on 1 GPU", value=tokens / (ms_step * 1e-3),
               unit="tokens/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=ms_step, higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype=cfg.dtype, data="synthetic",
               config=dict(workload=workload,
                           layers=[dict(layer=int(st["layer"]), zipf_s=st["cfg"].zipf_s, rank=int(st["rank"]),
                                        rank_slots=len(st["slots"]), rank_rows=w["M"],
                                        replicas=int(st["lay"]["n_replicas"]),
                                        tiles=list(st["fwd"].tile_choice()),
                                        balancedness_realized=float(np.mean(st["rows"]) / np.max(st["rows"])))
                                   for st, w in zip(states, work)],
                           rank_rows=M_all, rows_per_s=M_all / (ms_step * 1e-3), plan_ms=states[0]["plan_ms"],
                           weights=("E4M3 codes + row scales, packed at load" if e4m3 else "packed at load")
                           if packed else "row-major"),
               roofline=roof)
    if not args.no_cpu_baseline:
        base = cpu_baseline(states[0]["cfg"], states[0])
        base["cpu_model"] = cpu_model()
        base["build"] = "gcc -O2 -fopenmp, one thread per row of a slot"
        if n_l > 1:
            base["sample"] = f"layer {states[0]['layer']} of the {n_l} executed layers: " + base["sample"]
        out["cpu_baseline"] = base
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
