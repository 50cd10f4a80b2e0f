"""GPU parity: the HIP path, called through the C ABI, against the CPU checker on the same
seeded inputs.  Integer results (ids, counts, dispatch indices) are compared bit for bit;
gate weights to 1e-5 relative; the layer output to max|gpu-ref| <= tol * max|ref| with
tol = 1e-2 for bf16 storage (fp32 accumulation) and 1e-4 for fp32 storage."""

import numpy as np
import pytest

import oracle
from paper_2603_28768_amd import binding, synth

from cases import Case

pytestmark = pytest.mark.gpu

TOL = {"bf16": 1e-2, "f32": 1e-4}


def _np(t):
    return t.detach().float().cpu().numpy() if t.dtype.is_floating_point else t.detach().cpu().numpy()


# ----------------------------------------------------------------------- route

@pytest.mark.parametrize("T,E,k,quantum,renorm", [
    (256, 16, 2, None, True), (1000, 128, 8, None, True), (333, 256, 8, None, False),
    (97, 384, 8, None, True), (64, 100, 5, 0.5, True), (40, 7, 7, 1.0, False),
    (33, 1, 1, None, True), (31, 1000, 64, 0.25, True), (4096, 128, 8, None, True)])
def test_route_parity(torch_cuda, T, E, k, quantum, renorm):
    torch = torch_cuda
    print(f"route T={T} E={E} k={k} quantum={quantum} renorm={renorm}", flush=True)
    g = np.random.default_rng(T * 131 + E)
    l = (g.standard_normal((T, E)) * 2).astype(np.float32)
    if quantum:
        l = (np.round(l / quantum) * quantum).astype(np.float32)      # many exact ties
    ids, w = binding.route_topk(torch.from_numpy(l).cuda(), k, renorm)
    torch.cuda.synchronize()
    rid, rw = oracle.route(l, k, renorm)
    assert np.array_equal(_np(ids), rid)
    assert np.allclose(_np(w), rw, rtol=1e-5, atol=1e-30)


def test_route_reads_scores_that_are_not_16_byte_aligned(torch_cuda):
    # E % 4 == 0 lets the kernel read rows 16 bytes at a time, but only from a 16-byte aligned
    # base: a score matrix that starts 4 bytes into an allocation is read score by score
    torch = torch_cuda
    T, E, k = 300, 128, 8
    g = np.random.default_rng(77)
    l = (g.standard_normal((T, E)) * 2).astype(np.float32)
    flat = torch.empty(T * E + 1, dtype=torch.float32, device="cuda:0")
    view = flat[1:].view(T, E)
    view.copy_(torch.from_numpy(l))
    assert view.data_ptr() % 16 == 4 and view.is_contiguous()
    ids, w = binding.route_topk(view, k)
    rid, rw = oracle.route(l, k)
    assert np.array_equal(_np(ids), rid)
    assert np.allclose(_np(w), rw, rtol=1e-5, atol=1e-30)


# ---------------------------------------------------------------------- probes

def test_measurement_probes(torch_cuda):
    # the kernels of known work behind the benchmark's machine rates: the copy copies, the
    # other two run and report the work they were asked for
    torch = torch_cuda
    g = torch.Generator(device="cuda").manual_seed(3)
    a = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device="cuda:0", generator=g)
    b = torch.zeros_like(a)
    binding.probe_copy(a, b)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    sink = torch.zeros(4 * 256, dtype=torch.float32, device="cuda:0")
    assert binding.probe_mfma_bf16(10, sink, blocks=4) == 4 * 4 * 10 * 4 * 2 * 32 * 32 * 16
    isink = torch.zeros(4 * 256, dtype=torch.int32, device="cuda:0")
    small = torch.full((64 << 10,), 3, dtype=torch.uint8, device="cuda:0")
    assert binding.probe_read(small, 3, isink, blocks=4) == 4 * 3 * (64 << 10)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(sink).all())
    # every thread XORs the same number of equal words: an even count cancels
    assert int(isink.abs().sum()) == 0
    with pytest.raises(binding.CraftError):
        binding.probe_read(small[:1000], 1, isink, blocks=4)          # not a multiple of 32 KiB


# ------------------------------------------------------------------------ load

@pytest.mark.parametrize("L,T,k,E,bt", [
    (1, 256, 2, 16, 256), (3, 1000, 8, 128, 256), (2, 17, 3, 9, 5), (2, 9000, 8, 256, 4500),
    (1, 20000, 8, 384, 20000), (4, 4096, 8, 4096, 1024), (1, 7, 1, 1, 2)])
def test_expert_load_parity(torch_cuda, L, T, k, E, bt):
    torch = torch_cuda
    print(f"load L={L} T={T} k={k} E={E} bt={bt}", flush=True)
    g = np.random.default_rng(L * 7 + T)
    pop = synth.popularity(E, 1.3, 0)
    ids = g.choice(E, size=(L, T, k), p=pop).astype(np.int32)
    got = binding.expert_load(torch.from_numpy(ids).cuda(), E, bt)
    torch.cuda.synchronize()
    want = oracle.expert_load(ids, E, bt)
    assert np.array_equal(_np(got), want)


def test_expert_load_on_a_zipf_trace(torch_cuda):
    # the multi-layer stack's trace shape at reduced length: 58 layers x 256 experts, top-8
    torch = torch_cuda
    L, E, k, T, bt = 58, 256, 8, 8192, 4096
    s = synth.trace_layer_exponents(L, 5)
    ids = np.stack([synth.routing_trace_layer(E, k, T, s[l], 5, l) for l in range(L)])
    print("zipf trace", ids.shape, flush=True)
    got = _np(binding.expert_load(torch.from_numpy(ids).cuda(), E, bt))
    torch.cuda.synchronize()
    want = oracle.expert_load(ids, E, bt)
    assert np.array_equal(got, want)
    assert np.all(got.sum(-1) == bt * k)


# ------------------------------------------------------------- gating network

# fp32 accumulation of H products against the checker's double sum: the running sum stays of
# the size of the scores (a few units), each of the H/16 accumulator updates rounds it at
# 2^-24 relative, so the error is a few 1e-7 of the score scale in practice and H * 2^-24 of
# it at the very worst; 1e-4 of the largest score leaves room for both and is still a
# hundred times finer than a dropped or doubled term.
GATE_TOL = 1e-4


@pytest.mark.parametrize("dtype,T,H,E", [
    ("bf16", 100, 72, 5),            # one ragged block of experts, ragged tokens and slab
    ("bf16", 517, 520, 24),
    ("bf16", 96, 256, 130),          # two blocks per wave
    ("bf16", 70, 128, 384),          # three
    ("bf16", 40, 64, 512),           # four
    ("bf16", 33, 8, 1000),           # eight, a single 16-byte chunk per row
    ("bf16", 33000, 64, 128),        # workgroups to spare: two token fragments each
    ("bf16", 300, 2048, 200),        # with a workspace: the contraction split eight ways
    ("bf16", 200, 1000, 100),        # split, ragged last slab and a last split shorter than the rest
    ("bf16", 200, 1024, 384),        # split with three blocks of experts per wave
    ("f32", 50, 100, 12)])
def test_router_logits_parity(torch_cuda, dtype, T, H, E):
    cfg = synth.scaled(synth.CONFIGS["qwen3"], dtype=dtype, T=T, H=H, E=E)
    x, W = synth.activations(cfg), synth.gate_weights(cfg)
    xd, Wd = binding.to_device(x, dtype), binding.to_device(W, dtype)
    want = oracle.router_logits(x, W)
    U = np.zeros((E, H), dtype=np.float32)
    U[np.arange(E), np.arange(E) % H] = 1.0
    Ud = binding.to_device(U, dtype)
    ws = binding.router_logits_workspace(xd, Wd)
    print(f"  gate {dtype} T={T} H={H} E={E}: workspace {0 if ws is None else ws.numel()} bytes", flush=True)
    for workspace in ([None] if ws is None else [None, ws]):    # one workgroup per tile / split contraction
        got = _np(binding.router_logits(xd, Wd, workspace))
        assert got.shape == want.shape == (T, E)
        err = np.abs(got.astype(np.float64) - want).max()
        print(f"    max|ref|={np.abs(want).max():.3g} max|err|={err:.3g}", flush=True)
        assert err <= GATE_TOL * np.abs(want).max()
        # sums of a single term are exact: a gate of unit rows copies columns of x
        got = _np(binding.router_logits(xd, Ud, workspace))
        assert np.array_equal(got, x[:, np.arange(E) % H])
        # and the result depends on the arguments only
        assert np.array_equal(_np(binding.router_logits(xd, Wd, workspace)), _np(binding.router_logits(xd, Wd, workspace)))


def test_router_logits_empty_and_rejected(torch_cuda):
    torch = torch_cuda
    x = torch.zeros((0, 64), dtype=torch.bfloat16, device="cuda:0")
    W = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda:0")
    assert tuple(binding.router_logits(x, W).shape) == (0, 8)
    with pytest.raises(binding.CraftError):                       # bf16 rows must be whole 16-byte chunks
        binding.router_logits(torch.zeros((4, 12), dtype=torch.bfloat16, device="cuda:0"),
                              torch.zeros((8, 12), dtype=torch.bfloat16, device="cuda:0"))
    with pytest.raises(binding.CraftError):                       # more experts than the router takes
        binding.router_logits(torch.zeros((4, 8), dtype=torch.bfloat16, device="cuda:0"),
                              torch.zeros((1025, 8), dtype=torch.bfloat16, device="cuda:0"))


@pytest.mark.parametrize("name", ["qwen3", "kimi"])
def test_router_logits_full_size_feeds_the_router(torch_cuda, name):
    # full shapes; the checker affords a sample of the tokens.  The top-k decision is taken by
    # both sides on the same fp32 scores (the library's): ids bit-exact.
    torch = torch_cuda
    cfg = synth.CONFIGS[name]
    x, W = synth.activations(cfg), synth.gate_weights(cfg)
    xd, Wd = binding.to_device(x, cfg.dtype), binding.to_device(W, cfg.dtype)
    logits = binding.router_logits(xd, Wd, binding.router_logits_workspace(xd, Wd))
    toks = np.random.default_rng(5).choice(cfg.T, size=192, replace=False)
    toks = np.concatenate([toks, [0, cfg.T - 1]])
    want = oracle.router_logits(x[toks], W)
    got = _np(logits)
    err = np.abs(got[toks].astype(np.float64) - want).max()
    print(f"  gate {name}: max|ref|={np.abs(want).max():.3g} max|err|={err:.3g}", flush=True)
    assert err <= GATE_TOL * np.abs(want).max()
    ids, w = binding.route_topk(logits, cfg.k)
    ref_ids, ref_w = oracle.route(got, cfg.k)
    assert np.array_equal(_np(ids), ref_ids)
    assert np.allclose(_np(w), ref_w, rtol=1e-5, atol=1e-30)


@pytest.mark.parametrize("dtype,T,H,I,E,k,D,slots", [
    ("bf16", 600, 512, 384, 32, 4, 4, 4),
    ("bf16", 300, 2048, 64, 24, 2, 2, 2),        # the gate's contraction is split
    ("f32", 200, 96, 64, 12, 3, 2, 2)])
def test_forward_with_its_own_gating_network(torch_cuda, dtype, T, H, I, E, k, D, slots):
    # scores not handed in: the forward runs the gate first.  Its scores are the ones the
    # stand-alone call gives (same kernels, same workspace rule), and every decision after
    # them is taken on those fp32 scores by library and checker alike.
    torch = torch_cuda
    cfg = synth.scaled(synth.CONFIGS["qwen3"], dtype=dtype, T=T, H=H, I=I, E=E, k=k, D=D,
                       replica_slots=slots, zipf_s=1.2, profile_batches=2)
    case = Case(cfg)
    Wr = synth.gate_weights(cfg)
    Wrd = binding.to_device(Wr, dtype)
    packed = dtype == "bf16"
    for rank in range(D):
        own, x, _ = case.gpu_rank(rank, packed=packed, w_router=Wrd)
        out_own = own(x).clone()
        ids_own = own.debug["ids"].clone()
        logits = binding.router_logits(x, Wrd, binding.router_logits_workspace(x, Wrd))
        given, _, _ = case.gpu_rank(rank, packed=packed)
        out_given = given(x, logits)
        torch.cuda.synchronize()
        assert torch.equal(ids_own, given.debug["ids"]) and torch.equal(out_own, out_given)
        scores = _np(logits)
        want = oracle.router_logits(case.x, Wr)
        assert np.abs(scores - want).max() <= GATE_TOL * np.abs(want).max()
        ref = oracle.rank_forward(case.x, scores, cfg.k, case.slot_expert, case.rank_slot_off, rank,
                                  case.weights_of, True, None)
        assert np.array_equal(_np(ids_own), ref["ids"])
        assert np.array_equal(_np(own.debug["dest"]).reshape(-1), ref["dest"])
        assert own.result() == (ref["rows"], 0)
        err = np.abs(_np(out_own).astype(np.float64) - ref["out"]).max()
        assert err <= TOL[dtype] * np.abs(ref["out"]).max() + 1e-30


# --------------------------------------------------------------------- forward

def _row_units(case: Case, rank: int, heights):
    """Row ranges [a, b) (positions in the rank's row block) of everything the packed FFN
    schedules as a unit, for both ways a busy slot's fragments may be cut into row-tiles of the
    given heights (full tiles and a remainder, or shared evenly): the first and the last 32-row
    fragment of every row-tile of every slot with more than 64 rows, and every 32-row fragment
    of the slots with at most 64 rows (a tile of their own or a rider on a busy tile)."""
    p_lo, p_hi = case.rank_slot_off[rank], case.rank_slot_off[rank + 1]
    lo = int(case.slot_off[p_lo])
    units = []
    for p in range(p_lo, p_hi):
        a, n = int(case.slot_off[p]) - lo, int(case.slot_cnt[p])
        F = (n + 31) // 32
        if n == 0:
            continue
        if n <= 64:
            units += [(a + 32 * f, a + min(32 * f + 32, n)) for f in range(F)]
            continue
        for h in heights:
            f = h // 32
            m = (F + f - 1) // f
            for cut in ([min(i * f, F) for i in range(m + 1)], [i * F // m for i in range(m + 1)]):
                for f0, f1 in zip(cut[:-1], cut[1:]):
                    units.append((a + 32 * f0, a + min(32 * f0 + 32, n)))
                    units.append((a + 32 * (f1 - 1), a + min(32 * f1, n)))
    return units


def _assert_units_compared(case: Case, rank: int, tokens, heights):
    """Every unit of the FFN's work on this rank has at least one row whose token is among the
    compared ones (all tokens when `tokens` is None)."""
    cfg = case.cfg
    p_lo, p_hi = case.rank_slot_off[rank], case.rank_slot_off[rank + 1]
    lo, hi = int(case.slot_off[p_lo]), int(case.slot_off[p_hi])
    seen = np.zeros(hi - lo, dtype=bool)
    d = case.dest.reshape(cfg.T, cfg.k)
    d = d if tokens is None else d[np.asarray(tokens)]
    d = d[(d >= lo) & (d < hi)]
    seen[d - lo] = True
    units = _row_units(case, rank, heights)
    missed = [u for u in units if not seen[u[0]:u[1]].any()]
    assert units and not missed, missed[:5]
    return len(units)


def _tokens_covering_units(case: Case, rank: int, heights, extra: int = 0):
    """A token for the first and for the last row of every unit (see _row_units), a few tokens
    with no row on the rank, and `extra` random ones."""
    cfg = case.cfg
    lo = int(case.slot_off[case.rank_slot_off[rank]])
    hi = int(case.slot_off[case.rank_slot_off[rank + 1]])
    toks = set()
    for a, b in _row_units(case, rank, heights):
        toks.add(int(case.src[lo + a]) // cfg.k)
        toks.add(int(case.src[lo + b - 1]) // cfg.k)
    d = case.dest.reshape(cfg.T, cfg.k)
    off = np.nonzero(~((d >= lo) & (d < hi)).any(1))[0]
    toks.update(int(t) for t in off[:2])
    if extra:
        toks.update(int(t) for t in np.random.default_rng(1).choice(cfg.T, size=extra, replace=False))
    return sorted(toks)


def _check_rank(torch, case: Case, rank: int, tokens=None, max_rows=0, packed=False, knobs=None, ref=None,
                cover=False):
    """One forward of `rank` through the C ABI against the checker: integer results everywhere,
    the output on `tokens` (None: every token).  `ref`: a checker result for the same rank and
    tokens computed earlier.  `cover`: also assert that the compared tokens reach every
    row-tile, cold slot and rider unit of the two grouped GEMMs as this launch cuts them."""
    cfg = case.cfg
    fwd, x, logits = case.gpu_rank(rank, max_rows, packed=packed)
    for name, value in (knobs or {}).items():          # tuning knobs of the packed FFN
        setattr(fwd.args, name, value)
    if cover:
        rg, rd, ride_g, ride_d = fwd.tile_choice()
        n = _assert_units_compared(case, rank, tokens, sorted({rg, rd}))
        print(f"  rank {rank}: row-tiles of {rg} (gate/up) and {rd} (down) rows, riders {ride_g}/{ride_d}; "
              f"{n} units of work all have compared rows", flush=True)
    out = fwd(x, logits)
    rows, ovf = fwd.result()
    if ref is None:
        ref = case.oracle_rank(rank, tokens)
    d = {k: _np(v) for k, v in fwd.debug.items()}
    assert np.array_equal(d["ids"], ref["ids"])
    assert np.allclose(d["topk_w"], ref["w"], rtol=1e-5, atol=1e-30)
    assert np.array_equal(d["counts"], ref["counts"])
    assert np.array_equal(d["slot_cnt"], ref["slot_cnt"])
    assert np.array_equal(d["slot_off"], ref["slot_off"])
    assert np.array_equal(d["dest"].reshape(-1), ref["dest"])
    assert np.array_equal(d["src"], ref["src"])
    assert rows == ref["rows"] and ovf == 0
    got = _np(out).astype(np.float64)
    if tokens is not None:
        got = got[np.asarray(tokens)]
    scale = np.abs(ref["out"]).max()
    err = np.abs(got - ref["out"]).max()
    print(f"  rank {rank} packed={packed}: rows={rows} max|ref|={scale:.4g} max|err|={err:.3g} "
          f"rel={err / max(scale, 1e-30):.3g}", flush=True)
    assert err <= TOL[cfg.dtype] * scale + 1e-30
    return _np(out).astype(np.float64), ref


def test_tiny_layer_all_ranks(torch_cuda):
    # the tiny fp32 layer: every rank's share executes; their sum is the un-sharded layer
    case = Case(synth.CONFIGS["tiny"])
    cfg = case.cfg
    print("tiny", case.rows, flush=True)
    total = np.zeros((cfg.T, cfg.H))
    ref_total = np.zeros((cfg.T, cfg.H))
    for g in range(cfg.D):
        out, ref = _check_rank(torch_cuda, case, g)
        total += out
        ref_total += ref["out"]
    assert np.abs(total - ref_total).max() <= TOL["f32"] * np.abs(ref_total).max()


@pytest.mark.parametrize("dtype,T,H,I,E,k,D,slots", [
    ("bf16", 600, 512, 384, 32, 4, 4, 4),        # several row tiles, ragged last tile
    ("bf16", 517, 520, 200, 24, 8, 3, 5),        # ragged K (520, 200) and ragged N (200)
    ("bf16", 96, 256, 128, 8, 2, 8, 0),          # one expert per rank, no replicas
    ("f32", 300, 100, 60, 12, 3, 2, 3),          # fp32 path with ragged everything
    ("bf16", 1500, 256, 192, 16, 8, 1, 0),       # single rank holds everything
    ("bf16", 40, 128, 64, 6, 1, 2, 2)])          # top-1
def test_reduced_layers_every_rank(torch_cuda, dtype, T, H, I, E, k, D, slots):
    cfg = synth.scaled(synth.CONFIGS["qwen3"], dtype=dtype, T=T, H=H, I=I, E=E, k=k, D=D,
                       replica_slots=slots, zipf_s=1.2, profile_batches=2)
    print("reduced", cfg, flush=True)
    case = Case(cfg)
    for g in range(D):
        _check_rank(torch_cuda, case, g)
        if dtype == "bf16":
            _check_rank(torch_cuda, case, g, packed=True)


def test_forward_is_reproducible_bit_for_bit(torch_cuda):
    torch = torch_cuda
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=700, H=256, I=256, E=32, D=4, replica_slots=4,
                       profile_batches=2)
    case = Case(cfg)
    fwd, x, logits = case.gpu_rank(case.heaviest, packed=True)
    a = fwd(x, logits).clone()
    da = {k: v.clone() for k, v in fwd.debug.items()}
    for _ in range(3):
        b = fwd(x, logits)
        torch.cuda.synchronize()
        assert torch.equal(a, b)
        for k, v in fwd.debug.items():
            assert torch.equal(da[k], v), k


def test_forward_replays_from_a_hip_graph(torch_cuda):
    # the forward is launches only (counters are cleared by a kernel, not a memset node), so it
    # can be captured; every replay, with eager work and synchronisations in between, has to
    # give the bits of the eager forward on the same inputs
    torch = torch_cuda
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=700, H=256, I=256, E=32, D=4, replica_slots=4,
                       profile_batches=2)
    case = Case(cfg)
    fwd, x, logits = case.gpu_rank(case.heaviest, packed=True)
    sx, sl = x.clone(), logits.clone()                 # the captured launches read these buffers
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(2):
            fwd(sx, sl)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fwd(sx, sl)
    torch.cuda.synchronize()
    for shift in (0, 1, 37, 350):
        xs, ls = torch.roll(x, shift, 0), torch.roll(logits, shift, 0)   # other tokens, other routing
        want = fwd(xs, ls).clone()
        want_dest = fwd.debug["dest"].clone()
        torch.cuda.synchronize()
        sx.copy_(xs)
        sl.copy_(ls)
        fwd.out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(fwd.out, want), shift
        assert torch.equal(fwd.debug["dest"], want_dest), shift
    ref = case.oracle_rank(case.heaviest)
    sx.copy_(x)
    sl.copy_(logits)
    graph.replay()
    torch.cuda.synchronize()
    out = fwd.out.float().cpu().numpy().astype(np.float64)
    assert np.abs(out - ref["out"]).max() <= TOL[cfg.dtype] * np.abs(ref["out"]).max()


def test_one_expert_layer_is_the_dense_ffn(torch_cuda):
    # E = 1, k = 1: every token goes to the one expert with weight 1, which is how a dense
    # (shared) expert runs through the same entry point.  Alone on one rank the layer is the
    # plain SwiGLU FFN of every token; replicated on two ranks each takes every other token
    # (the i-th assignment goes to copy i mod 2) and the two outputs add up to it.
    for D, slots in ((1, 0), (2, 1)):
        cfg = synth.scaled(synth.CONFIGS["qwen3"], T=600, H=512, I=384, E=1, k=1, D=D,
                           replica_slots=slots, profile_batches=2)
        case = Case(cfg)
        dense = oracle.ffn_rows(case.x.astype(np.float32), *synth.expert_weights(cfg, 0))
        total = np.zeros_like(dense)
        for g in range(D):
            out, ref = _check_rank(torch_cuda, case, g, packed=True)
            assert ref["rows"] == cfg.T // D
            total += out
        assert np.abs(total - dense).max() <= TOL["bf16"] * np.abs(dense).max()


def test_rank_without_rows_and_unused_experts(torch_cuda):
    # strong skew on few tokens: some experts (and with D = E some ranks) get nothing
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=24, H=128, I=64, E=16, k=2, D=16,
                       replica_slots=0, zipf_s=3.0, profile_batches=1)
    case = Case(cfg)
    assert min(case.rows) == 0
    for g in (int(np.argmin(case.rows)), case.heaviest):
        out, _ = _check_rank(torch_cuda, case, g, packed=True)
        if case.rows[g] == 0:
            assert np.all(out == 0)


def test_packed_weights_layout(torch_cuda):
    # the packed stream against its stated layout, element by element
    torch = torch_cuda
    H, I = 72, 40                                   # ragged in every direction
    g = np.random.default_rng(5)
    mats = [synth.round_to_storage(g.standard_normal(s).astype(np.float32), "bf16")
            for s in ((I, H), (I, H), (H, I))]
    dev = [binding.to_device(m, "bf16") for m in mats]
    pgu, pdn = binding.pack_weights(*dev)
    torch.cuda.synchronize()
    pgu = synth.bf16_bits_to_f32(pgu.cpu().numpy().view(np.uint16))
    pdn = synth.bf16_bits_to_f32(pdn.cpu().numpy().view(np.uint16))
    Wg, Wu, Wd = mats

    def expect(groups, ksteps, row_of, K):
        # [32-wide step][column group][half][lane][8 values]
        out = np.zeros((ksteps, groups, 2, 64, 8), np.float32)
        for gi in range(groups):
            for s in range(ksteps):
                for h in range(2):
                    for l in range(64):
                        src = row_of(gi, h, l & 15)
                        k0 = 32 * s + 8 * (l >> 4)
                        if src is not None and k0 < K:
                            out[s, gi, h, l] = src[k0:k0 + 8]
        return out.reshape(-1)

    gu = expect(((I + 15) // 16 + 7) // 8 * 8, (H + 255) // 256 * 8,
                lambda gi, h, r: (Wu if h else Wg)[16 * gi + r] if 16 * gi + r < I else None, H)
    dn = expect(((H + 31) // 32 + 7) // 8 * 8, (I + 255) // 256 * 8,
                lambda gi, h, r: Wd[32 * gi + 16 * h + r] if 32 * gi + 16 * h + r < H else None, I)
    assert np.array_equal(pgu, gu) and np.array_equal(pdn, dn)


def test_empty_batch(torch_cuda):
    torch = torch_cuda
    cfg = synth.scaled(synth.CONFIGS["tiny"], T=0)
    W = np.ones((1, 1, cfg.E), dtype=np.int64)
    plan = binding.Plan(W, cfg.D, 0)
    ws = [torch.zeros((cfg.I, cfg.H), device="cuda") for _ in range(4)]
    wd = [torch.zeros((cfg.H, cfg.I), device="cuda") for _ in range(4)]
    fwd = binding.RankForward(plan, 0, 0, "f32", 0, cfg.H, cfg.I, cfg.k, ws, ws, wd)
    out = fwd(torch.empty((0, cfg.H), device="cuda"), torch.empty((0, cfg.E), device="cuda"))
    rows, ovf = fwd.result()
    assert tuple(out.shape) == (0, cfg.H) and rows == 0 and ovf == 0


def test_overflow_is_reported_not_computed(torch_cuda):
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=256, H=128, I=64, E=8, k=2, D=2,
                       replica_slots=0, profile_batches=1)
    case = Case(cfg)
    g = case.heaviest
    fwd, x, logits = case.gpu_rank(g, max_rows=case.rows[g] - 1)
    out = fwd(x, logits)
    rows, ovf = fwd.result()
    assert rows == case.rows[g] and ovf == 1
    assert np.all(_np(out) == 0)
    fwd2, x, logits = case.gpu_rank(g, max_rows=case.rows[g])      # exactly enough
    fwd2(x, logits)
    assert fwd2.result() == (case.rows[g], 0)


def test_forward_rejects_foreign_tables(torch_cuda):
    torch = torch_cuda
    cfg = synth.scaled(synth.CONFIGS["tiny"], T=64)
    case = Case(cfg)
    fwd, x, logits = case.gpu_rank(0)
    other = case.plan.upload_tables(0, 1)
    fwd.args.tables = other.data_ptr()                              # tables of another rank
    with pytest.raises(binding.CraftError):
        fwd(x, logits)
    fwd.args.tables = x.data_ptr()                                  # not a table buffer at all
    with pytest.raises(binding.CraftError):
        fwd(x, logits)
    # a buffer filled again for another rank counts for that rank only; filled again for the
    # same rank it stays good
    import ctypes
    mine = fwd.tables
    n = ctypes.c_size_t()
    lib = binding.lib()
    assert lib.craft_plan_tables_bytes(case.plan._h, 0, 1, ctypes.byref(n)) == 0
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert lib.craft_plan_tables_upload(case.plan._h, 0, 1, ctypes.c_void_p(mine.data_ptr()), n.value, stream) == 0
    fwd.args.tables = mine.data_ptr()
    with pytest.raises(binding.CraftError):
        fwd(x, logits)
    for _ in range(2):
        assert lib.craft_plan_tables_upload(case.plan._h, 0, 0, ctypes.c_void_p(mine.data_ptr()), n.value, stream) == 0
    ref = case.oracle_rank(0)
    out = fwd(x, logits)
    torch.cuda.synchronize()
    assert np.abs(_np(out).astype(np.float64) - ref["out"]).max() <= TOL[cfg.dtype] * np.abs(ref["out"]).max()


def test_rank_with_more_slots_than_the_tile_tables_in_lds(torch_cuda):
    # above 256 slots on a rank the FFN walks its tile tables in global memory
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=700, H=64, I=64, E=300, k=4, D=1, replica_slots=6,
                       zipf_s=1.1, profile_batches=2)
    case = Case(cfg)
    rows = case.slot_cnt
    assert len(rows) > 256 and (rows > 64).any() and ((rows > 0) & (rows <= 32)).any()
    outs = [_check_rank(torch_cuda, case, 0, packed=True, knobs=knobs)[0]
            for knobs in (dict(riders_gateup=-1, riders_down=-1),
                          dict(tile_rows_gateup=128, tile_rows_down=128, riders_gateup=1, riders_down=1))]
    assert np.array_equal(outs[0], outs[1])
    _check_rank(torch_cuda, case, 0, packed=False)


@pytest.mark.parametrize("T,E,k,D,slots", [
    (3000, 160, 4, 4, 6),        # three expert groups share the waves five each; 19 blocks per wave
    (4100, 128, 8, 8, 16),       # two groups, 17 blocks per wave: one more than the registers keep
    (8192, 384, 8, 8, 24),       # six groups, 128 blocks per wave, four waves idle
    (2000, 1024, 2, 16, 32),     # a wave per group, every block of the batch
    (8200, 72, 4, 2, 5),         # one block more than a chunk: two workgroups per group, ragged group
    (20000, 200, 3, 4, 9)])      # three chunks of four groups
def test_dispatch_over_block_and_expert_shapes(torch_cuda, T, E, k, D, slots):
    # how the per-block counts are dealt to the waves depends on the number of 32-token blocks
    # and of 64-expert groups: integer results against the checker on every rank, narrow FFN
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=T, H=64, I=32, E=E, k=k, D=D, replica_slots=slots,
                       zipf_s=1.0, profile_batches=2)
    print("dispatch shapes", cfg, flush=True)
    case = Case(cfg)
    toks = list(range(0, T, max(1, T // 16)))
    for g in (0, D - 1):
        _check_rank(torch_cuda, case, g, tokens=toks, packed=True)


@pytest.mark.parametrize("w8", [False, True])
@pytest.mark.parametrize("T,H,I,E,k,D,slots,zipf", [
    (240, 128, 192, 32, 4, 1, 0, 1.0),     # fewer busy tiles than units of the two-fragment slots
    (400, 128, 64, 48, 6, 1, 0, 1.5),      # more units than busy tiles: some cold tiles remain
    (900, 256, 320, 32, 4, 2, 2, 1.8)])    # three column tiles, replicas
def test_cold_slots_riding_with_busy_tiles(torch_cuda, T, H, I, E, k, D, slots, zipf, w8):
    # slots with at most 64 rows are carried by the tiles of busy slots or get tiles of their
    # own: every way of cutting the work gives the same bits, and those match the checker
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=T, H=H, I=I, E=E, k=k, D=D, replica_slots=slots,
                       zipf_s=zipf, profile_batches=2)
    case = Case(cfg, w8=w8)
    for g in range(D):
        rows = case.slot_cnt[case.rank_slot_off[g]:case.rank_slot_off[g + 1]]
        assert (rows > 64).any() and ((rows > 0) & (rows <= 32)).any()
        if D == 1:
            assert ((rows > 32) & (rows <= 64)).any()
        outs = []
        for knobs in (dict(riders_gateup=-1, riders_down=-1),
                      dict(tile_rows_gateup=128, tile_rows_down=160, riders_gateup=1, riders_down=1),
                      dict(tile_rows_gateup=224, tile_rows_down=224, riders_gateup=1, riders_down=-1),
                      dict(tile_rows_gateup=256, tile_rows_down=192, riders_gateup=1, riders_down=1)):
            print(" ", knobs, flush=True)
            outs.append(_check_rank(torch_cuda, case, g, packed=True, knobs=knobs)[0])
        for o in outs[1:]:
            assert np.array_equal(outs[0], o)


def test_block_ordered_tile_list_with_ragged_bands(torch_cuda):
    # more than two rounds of busy tiles over the CUs: the kernels walk every slot's tiles block
    # by block (bands of 8 row-tiles, blocks of 8 column tiles).  Four slots whose row-tile counts
    # are no multiples of 8 and 10 column tiles per slot in both GEMMs give ragged last bands and
    # a ragged last block of columns; every token is compared.
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=16000, H=2560, I=1280, E=4, k=1, D=1, replica_slots=0,
                       zipf_s=1.0, profile_batches=1)
    case = Case(cfg)
    rows = case.slot_cnt[case.rank_slot_off[0]:case.rank_slot_off[1]]
    fwd, _, _ = case.gpu_rank(0, packed=True)
    rg, rd, _, _ = fwd.tile_choice()
    for height, nt in ((rg, (cfg.I + 127) // 128), (rd, (cfg.H + 255) // 256)):
        row_tiles = [(int(r) + height - 1) // height for r in rows if r > 64]
        assert sum(row_tiles) * nt > 2 * 256 and any(m % 8 for m in row_tiles) and nt % 8
    print(f"  slot rows {rows.tolist()}, row-tiles of {rg}/{rd} rows", flush=True)
    _check_rank(torch_cuda, case, 0, packed=True, cover=True)


# -------------------------------------------------- full-size configurations

@pytest.mark.parametrize("name", ["qwen3", "dsv3", "kimi"])
def test_full_size_heaviest_rank_every_token(torch_cuda, name):
    # the launch configuration the benchmark times: full shapes, the heaviest rank's share, the
    # tile heights and rider switches the library picks by itself.  Integer results and the
    # output of EVERY token are compared (the checker does a rank's rows in seconds), so every
    # row of every row-tile, cold slot and rider unit of both GEMMs is looked at.
    import time
    cfg = synth.CONFIGS[name]
    print("full size", cfg, flush=True)
    case = Case(cfg)
    g = case.heaviest
    print(f"  rows per rank: max={max(case.rows)} mean={np.mean(case.rows):.0f} heaviest={g} "
          f"slot rows={case.slot_cnt[case.rank_slot_off[g]:case.rank_slot_off[g + 1]].tolist()}", flush=True)
    t0 = time.perf_counter()
    ref = case.oracle_rank(g)
    print(f"  checker: all {ref['rows']} rows, {cfg.T} tokens in {time.perf_counter() - t0:.1f} s", flush=True)
    _check_rank(torch_cuda, case, g, packed=True, ref=ref, cover=True)
    _check_rank(torch_cuda, case, g, packed=False, ref=ref)


# ------------------------------------------------------------- 8-bit expert weights

@pytest.mark.parametrize("rows,K,scale", [(7, 64, 1.0), (33, 520, 0.02), (5, 4096, 30.0), (1, 8, 1.0)])
def test_quantize_e4m3_parity(torch_cuda, rows, K, scale):
    torch = torch_cuda
    g = np.random.default_rng(rows * 1000 + K)
    W = synth.round_to_storage((g.standard_normal((rows, K)) * scale).astype(np.float32), "bf16")
    W[0, :8] = [0.0, -0.0, 1.0625, 1.1875, -1.0625, 448.0, 2.0 ** -10, 3 * 2.0 ** -10]   # zeros, ties, top
    if rows > 2:
        W[2] = 0.0                                                    # an all-zero row: scale 1
    codes, sc = binding.quantize_e4m3(binding.to_device(W, "bf16", "cuda:0"))
    want_c, want_s = oracle.quantize_e4m3(W)
    assert np.array_equal(sc.cpu().numpy(), want_s)
    assert np.array_equal(codes.cpu().numpy(), want_c)


@pytest.mark.parametrize("T,H,I,E,k,D,slots", [
    (600, 512, 384, 32, 4, 4, 4),          # several row tiles, ragged last tile
    (517, 520, 200, 24, 8, 3, 5),          # ragged K and N
    (40, 128, 64, 6, 1, 2, 2)])            # top-1, cold slots only
def test_reduced_layers_with_e4m3_weights(torch_cuda, T, H, I, E, k, D, slots):
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=T, H=H, I=I, E=E, k=k, D=D, replica_slots=slots,
                       zipf_s=1.2, profile_batches=2)
    case = Case(cfg, w8=True)
    for g in range(D):
        _check_rank(torch_cuda, case, g, packed=True)


def test_full_size_qwen3_with_e4m3_weights(torch_cuda):
    case = Case(synth.CONFIGS["qwen3"], w8=True)
    g = case.heaviest
    _check_rank(torch_cuda, case, g, packed=True, cover=True)          # every token
