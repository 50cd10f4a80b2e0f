"""craft_moe_rank_forward_static: the forward on the library's own device scratch, for callers
that cannot allocate.  Its results are those of craft_moe_rank_forward on a caller workspace
(same kernels): compared bit for bit, on two calls in a row, the second with a smaller input,
so that whatever the first call left in the shared scratch is seen not to matter."""
import numpy as np
import pytest

from paper_2603_28768_amd import binding, synth

from cases import Case

pytestmark = pytest.mark.gpu


def _both_ways(torch, cfg, packed):
    case = Case(cfg)
    rank = case.heaviest
    fwd, x, logits = case.gpu_rank(rank, packed=packed)
    want = fwd(x, logits).clone()
    want_dbg = {k: v.clone() for k, v in fwd.debug.items()}
    rows, ovf = fwd.result()
    assert ovf == 0 and rows == case.rows[rank] > 0
    fwd.out.zero_()
    for v in fwd.debug.values():
        v.zero_()
    fwd.workspace.fill_(0xAB)                      # the caller's workspace is not used any more
    fwd.args.workspace, fwd.args.workspace_bytes = None, 0
    got = fwd(x, logits, static_scratch=True)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    for k, v in fwd.debug.items():
        assert torch.equal(v, want_dbg[k]), k
    so = fwd.debug["slot_off"].cpu().numpy()
    assert so[case.rank_slot_off[rank + 1]] - so[case.rank_slot_off[rank]] == rows
    return case, rank, got


def test_static_scratch_forward_matches_the_workspace_forward_twice(torch_cuda):
    torch = torch_cuda
    big = synth.scaled(synth.CONFIGS["qwen3"], T=1500, H=512, I=384, E=32, k=4, D=2, replica_slots=3,
                       zipf_s=1.3, profile_batches=2)
    small = synth.scaled(synth.CONFIGS["qwen3"], T=300, H=256, I=128, E=16, k=2, D=2, replica_slots=1,
                         zipf_s=1.1, profile_batches=2)
    print("static scratch, first call", big, flush=True)
    _both_ways(torch, big, packed=True)
    print("static scratch, second (smaller) call", small, flush=True)
    case, rank, got = _both_ways(torch, small, packed=True)
    # and against the checker, like every other forward
    ref = case.oracle_rank(rank)
    err = np.abs(got.float().cpu().numpy().astype(np.float64) - ref["out"]).max()
    assert err <= 1e-2 * np.abs(ref["out"]).max()
    # fp32 through the row-major kernels, smaller again
    tiny = synth.scaled(synth.CONFIGS["tiny"], T=100)
    _both_ways(torch, tiny, packed=False)


def test_static_scratch_forward_refuses_a_full_size_request(torch_cuda):
    cfg = synth.CONFIGS["qwen3"]
    W = np.ones((1, 1, cfg.E), dtype=np.int64)
    plan = binding.Plan(W, cfg.D, 0)
    import ctypes
    a = binding.FwdArgs()
    a.dtype, a.T, a.H, a.I, a.k = binding.CRAFT_BF16, cfg.T, cfg.H, cfg.I, cfg.k
    a.logits = 0x1000
    assert binding.lib().craft_moe_rank_forward_static(plan._h, 0, 0, ctypes.byref(a), None) == -5
