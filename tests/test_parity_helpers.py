"""CPU checks of the helpers the full-size GPU parity tests rely on: the list of work units
(row-tiles, cold slots' fragments, rider units) and the assertion that compared tokens reach
every one of them."""
import numpy as np
import pytest

from paper_2603_28768_amd import synth

from cases import Case
import test_gpu_parity as tp


@pytest.fixture(scope="module")
def case():
    cfg = synth.scaled(synth.CONFIGS["qwen3"], T=2000, H=64, I=32, E=32, k=4, D=2, replica_slots=3,
                       zipf_s=1.3, profile_batches=2)
    return Case(cfg)


def test_units_tile_the_rank_rows(case):
    g = case.heaviest
    rows = case.slot_cnt[case.rank_slot_off[g]:case.rank_slot_off[g + 1]]
    assert (rows > 64).any() and ((rows > 0) & (rows <= 64)).any()
    units = tp._row_units(case, g, [224, 160])
    M = int(rows.sum())
    assert all(0 <= a < b <= M and b - a <= 32 for a, b in units)
    # each unit lies inside one slot
    off = np.concatenate([[0], np.cumsum(rows)])
    for a, b in units:
        p = np.searchsorted(off, a, side="right") - 1
        assert b <= off[p + 1]
    # a cold slot contributes each of its fragments, a busy one at least its first and last
    for p, n in enumerate(rows):
        mine = [(a, b) for a, b in units if off[p] <= a < off[p + 1]]
        if 0 < n <= 64:
            assert sorted(set(mine)) == [(off[p] + 32 * f, off[p] + min(32 * f + 32, n)) for f in range((n + 31) // 32)]
        elif n > 64:
            assert (off[p], off[p] + 32) in mine and any(b == off[p + 1] for _, b in mine)


def test_compared_tokens_must_reach_every_unit(case):
    g = case.heaviest
    n = tp._assert_units_compared(case, g, None, [224, 160])          # every token: trivially all
    toks = tp._tokens_covering_units(case, g, [224, 160])
    assert tp._assert_units_compared(case, g, toks, [224, 160]) == n
    with pytest.raises(AssertionError):
        tp._assert_units_compared(case, g, toks[:5], [224, 160])
