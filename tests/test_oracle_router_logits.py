"""Pins for the checker's gating-network scores (Sec. 2.1, read as a linear gate): values the
mathematics fixes, exact rational arithmetic on small cases, an independent library routine."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2603_28768_amd import synth


def _bf16_values(g, shape, scale=1.0):
    return synth.round_to_storage((g.standard_normal(shape) * scale).astype(np.float32), "bf16")


def test_unit_rows_select_columns_of_x():
    # W_r[e] = unit vector of coordinate c_e  =>  score[t][e] = x[t][c_e], exactly
    g = np.random.default_rng(1)
    T, H, E = 7, 24, 5
    x = _bf16_values(g, (T, H))
    cols = [3, 0, 23, 11, 3]
    W = np.zeros((E, H), dtype=np.float32)
    W[np.arange(E), cols] = 1.0
    got = oracle.router_logits(x, W)
    assert got.shape == (T, E) and got.dtype == np.float32
    assert np.array_equal(got, x[:, cols])


def test_one_hot_tokens_read_columns_of_the_gate():
    # x[t] = 2 * unit vector of coordinate h_t  =>  score[t][e] = 2 * W_r[e][h_t], exactly: a
    # transposed operand or a swapped index cannot pass both this and the test above
    g = np.random.default_rng(2)
    T, H, E = 4, 16, 9
    W = _bf16_values(g, (E, H), 0.25)
    hs = [15, 2, 2, 7]
    x = np.zeros((T, H), dtype=np.float32)
    x[np.arange(T), hs] = 2.0
    assert np.array_equal(oracle.router_logits(x, W), 2.0 * W[:, hs].T)


def test_exact_rational_arithmetic_on_small_cases():
    # bf16 values are dyadic rationals: the exact dot product, rounded once to fp32, is what a
    # double accumulation of at most a few dozen such products gives (53 bits hold it exactly)
    g = np.random.default_rng(3)
    for T, H, E in ((3, 8, 4), (2, 40, 3), (5, 16, 1)):
        x, W = _bf16_values(g, (T, H)), _bf16_values(g, (E, H), 0.3)
        got = oracle.router_logits(x, W)
        for t in range(T):
            for e in range(E):
                exact = sum(Fraction(float(x[t, h])) * Fraction(float(W[e, h])) for h in range(H))
                assert got[t, e] == np.float32(float(exact))


def test_against_a_library_matrix_product_and_linearity():
    g = np.random.default_rng(4)
    T, H, E = 33, 520, 24                      # nothing square, H not a power of two
    x, W = _bf16_values(g, (T, H)), _bf16_values(g, (E, H), H ** -0.5)
    got = oracle.router_logits(x, W).astype(np.float64)
    want = x.astype(np.float64) @ W.astype(np.float64).T
    assert np.abs(got - want).max() <= 2.0 ** -23 * np.abs(want).max()
    # additivity in the tokens (exact for power-of-two scaling): score(2x) = 2 score(x)
    assert np.array_equal(oracle.router_logits(2.0 * x, W), 2.0 * oracle.router_logits(x, W))
    # a dropped tail of the contraction shows: the last coordinate matters
    x2 = x.copy(); x2[:, -1] += 1.0
    assert np.allclose(oracle.router_logits(x2, W) - got, W[:, -1][None, :], atol=1e-5)


def test_feeds_the_router():
    # scores -> top-k: with a gate whose rows are scaled unit vectors the picked experts are
    # the ones the construction says
    H, E = 8, 8
    W = np.diag(np.arange(1, E + 1)).astype(np.float32)       # score[e] = (e+1) * x[e]
    x = np.ones((1, H), dtype=np.float32)
    ids, w = oracle.route(oracle.router_logits(x, W), 3)
    assert ids.tolist() == [[7, 6, 5]] and abs(float(w.sum()) - 1.0) < 1e-6


def test_rejects_mismatched_shapes():
    with pytest.raises(ValueError):
        oracle.router_logits(np.zeros((2, 8), np.float32), np.zeros((3, 9), np.float32))
