"""Pins for the CPU checker's 8-bit weight storage (OCP FP8 E4M3 with a scale per row).

The format is a published one, so the pins are what its specification fixes (special
values, ranges, spacing) and an independent implementation of the same format
(torch.float8_e4m3fn), plus brute-force nearest-value checks of the rounding."""
import numpy as np
import pytest
import torch

import oracle


def _table():
    return np.array([oracle.e4m3_value(c) for c in range(256)])


def test_values_the_format_fixes():
    t = _table()
    assert t[0x38] == 1.0 and t[0x3c] == 1.5 and t[0xb8] == -1.0
    assert t[0x7e] == 448.0 and t[0xfe] == -448.0               # largest finite magnitude
    assert t[0x08] == 2.0 ** -6 and t[0x01] == 2.0 ** -9          # smallest normal, smallest subnormal
    assert t[0x00] == 0.0 and t[0x80] == 0.0 and np.signbit(t[0x80])
    assert np.isnan(t[0x7f]) and np.isnan(t[0xff])               # the only NaNs; no infinities
    assert np.isfinite(np.delete(t, [0x7f, 0xff])).all()
    pos = t[:0x7f]
    assert (np.diff(pos) > 0).all()                              # codes order like their values
    assert np.array_equal(t[0x80:0xff], -pos)
    for ex in range(1, 15):                                      # 8 equally spaced values per binade
        b = pos[ex * 8:(ex + 1) * 8]
        assert b[0] == 2.0 ** (ex - 7) and np.allclose(np.diff(b), b[0] / 8, rtol=0, atol=0)
    assert np.allclose(np.diff(pos[:9]), 2.0 ** -9, rtol=0, atol=0)   # subnormals continue the grid


def test_values_match_an_independent_implementation():
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    t = _table()
    same = (t == ref) | (np.isnan(t) & np.isnan(ref))
    assert same.all()
    ok = ~np.isnan(t)
    assert np.array_equal(np.signbit(t[ok]), np.signbit(ref[ok]))


@pytest.mark.parametrize("seed", range(4))
def test_quantisation_is_nearest_with_ties_to_even(seed):
    g = np.random.default_rng(seed)
    W = (g.standard_normal((6, 97)) * g.choice([1e-3, 1.0, 50.0], size=(6, 1))).astype(np.float32)
    W[0, :8] = [0.0, -0.0, 1e-30, -1e-30, W[0].max(), W[0].min(), 0.5, -0.5]
    codes, scale = oracle.quantize_e4m3(W)
    amax = np.abs(W).max(axis=1)
    assert np.array_equal(scale, (amax / np.float32(448.0)).astype(np.float32))
    t = _table()
    finite = np.array([c for c in range(0x7f)])
    q = (W / scale[:, None]).astype(np.float32).astype(np.float64)          # the float quotient
    for r in range(W.shape[0]):
        for k in range(W.shape[1]):
            a = abs(q[r, k])
            d = np.abs(t[finite] - a)
            best = d.min()
            c = int(codes[r, k])
            assert abs(abs(t[c]) - a) == best                                 # a nearest value ...
            ties = finite[d == best]
            if len(ties) == 2:
                assert (c & 0x7f) == ties[ties % 2 == 0][0]                   # ... the even one on a tie
            assert bool(c & 0x80) == bool(np.signbit(q[r, k]))
    # the largest magnitude of a row lands on +-448 exactly
    top = np.abs(oracle.dequantize_e4m3(codes, scale)).max(axis=1)
    assert np.array_equal(top.astype(np.float32), (np.float32(448.0) * scale).astype(np.float32))


def test_quantisation_matches_an_independent_implementation_in_range():
    g = np.random.default_rng(9)
    W = g.standard_normal((5, 256)).astype(np.float32)
    codes, scale = oracle.quantize_e4m3(W)
    q = torch.from_numpy((W / scale[:, None]).astype(np.float32))
    ref = q.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(codes, ref)


def test_exact_ties_and_special_rows():
    # halfway between 1.0 (0x38, even) and 1.125 (0x39): to 1.0; between 1.125 and 1.25 (0x3a): to 1.25
    W = np.array([[448.0, 1.0625, 1.1875, -1.0625, 2.0 ** -10, 3 * 2.0 ** -10]], np.float32)
    codes, scale = oracle.quantize_e4m3(W)
    assert scale[0] == 1.0
    assert codes[0].tolist() == [0x7e, 0x38, 0x3a, 0xb8, 0x00, 0x02]        # 2^-10 ties to 0, 3*2^-10 to 2^-8
    z, s = oracle.quantize_e4m3(np.zeros((2, 5), np.float32))
    assert (z == 0).all() and (s == 1.0).all()
    W = np.array([[0.0, -0.0, 7.0]], np.float32)
    c, _ = oracle.quantize_e4m3(W)
    assert c[0].tolist() == [0x00, 0x80, 0x7e]


def test_round_trip_error_bound():
    g = np.random.default_rng(10)
    W = g.standard_normal((8, 512)).astype(np.float32)
    codes, scale = oracle.quantize_e4m3(W)
    back = oracle.dequantize_e4m3(codes, scale)
    # half a mantissa step relative for normal values, half a subnormal step absolute below
    bound = np.maximum(np.abs(W) * 2.0 ** -4, scale[:, None] * 2.0 ** -10) * (1 + 1e-6)
    assert (np.abs(back - W) <= bound).all()
