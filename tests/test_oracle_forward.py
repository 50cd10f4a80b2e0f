"""Pins for the CPU checker's forward steps (route, load, dispatch, FFN, combine).

Each check ties a checker function to something outside itself: a library routine
that computes the same thing in a special case, a closed form, brute force, or an
invariant the method fixes.  Some checks plant a plausible mistake into a copy of
the checker's result and confirm the pin would have caught it.
"""
import numpy as np
import pytest
import scipy.special

import oracle
from paper_2603_28768_amd import synth


# --------------------------------------------------------------------- route

def _logits(T, E, seed, quantum=None):
    g = np.random.default_rng(seed)
    l = g.standard_normal((T, E)).astype(np.float32)
    if quantum:                       # force many exact ties
        l = (np.round(l / quantum) * quantum).astype(np.float32)
    return l


@pytest.mark.parametrize("T,E,k,quantum", [(64, 16, 2, None), (50, 128, 8, None),
                                           (40, 24, 5, 0.5), (8, 7, 7, 1.0), (3, 1, 1, None)])
def test_route_ids_equal_full_stable_sort(T, E, k, quantum):
    # Sec. 2.1: the k largest scores.  A full stable sort of the negated row puts
    # equal scores in ascending expert order, which is the tie rule.
    l = _logits(T, E, 1, quantum)
    ids, _ = oracle.route(l, k)
    ref = np.argsort(-l.astype(np.float64), axis=1, kind="stable")[:, :k]
    assert np.array_equal(ids, ref)
    for t in range(T):
        assert len(set(ids[t])) == k
        assert np.all(np.diff(l[t, ids[t]]) <= 0)


def test_route_weights_closed_forms():
    T, E, k = 70, 32, 4
    l = _logits(T, E, 2) * 3.0
    ids, w = oracle.route(l, k, True)
    # renormalised weights = softmax over the k picked scores (the full denominator cancels)
    picked = np.take_along_axis(l.astype(np.float64), ids.astype(np.int64), axis=1)
    ref = scipy.special.softmax(picked, axis=1)
    assert np.allclose(w, ref, rtol=2e-7, atol=0)
    assert np.allclose(w.astype(np.float64).sum(1), 1.0, atol=1e-6)
    # without renormalisation = full softmax gathered at the picked experts
    _, w2 = oracle.route(l, k, False)
    full = scipy.special.softmax(l.astype(np.float64), axis=1)
    assert np.allclose(w2, np.take_along_axis(full, ids.astype(np.int64), axis=1), rtol=2e-7)
    # k = E: plain softmax, in descending order of score
    ids3, w3 = oracle.route(l, E, True)
    assert np.allclose(np.take_along_axis(full, ids3.astype(np.int64), axis=1), w3, rtol=2e-7)


def test_route_large_scores_do_not_overflow():
    l = np.array([[1000.0, 999.0, -1000.0, 0.0]], dtype=np.float32)
    ids, w = oracle.route(l, 2, True)
    assert ids.tolist() == [[0, 1]]
    e = np.exp(-1.0)
    assert np.allclose(w, [[1 / (1 + e), e / (1 + e)]], rtol=1e-6)


# ---------------------------------------------------------------------- load

@pytest.mark.parametrize("L,T,k,E,bt", [(1, 64, 2, 16, 64), (3, 1000, 8, 128, 256), (2, 17, 4, 9, 5)])
def test_expert_load_equals_bincount_and_sums(L, T, k, E, bt):
    g = np.random.default_rng(3)
    ids = g.integers(0, E, size=(L, T, k)).astype(np.int32)
    c = oracle.expert_load(ids, E, bt)
    B = -(-T // bt)
    assert c.shape == (B, L, E) and c.dtype == np.int64
    for b in range(B):
        t0, t1 = b * bt, min(T, (b + 1) * bt)
        for l in range(L):
            assert np.array_equal(c[b, l], np.bincount(ids[l, t0:t1].reshape(-1), minlength=E))
            assert c[b, l].sum() == (t1 - t0) * k          # counts sum to tokens * k
    with pytest.raises(ValueError):
        bad = ids.copy()
        bad[0, 0, 0] = E
        oracle.expert_load(bad, E, bt)


# ------------------------------------------------------------------ dispatch

def _slots(E, extra, D, seed):
    """A random but valid slot table: every expert once, `extra` more copies."""
    g = np.random.default_rng(seed)
    se = list(range(E)) + list(g.integers(0, E, size=extra))
    g.shuffle(se)
    return np.array(se, dtype=np.int32)


@pytest.mark.parametrize("T,k,E,extra", [(200, 2, 16, 4), (333, 8, 64, 9), (50, 4, 8, 0), (0, 2, 4, 1)])
def test_dispatch_invariants_and_closed_form(T, k, E, extra):
    g = np.random.default_rng(4)
    pop = synth.popularity(E, 1.2, 0)
    ids = np.stack([g.choice(E, size=k, replace=False, p=pop) for _ in range(T)]).astype(np.int32) \
        if T else np.zeros((0, k), np.int32)
    se = _slots(E, extra, 4, 5)
    dest, src, cnt, off = oracle.dispatch(ids, E, se)
    A, S = T * k, se.size
    flat = ids.reshape(-1)
    # bijection, inverse pair
    assert sorted(dest.tolist()) == list(range(A))
    assert np.array_equal(src[dest], np.arange(A))
    assert off[0] == 0 and off[-1] == A and np.array_equal(np.diff(off), cnt)
    copies = np.bincount(se, minlength=E)
    slots_of = [np.nonzero(se == e)[0] for e in range(E)]
    for p in range(S):
        seg = src[off[p]:off[p + 1]]
        assert np.all(flat[seg] == se[p])                  # a slot only sees its expert
        assert np.all(np.diff(seg) > 0)                    # stable: source order kept
    for e in range(E):                                     # shares differ by at most one
        shares = cnt[slots_of[e]]
        assert shares.max() - shares.min() <= 1
        assert np.all(np.diff(shares) <= 0)                # earlier copies fill first
    # closed form: dest = slot_off[slots(e)[i mod c]] + i div c
    seen = np.zeros(E, dtype=np.int64)
    for a in range(A):
        e = flat[a]
        i = seen[e]
        seen[e] += 1
        assert dest[a] == off[slots_of[e][i % copies[e]]] + i // copies[e]


def test_dispatch_without_replicas_is_a_stable_sort():
    T, k, E = 300, 4, 32
    g = np.random.default_rng(6)
    ids = g.integers(0, E, size=(T, k)).astype(np.int32)
    perm = g.permutation(E).astype(np.int32)               # slot p holds expert perm[p]
    dest, src, cnt, off = oracle.dispatch(ids, E, perm)
    slot_of_expert = np.argsort(perm)
    ref = np.argsort(slot_of_expert[ids.reshape(-1)], kind="stable")
    assert np.array_equal(src, ref)


def test_dispatch_pin_catches_modulo_direction_mistake():
    # a checker that sent token i to copy (i div share) instead of (i mod c) would
    # break "shares differ by <= 1 and earlier copies fill first" only sometimes, but
    # always breaks the closed form; plant it and see the closed form disagree.
    ids = np.zeros((10, 1), dtype=np.int32)
    se = np.array([0, 0, 0], dtype=np.int32)
    dest, *_ = oracle.dispatch(ids, 1, se)
    assert dest.tolist() == [0, 4, 7, 1, 5, 8, 2, 6, 9, 3]
    blocked = [i // 4 * 4 + i % 4 for i in range(10)]       # contiguous blocks instead
    assert blocked != dest.tolist()


# -------------------------------------------------------------- FFN + combine

def _dense_moe(x, logits, k, weights):
    """The un-sharded layer written with library matmuls: no plan, no dispatch."""
    x64 = x.astype(np.float64)
    order = np.argsort(-logits.astype(np.float64), axis=1, kind="stable")[:, :k]
    picked = np.take_along_axis(logits.astype(np.float64), order, axis=1)
    gate = scipy.special.softmax(picked, axis=1)
    out = np.zeros_like(x64)
    for e, (Wg, Wu, Wd) in enumerate(weights):
        g = x64 @ Wg.astype(np.float64).T
        u = x64 @ Wu.astype(np.float64).T
        y = (g * scipy.special.expit(g) * u) @ Wd.astype(np.float64).T
        for j in range(k):
            sel = order[:, j] == e
            out[sel] += gate[sel, j][:, None] * y[sel]
    return out


def _tiny_layer(T=48, H=24, E=6, k=2, I=40, seed=7):
    cfg = synth.scaled(synth.CONFIGS["tiny"], T=T, H=H, E=E, k=k, I=I)
    pop = synth.layer_popularity(cfg)
    logits = synth.router_logits(cfg, pop, "eval")
    x = synth.activations(cfg)
    weights = [synth.expert_weights(cfg, e) for e in range(E)]
    return cfg, logits, x, weights


def test_single_expert_is_a_swiglu_mlp():
    # E = 1, k = 1, one rank: the layer is one SwiGLU MLP with gate weight 1
    cfg, logits, x, weights = _tiny_layer(T=9, E=1, k=1)
    r = oracle.rank_forward(x, logits, 1, [0], [0, 1], 0, lambda e: weights[e])
    Wg, Wu, Wd = (w.astype(np.float64) for w in weights[0])
    g = x.astype(np.float64) @ Wg.T
    ref = (g / (1 + np.exp(-g)) * (x.astype(np.float64) @ Wu.T)) @ Wd.T
    assert np.allclose(r["out"], ref, rtol=1e-12, atol=1e-12)
    assert np.allclose(r["w"], 1.0)


def test_ffn_operand_orientation():
    # non-square shapes with distinct gate/up so that a transposed operand or a
    # swapped gate/up pair cannot pass
    g = np.random.default_rng(8)
    X = g.standard_normal((5, 7)).astype(np.float32)
    Wg = g.standard_normal((11, 7)).astype(np.float32)
    Wu = g.standard_normal((11, 7)).astype(np.float32)
    Wd = g.standard_normal((7, 11)).astype(np.float32)
    Y = oracle.ffn_rows(X, Wg, Wu, Wd)
    G = X.astype(np.float64) @ Wg.astype(np.float64).T
    U = X.astype(np.float64) @ Wu.astype(np.float64).T
    ref = (G * scipy.special.expit(G) * U) @ Wd.astype(np.float64).T
    assert np.allclose(Y, ref, rtol=1e-12, atol=1e-13)
    swapped = (U * scipy.special.expit(U) * G) @ Wd.astype(np.float64).T
    assert not np.allclose(Y, swapped, rtol=1e-3)


@pytest.mark.parametrize("D,extra", [(1, 0), (3, 0), (3, 4), (4, 7)])
def test_rank_shares_sum_to_the_unsharded_layer(D, extra):
    # whatever the plan, the ranks' partial outputs add up to the plain MoE layer
    cfg, logits, x, weights = _tiny_layer()
    E, k = cfg.E, cfg.k
    se = _slots(E, extra, D, 9)
    S = se.size
    bounds = [0] + sorted(np.random.default_rng(10).choice(np.arange(1, S), size=D - 1,
                                                            replace=False).tolist()) + [S]
    total = np.zeros((cfg.T, cfg.H))
    rows = 0
    for g in range(D):
        r = oracle.rank_forward(x, logits, k, se, bounds, g, lambda e: weights[e])
        total += r["out"]
        rows += r["rows"]
    assert rows == cfg.T * k
    ref = _dense_moe(x, logits, k, weights)
    # the checker stores gate weights as fp32 (2^-24 relative); everything else is double
    assert np.allclose(total, ref, rtol=0, atol=4e-7 * np.abs(ref).max())


def test_rank_forward_token_subset_matches_full():
    cfg, logits, x, weights = _tiny_layer()
    se = _slots(cfg.E, 3, 2, 11)
    off = [0, 4, se.size]
    full = oracle.rank_forward(x, logits, cfg.k, se, off, 1, lambda e: weights[e])
    toks = [0, 5, 17, 47]
    part = oracle.rank_forward(x, logits, cfg.k, se, off, 1, lambda e: weights[e], tokens=toks)
    assert np.array_equal(part["out"], full["out"][toks])


def test_combine_skips_foreign_rows_and_orders_terms():
    Y = np.arange(12, dtype=np.float64).reshape(3, 4) + 1
    dest = np.array([[5, 0], [6, 7], [1, 2]], dtype=np.int32)   # rank owns positions 5..7
    w = np.array([[0.25, 0.75], [0.5, 0.5], [0.1, 0.9]], dtype=np.float32)
    out = oracle.combine(Y, 5, dest, w, 3, 2)
    assert np.allclose(out[0], 0.25 * Y[0])
    assert np.allclose(out[1], 0.5 * Y[1] + 0.5 * Y[2])
    assert np.all(out[2] == 0)


def test_double_accumulation_error_is_far_below_the_gate():
    # the checker's own rounding: a float64 run against exact rational arithmetic on a
    # tiny case (fractions), to show its error is many orders below the 1e-2 gate
    from fractions import Fraction
    g = np.random.default_rng(12)
    X = g.standard_normal((1, 6)).astype(np.float32)
    Wg = g.standard_normal((4, 6)).astype(np.float32)
    Wu = g.standard_normal((4, 6)).astype(np.float32)
    Wd = g.standard_normal((6, 4)).astype(np.float32)
    Y = oracle.ffn_rows(X, Wg, Wu, Wd)[0]
    F = lambda a: Fraction(float(a))
    gs = [sum(F(X[0, h]) * F(Wg[i, h]) for h in range(6)) for i in range(4)]
    us = [sum(F(X[0, h]) * F(Wu[i, h]) for h in range(6)) for i in range(4)]
    import math
    act = [Fraction(float(gi) / (1 + math.exp(-float(gi)))) * ui for gi, ui in zip(gs, us)]
    ref = [float(sum(act[i] * F(Wd[h, i]) for i in range(4))) for h in range(6)]
    assert np.allclose(Y, ref, rtol=1e-13, atol=1e-15)
