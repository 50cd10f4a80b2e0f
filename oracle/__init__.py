"""CPU checker ("oracle") for the MoE rank-forward path and its planner.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  It never imports the HIP library or its binding,
and the library never imports this package.

`moe_oracle.c` holds the per-step definitions (route, load, dispatch, FFN,
combine); `plan_oracle.py` holds the planner.  This file only marshals numpy
arrays into the C functions and strings the steps together for one rank.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import plan_oracle  # noqa: F401  (re-exported)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile moe_oracle.c with gcc (plain -O2, OpenMP over FFN rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_i32, c_i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        lib.oracle_route.argtypes = [vp, c_i64, c_i32, c_i32, c_i32, vp, vp]
        lib.oracle_expert_load.argtypes = [vp, c_i32, c_i64, c_i32, c_i32, c_i64, vp]
        lib.oracle_dispatch.argtypes = [vp, c_i64, c_i32, c_i32, vp, vp, vp, vp, vp]
        lib.oracle_ffn_rows.argtypes = [vp, c_i64, c_i32, c_i32, vp, vp, vp, vp]
        lib.oracle_combine.argtypes = [vp, c_i64, c_i64, vp, vp, c_i64, c_i32, c_i32, vp]
        lib.oracle_router_logits.argtypes = [vp, vp, c_i64, c_i32, c_i32, vp]
        lib.oracle_router_logits.restype = ctypes.c_int
        lib.oracle_quantize_e4m3.argtypes = [vp, c_i64, c_i64, vp, vp]
        lib.oracle_quantize_e4m3.restype = ctypes.c_int
        lib.oracle_e4m3_value.argtypes = [ctypes.c_uint8]
        lib.oracle_e4m3_value.restype = ctypes.c_double
        for f in (lib.oracle_route, lib.oracle_expert_load, lib.oracle_dispatch,
                  lib.oracle_ffn_rows, lib.oracle_combine, lib.oracle_num_threads):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def router_logits(x: np.ndarray, w_router: np.ndarray) -> np.ndarray:
    """fp32 scores [T][E] of the linear gate: x [T][H] against w_router [E][H]."""
    x, w_router = _c(x, np.float32), _c(w_router, np.float32)
    (T, H), (E, H2) = x.shape, w_router.shape
    if H != H2:
        raise ValueError("x and w_router disagree on the hidden size")
    out = np.empty((T, E), dtype=np.float32)
    rc = _load().oracle_router_logits(_p(x), _p(w_router), T, H, E, _p(out))
    if rc:
        raise ValueError(f"oracle_router_logits failed ({rc})")
    return out


def route(logits: np.ndarray, k: int, renormalize: bool = True) -> Tuple[np.ndarray, np.ndarray]:
    """(ids int32 [T][k], w float32 [T][k]) from fp32 router scores [T][E]."""
    logits = _c(logits, np.float32)
    T, E = logits.shape
    ids = np.empty((T, k), dtype=np.int32)
    w = np.empty((T, k), dtype=np.float32)
    rc = _load().oracle_route(_p(logits), T, E, k, int(bool(renormalize)), _p(ids), _p(w))
    if rc:
        raise ValueError(f"oracle_route failed ({rc})")
    return ids, w


def expert_load(ids: np.ndarray, E: int, batch_tokens: int) -> np.ndarray:
    """counts int64 [B][L][E] from ids int32 [L][T][k]."""
    ids = _c(ids, np.int32)
    L, T, k = ids.shape
    B = (T + batch_tokens - 1) // batch_tokens
    counts = np.empty((B, L, E), dtype=np.int64)
    rc = _load().oracle_expert_load(_p(ids), L, T, k, E, batch_tokens, _p(counts))
    if rc:
        raise ValueError(f"oracle_expert_load failed ({rc})")
    return counts


def dispatch(ids: np.ndarray, E: int, slot_expert: Sequence[int]):
    """(dest [A], src [A], slot_cnt [S], slot_off [S+1]), all int32."""
    flat = _c(ids, np.int32).reshape(-1)
    se = _c(slot_expert, np.int32)
    A, S = flat.size, se.size
    dest = np.empty(A, dtype=np.int32)
    src = np.empty(A, dtype=np.int32)
    cnt = np.empty(S, dtype=np.int32)
    off = np.empty(S + 1, dtype=np.int32)
    rc = _load().oracle_dispatch(_p(flat), A, E, S, _p(se), _p(dest), _p(src), _p(cnt), _p(off))
    if rc:
        raise ValueError(f"oracle_dispatch failed ({rc})")
    return dest, src, cnt, off


def ffn_rows(X: np.ndarray, Wg: np.ndarray, Wu: np.ndarray, Wd: np.ndarray) -> np.ndarray:
    """double [rows][H] = down(silu(gate X) * up X) for one expert."""
    X, Wg, Wu, Wd = (_c(a, np.float32) for a in (X, Wg, Wu, Wd))
    rows, H = X.shape
    I = Wg.shape[0]
    assert Wg.shape == (I, H) and Wu.shape == (I, H) and Wd.shape == (H, I)
    Y = np.empty((rows, H), dtype=np.float64)
    rc = _load().oracle_ffn_rows(_p(X), rows, H, I, _p(Wg), _p(Wu), _p(Wd), _p(Y))
    if rc:
        raise ValueError(f"oracle_ffn_rows failed ({rc})")
    return Y


def e4m3_value(code: int) -> float:
    return float(_load().oracle_e4m3_value(int(code)))


def quantize_e4m3(W: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """(codes uint8 [rows][K], scale float32 [rows]) of a weight matrix, one scale per row."""
    W = _c(W, np.float32)
    rows, K = W.shape
    codes = np.empty((rows, K), dtype=np.uint8)
    scale = np.empty(rows, dtype=np.float32)
    rc = _load().oracle_quantize_e4m3(_p(W), rows, K, _p(codes), _p(scale))
    if rc:
        raise ValueError(f"oracle_quantize_e4m3 failed ({rc})")
    return codes, scale


def dequantize_e4m3(codes: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """float64 [rows][K]: code value times the row's scale, exactly."""
    table = np.array([e4m3_value(c) for c in range(256)], dtype=np.float64)
    return table[codes] * scale.astype(np.float64)[:, None]


def combine(Y: np.ndarray, lo: int, dest: np.ndarray, w: np.ndarray, T: int, k: int) -> np.ndarray:
    """double [T][H]: weighted sum of the rank's rows (global positions lo .. lo+M-1)."""
    Y = _c(Y, np.float64)
    M, H = Y.shape
    dest = _c(dest, np.int32).reshape(-1)
    w = _c(w, np.float32).reshape(-1)
    out = np.empty((T, H), dtype=np.float64)
    rc = _load().oracle_combine(_p(Y), M, lo, _p(dest), _p(w), T, k, H, _p(out))
    if rc:
        raise ValueError(f"oracle_combine failed ({rc})")
    return out


def rank_forward(x: np.ndarray, logits: np.ndarray, k: int, slot_expert: Sequence[int],
                 rank_slot_off: Sequence[int], rank: int, weights_of, renormalize: bool = True,
                 tokens: Optional[Sequence[int]] = None) -> dict:
    """One rank's share of one layer, step by step.

    weights_of(e) -> (Wg, Wu, Wd) float32 arrays of expert e.
    tokens: when given, the FFN and the combine are evaluated only for the rows
    that feed these tokens, and `out` holds just those tokens (in that order);
    routing and dispatch always cover the whole batch.
    """
    x = _c(x, np.float32)
    T, H = x.shape
    E = logits.shape[1]
    ids, w = route(logits, k, renormalize)
    dest, src, cnt, off = dispatch(ids, E, slot_expert)
    p_lo, p_hi = rank_slot_off[rank], rank_slot_off[rank + 1]
    lo, hi = int(off[p_lo]), int(off[p_hi])
    M = hi - lo
    if tokens is None:
        need = np.ones(M, dtype=bool)
    else:
        need = np.zeros(M, dtype=bool)
        for t in tokens:
            d = dest[t * k:(t + 1) * k]
            d = d[(d >= lo) & (d < hi)]
            need[d - lo] = True
    Y = np.zeros((M, H), dtype=np.float64)
    for p in range(p_lo, p_hi):
        r0, r1 = int(off[p]) - lo, int(off[p + 1]) - lo
        rows = np.nonzero(need[r0:r1])[0] + r0
        if rows.size == 0:
            continue
        Wg, Wu, Wd = weights_of(int(slot_expert[p]))
        Y[rows] = ffn_rows(x[src[rows + lo] // k], Wg, Wu, Wd)
    if tokens is None:
        out = combine(Y, lo, dest, w, T, k)
    else:
        tok = np.asarray(tokens, dtype=np.int64)
        sub_dest = dest.reshape(T, k)[tok]
        sub_w = w.reshape(T, k)[tok]
        out = combine(Y, lo, sub_dest, sub_w, tok.size, k)
    return dict(ids=ids, w=w, dest=dest, src=src, slot_cnt=cnt, slot_off=off,
                lo=lo, rows=M, Y=Y, out=out, counts=expert_load(ids[None], E, max(T, 1))[0, 0])
