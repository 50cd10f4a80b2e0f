"""Thin ctypes binding over libcraft.so: argument marshalling only.

Every step of the path runs inside the library's HIP kernels (or, for the planner, its
host C++).  PyTorch is used for device memory and streams only.  There is no fallback: if
the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcraft.so")

CRAFT_F32, CRAFT_BF16 = 0, 1
CRAFT_W_BF16, CRAFT_W_E4M3 = 0, 1
KERNEL_NAMES = ["route", "scan", "dispatch", "gateup", "down", "combine", "gate"]

c_i32, c_i64, c_vp, c_sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
P = ctypes.POINTER


class PlanParams(ctypes.Structure):
    _fields_ = [("L", c_i32), ("E", c_i32), ("D", c_i32), ("gpus_per_node", c_i32), ("B", c_i64),
                ("load", c_vp), ("bytes_per_replica", c_vp), ("budget_bytes", c_i64),
                ("objective", c_i32), ("auto_r", c_i32)]


class FwdArgs(ctypes.Structure):
    _fields_ = [("dtype", c_i32), ("T", c_i64), ("H", c_i32), ("I", c_i32), ("k", c_i32),
                ("renormalize", c_i32), ("x", c_vp), ("logits", c_vp), ("w_router", c_vp), ("w_gate", c_vp),
                ("w_up", c_vp), ("w_down", c_vp), ("w_gateup_packed", c_vp), ("w_down_packed", c_vp),
                ("weight_format", c_i32),
                ("out", c_vp), ("ids", c_vp), ("topk_w", c_vp),
                ("dest", c_vp), ("src", c_vp), ("counts", c_vp), ("slot_cnt", c_vp),
                ("slot_off", c_vp), ("max_rows", c_i64), ("tile_rows_gateup", c_i32),
                ("tile_rows_down", c_i32), ("riders_gateup", c_i32), ("riders_down", c_i32),
                ("tables", c_vp), ("workspace", c_vp),
                ("workspace_bytes", c_sz)]


EXPORTS = {
    "craft_status_str": (ctypes.c_char_p, [ctypes.c_int]),
    "craft_router_logits_workspace": (ctypes.c_int, [c_i32, c_i64, c_i32, c_i32, P(c_sz)]),
    "craft_router_logits": (ctypes.c_int, [c_i32, c_vp, c_vp, c_i64, c_i32, c_i32, c_vp, c_vp, c_sz, c_vp]),
    "craft_route_topk": (ctypes.c_int, [c_vp, c_i64, c_i32, c_i32, c_i32, c_vp, c_vp, c_vp]),
    "craft_expert_load": (ctypes.c_int, [c_vp, c_i32, c_i64, c_i32, c_i32, c_i64, c_vp, c_vp]),
    "craft_load_accumulate": (ctypes.c_int, [c_vp, c_i64, c_vp, c_vp]),
    "craft_plan": (ctypes.c_int, [P(PlanParams), P(c_vp)]),
    "craft_plan_diff": (ctypes.c_int, [c_vp, c_vp, c_i32, c_i32, c_vp, P(c_i32), P(c_i32)]),
    "craft_plan_destroy": (None, [c_vp]),
    "craft_plan_summary": (ctypes.c_int, [c_vp, P(c_i32), P(c_i32), P(c_i32), P(c_i64),
                                          P(ctypes.c_double), P(ctypes.c_double)]),
    "craft_plan_layer_info": (ctypes.c_int, [c_vp, c_i32, P(c_i32), P(c_i32), P(ctypes.c_double),
                                             P(c_i64)]),
    "craft_plan_layer_tables": (ctypes.c_int, [c_vp, c_i32, c_vp, c_vp, c_vp, c_vp]),
    "craft_plan_greedy_order": (ctypes.c_int, [c_vp, c_vp, c_i64, P(c_i64)]),
    "craft_plan_benefit": (ctypes.c_int, [c_vp, P(c_i32), c_vp, c_vp, c_vp, P(ctypes.c_double),
                                          P(c_i32)]),
    "craft_plan_rank_rows": (ctypes.c_int, [c_vp, c_i32, c_vp, c_vp, P(c_i32)]),
    "craft_plan_tables_bytes": (ctypes.c_int, [c_vp, c_i32, c_i32, P(c_sz)]),
    "craft_plan_tables_upload": (ctypes.c_int, [c_vp, c_i32, c_i32, c_vp, c_sz, c_vp]),
    "craft_pack_weights_bytes": (ctypes.c_int, [c_i32, c_i32, c_i32, P(c_sz), P(c_sz)]),
    "craft_pack_weights": (ctypes.c_int, [c_i32, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp]),
    "craft_quantize_e4m3": (ctypes.c_int, [c_vp, c_i64, c_i32, c_vp, c_vp, c_vp]),
    "craft_pack_weights_e4m3_bytes": (ctypes.c_int, [c_i32, c_i32, P(c_sz), P(c_sz)]),
    "craft_pack_weights_e4m3": (ctypes.c_int, [c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp,
                                               c_vp]),
    "craft_moe_rank_forward_workspace": (ctypes.c_int, [c_vp, c_i32, c_i32, P(FwdArgs), P(c_sz)]),
    "craft_moe_rank_forward": (ctypes.c_int, [c_vp, c_i32, c_i32, P(FwdArgs), c_vp]),
    "craft_moe_rank_forward_static": (ctypes.c_int, [c_vp, c_i32, c_i32, P(FwdArgs), c_vp]),
    "craft_moe_rank_forward_tiles": (ctypes.c_int, [c_vp, c_i32, c_i32, P(FwdArgs), P(c_i32), P(c_i32),
                                                    P(c_i32), P(c_i32)]),
    "craft_moe_rank_forward_result": (ctypes.c_int, [c_vp, P(c_i64), P(c_i32)]),
    "craft_probe_copy": (ctypes.c_int, [c_vp, c_vp, c_i64, c_vp]),
    "craft_probe_read": (ctypes.c_int, [c_vp, c_i64, c_i32, c_i32, c_vp, P(ctypes.c_double), c_vp]),
    "craft_probe_mfma_bf16": (ctypes.c_int, [c_i32, c_i32, c_vp, P(ctypes.c_double), c_vp]),
    "craft_probe_mfma_operands": (ctypes.c_int, [c_i32, c_i32, c_i32, c_i32, c_vp, P(ctypes.c_double), c_vp]),
    "craft_timing_enable": (ctypes.c_int, [c_i32, c_i32]),
    "craft_timing_read": (ctypes.c_int, [P(ctypes.c_double), P(c_i64)]),
}

_lib = None


class CraftError(RuntimeError):
    pass


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise CraftError(f"{LIB_PATH} is missing: build it first "
                             "(python -m paper_2603_28768_amd.build)")
        # torch first: the library has to bind to the HIP runtime torch brings along, or
        # streams and device pointers made by one runtime meet kernels registered in another
        import torch  # noqa: F401
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            f = getattr(l, name)
            f.restype, f.argtypes = res, args
        _lib = l
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise CraftError(f"{what}: {lib().craft_status_str(rc).decode()} ({rc})")


def _stream_ptr(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev(t):
    """Device pointer of a CUDA tensor (or NULL)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous()
    return ctypes.c_void_p(t.data_ptr())


# ------------------------------------------------------------------------ routing

def router_logits_workspace(x, w_router):
    """A workspace tensor of the size craft_router_logits splits its contraction with, or None
    when this shape is not split."""
    import torch
    T, H = x.shape
    n = c_sz()
    _check(lib().craft_router_logits_workspace(CRAFT_BF16 if x.dtype == torch.bfloat16 else CRAFT_F32,
                                               T, H, w_router.shape[0], n), "craft_router_logits_workspace")
    return torch.empty(n.value, dtype=torch.uint8, device=x.device) if n.value else None


def router_logits(x, w_router, workspace=None, stream=None):
    """x: cuda [T][H], w_router: cuda [E][H] (both float32 or both bfloat16) -> float32 [T][E].
    `workspace`: a tensor from router_logits_workspace (the faster, split form) or None."""
    import torch
    assert x.dim() == 2 and w_router.dim() == 2 and x.shape[1] == w_router.shape[1]
    assert x.dtype == w_router.dtype and x.dtype in (torch.float32, torch.bfloat16)
    assert x.is_contiguous() and w_router.is_contiguous()
    T, H = x.shape
    E = w_router.shape[0]
    logits = torch.empty((T, E), dtype=torch.float32, device=x.device)
    _check(lib().craft_router_logits(CRAFT_BF16 if x.dtype == torch.bfloat16 else CRAFT_F32, _dev(x),
                                     _dev(w_router), T, H, E, _dev(logits),
                                     _dev(workspace) if workspace is not None else None,
                                     workspace.numel() if workspace is not None else 0,
                                     _stream_ptr(stream)),
           "craft_router_logits")
    return logits


def route_topk(logits, k: int, renormalize: bool = True, stream=None):
    """logits: cuda float32 [T][E] -> (ids int32 [T][k], w float32 [T][k])."""
    import torch
    assert logits.dtype == torch.float32 and logits.dim() == 2
    T, E = logits.shape
    ids = torch.empty((T, k), dtype=torch.int32, device=logits.device)
    w = torch.empty((T, k), dtype=torch.float32, device=logits.device)
    _check(lib().craft_route_topk(_dev(logits), T, E, k, int(renormalize), _dev(ids), _dev(w),
                                  _stream_ptr(stream)), "craft_route_topk")
    return ids, w


def expert_load(topk_ids, E: int, batch_tokens: int, stream=None):
    """topk_ids: cuda int32 [L][T][k] -> counts cuda int64 [B][L][E]."""
    import torch
    assert topk_ids.dtype == torch.int32 and topk_ids.dim() == 3
    L, T, k = topk_ids.shape
    B = (T + batch_tokens - 1) // batch_tokens
    counts = torch.empty((B, L, E), dtype=torch.int64, device=topk_ids.device)
    _check(lib().craft_expert_load(_dev(topk_ids), L, T, k, E, batch_tokens, _dev(counts),
                                   _stream_ptr(stream)), "craft_expert_load")
    return counts


def load_accumulate(counts, window, stream=None):
    """window (cuda int64) += counts (cuda int32), element by element."""
    import torch
    assert counts.dtype == torch.int32 and window.dtype == torch.int64
    assert counts.numel() == window.numel() and counts.is_contiguous() and window.is_contiguous()
    _check(lib().craft_load_accumulate(_dev(counts), counts.numel(), _dev(window),
                                       _stream_ptr(stream)), "craft_load_accumulate")
    return window


# ----------------------------------------------------------------------- planning

class Plan:
    """Owner of a craft_plan_t."""

    def __init__(self, load: np.ndarray, D: int, budget_bytes: int,
                 bytes_per_replica: Optional[Sequence[int]] = None, gpus_per_node: int = 8,
                 objective: int = 0, auto_r: bool = False):
        load = np.ascontiguousarray(load, dtype=np.int64)
        assert load.ndim == 3
        B, L, E = load.shape
        bpr = None if bytes_per_replica is None else np.ascontiguousarray(bytes_per_replica, np.int64)
        pp = PlanParams(L, E, D, gpus_per_node, B, load.ctypes.data,
                        None if bpr is None else bpr.ctypes.data, int(budget_bytes), objective,
                        1 if auto_r else 0)
        h = c_vp()
        _check(lib().craft_plan(ctypes.byref(pp), ctypes.byref(h)), "craft_plan")
        self._h = h
        self.L, self.E, self.D = L, E, D
        self._keep = []          # device table buffers stay alive with the plan

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h is not None and _lib is not None:
            _lib.craft_plan_destroy(h)

    def summary(self) -> dict:
        L, E, D = c_i32(), c_i32(), c_i32()
        tot, rf, ms = c_i64(), ctypes.c_double(), ctypes.c_double()
        _check(lib().craft_plan_summary(self._h, L, E, D, tot, rf, ms), "craft_plan_summary")
        return dict(L=L.value, E=E.value, D=D.value, total_replicas=tot.value,
                    replication_factor=rf.value, memory_saving_vs_uniform=ms.value)

    def layer(self, layer: int) -> dict:
        n, S, bal, mx = c_i32(), c_i32(), ctypes.c_double(), c_i64()
        _check(lib().craft_plan_layer_info(self._h, layer, n, S, bal, mx), "craft_plan_layer_info")
        copies = np.empty(self.E, np.int32)
        slot_expert = np.empty(S.value, np.int32)
        off = np.empty(self.D + 1, np.int32)
        load = np.empty(self.D, np.int64)
        _check(lib().craft_plan_layer_tables(self._h, layer, copies.ctypes.data,
                                             slot_expert.ctypes.data, off.ctypes.data,
                                             load.ctypes.data), "craft_plan_layer_tables")
        return dict(n_replicas=n.value, n_slots=S.value, est_balancedness=bal.value,
                    est_max_rank_load=mx.value, copies=copies, slot_expert=slot_expert,
                    rank_slot_off=off, rank_load=load)

    def greedy_order(self) -> np.ndarray:
        n = c_i64()
        _check(lib().craft_plan_greedy_order(self._h, None, 0, n), "craft_plan_greedy_order")
        out = np.empty(n.value, np.int32)
        _check(lib().craft_plan_greedy_order(self._h, out.ctypes.data, n.value, n),
               "craft_plan_greedy_order")
        return out

    def diff(self, new: "Plan", layer: int, rank: int) -> dict:
        """What `rank` does to its weights of `layer` when this plan is replaced by `new`."""
        off = new.layer(layer)["rank_slot_off"]
        reuse = np.empty(int(off[rank + 1] - off[rank]), np.int32)
        nf, nd = c_i32(), c_i32()
        _check(lib().craft_plan_diff(self._h, new._h, layer, rank, reuse.ctypes.data, nf, nd),
               "craft_plan_diff")
        return dict(reuse=reuse, n_fetch=nf.value, n_drop=nd.value)

    def benefit(self) -> dict:
        """Alg. 1's matrix as kept by an objective-1 plan."""
        K, tot, aR = c_i32(), ctypes.c_double(), c_i32()
        _check(lib().craft_plan_benefit(self._h, K, None, None, None, tot, aR), "craft_plan_benefit")
        counts = np.empty(K.value, np.int32)
        base = np.empty(self.L, np.float64)
        gain = np.empty((K.value, self.L), np.float64)
        _check(lib().craft_plan_benefit(self._h, K, counts.ctypes.data, base.ctypes.data,
                                        gain.ctypes.data, tot, aR), "craft_plan_benefit")
        return dict(counts=counts, base=base, gain=gain, total_gain=tot.value, auto_R=aR.value)

    def rank_rows(self, layer: int, counts: np.ndarray):
        counts = np.ascontiguousarray(counts, dtype=np.int64)
        assert counts.shape == (self.E,)
        rows = np.empty(self.D, np.int64)
        top = c_i32()
        _check(lib().craft_plan_rank_rows(self._h, layer, counts.ctypes.data, rows.ctypes.data, top),
               "craft_plan_rank_rows")
        return rows, top.value

    def upload_tables(self, layer: int, rank: int, device="cuda:0", stream=None):
        """Device tensor holding the tables of (layer, rank)."""
        import torch
        n = c_sz()
        _check(lib().craft_plan_tables_bytes(self._h, layer, rank, n), "craft_plan_tables_bytes")
        buf = torch.empty(n.value + 256, dtype=torch.uint8, device=device)
        _check(lib().craft_plan_tables_upload(self._h, layer, rank, _dev(buf), n.value,
                                              _stream_ptr(stream)), "craft_plan_tables_upload")
        self._keep.append(buf)
        return buf


# ---------------------------------------------------------------------- execution

def _torch_dtype(dtype: str):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def to_device(a: np.ndarray, dtype: str, device="cuda:0"):
    """Host float32 values (already representable in `dtype`) -> device tensor of `dtype`."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(device=device, dtype=_torch_dtype(dtype)).contiguous()


def pack_weights(w_gate, w_up, w_down, stream=None):
    """bf16 device matrices of one expert -> (packed_gateup, packed_down) device buffers."""
    import torch
    I, H = w_gate.shape
    assert w_gate.dtype == torch.bfloat16 and tuple(w_up.shape) == (I, H) and tuple(w_down.shape) == (H, I)
    a, b = c_sz(), c_sz()
    _check(lib().craft_pack_weights_bytes(CRAFT_BF16, H, I, a, b), "craft_pack_weights_bytes")
    pgu = torch.empty(a.value, dtype=torch.uint8, device=w_gate.device)
    pdn = torch.empty(b.value, dtype=torch.uint8, device=w_gate.device)
    _check(lib().craft_pack_weights(CRAFT_BF16, H, I, _dev(w_gate), _dev(w_up), _dev(w_down),
                                    _dev(pgu), _dev(pdn), _stream_ptr(stream)), "craft_pack_weights")
    return pgu, pdn


def quantize_e4m3(w, stream=None):
    """bf16 device matrix [rows][K] -> (codes uint8 [rows][K], scale fp32 [rows])."""
    import torch
    assert w.dtype == torch.bfloat16 and w.dim() == 2 and w.is_contiguous()
    rows, K = w.shape
    codes = torch.empty((rows, K), dtype=torch.uint8, device=w.device)
    scale = torch.empty(rows, dtype=torch.float32, device=w.device)
    _check(lib().craft_quantize_e4m3(_dev(w), rows, K, _dev(codes), _dev(scale), _stream_ptr(stream)),
           "craft_quantize_e4m3")
    return codes, scale


def pack_weights_e4m3(w_gate, w_up, w_down, stream=None):
    """bf16 device matrices of one expert -> E4M3-packed (gateup, down) device buffers."""
    import torch
    I, H = w_gate.shape
    q = [quantize_e4m3(m, stream) for m in (w_gate, w_up, w_down)]
    a, b = c_sz(), c_sz()
    _check(lib().craft_pack_weights_e4m3_bytes(H, I, a, b), "craft_pack_weights_e4m3_bytes")
    pgu = torch.empty(a.value, dtype=torch.uint8, device=w_gate.device)
    pdn = torch.empty(b.value, dtype=torch.uint8, device=w_gate.device)
    _check(lib().craft_pack_weights_e4m3(H, I, _dev(q[0][0]), _dev(q[1][0]), _dev(q[2][0]),
                                         _dev(q[0][1]), _dev(q[1][1]), _dev(q[2][1]),
                                         _dev(pgu), _dev(pdn), _stream_ptr(stream)),
           "craft_pack_weights_e4m3")
    return pgu, pdn


class RankForward:
    """Buffers and argument block for repeated forwards of one (plan, layer, rank)."""

    def __init__(self, plan: Plan, layer: int, rank: int, dtype: str, T: int, H: int, I: int,
                 k: int, w_gate: Sequence, w_up: Sequence, w_down: Sequence,
                 renormalize: bool = True, max_rows: int = 0, device="cuda:0",
                 want_debug_outputs: bool = False, packed: Optional[Sequence] = None,
                 weight_format: int = 0, w_router=None):
        import torch
        self.plan, self.layer, self.rank = plan, layer, rank
        self.dtype, self.T, self.H, self.I, self.k = dtype, T, H, I, k
        info = plan.layer(layer)
        self.S = info["n_slots"]
        off = info["rank_slot_off"]
        self.nslots = int(off[rank + 1] - off[rank])
        assert len(w_gate) == len(w_up) == len(w_down) == self.nslots
        td = _torch_dtype(dtype)
        for wg, wu, wd in zip(w_gate, w_up, w_down):
            assert wg.dtype == td and tuple(wg.shape) == (I, H) and wg.is_contiguous()
            assert wu.dtype == td and tuple(wu.shape) == (I, H) and wu.is_contiguous()
            assert wd.dtype == td and tuple(wd.shape) == (H, I) and wd.is_contiguous()
        self._weights = (list(w_gate), list(w_up), list(w_down))
        mk = lambda ws: torch.tensor([w.data_ptr() for w in ws] or [0], dtype=torch.int64,
                                     device=device)
        self._ptrs = (mk(w_gate), mk(w_up), mk(w_down))
        self._packed = None
        if packed is not None:           # list of (packed_gateup, packed_down) per slot
            assert len(packed) == self.nslots and dtype == "bf16"
            self._packed = (list(packed), mk([p[0] for p in packed]), mk([p[1] for p in packed]))
        self.tables = plan.upload_tables(layer, rank, device)
        self.out = torch.empty((T, H), dtype=td, device=device)
        self.debug = {}
        if want_debug_outputs:
            i32 = dict(dtype=torch.int32, device=device)
            self.debug = dict(ids=torch.empty((T, k), **i32),
                              topk_w=torch.empty((T, k), dtype=torch.float32, device=device),
                              dest=torch.empty((T, k), **i32), src=torch.empty((T * k,), **i32),
                              counts=torch.empty((plan.E,), **i32),
                              slot_cnt=torch.empty((self.S,), **i32),
                              slot_off=torch.empty((self.S + 1,), **i32))
        a = FwdArgs()
        a.dtype = CRAFT_BF16 if dtype == "bf16" else CRAFT_F32
        a.T, a.H, a.I, a.k = T, H, I, k
        a.renormalize = int(renormalize)
        a.w_gate, a.w_up, a.w_down = (p.data_ptr() for p in self._ptrs)
        if self._packed is not None:
            a.w_gateup_packed, a.w_down_packed = self._packed[1].data_ptr(), self._packed[2].data_ptr()
            a.weight_format = weight_format
        a.out = self.out.data_ptr()
        # scores come with every call, unless the forward runs the gating network itself
        self.w_router = w_router
        if w_router is not None:
            assert w_router.dtype == td and tuple(w_router.shape) == (plan.E, H) and w_router.is_contiguous()
            a.w_router = w_router.data_ptr()
        else:
            a.logits = self.out.data_ptr()       # stands in for "given" while the workspace is sized
        for name, t in self.debug.items():
            setattr(a, name, t.data_ptr())
        a.max_rows = max_rows
        a.tables = self.tables.data_ptr()
        n = c_sz()
        _check(lib().craft_moe_rank_forward_workspace(plan._h, layer, rank, ctypes.byref(a), n),
               "craft_moe_rank_forward_workspace")
        self.workspace = torch.empty(n.value + 256, dtype=torch.uint8, device=device)
        a.workspace = self.workspace.data_ptr()
        a.workspace_bytes = n.value
        self.args = a

    def __call__(self, x, logits=None, stream=None, static_scratch=False):
        """Enqueue one forward; returns the (reused) output tensor.  `logits` is left out by a
        forward that was given the gate's weights.  static_scratch: go through
        craft_moe_rank_forward_static (the library's own scratch instead of the workspace)."""
        import torch
        assert x.dtype == _torch_dtype(self.dtype) and tuple(x.shape) == (self.T, self.H)
        assert x.is_contiguous()
        self.args.x = x.data_ptr()
        if self.w_router is None:
            assert logits.dtype == torch.float32 and tuple(logits.shape) == (self.T, self.plan.E)
            assert logits.is_contiguous()
            self.args.logits = logits.data_ptr()
        else:
            assert logits is None
            self.args.logits = None
        entry = lib().craft_moe_rank_forward_static if static_scratch else lib().craft_moe_rank_forward
        _check(entry(self.plan._h, self.layer, self.rank, ctypes.byref(self.args), _stream_ptr(stream)),
               "craft_moe_rank_forward_static" if static_scratch else "craft_moe_rank_forward")
        return self.out

    def tile_choice(self):
        """Row-tile heights and rider switches the forward uses: (rows gate/up, rows down,
        riders gate/up, riders down)."""
        g, d, rg, rd = c_i32(), c_i32(), c_i32(), c_i32()
        _check(lib().craft_moe_rank_forward_tiles(self.plan._h, self.layer, self.rank,
                                                  ctypes.byref(self.args), g, d, rg, rd),
               "craft_moe_rank_forward_tiles")
        return g.value, d.value, rg.value, rd.value

    def tile_rows(self):
        """(gate/up, down) row-tile heights the forward uses."""
        return self.tile_choice()[:2]

    def result(self):
        """(rows routed to the rank, overflow flag) of the last forward; synchronises."""
        import torch
        torch.cuda.synchronize()
        rows, ovf = c_i64(), c_i32()
        _check(lib().craft_moe_rank_forward_result(_dev(self.workspace), rows, ovf),
               "craft_moe_rank_forward_result")
        return rows.value, ovf.value


def probe_copy(src, dst, stream=None):
    """dst <- src (device uint8 tensors of equal size, a multiple of 16 bytes)."""
    assert src.numel() == dst.numel() and src.element_size() == dst.element_size() == 1
    _check(lib().craft_probe_copy(_dev(src), _dev(dst), src.numel(), _stream_ptr(stream)), "craft_probe_copy")


def probe_read(src, passes: int, sink, blocks: int = 0, stream=None) -> float:
    """Enqueue the read loop over src (device uint8, a multiple of 32 KiB); returns the bytes it
    requests.  sink: device int32 tensor with at least blocks * 256 elements (0: 8 per CU)."""
    n = ctypes.c_double()
    _check(lib().craft_probe_read(_dev(src), src.numel(), passes, blocks, _dev(sink), n, _stream_ptr(stream)),
           "craft_probe_read")
    return n.value


def probe_mfma_bf16(iters: int, sink, blocks: int = 0, stream=None) -> float:
    """Enqueue the register-only MFMA loop; returns the floating-point operations it performs.
    sink: device float32 tensor with at least blocks * 256 elements (blocks = 0: 2 per CU)."""
    fl = ctypes.c_double()
    _check(lib().craft_probe_mfma_bf16(blocks, iters, _dev(sink), fl, _stream_ptr(stream)),
           "craft_probe_mfma_bf16")
    return fl.value


def probe_mfma_operands(shape: int, data: int, iters: int, sink, blocks: int = 0, stream=None) -> float:
    """Enqueue the matrix loop of the given instruction shape (0: 32x32x16, 1: 16x16x32) on operands
    of the given contents (0 zeros, 1 small values, 2 random); returns its floating-point operations.
    sink: device float32 tensor with at least blocks * 256 elements (blocks = 0: 1 per CU)."""
    fl = ctypes.c_double()
    _check(lib().craft_probe_mfma_operands(shape, data, blocks, iters, _dev(sink), fl, _stream_ptr(stream)),
           "craft_probe_mfma_operands")
    return fl.value


def timing_enable(level: int, max_forwards: int = 0):
    _check(lib().craft_timing_enable(level, max_forwards), "craft_timing_enable")


def timing_read() -> dict:
    ms = (ctypes.c_double * len(KERNEL_NAMES))()
    n = (c_i64 * len(KERNEL_NAMES))()
    _check(lib().craft_timing_read(ms, n), "craft_timing_read")
    return {name: dict(ms=ms[i], launches=n[i]) for i, name in enumerate(KERNEL_NAMES)}
