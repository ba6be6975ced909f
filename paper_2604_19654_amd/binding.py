"""ctypes binding of libfeplb.so.  Argument marshalling only: every step of the
path runs in the library's HIP kernels (or, for the plan, its host C++).  Torch
tensors provide device memory and streams; nothing here computes.

The library must have been built (python -m paper_2604_19654_amd.build, or
__graft_entry__.build()); loading fails loudly otherwise -- there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
ORD_MAX = 2**31 - 1
MAX_GROUPS = 128   # FEPLB_MAX_GROUPS
F32, BF16 = 0, 1
FFN_GATE_UP, FFN_DOWN, FFN_SCHEDULE, FFN_ALL = 1, 2, 4, 7
BWD_SCHEDULE, BWD_TRANSPOSE, BWD_DGRAD, BWD_WGRAD, BWD_ALL = 1, 2, 4, 8, 15
BWD_ACCUMULATE = 16
PLAN_WHOLE, PLAN_OVERFLOW = 0, 1


class FeplbError(RuntimeError):
    pass


class Group(C.Structure):
    _fields_ = [("expert", C.c_int32), ("ord_lo", C.c_int32), ("ord_hi", C.c_int32)]


class Move(C.Structure):
    _fields_ = [("expert", C.c_int32), ("src", C.c_int32), ("dst", C.c_int32),
                ("reserved", C.c_int32), ("rows", C.c_int64), ("ord_lo", C.c_int64)]


_LIB = None


def lib_path() -> str:
    return os.path.join(HERE, "libfeplb.so")


def lib():
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise FeplbError(f"{path} is missing: build it with `python -m paper_2604_19654_amd.build`")
        L = C.CDLL(path)
        vp, i32, sz, i64 = C.c_void_p, C.c_int32, C.c_size_t, C.c_int64
        L.feplb_version.restype = C.c_char_p
        L.feplb_last_error.restype = C.c_char_p
        L.feplb_route_topk.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp]
        L.feplb_permute_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.feplb_permute_workspace_bytes.restype = sz
        L.feplb_permute.argtypes = [vp, i32, i32, i32, C.POINTER(Group), i32, vp, i32, vp, i32,
                                    vp, vp, vp, vp, sz, vp]
        L.feplb_permute_append.argtypes = L.feplb_permute.argtypes
        L.feplb_grouped_ffn_workspace_bytes.argtypes = [i32, i32]
        L.feplb_grouped_ffn_workspace_bytes.restype = sz
        L.feplb_grouped_ffn.argtypes = [vp, vp, i32, i32, vp, i32, i32, i32, i32, i32, C.POINTER(vp), C.POINTER(vp),
                                        C.POINTER(vp), vp, vp, i32, i32, vp, sz, vp]
        L.feplb_grouped_ffn_static.argtypes = [vp, vp, i32, i32, vp, i32, i32, i32, i32, i32, C.POINTER(vp), C.POINTER(vp),
                                               C.POINTER(vp), vp, vp, i32, i32, vp]
        L.feplb_grouped_ffn_train.argtypes = [vp, vp, i32, i32, vp, i32, i32, i32, i32, i32, C.POINTER(vp), C.POINTER(vp),
                                              C.POINTER(vp), vp, vp, vp, i32, i32, vp, sz, vp]
        L.feplb_grouped_ffn_backward_wt_bytes.argtypes = [i32, i32, i32]
        L.feplb_grouped_ffn_backward_wt_bytes.restype = sz
        L.feplb_grouped_ffn_backward.argtypes = [vp, vp, i32, i32, i32, i32, i32, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                                 vp, vp, vp, vp, i32, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                                 vp, sz, i32, vp, sz, vp]
        L.feplb_unpermute_combine.argtypes = [vp, i32, i32, vp, vp, i32, i32, i32, vp, vp]
        L.feplb_combine_backward.argtypes = [vp, vp, i32, i32, vp, vp, i32, i32, i32, vp, vp, vp]
        L.feplb_route_topk_backward.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
        L.feplb_stage_weights.argtypes = [vp, vp, sz, vp, vp]
        L.feplb_stream_wait.argtypes = [vp, vp]
        L.feplb_expert_bytes.argtypes = [i32, i32, i32]
        L.feplb_expert_bytes.restype = sz
        L.feplb_plan.argtypes = [i32, i32, vp, vp, vp, vp, i64, i32, i32, C.POINTER(Move), i32,
                                 C.POINTER(i32), vp, vp, C.POINTER(i32)]
        L.feplb_history_update.argtypes = [i32, vp, vp, i32]
        L.feplb_place.argtypes = [i32, i32, vp, i32, vp, vp, vp, vp, C.POINTER(i32)]
        L.feplb_mark_dynamic.argtypes = [i32, i32, vp, vp, i32, vp]
        L.feplb_apply_moves.argtypes = [i32, i32, vp, C.POINTER(Move), i32, vp]
        L.feplb_straggler.argtypes = [i32, vp, C.POINTER(C.c_double)]
        for name in ("feplb_history_update", "feplb_place", "feplb_mark_dynamic", "feplb_apply_moves", "feplb_straggler"):
            getattr(L, name).restype = i32
        for name in ("feplb_route_topk", "feplb_permute", "feplb_permute_append", "feplb_grouped_ffn", "feplb_grouped_ffn_static", "feplb_grouped_ffn_train",
                     "feplb_grouped_ffn_backward", "feplb_unpermute_combine", "feplb_combine_backward",
                     "feplb_route_topk_backward",
                     "feplb_stage_weights", "feplb_stream_wait", "feplb_plan"):
            getattr(L, name).restype = i32
        _LIB = L
    return _LIB


_HIP = None


def hip_runtime():
    """The HIP runtime torch already loaded (so that streams and events are shared)."""
    global _HIP
    if _HIP is None:
        path = None
        with open("/proc/self/maps") as fh:
            for line in fh:
                if "libamdhip64" in line:
                    path = line.split()[-1]
                    break
        _HIP = C.CDLL(path or "libamdhip64.so")
        _HIP.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        _HIP.hipEventDestroy.argtypes = [C.c_void_p]
        _HIP.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        _HIP.hipEventSynchronize.argtypes = [C.c_void_p]
        _HIP.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
    return _HIP


class HipEvent:
    """A plain hipEvent_t (timing enabled), recordable on any stream."""

    def __init__(self):
        self.handle = C.c_void_p()
        rc = hip_runtime().hipEventCreate(C.byref(self.handle))
        if rc != 0:
            raise FeplbError(f"hipEventCreate failed: {rc}")

    def record(self, stream=None):
        rc = hip_runtime().hipEventRecord(self.handle, _stream(stream))
        if rc != 0:
            raise FeplbError(f"hipEventRecord failed: {rc}")

    def synchronize(self):
        rc = hip_runtime().hipEventSynchronize(self.handle)
        if rc != 0:
            raise FeplbError(f"hipEventSynchronize failed: {rc}")

    def elapsed_ms(self, later: "HipEvent") -> float:
        ms = C.c_float(0.0)
        rc = hip_runtime().hipEventElapsedTime(C.byref(ms), self.handle, later.handle)
        if rc != 0:
            raise FeplbError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def __del__(self):
        try:
            if self.handle:
                hip_runtime().hipEventDestroy(self.handle)
        except Exception:
            pass


def version() -> str:
    return lib().feplb_version().decode()


def _check(rc: int, what: str):
    if rc != 0:
        raise FeplbError(f"{what} failed with code {rc}: {lib().feplb_last_error().decode()}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_contiguous():
        raise FeplbError("tensors passed to the library must be contiguous")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _need(t: torch.Tensor, dtype, name: str):
    if not t.is_cuda or t.dtype != dtype:
        raise FeplbError(f"{name}: expected a CUDA tensor of {dtype}, got {t.dtype} on {t.device}")


def feplb_route_topk(logits, k, topk_ids=None, topk_w=None, counts=None, want_counts=True, stream=None):
    """logits fp32 [T,E] -> (topk_ids int32 [T,k], topk_w fp32 [T,k], counts int32 [E] or None)."""
    _need(logits, torch.float32, "logits")
    T, E = logits.shape
    dev = logits.device
    if topk_ids is None:
        topk_ids = torch.empty((T, k), dtype=torch.int32, device=dev)
    if topk_w is None:
        topk_w = torch.empty((T, k), dtype=torch.float32, device=dev)
    if counts is None and want_counts:
        counts = torch.empty((E,), dtype=torch.int32, device=dev)
    _check(lib().feplb_route_topk(_ptr(logits), T, E, k, _ptr(topk_ids), _ptr(topk_w), _ptr(counts),
                                  _stream(stream)), "feplb_route_topk")
    return topk_ids, topk_w, counts


def feplb_permute_workspace_bytes(T, k, E, G) -> int:
    return int(lib().feplb_permute_workspace_bytes(T, k, E, G))


def _group_array(groups: Sequence):
    arr = (Group * max(len(groups), 1))()
    for i, g in enumerate(groups):
        e, lo, hi = (g.expert, g.ord_lo, g.ord_hi) if isinstance(g, Group) else g
        arr[i] = Group(int(e), int(lo), int(hi))
    return arr


def feplb_permute(topk_ids, E, groups, X, R_cap, Xp=None, offsets=None, row_src=None, inv=None,
                  ws=None, stream=None, append=False):
    """-> (Xp bf16 [R_cap,d], offsets int32 [G+1], row_src int32 [R_cap], inv int32 [T*k]).
    append=True calls feplb_permute_append: offsets[0] is then the (device-side) row these groups
    start at, and offsets, row_src and inv must be the earlier call's buffers."""
    if append and (offsets is None or row_src is None or inv is None):
        raise FeplbError("feplb_permute(append=True) continues an earlier call: pass its offsets view, row_src and inv")
    _need(topk_ids, torch.int32, "topk_ids")
    T, k = topk_ids.shape
    G = len(groups)
    dev = topk_ids.device
    d = 0
    if X is not None:
        _need(X, torch.bfloat16, "X")
        d = X.shape[1]
        if Xp is None:
            Xp = torch.empty((R_cap, d), dtype=torch.bfloat16, device=dev)
    if offsets is None:
        offsets = torch.empty((G + 1,), dtype=torch.int32, device=dev)
    if row_src is None:
        row_src = torch.empty((max(R_cap, 1),), dtype=torch.int32, device=dev)
    if inv is None:
        inv = torch.empty((max(T * k, 1),), dtype=torch.int32, device=dev)
    need = feplb_permute_workspace_bytes(T, k, E, G)
    if ws is None:
        ws = torch.empty((need,), dtype=torch.uint8, device=dev)
    fn = lib().feplb_permute_append if append else lib().feplb_permute
    _check(fn(_ptr(topk_ids), T, k, E, _group_array(groups), G, _ptr(X), d, _ptr(Xp),
              R_cap, _ptr(offsets), _ptr(row_src), _ptr(inv), _ptr(ws), ws.numel(),
              _stream(stream)), "feplb_permute_append" if append else "feplb_permute")
    return Xp, offsets, row_src, inv


def feplb_grouped_ffn_workspace_bytes(R_cap, G) -> int:
    return int(lib().feplb_grouped_ffn_workspace_bytes(R_cap, G))


def _ptr_array(tensors: Sequence[Optional[torch.Tensor]]):
    arr = (C.c_void_p * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else (t if isinstance(t, int) else _ptr(t))
    return arr


def feplb_grouped_ffn(Xp, offsets, g_begin, g_end, d, f, w_gate, w_up, w_down, H, Yp,
                      phases=FFN_ALL, ws=None, stream=None, row_src=None, k=0, AB=None):
    """Runs groups [g_begin, g_end).  w_* are sequences (indexed by group) of bf16
    tensors or raw device addresses.  H bf16 [R_cap,f]; Yp fp32 or bf16 [R_cap,d].
    With row_src (int32 [R_cap], from feplb_permute) and k, Xp is the unpermuted X [T,d] and the
    rows X[row_src[r] // k] are gathered as the gate/up GEMM loads them.
    With AB (bf16 [R_cap,2f]) the call is feplb_grouped_ffn_train: the derivatives of the SwiGLU
    product with respect to the gate and up products are kept in AB for feplb_grouped_ffn_backward."""
    R_cap = H.shape[0]
    yp_dtype = F32
    if Yp is not None:
        yp_dtype = {torch.float32: F32, torch.bfloat16: BF16}[Yp.dtype]
    if ws is None:
        ws = torch.empty((feplb_grouped_ffn_workspace_bytes(R_cap, g_end),), dtype=torch.uint8,
                         device=H.device)
    n_src = int(Xp.shape[0]) if row_src is not None else 0
    if AB is not None:
        _need(AB, torch.bfloat16, "AB")
        if tuple(AB.shape) != (R_cap, 2 * f):
            raise FeplbError("AB must be [R_cap, 2f]")
        _check(lib().feplb_grouped_ffn_train(_ptr(Xp), _ptr(row_src), n_src, k, _ptr(offsets), g_begin, g_end, R_cap, d, f,
                                             _ptr_array(w_gate), _ptr_array(w_up), _ptr_array(w_down),
                                             _ptr(H), _ptr(AB), _ptr(Yp), yp_dtype, phases, _ptr(ws), ws.numel(),
                                             _stream(stream)), "feplb_grouped_ffn_train")
        return H, Yp
    _check(lib().feplb_grouped_ffn(_ptr(Xp), _ptr(row_src), n_src, k, _ptr(offsets), g_begin, g_end, R_cap, d, f,
                                   _ptr_array(w_gate), _ptr_array(w_up), _ptr_array(w_down),
                                   _ptr(H), _ptr(Yp), yp_dtype, phases, _ptr(ws), ws.numel(),
                                   _stream(stream)), "feplb_grouped_ffn")
    return H, Yp


STATIC_WS_BYTES = 262144   # FEPLB_STATIC_WS_BYTES


def feplb_grouped_ffn_static(Xp, offsets, g_begin, g_end, d, f, w_gate, w_up, w_down, H, Yp,
                             phases=FFN_ALL, stream=None, row_src=None, k=0):
    """feplb_grouped_ffn without a workspace: the tile table lives in device memory that is part of
    the library (for callers that cannot allocate).  Same arguments and results otherwise."""
    R_cap = H.shape[0]
    yp_dtype = F32
    if Yp is not None:
        yp_dtype = {torch.float32: F32, torch.bfloat16: BF16}[Yp.dtype]
    n_src = int(Xp.shape[0]) if row_src is not None else 0
    _check(lib().feplb_grouped_ffn_static(_ptr(Xp), _ptr(row_src), n_src, k, _ptr(offsets), g_begin, g_end, R_cap, d, f,
                                          _ptr_array(w_gate), _ptr_array(w_up), _ptr_array(w_down),
                                          _ptr(H), _ptr(Yp), yp_dtype, phases, _stream(stream)),
           "feplb_grouped_ffn_static")
    return H, Yp


def feplb_grouped_ffn_backward_wt_bytes(n_groups, d, f) -> int:
    return int(lib().feplb_grouped_ffn_backward_wt_bytes(n_groups, d, f))


def feplb_grouped_ffn_backward(Xp, offsets, g_begin, g_end, d, f, w_gate, w_up, w_down, H, AB, dYp, dXp,
                               dw_gate, dw_up, dw_down, WT=None, phases=BWD_ALL, ws=None, stream=None):
    """Backward of groups [g_begin, g_end).  Xp bf16 [R_cap,d] (materialised), H bf16 [R_cap,f] and
    AB bf16 [R_cap,2f] as left by feplb_grouped_ffn(..., AB=AB), dYp bf16 [R_cap,d].  Writes dXp
    (fp32 or bf16 [R_cap,d]), da | db over AB, and the fp32 weight gradients dw_*[g]."""
    R_cap = H.shape[0]
    dev = H.device
    dxp_dtype = F32
    if dXp is not None:
        dxp_dtype = {torch.float32: F32, torch.bfloat16: BF16}[dXp.dtype]
    if WT is None:
        WT = torch.empty((max(feplb_grouped_ffn_backward_wt_bytes(g_end - g_begin, d, f), 16),), dtype=torch.uint8, device=dev)
    if ws is None:
        ws = torch.empty((feplb_grouped_ffn_workspace_bytes(R_cap, g_end),), dtype=torch.uint8, device=dev)
    _check(lib().feplb_grouped_ffn_backward(_ptr(Xp), _ptr(offsets), g_begin, g_end, R_cap, d, f,
                                            _ptr_array(w_gate), _ptr_array(w_up), _ptr_array(w_down),
                                            _ptr(H), _ptr(AB), _ptr(dYp), _ptr(dXp), dxp_dtype,
                                            _ptr_array(dw_gate), _ptr_array(dw_up), _ptr_array(dw_down),
                                            _ptr(WT), WT.numel(), phases, _ptr(ws), ws.numel(), _stream(stream)),
           "feplb_grouped_ffn_backward")
    return dXp


def feplb_unpermute_combine(Yp, inv, topk_w, T, k, d, Y=None, stream=None):
    """-> Y bf16 [T,d]."""
    yp_dtype = {torch.float32: F32, torch.bfloat16: BF16}[Yp.dtype]
    if Y is None:
        Y = torch.empty((T, d), dtype=torch.bfloat16, device=Yp.device)
    _check(lib().feplb_unpermute_combine(_ptr(Yp), yp_dtype, int(Yp.shape[0]), _ptr(inv), _ptr(topk_w), T, k, d, _ptr(Y),
                                         _stream(stream)), "feplb_unpermute_combine")
    return Y


def feplb_combine_backward(dY, Yp, inv, topk_w, T, k, d, dYp, dw=None, stream=None):
    """dY bf16 [T,d], Yp [R_cap,d] (fp32 or bf16) -> dYp bf16 [R_cap,d] (written in place), dw fp32 [T,k]."""
    _need(dY, torch.bfloat16, "dY")
    _need(dYp, torch.bfloat16, "dYp")
    yp_dtype = {torch.float32: F32, torch.bfloat16: BF16}[Yp.dtype]
    if dw is None:
        dw = torch.empty((T, k), dtype=torch.float32, device=dY.device)
    if dYp.shape[0] != Yp.shape[0]:
        raise FeplbError("Yp and dYp must hold the same number of rows")
    _check(lib().feplb_combine_backward(_ptr(dY), _ptr(Yp), yp_dtype, int(Yp.shape[0]), _ptr(inv), _ptr(topk_w), T, k, d,
                                        _ptr(dYp), _ptr(dw), _stream(stream)), "feplb_combine_backward")
    return dYp, dw


def feplb_route_topk_backward(topk_ids, topk_w, dw, E, dlogits=None, stream=None):
    """-> dlogits fp32 [T,E]."""
    T, k = topk_ids.shape
    if dlogits is None:
        dlogits = torch.empty((T, E), dtype=torch.float32, device=topk_ids.device)
    _check(lib().feplb_route_topk_backward(_ptr(topk_ids), _ptr(topk_w), _ptr(dw), T, E, k, _ptr(dlogits),
                                           _stream(stream)), "feplb_route_topk_backward")
    return dlogits


def feplb_stage_weights(slot: torch.Tensor, src: torch.Tensor, side_stream, done_event: "HipEvent" = None):
    """Async copy src -> slot on side_stream; records done_event there if given."""
    nbytes = src.numel() * src.element_size()
    if slot.numel() * slot.element_size() < nbytes:
        raise FeplbError("staging slot smaller than the source")
    _check(lib().feplb_stage_weights(_ptr(slot), _ptr(src), nbytes, _stream(side_stream),
                                     done_event.handle if done_event is not None else None),
           "feplb_stage_weights")


def feplb_stream_wait(stream, event: "HipEvent"):
    _check(lib().feplb_stream_wait(_stream(stream), event.handle), "feplb_stream_wait")


def feplb_expert_bytes(d, f, elem_bytes=2) -> int:
    return int(lib().feplb_expert_bytes(d, f, elem_bytes))


def feplb_plan(P, owner, n, dyn_flag, slots, tau=0, mode=PLAN_WHOLE, this_rank=-1, max_moves=None):
    """Host-only.  Returns (moves [(expert, src, dst, rows, ord_lo)], load_before, load_after, chosen_rank)."""
    owner = np.ascontiguousarray(owner, dtype=np.int32)
    n = np.ascontiguousarray(n, dtype=np.int64)
    dyn_flag = np.ascontiguousarray(dyn_flag, dtype=np.uint8)
    slots = np.ascontiguousarray(slots, dtype=np.int32)
    E = int(n.shape[0])
    if owner.shape[0] != E or dyn_flag.shape[0] != E or slots.shape[0] != P:
        raise FeplbError("feplb_plan: array lengths do not match P/E")
    if max_moves is None:
        max_moves = int(slots.sum()) if mode == PLAN_WHOLE else int(slots[this_rank] if this_rank >= 0 else slots.max(initial=0))
        max_moves = max(max_moves, 1)
    moves = (Move * max_moves)()
    n_moves = C.c_int32(0)
    chosen = C.c_int32(-1)
    before = np.zeros(P, dtype=np.int64)
    after = np.zeros(P, dtype=np.int64)
    _check(lib().feplb_plan(P, E, owner.ctypes.data, n.ctypes.data, dyn_flag.ctypes.data,
                            slots.ctypes.data, int(tau), int(mode), int(this_rank), moves, max_moves,
                            C.byref(n_moves), before.ctypes.data, after.ctypes.data, C.byref(chosen)),
           "feplb_plan")
    out = [(m.expert, m.src, m.dst, int(m.rows), int(m.ord_lo)) for m in moves[: n_moves.value]]
    return out, before, after, chosen.value


HIST_FRAC_BITS = 16   # FEPLB_HIST_FRAC_BITS


def feplb_history_update(hist: np.ndarray, n, shift: int) -> np.ndarray:
    """Host-only.  Updates the int64 history array in place (and returns it)."""
    if hist.dtype != np.int64 or not hist.flags.c_contiguous:
        raise FeplbError("feplb_history_update: hist must be a contiguous int64 array")
    n = np.ascontiguousarray(n, dtype=np.int64)
    if n.shape != hist.shape:
        raise FeplbError("feplb_history_update: hist and n differ in length")
    _check(lib().feplb_history_update(int(hist.shape[0]), hist.ctypes.data, n.ctypes.data, int(shift)),
           "feplb_history_update")
    return hist


def feplb_place(P, hist, cap, owner_in):
    """Host-only.  Returns (owner_out int32 [E], load_before, load_after, migrated)."""
    hist = np.ascontiguousarray(hist, dtype=np.int64)
    owner_in = np.ascontiguousarray(owner_in, dtype=np.int32)
    E = int(hist.shape[0])
    if owner_in.shape[0] != E:
        raise FeplbError("feplb_place: array lengths differ")
    owner_out = np.zeros(E, dtype=np.int32)
    before = np.zeros(P, dtype=np.int64)
    after = np.zeros(P, dtype=np.int64)
    moved = C.c_int32(0)
    _check(lib().feplb_place(P, E, hist.ctypes.data, int(cap), owner_in.ctypes.data, owner_out.ctypes.data,
                             before.ctypes.data, after.ctypes.data, C.byref(moved)), "feplb_place")
    return owner_out, before, after, int(moved.value)


def feplb_mark_dynamic(P, owner, hist, dyn) -> np.ndarray:
    """Host-only.  -> uint8 [E] flags."""
    owner = np.ascontiguousarray(owner, dtype=np.int32)
    hist = np.ascontiguousarray(hist, dtype=np.int64)
    flag = np.zeros(owner.shape[0], dtype=np.uint8)
    if hist.shape != owner.shape:
        raise FeplbError("feplb_mark_dynamic: array lengths differ")
    _check(lib().feplb_mark_dynamic(P, int(owner.shape[0]), owner.ctypes.data, hist.ctypes.data, int(dyn),
                                    flag.ctypes.data), "feplb_mark_dynamic")
    return flag


def feplb_apply_moves(P, owner, moves) -> np.ndarray:
    """Host-only.  moves as returned by feplb_plan.  -> int32 [E]: the rank that runs each expert."""
    owner = np.ascontiguousarray(owner, dtype=np.int32)
    arr = (Move * max(len(moves), 1))()
    for i, (e, src, dst, rows, lo) in enumerate(moves):
        arr[i] = Move(int(e), int(src), int(dst), 0, int(rows), int(lo))
    home = np.zeros(owner.shape[0], dtype=np.int32)
    _check(lib().feplb_apply_moves(P, int(owner.shape[0]), owner.ctypes.data, arr, len(moves), home.ctypes.data),
           "feplb_apply_moves")
    return home


def feplb_straggler(values) -> float:
    """Host-only.  max - mean of a per-rank quantity."""
    v = np.ascontiguousarray(values, dtype=np.float64)
    out = C.c_double(0.0)
    _check(lib().feplb_straggler(int(v.shape[0]), v.ctypes.data, C.byref(out)), "feplb_straggler")
    return float(out.value)
