"""ctypes binding of liboptstage.so: the same names as include/optstage.h and
include/optstage_ops.h, argument marshalling only.  Every step of the path runs in the
library's HIP kernels; there is no fallback — if the library is missing, importing this
module's `lib()` raises."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liboptstage.so")

OK, E_ARG, E_ORDER, E_BUDGET, E_HOSTPOOL, E_HIP, E_STATE, E_ARENA = 0, -1, -2, -3, -4, -5, -6, -7
OP_F, OP_B, OP_W, OP_O, OP_OWAIT, OP_R = range(6)
OP_CODE = {"F": OP_F, "B": OP_B, "W": OP_W, "O": OP_O, "OWAIT": OP_OWAIT, "R": OP_R}
KINDS = ("X_IN", "N1", "QKV", "O", "LSE", "X_MID", "N2", "GU", "A", "STATS", "DY", "DX_MID")
KIND_ID = {k: i for i, k in enumerate(KINDS)}
N_KINDS, N_F_KINDS = 12, 10
WEIGHTS = ("g1", "b1", "wqkv", "wo", "g2", "b2", "wgu", "wd")
WEIGHT_ID = {k: i for i, k in enumerate(WEIGHTS)}
KERNEL_CLASSES = ("gemm_nt_store", "gemm_nt_resid", "gemm_tn_accum", "attn_fwd", "attn_bwd", "norm_fwd", "norm_bwd",
                  "act_fwd", "act_bwd", "rope", "gemm_nt_qkv", "gemm_nt_gu")
GEMM_NT, GEMM_TN, GEMM_NT_SLAB = 0, 1, 2
EPI_STORE, EPI_RESID, EPI_ACCUM = 0, 1, 2


class Desc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("family", C.c_uint32), ("dtype", C.c_uint32),
                ("n_layers", C.c_uint32), ("hidden", C.c_uint32), ("n_q_heads", C.c_uint32),
                ("n_kv_heads", C.c_uint32), ("head_dim", C.c_uint32), ("ffn", C.c_uint32), ("seq", C.c_uint32),
                ("micro_batch", C.c_uint32), ("stage_index", C.c_uint32), ("n_stages", C.c_uint32),
                ("n_microbatches", C.c_uint32), ("norm_eps", C.c_float), ("rope_base", C.c_float),
                ("recompute", C.c_uint32), ("n_chunks", C.c_uint32), ("no_fusion", C.c_uint32), ("reserved", C.c_uint32),
                ("hbm_budget_bytes", C.c_uint64), ("arena", C.c_void_p), ("arena_bytes", C.c_uint64),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_uint64), ("host_pool", C.c_void_p),
                ("host_pool_bytes", C.c_uint64), ("compute_stream", C.c_void_p), ("copy_stream", C.c_void_p),
                ("reload_stream", C.c_void_p)]


class GemmProblem(C.Structure):
    _fields_ = [("A", C.c_void_p), ("B", C.c_void_p), ("C", C.c_void_p), ("R", C.c_void_p),
                ("M", C.c_uint32), ("N", C.c_uint32), ("lda", C.c_uint32), ("ldb", C.c_uint32), ("ldc", C.c_uint32)]


class Event(C.Structure):
    _fields_ = [("op", C.c_uint32), ("microbatch", C.c_uint32), ("layer", C.c_uint32), ("kind_mask", C.c_uint32)]


class Stats(C.Structure):
    _fields_ = [("live_bytes", C.c_uint64), ("peak_bytes", C.c_uint64), ("bytes_offloaded", C.c_uint64),
                ("bytes_reloaded", C.c_uint64), ("n_ops", C.c_uint64 * 6), ("ms_ops", C.c_double * 6),
                ("arena_high_water", C.c_uint64), ("kernel_launches", C.c_uint64 * 12),
                ("kernel_ms", C.c_double * 12), ("kernel_work", C.c_double * 12),
                ("min_live_bytes", C.c_uint64), ("avg_live_bytes", C.c_double), ("stall_ms", C.c_double * 2),
                ("n_trace", C.c_uint64)]


class TraceEntry(C.Structure):
    _fields_ = [("op", C.c_uint32), ("microbatch", C.c_uint32), ("layer", C.c_uint32), ("kind_mask", C.c_uint32),
                ("live_bytes", C.c_uint64), ("start_ms", C.c_double), ("end_ms", C.c_double), ("stall_ms", C.c_double)]


class OptstageError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"optstage status {status}: {msg}")
        self.status = status


_lib = None
_vp, _u32, _u64, _f32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_float

_SIGS = {
    "optstage_query_sizes": [C.POINTER(Desc), C.POINTER(_u64), C.POINTER(_u64), C.POINTER(_u64)],
    "optstage_create": [C.POINTER(Desc), C.POINTER(_vp)],
    "optstage_set_weight": [_vp, _u32, _u32, _vp, _vp],
    "optstage_bind_io": [_vp, _u32, _vp, _vp, _vp, _vp],
    "optstage_bind_io_chunk": [_vp, _u32, _u32, _vp, _vp, _vp, _vp],
    "optstage_validate": [_vp, C.POINTER(Event), C.c_size_t, C.POINTER(C.c_size_t)],
    "optstage_run": [_vp, C.POINTER(Event), C.c_size_t],
    "optstage_forward": [_vp, _u32],
    "optstage_backward_input": [_vp, _u32],
    "optstage_backward_weight": [_vp, _u32],
    "optstage_offload": [_vp, _u32, _u32, _u32],
    "optstage_offload_wait": [_vp, _u32, _u32, _u32],
    "optstage_reload": [_vp, _u32, _u32, _u32],
    "optstage_synchronize": [_vp],
    "optstage_reset": [_vp],
    "optstage_get_stats": [_vp, C.POINTER(Stats)],
    "optstage_set_kernel_timing": [_vp, _u32],
    "optstage_get_trace": [_vp, C.POINTER(TraceEntry), C.c_size_t, C.POINTER(C.c_size_t)],
    "optstage_set_grad_overwrite": [_vp, _u32],
    "optstage_debug_checksum": [_vp, _u32, _u32, _u32, _u32, C.POINTER(_u64)],
    "optstage_debug_read": [_vp, _u32, _u32, _u32, _vp, _u64],
    "optstage_plan": [C.POINTER(Desc), C.POINTER(Event), C.c_size_t, C.POINTER(C.c_size_t), C.POINTER(_u64), C.POINTER(_u64)],
    "optstage_op_gemm": [_u32, _u32, _u32, _vp, _vp, _vp, _vp, _u32, _u32, _u32, _u32, _u32, _u32, _vp],
    "optstage_op_gemm_rope": [_u32, _vp, _vp, _vp, _u32, _u32, _u32, _u32, _u32, _u32, _vp, _u32, _u32, _vp],
    "optstage_op_gemm_swiglu": [_vp, _vp, _vp, _vp, _u32, _u32, _u32, _u32, _vp],
    "optstage_op_gemm_grouped": [_u32, _u32, _u32, _vp, _u32, _vp],
    "optstage_op_weight_slabs": [_vp, _vp, _u32, _u32, _u32, _vp],
    "optstage_op_norm_fwd": [_u32, _u32, _vp, _vp, _vp, _vp, _vp, _u32, _u32, _f32, _vp],
    "optstage_op_norm_bwd": [_u32, _u32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _u32, _u32, _vp],
    "optstage_op_norm_bwd_static": [_u32, _u32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _u32, _u32, _vp],
    "optstage_op_act_fwd": [_u32, _u32, _vp, _vp, _u32, _u32, _vp],
    "optstage_op_act_bwd": [_u32, _u32, _vp, _vp, _vp, _u32, _u32, _vp],
    "optstage_op_rope_table": [_vp, _u32, _u32, _f32, _vp],
    "optstage_op_rope": [_u32, _vp, _vp, _vp, _u32, _u32, _u32, _u32, _u32, _u32, _vp],
    "optstage_op_attn_fwd": [_u32, _vp, _vp, _vp, _u32, _u32, _u32, _u32, _u32, _vp],
    "optstage_op_attn_bwd": [_u32, _vp, _vp, _vp, _vp, _vp, _vp, _u32, _u32, _u32, _u32, _u32, _vp],
    "optstage_op_checksum": [_vp, _u64, _vp, _vp],
}
EXPORTS = tuple(_SIGS) + ("optstage_destroy", "optstage_last_error", "optstage_op_attn_bwd_ws_floats")


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OptstageError(E_STATE, f"{LIB_PATH} is missing: run `python -m paper_2510_05186_amd.build` "
                                         "(there is no CPU fallback)")
        # PyTorch supplies the device memory and the streams this library works on, and it ships a HIP runtime of its
        # own: that runtime has to be the one in the process before liboptstage.so is mapped (a second runtime, pulled
        # in by this library's own dependency when it is loaded first, sees no device)
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        for name, args in _SIGS.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = C.c_int
        L.optstage_destroy.argtypes = [_vp]
        L.optstage_destroy.restype = None
        L.optstage_last_error.argtypes = []
        L.optstage_last_error.restype = C.c_char_p
        L.optstage_op_attn_bwd_ws_floats.argtypes = [_u32] * 5
        L.optstage_op_attn_bwd_ws_floats.restype = _u64
        _lib = L
    return _lib


def check(status):
    if status != OK:
        raise OptstageError(status, lib().optstage_last_error().decode())


def make_events(events) -> "C.Array":
    """events: iterable of ("F", j) / ("F", j, chunk) / ("O", j, layer, kinds) tuples (kinds = names or ids)."""
    events = list(events)
    arr = (Event * max(1, len(events)))()
    for n, ev in enumerate(events):
        arr[n].op = OP_CODE[ev[0]] if isinstance(ev[0], str) else int(ev[0])
        arr[n].microbatch = ev[1]
        if len(ev) == 3:
            arr[n].layer = ev[2]                       # compute op of a model chunk
        elif len(ev) > 3:
            arr[n].layer = ev[2]
            mask = 0
            for k in ev[3]:
                mask |= 1 << (KIND_ID[k] if isinstance(k, str) else int(k))
            arr[n].kind_mask = mask
    return arr


def make_desc(cfg, budget=0, arena=0, arena_bytes=0, workspace=0, workspace_bytes=0, host_pool=0,
              host_pool_bytes=0, compute_stream=0, copy_stream=0, reload_stream=0, recompute=0, n_chunks=1,
              no_fusion=0) -> Desc:
    d = Desc()
    d.struct_size = C.sizeof(Desc)
    d.family, d.dtype = cfg.family, cfg.dtype
    d.n_layers, d.hidden, d.n_q_heads, d.n_kv_heads = cfg.n_layers, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads
    d.head_dim, d.ffn, d.seq, d.micro_batch = cfg.head_dim, cfg.ffn, cfg.seq, cfg.micro_batch
    d.stage_index, d.n_stages, d.n_microbatches = cfg.stage_index, cfg.n_stages, cfg.n_microbatches
    d.norm_eps, d.rope_base = cfg.norm_eps, cfg.rope_base
    d.hbm_budget_bytes = int(budget)
    d.arena, d.arena_bytes = arena, arena_bytes
    d.workspace, d.workspace_bytes = workspace, workspace_bytes
    d.host_pool, d.host_pool_bytes = host_pool, host_pool_bytes
    d.compute_stream, d.copy_stream = compute_stream, copy_stream
    d.reload_stream = reload_stream
    d.recompute = int(recompute)
    d.n_chunks = int(n_chunks)
    d.no_fusion = int(no_fusion)
    return d


def query_sizes(cfg, recompute=0):
    """-> (min_workspace, act_bytes_per_mb, {kind: bytes})"""
    d = make_desc(cfg, recompute=recompute)
    ws, act = _u64(), _u64()
    kinds = (_u64 * N_KINDS)()
    check(lib().optstage_query_sizes(C.byref(d), C.byref(ws), C.byref(act), kinds))
    return ws.value, act.value, {k: kinds[i] for i, k in enumerate(KINDS)}


def plan(cfg, events, budget=0, recompute=0, n_chunks=1):
    """Pure-host validation + accounting.  -> (status, first_bad, peak_bytes, live_after list)."""
    d = make_desc(cfg, budget=budget, recompute=recompute, n_chunks=n_chunks)
    arr = make_events(events)
    n = len(list(events)) if not isinstance(events, list) else len(events)
    bad = C.c_size_t(0)
    peak = _u64(0)
    live = (_u64 * max(1, n))()
    st = lib().optstage_plan(C.byref(d), arr, n, C.byref(bad), C.byref(peak), live)
    return st, bad.value, peak.value, [live[i] for i in range(n)]
