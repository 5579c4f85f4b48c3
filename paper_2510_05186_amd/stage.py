"""Thin convenience layer over the C-ABI: obtains device / pinned memory and streams from
PyTorch, hands raw pointers to liboptstage and keeps the tensors alive.  No arithmetic
happens here."""
from __future__ import annotations

import ctypes as C

import numpy as np
import torch

from . import binding as B

_TORCH_DT = {0: torch.float32, 1: torch.bfloat16}
_STREAMS = []   # one (compute, offload, reload) triple per process: every Stage shares it, so the streams keep
                # the distinct hardware queues they were given when created and copies overlap compute


def _streams():
    if not _STREAMS:
        _STREAMS.extend([torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()])
    return _STREAMS


def to_device(a: np.ndarray, dtype: int) -> torch.Tensor:
    """float32 numpy (already rounded to the stage dtype) -> device tensor of the stage dtype."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(device="cuda", dtype=_TORCH_DT[dtype]).contiguous()


def to_numpy(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(dtype=torch.float32, device="cpu").numpy().astype(np.float64)


class Stage:
    def __init__(self, cfg, budget: int = 0, arena_bytes: int | None = None, host_pool_bytes: int = 0,
                 duplex: bool = False, recompute: bool = False, n_chunks: int = 1, grad_overwrite: bool = False,
                 host_pool: torch.Tensor | None = None, no_fusion: bool = False):
        """duplex: reloads get a stream of their own instead of sharing the offloads' (single channel).
        recompute: F keeps no norm outputs and no MLP activation output; B rebuilds them for W.
        n_chunks: model chunks on this stage (cfg.n_layers counts all of them).
        grad_overwrite: the first B / W of an iteration store the parameter gradients instead of adding to them, so
        the accumulators need no clearing between iterations.
        no_fusion: rotary and the MLP activation always run as kernels of their own (by default they run in the
        epilogues of the QKV and gate / up projections where the shapes allow it).
        host_pool: a pinned uint8 tensor to use as the offload pool instead of allocating host_pool_bytes (a process
        that runs several stages one after the other can hand the same block to each)."""
        if not torch.cuda.is_available():
            raise RuntimeError("optstage needs a GPU: there is no CPU path")
        self.cfg = cfg
        self.lib = B.lib()
        self.recompute = bool(recompute)
        ws_bytes, act_per_mb, self.kind_bytes = B.query_sizes(cfg, recompute=int(recompute))
        self.act_bytes_per_mb = act_per_mb
        if arena_bytes is None:
            full = act_per_mb if not recompute else B.query_sizes(cfg)[1]   # B and W hold the rebuilt kinds too
            arena_bytes = int((budget if budget else full * cfg.n_microbatches) * 1.25) + (64 << 20)
        self.n_chunks = int(n_chunks)
        self.arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        if host_pool is not None:
            if not host_pool.is_pinned() or host_pool.dtype != torch.uint8:
                raise ValueError("host_pool must be a pinned uint8 tensor")
            self.host_pool, host_pool_bytes = host_pool, host_pool.numel()
        else:
            self.host_pool = torch.empty(host_pool_bytes, dtype=torch.uint8, pin_memory=True) if host_pool_bytes else None
        self.compute_stream, self.copy_stream, self.reload_stream = _streams()
        self.desc = B.make_desc(
            cfg, budget=budget, arena=self.arena.data_ptr(), arena_bytes=arena_bytes,
            workspace=self.workspace.data_ptr(), workspace_bytes=ws_bytes,
            host_pool=self.host_pool.data_ptr() if self.host_pool is not None else 0,
            host_pool_bytes=host_pool_bytes, compute_stream=self.compute_stream.cuda_stream,
            copy_stream=self.copy_stream.cuda_stream,
            reload_stream=self.reload_stream.cuda_stream if duplex else 0, recompute=int(recompute),
            n_chunks=self.n_chunks, no_fusion=int(no_fusion))
        h = C.c_void_p()
        B.check(self.lib.optstage_create(C.byref(self.desc), C.byref(h)))
        self.h = h
        if grad_overwrite:
            B.check(self.lib.optstage_set_grad_overwrite(self.h, 1))
        self.weights, self.grads = [], []
        self.x, self.dy, self.y, self.dx = {}, {}, {}, {}

    def close(self):
        if getattr(self, "h", None):
            torch.cuda.synchronize()
            self.lib.optstage_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- setup
    def set_weights(self, weights: list):
        """weights: per layer dict name -> float32 numpy (rounded to the stage dtype)."""
        self.weights, self.grads = [], []
        for l, w in enumerate(weights):
            dw, dg = {}, {}
            for name, arr in w.items():
                dw[name] = to_device(arr, self.cfg.dtype)
                dg[name] = torch.zeros(arr.shape, dtype=torch.float32, device="cuda")
                self._order_after_torch()
                B.check(self.lib.optstage_set_weight(self.h, l, B.WEIGHT_ID[name], dw[name].data_ptr(), dg[name].data_ptr()))
            self.weights.append(dw)
            self.grads.append(dg)
        torch.cuda.synchronize()

    def set_weights_device(self, weights: list):
        """weights: per layer dict name -> device tensor already in the stage dtype."""
        self.weights, self.grads = [], []
        self._order_after_torch()
        for l, w in enumerate(weights):
            dg = {}
            for name, t in w.items():
                dg[name] = torch.zeros(t.shape, dtype=torch.float32, device="cuda")
                B.check(self.lib.optstage_set_weight(self.h, l, B.WEIGHT_ID[name], t.data_ptr(), dg[name].data_ptr()))
            self.weights.append(w)
            self.grads.append(dg)
        torch.cuda.synchronize()

    def zero_grads_async(self):
        """Clears the fp32 gradient accumulators on torch's current stream (no synchronisation)."""
        for g in self.grads:
            for t in g.values():
                t.zero_()

    def zero_grads(self):
        for g in self.grads:
            for t in g.values():
                t.zero_()
        torch.cuda.synchronize()

    def bind(self, mb: int, x: np.ndarray | torch.Tensor, dy: np.ndarray | torch.Tensor, chunk: int = 0):
        """Boundary tensors of micro-batch mb (of model chunk `chunk`); the dicts x, dy, y, dx are keyed by mb for
        chunk 0 and by (chunk, mb) otherwise."""
        dt = self.cfg.dtype
        key = mb if chunk == 0 else (chunk, mb)
        self.x[key] = x if isinstance(x, torch.Tensor) else to_device(x, dt)
        self.dy[key] = dy if isinstance(dy, torch.Tensor) else to_device(dy, dt)
        self.y[key] = torch.empty_like(self.x[key])
        self.dx[key] = torch.empty_like(self.x[key])
        B.check(self.lib.optstage_bind_io_chunk(self.h, chunk, mb, self.x[key].data_ptr(), self.dy[key].data_ptr(),
                                                self.y[key].data_ptr(), self.dx[key].data_ptr()))

    def _order_after_torch(self):
        """The library's streams know nothing of torch's: work torch has queued on its current stream (tensor
        creation, copies, fills) must finish before the library reads those tensors."""
        cur = torch.cuda.current_stream()
        self.compute_stream.wait_stream(cur)
        self.copy_stream.wait_stream(cur)
        self.reload_stream.wait_stream(cur)

    # ---- execution
    def validate(self, events):
        arr = B.make_events(events)
        bad = C.c_size_t(0)
        st = self.lib.optstage_validate(self.h, arr, len(events), C.byref(bad))
        return st, bad.value

    def run(self, events):
        arr = events if not isinstance(events, (list, tuple)) else B.make_events(events)
        n = len(events) if isinstance(events, (list, tuple)) else len(arr)
        self._order_after_torch()
        B.check(self.lib.optstage_run(self.h, arr, n))

    def run_raw(self, arr, n):
        self._order_after_torch()
        B.check(self.lib.optstage_run(self.h, arr, n))

    def synchronize(self):
        B.check(self.lib.optstage_synchronize(self.h))

    def reset(self):
        B.check(self.lib.optstage_reset(self.h))

    def stats(self) -> B.Stats:
        s = B.Stats()
        B.check(self.lib.optstage_get_stats(self.h, C.byref(s)))
        return s

    def trace(self) -> list:
        """Executed events since the last reset: (op name, micro-batch, layer or chunk, kind_mask, live bytes after the
        event, start ms, end ms, stall ms); times are valid after synchronize()."""
        n = C.c_size_t(0)
        B.check(self.lib.optstage_get_trace(self.h, None, 0, C.byref(n)))
        arr = (B.TraceEntry * max(1, n.value))()
        B.check(self.lib.optstage_get_trace(self.h, arr, n.value, None))
        names = {v: k for k, v in B.OP_CODE.items()}
        return [(names[e.op], e.microbatch, e.layer, e.kind_mask, e.live_bytes, e.start_ms, e.end_ms, e.stall_ms)
                for e in arr[:n.value]]

    def checksum(self, mb, layer, kind, where=0):
        out = (C.c_uint64 * 2)()
        B.check(self.lib.optstage_debug_checksum(self.h, mb, layer, B.KIND_ID[kind], where, out))
        return out[0], out[1]

    def read(self, mb, layer, kind) -> np.ndarray:
        n = self.kind_bytes[kind]
        buf = np.empty(n, dtype=np.uint8)
        B.check(self.lib.optstage_debug_read(self.h, mb, layer, B.KIND_ID[kind], buf.ctypes.data, n))
        return buf
