"""Thin ctypes binding of libfae.so: same names as the C ABI (include/fae.h), argument
marshalling only.  Every step of the path runs in the library's HIP kernels; torch
is used for device memory and the stream.  There is no CPU fallback: if the
library is missing and cannot be built, importing a function raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfae.so")

FAE_OK, FAE_EINVAL, FAE_ERANGE, FAE_ENOSPC, FAE_EHIP = 0, -1, -2, -3, -4
FAE_MAX_TABLES = 64
FAE_SRC_DEVICE, FAE_SRC_PROCEDURAL = 0, 1
FAE_SYNC_HOT_TO_FULL, FAE_SYNC_FULL_TO_HOT = 0, 1
FAE_POOL_SUM, FAE_POOL_MEAN = 0, 1
FAE_OPT_SGD, FAE_OPT_ROWWISE_ADAGRAD = 0, 1

EXPORTS = [
    "fae_create", "fae_destroy", "fae_last_error", "fae_version", "fae_sync", "fae_set_option",
    "fae_timing_enable", "fae_timing_reset", "fae_timing_read", "fae_kernel_name", "fae_copy_probe", "fae_read_probe", "fae_fill_probe",
    "fae_profile", "fae_choose_cutoff_workspace_bytes", "fae_choose_cutoff", "fae_count_hot",
    "fae_build_workspace_bytes", "fae_build_hot_tables", "fae_partition_workspace_bytes",
    "fae_partition_batch", "fae_embbag_fwd", "fae_bwd_workspace_bytes", "fae_embbag_bwd_presort",
    "fae_embbag_fwd_presort",
    "fae_embbag_bwd_sgd", "fae_bwd_static_workspace_bytes", "fae_embbag_bwd_sgd_static",
    "fae_sync_hot_rows", "fae_estimate_workspace_bytes", "fae_estimate_hot", "fae_choose_cutoff_sampled",
    "fae_t_quantile", "fae_sched_init", "fae_sched_report", "fae_sched_segment",
    "fae_embbag_fwd_opts", "fae_embbag_bwd_opts",
]


class FaeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libfae error {code}: {msg}")
        self.code = code


class _Tables(C.Structure):
    _fields_ = [("n_tables", C.c_int32), ("dim", C.c_int32), ("h_rows", C.POINTER(C.c_int64))]


class _Batch(C.Structure):
    _fields_ = [("n_samples", C.c_int64), ("h_indices", C.POINTER(C.c_void_p)),
                ("h_offsets", C.POINTER(C.c_void_p)), ("h_n_lookups", C.POINTER(C.c_int64)),
                ("index_bits", C.c_int32)]


class _WeightSrc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("h_W", C.POINTER(C.c_void_p)), ("seed", C.c_uint64)]


class _BwdDebug(C.Structure):
    _fields_ = [("uniq", C.c_void_p), ("runlen", C.c_void_p), ("table_start", C.c_void_p)]


class _HotEstimate(C.Structure):
    _fields_ = [("rows", C.c_double), ("half_rows", C.c_double), ("ybar", C.c_double), ("s", C.c_double),
                ("N", C.c_int64), ("n", C.c_int64)]


class _StepOpts(C.Structure):
    _fields_ = [("pooling", C.c_int32), ("optimizer", C.c_int32), ("lr", C.c_float), ("eps", C.c_float),
                ("h_state", C.POINTER(C.c_void_p))]


class _Sched(C.Structure):
    _fields_ = [("rate", C.c_double), ("prev", C.c_double), ("u", C.c_int32), ("falls", C.c_int32),
                ("reports", C.c_int32)]


_lib = None


def load():
    """Load libfae.so (building it first if it has never been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libfae.so is missing and could not be built; run __graft_entry__.build()")
    lib = C.CDLL(LIB_PATH)
    lib.fae_last_error.restype = C.c_char_p
    lib.fae_last_error.argtypes = [C.c_void_p]
    lib.fae_version.restype = C.c_char_p
    for name in ("fae_choose_cutoff_workspace_bytes", "fae_build_workspace_bytes",
                 "fae_partition_workspace_bytes", "fae_bwd_workspace_bytes", "fae_estimate_workspace_bytes",
                 "fae_bwd_static_workspace_bytes"):
        getattr(lib, name).restype = C.c_size_t
    lib.fae_destroy.restype = None
    lib.fae_kernel_name.restype = C.c_char_p
    lib.fae_t_quantile.restype = C.c_double
    lib.fae_t_quantile.argtypes = [C.c_double, C.c_int64]
    lib.fae_sched_report.restype = C.c_double
    lib.fae_sched_report.argtypes = [C.c_void_p, C.c_double]
    lib.fae_sched_init.argtypes = [C.c_void_p, C.c_double, C.c_int32]
    lib.fae_sched_segment.restype = C.c_int64
    lib.fae_sched_segment.argtypes = [C.c_void_p, C.c_int64]
    _lib = lib
    return lib


# ------------------------------------------------------------------------------------
# marshalling helpers
# ------------------------------------------------------------------------------------
@dataclass
class Tables:
    rows: Sequence[int]
    dim: int

    def c(self):
        key = (tuple(int(r) for r in self.rows), int(self.dim))
        cached = getattr(self, "_c", None)
        if cached is None or cached[0] != key:     # marshal once; re-marshal if the shape changed
            rows = (C.c_int64 * len(self.rows))(*key[0])
            t = _Tables(len(self.rows), int(self.dim), rows)
            t._keep = rows
            self._c = (key, t)
        return self._c[1]


@dataclass
class Batch:
    n_samples: int
    indices: List[torch.Tensor]                 # per table, device int32 (or int64 with index_bits=64)
    offsets: List[Optional[torch.Tensor]]       # per table, device int32[S+1] or None
    n_lookups: Sequence[int]
    index_bits: int = 32

    def c(self):
        """Marshalled once per Batch object (the tensors must stay alive and in place)."""
        if getattr(self, "_c", None) is None:
            nt = len(self.indices)
            idx = _ptrs(self.indices, torch.int64 if self.index_bits == 64 else torch.int32)
            off = _ptrs(self.offsets, torch.int32) if any(o is not None for o in self.offsets) else None
            nl = (C.c_int64 * nt)(*[int(n) for n in self.n_lookups])
            b = _Batch(int(self.n_samples), idx, off, nl, int(self.index_bits))
            b._keep = (idx, off, nl)
            self._c = b
        return self._c


def _ptrs(tensors: Sequence[Optional[torch.Tensor]], dtype):
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        if t is None:
            arr[i] = None
            continue
        if t.dtype != dtype or not t.is_contiguous() or not t.is_cuda:
            raise TypeError(f"tensor {i}: need a contiguous device tensor of {dtype}, got {t.dtype} on {t.device}")
        arr[i] = t.data_ptr() if t.numel() > 0 else None
    return arr


def _ptr(t: Optional[torch.Tensor], dtype):
    if t is None:
        return None
    if t.dtype != dtype or not t.is_contiguous() or not t.is_cuda:
        raise TypeError(f"need a contiguous device tensor of {dtype}, got {t.dtype} on {t.device}")
    return C.c_void_p(t.data_ptr())


# ------------------------------------------------------------------------------------
# the ABI, name for name
# ------------------------------------------------------------------------------------
class Context:
    """Owns a fae_ctx bound to a device and a stream (default: torch's current stream)."""

    def __init__(self, device: int = 0, stream: Optional[int] = None):
        lib = load()
        if not torch.cuda.is_available():
            raise RuntimeError("libfae needs a GPU: torch.cuda.is_available() is False")
        if stream is None:
            stream = torch.cuda.current_stream(device).cuda_stream
        self.device = device
        self._h = C.c_void_p()
        rc = lib.fae_create(C.byref(self._h), C.c_int32(device), C.c_void_p(stream))
        if rc != FAE_OK:
            raise FaeError(rc, "fae_create failed")

    def close(self):
        if self._h:
            load().fae_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, rc: int):
        if rc != FAE_OK:
            raise FaeError(rc, load().fae_last_error(self._h).decode())


def fae_version() -> str:
    return load().fae_version().decode()


def fae_sync(ctx: Context):
    ctx.check(load().fae_sync(ctx._h))


def fae_set_option(ctx: Context, name: str, value: int):
    ctx.check(load().fae_set_option(ctx._h, name.encode(), C.c_int64(value)))


FAE_K_COUNT = 19


def fae_kernel_name(kernel_class: int) -> str:
    return load().fae_kernel_name(C.c_int32(kernel_class)).decode()


def fae_timing_enable(ctx: Context, on: bool):
    ctx.check(load().fae_timing_enable(ctx._h, C.c_int32(1 if on else 0)))


def fae_timing_reset(ctx: Context):
    ctx.check(load().fae_timing_reset(ctx._h))


def fae_timing_read(ctx: Context, kernel_class: int):
    """(total milliseconds, launches) of one kernel class since the last reset."""
    ms, n = C.c_double(0.0), C.c_int64(0)
    ctx.check(load().fae_timing_read(ctx._h, C.c_int32(kernel_class), C.byref(ms), C.byref(n)))
    return float(ms.value), int(n.value)


def fae_copy_probe(ctx: Context, dst: torch.Tensor, src: torch.Tensor):
    assert dst.numel() * dst.element_size() == src.numel() * src.element_size()
    ctx.check(load().fae_copy_probe(ctx._h, C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()),
                                    C.c_size_t(src.numel() * src.element_size())))


def fae_read_probe(ctx: Context, src: torch.Tensor, sink: torch.Tensor):
    ctx.check(load().fae_read_probe(ctx._h, C.c_void_p(src.data_ptr()), C.c_size_t(src.numel() * src.element_size()),
                                    _ptr(sink, torch.float32)))


def fae_fill_probe(ctx: Context, dst: torch.Tensor, value: float = 0.0):
    ctx.check(load().fae_fill_probe(ctx._h, C.c_void_p(dst.data_ptr()), C.c_size_t(dst.numel() * dst.element_size()),
                                    C.c_float(value)))


def fae_profile(ctx: Context, tables: Tables, chunk: Batch, counts: List[torch.Tensor]):
    t, b = tables.c(), chunk.c()
    ctx.check(load().fae_profile(ctx._h, C.byref(t), C.byref(b), _ptrs(counts, torch.int32)))


def fae_choose_cutoff_workspace_bytes(tables: Tables) -> int:
    t = tables.c()
    return int(load().fae_choose_cutoff_workspace_bytes(C.byref(t)))


def fae_choose_cutoff(ctx: Context, tables: Tables, counts: List[torch.Tensor], T: Sequence[int],
                      t_denom: int, budget_bytes: int, small_table_bytes: int, ws: torch.Tensor):
    """Returns (c, cutoff[z], n_hot[z]) as Python ints."""
    nt = len(tables.rows)
    t = tables.c()
    Ta = (C.c_int64 * nt)(*[int(v) for v in T])
    c_out = C.c_int64(0)
    cut = (C.c_uint32 * nt)()
    nh = (C.c_int64 * nt)()
    ctx.check(load().fae_choose_cutoff(ctx._h, C.byref(t), _ptrs(counts, torch.int32), Ta,
                                       C.c_int64(t_denom), C.c_int64(budget_bytes),
                                       C.c_int64(small_table_bytes), C.byref(c_out), cut, nh,
                                       _ptr(ws, torch.uint8), C.c_size_t(ws.numel())))
    return int(c_out.value), list(cut), list(nh)


def fae_count_hot(ctx: Context, tables: Tables, counts: List[torch.Tensor], cutoff: Sequence[int],
                  ws: torch.Tensor) -> List[int]:
    nt = len(tables.rows)
    t = tables.c()
    cut = (C.c_uint32 * nt)(*[int(v) for v in cutoff])
    nh = (C.c_int64 * nt)()
    ctx.check(load().fae_count_hot(ctx._h, C.byref(t), _ptrs(counts, torch.int32), cut, nh,
                                   _ptr(ws, torch.uint8), C.c_size_t(ws.numel())))
    return list(nh)


def fae_build_workspace_bytes(tables: Tables) -> int:
    t = tables.c()
    return int(load().fae_build_workspace_bytes(C.byref(t)))


def fae_build_hot_tables(ctx: Context, tables: Tables, counts: List[torch.Tensor], cutoff: Sequence[int],
                         src_kind: int, src_W: Optional[List[torch.Tensor]], seed: int,
                         remap: List[torch.Tensor], hot_ids: List[torch.Tensor], hotW: List[torch.Tensor],
                         cap: Sequence[int], ws: torch.Tensor) -> List[int]:
    nt = len(tables.rows)
    t = tables.c()
    cut = (C.c_uint32 * nt)(*[int(v) for v in cutoff])
    capa = (C.c_int64 * nt)(*[int(v) for v in cap])
    nh = (C.c_int64 * nt)()
    wp = _ptrs(src_W, torch.float32) if src_W is not None else None
    src = _WeightSrc(int(src_kind), wp, C.c_uint64(seed & ((1 << 64) - 1)))
    ctx.check(load().fae_build_hot_tables(ctx._h, C.byref(t), _ptrs(counts, torch.int32), cut, C.byref(src),
                                          _ptrs(remap, torch.int32), _ptrs(hot_ids, torch.int32),
                                          _ptrs(hotW, torch.float32), capa, nh,
                                          _ptr(ws, torch.uint8), C.c_size_t(ws.numel())))
    return list(nh)


def fae_partition_workspace_bytes(tables: Tables, n_samples: int) -> int:
    t = tables.c()
    return int(load().fae_partition_workspace_bytes(C.byref(t), C.c_int64(n_samples)))


def fae_partition_batch(ctx: Context, tables: Tables, batch: Batch, remap: List[torch.Tensor],
                        hot_samples: torch.Tensor, cold_samples: torch.Tensor,
                        slots: List[torch.Tensor], hoffsets: List[torch.Tensor], ws: torch.Tensor):
    """Returns (n_hot_samples, n_hot_lookups[z])."""
    nt = len(tables.rows)
    t, b = tables.c(), batch.c()
    n_hot = C.c_int64(0)
    nl = (C.c_int64 * nt)()
    ctx.check(load().fae_partition_batch(ctx._h, C.byref(t), C.byref(b), _ptrs(remap, torch.int32),
                                         _ptr(hot_samples, torch.int32), _ptr(cold_samples, torch.int32),
                                         C.byref(n_hot), _ptrs(slots, torch.int32), _ptrs(hoffsets, torch.int32),
                                         nl, _ptr(ws, torch.uint8), C.c_size_t(ws.numel())))
    return int(n_hot.value), list(nl)


def fae_embbag_fwd(ctx: Context, hot_tables: Tables, hotW: List[torch.Tensor], hot_batch: Batch,
                   out: torch.Tensor, out_row_stride: int):
    t, b = hot_tables.c(), hot_batch.c()
    ctx.check(load().fae_embbag_fwd(ctx._h, C.byref(t), _ptrs(hotW, torch.float32), C.byref(b),
                                    _ptr(out, torch.float32), C.c_int64(out_row_stride)))


def fae_bwd_workspace_bytes(hot_tables: Tables, n_samples: int, n_lookups: Sequence[int]) -> int:
    t = hot_tables.c()
    nl = (C.c_int64 * len(n_lookups))(*[int(n) for n in n_lookups])
    return int(load().fae_bwd_workspace_bytes(C.byref(t), C.c_int64(n_samples), nl))


def fae_embbag_bwd_presort(ctx: Context, hot_tables: Tables, hot_batch: Batch, ws: torch.Tensor):
    t, b = hot_tables.c(), hot_batch.c()
    ctx.check(load().fae_embbag_bwd_presort(ctx._h, C.byref(t), C.byref(b), _ptr(ws, torch.uint8),
                                            C.c_size_t(ws.numel())))


def fae_embbag_fwd_presort(ctx: Context, hot_tables: Tables, hotW: List[torch.Tensor], hot_batch: Batch,
                           out: torch.Tensor, out_row_stride: int, ws: torch.Tensor):
    t, b = hot_tables.c(), hot_batch.c()
    ctx.check(load().fae_embbag_fwd_presort(ctx._h, C.byref(t), _ptrs(hotW, torch.float32), C.byref(b),
                                            _ptr(out, torch.float32), C.c_int64(out_row_stride),
                                            _ptr(ws, torch.uint8), C.c_size_t(ws.numel())))


def fae_embbag_bwd_sgd(ctx: Context, hot_tables: Tables, hotW: List[torch.Tensor], hot_batch: Batch,
                       gout: torch.Tensor, gout_row_stride: int, lr: float, ws: torch.Tensor,
                       dbg_uniq: Optional[torch.Tensor] = None, dbg_runlen: Optional[torch.Tensor] = None,
                       dbg_table_start: Optional[torch.Tensor] = None):
    t, b = hot_tables.c(), hot_batch.c()
    dbg = None
    if dbg_uniq is not None:
        d = _BwdDebug(_ptr(dbg_uniq, torch.int32), _ptr(dbg_runlen, torch.int32), _ptr(dbg_table_start, torch.int32))
        dbg = C.byref(d)
    ctx.check(load().fae_embbag_bwd_sgd(ctx._h, C.byref(t), _ptrs(hotW, torch.float32), C.byref(b),
                                        _ptr(gout, torch.float32), C.c_int64(gout_row_stride), C.c_float(lr),
                                        dbg, _ptr(ws, torch.uint8), C.c_size_t(ws.numel())))


def fae_bwd_static_workspace_bytes() -> int:
    return int(load().fae_bwd_static_workspace_bytes())


def fae_embbag_bwd_sgd_static(ctx: Context, hot_tables: Tables, hotW: List[torch.Tensor], hot_batch: Batch,
                              gout: torch.Tensor, gout_row_stride: int, lr: float):
    """fae_embbag_bwd_sgd on the library's built-in workspace (nothing is allocated)."""
    t, b = hot_tables.c(), hot_batch.c()
    ctx.check(load().fae_embbag_bwd_sgd_static(ctx._h, C.byref(t), _ptrs(hotW, torch.float32), C.byref(b),
                                               _ptr(gout, torch.float32), C.c_int64(gout_row_stride), C.c_float(lr)))


def _step_opts(pooling: int, optimizer: int, lr: float, eps: float, state: Optional[List[torch.Tensor]]):
    sp = _ptrs(state, torch.float32) if state is not None else None
    o = _StepOpts(int(pooling), int(optimizer), float(lr), float(eps), sp)
    o._keep = sp
    return o


def fae_embbag_fwd_opts(ctx: Context, hot_tables: Tables, hotW: List[torch.Tensor], hot_batch: Batch,
                        out: torch.Tensor, out_row_stride: int, pooling: int):
    t, b = hot_tables.c(), hot_batch.c()
    o = _step_opts(pooling, FAE_OPT_SGD, 0.0, 0.0, None)
    ctx.check(load().fae_embbag_fwd_opts(ctx._h, C.byref(t), _ptrs(hotW, torch.float32), C.byref(b),
                                         _ptr(out, torch.float32), C.c_int64(out_row_stride), C.byref(o)))


def fae_embbag_bwd_opts(ctx: Context, hot_tables: Tables, hotW: List[torch.Tensor], hot_batch: Batch,
                        gout: torch.Tensor, gout_row_stride: int, lr: float, ws: torch.Tensor,
                        pooling: int = FAE_POOL_SUM, optimizer: int = FAE_OPT_SGD, eps: float = 0.0,
                        state: Optional[List[torch.Tensor]] = None,
                        dbg_uniq: Optional[torch.Tensor] = None, dbg_runlen: Optional[torch.Tensor] = None,
                        dbg_table_start: Optional[torch.Tensor] = None):
    t, b = hot_tables.c(), hot_batch.c()
    o = _step_opts(pooling, optimizer, lr, eps, state)
    dbg = None
    if dbg_uniq is not None:
        d = _BwdDebug(_ptr(dbg_uniq, torch.int32), _ptr(dbg_runlen, torch.int32), _ptr(dbg_table_start, torch.int32))
        dbg = C.byref(d)
    ctx.check(load().fae_embbag_bwd_opts(ctx._h, C.byref(t), _ptrs(hotW, torch.float32), C.byref(b),
                                         _ptr(gout, torch.float32), C.c_int64(gout_row_stride), C.byref(o),
                                         dbg, _ptr(ws, torch.uint8), C.c_size_t(ws.numel())))


def fae_sync_hot_rows(ctx: Context, tables: Tables, n_hot: Sequence[int], hot_ids: List[torch.Tensor],
                      hotW: List[torch.Tensor], W: List[torch.Tensor], direction: int):
    nt = len(tables.rows)
    t = tables.c()
    nh = (C.c_int64 * nt)(*[int(v) for v in n_hot])
    ctx.check(load().fae_sync_hot_rows(ctx._h, C.byref(t), nh, _ptrs(hot_ids, torch.int32),
                                       _ptrs(hotW, torch.float32), _ptrs(W, torch.float32), C.c_int32(direction)))


def _chunk_args(chunks: Sequence[Sequence[int]]):
    nt = len(chunks)
    n = (C.c_int64 * nt)(*[len(c) for c in chunks])
    arrs = [(C.c_int64 * max(len(c), 1))(*[int(v) for v in c]) for c in chunks]
    ptrs = (C.c_void_p * nt)(*[C.cast(a, C.c_void_p) for a in arrs])
    return n, ptrs, arrs


def fae_estimate_workspace_bytes(tables: Tables, n_chunks: Sequence[int]) -> int:
    t = tables.c()
    n = (C.c_int64 * len(n_chunks))(*[int(v) for v in n_chunks])
    return int(load().fae_estimate_workspace_bytes(C.byref(t), n))


def _estimates(out, nt):
    return [dict(rows=out[z].rows, half_rows=out[z].half_rows, ybar=out[z].ybar, s=out[z].s,
                 N=int(out[z].N), n=int(out[z].n)) for z in range(nt)]


def fae_estimate_hot(ctx: Context, tables: Tables, counts: List[torch.Tensor], cutoff: Sequence[int], m: int,
                     chunks: Sequence[Sequence[int]], confidence: float, ws: torch.Tensor):
    """Returns (estimates[z] as dicts, C[z] lists of chunk counts)."""
    nt = len(tables.rows)
    t = tables.c()
    cut = (C.c_uint32 * nt)(*[int(v) for v in cutoff])
    n, ptrs, keep = _chunk_args(chunks)
    out = (_HotEstimate * nt)()
    total = sum(len(c) for c in chunks)
    Cout = (C.c_int32 * max(total, 1))()
    ctx.check(load().fae_estimate_hot(ctx._h, C.byref(t), _ptrs(counts, torch.int32), cut, C.c_int64(m), n, ptrs,
                                      C.c_double(confidence), out, Cout, _ptr(ws, torch.uint8),
                                      C.c_size_t(ws.numel())))
    Cs, pos = [], 0
    for c in chunks:
        Cs.append(list(Cout[pos:pos + len(c)]))
        pos += len(c)
    return _estimates(out, nt), Cs


def fae_choose_cutoff_sampled(ctx: Context, tables: Tables, counts: List[torch.Tensor], T: Sequence[int],
                              t_denom: int, budget_bytes: int, small_table_bytes: int, m: int,
                              chunks: Sequence[Sequence[int]], confidence: float, ws: torch.Tensor):
    """Returns (c, cutoff[z], estimates[z])."""
    nt = len(tables.rows)
    t = tables.c()
    Ta = (C.c_int64 * nt)(*[int(v) for v in T])
    n, ptrs, keep = _chunk_args(chunks)
    c_out = C.c_int64(0)
    cut = (C.c_uint32 * nt)()
    out = (_HotEstimate * nt)()
    ctx.check(load().fae_choose_cutoff_sampled(ctx._h, C.byref(t), _ptrs(counts, torch.int32), Ta, C.c_int64(t_denom),
                                               C.c_int64(budget_bytes), C.c_int64(small_table_bytes), C.c_int64(m),
                                               n, ptrs, C.c_double(confidence), C.byref(c_out), cut, out,
                                               _ptr(ws, torch.uint8), C.c_size_t(ws.numel())))
    return int(c_out.value), list(cut), _estimates(out, nt)


def fae_t_quantile(confidence: float, df: int) -> float:
    return float(load().fae_t_quantile(C.c_double(confidence), C.c_int64(df)))


class Sched:
    """fae_sched and its three calls (host only; needs no GPU)."""

    def __init__(self, p0: float = 50.0, u: int = 4):
        self._s = _Sched()
        rc = load().fae_sched_init(C.byref(self._s), C.c_double(p0), C.c_int32(u))
        if rc != FAE_OK:
            raise FaeError(rc, "fae_sched_init: bad argument")

    @property
    def rate(self) -> float:
        return float(self._s.rate)

    def report(self, test_loss: float) -> float:
        r = float(load().fae_sched_report(C.byref(self._s), C.c_double(test_loss)))
        if r < 0:
            raise FaeError(FAE_EINVAL, "fae_sched_report: bad argument")
        return r

    def segment(self, n_total: int) -> int:
        return int(load().fae_sched_segment(C.byref(self._s), C.c_int64(n_total)))
