"""Thin ctypes binding of libdqrm.so: argument marshalling only.

Every function has the name of the C entry point it calls (``include/dqrm.h``)
and passes device pointers of torch tensors plus the current HIP stream.  No
step of the path runs in Python or in torch; torch only owns device memory and
streams.  There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np
import torch

from . import build as _build

OK = 0
ERR_INVALID_ARG = -1
ERR_UNSUPPORTED = -2
ERR_WORKSPACE_TOO_SMALL = -3
ERR_INDEX_OUT_OF_RANGE = -4
ERR_HIP = -5
ERR_CAPACITY = -6
ERR_BAD_OFFSETS = -7
ERR_SCRATCH_LIMIT = -8
_NAMES = {0: "OK", -1: "INVALID_ARG", -2: "UNSUPPORTED", -3: "WORKSPACE_TOO_SMALL", -4: "INDEX_OUT_OF_RANGE",
          -5: "HIP_ERROR", -6: "CAPACITY", -7: "BAD_OFFSETS", -8: "SCRATCH_LIMIT"}

FWD_MASTER = 0
FWD_PACKED = 1
SEG_CHUNK = 32
MAX_TABLE_LOOKUPS = 65536
MAX_TABLES = 1024
MAX_DIM = 256
NOALLOC_SCRATCH_BYTES = 8 << 20

EXPORTS = ("dqrm_find_scale", "dqrm_pack_int4", "dqrm_embbag_fwd", "dqrm_embbag_bwd_workspace_bytes",
           "dqrm_embbag_bwd", "dqrm_embbag_bwd_noalloc", "dqrm_dedupe", "dqrm_dedupe_multi", "dqrm_segment_sum", "dqrm_segment_sum_multi",
           "dqrm_grad_quant_int8", "dqrm_grad_quant_int8_multi",
           "dqrm_sparse_update", "dqrm_sparse_merge_workspace_bytes", "dqrm_sparse_merge", "dqrm_sparse_update_sums",
           "dqrm_quant_update", "dqrm_dense_workspace_bytes", "dqrm_dense_step",
           "dqrm_dense_param_count", "dqrm_dense_step_quant", "dqrm_check_status", "dqrm_last_hip_error", "dqrm_version")


class DqrmError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        self.code = code
        super().__init__(f"{where}: DQRM_ERR_{_NAMES.get(code, code)}" + (f" ({detail})" if detail else ""))


class dqrm_tables_t(C.Structure):
    _fields_ = [("num_tables", C.c_int32), ("dim", C.c_int32), ("row_offsets_host", C.c_void_p),
                ("row_offsets_dev", C.c_void_p), ("master", C.c_void_p), ("packed", C.c_void_p),
                ("w_scale", C.c_void_p)]


class dqrm_sparse_block_t(C.Structure):
    _fields_ = [("uniq_rows", C.c_void_p), ("table_uniq_offsets", C.c_void_p), ("gq", C.c_void_p),
                ("capacity", C.c_int64)]


class dqrm_dedupe_batch_t(C.Structure):
    _fields_ = [("indices", C.c_void_p), ("offsets", C.c_void_p), ("num_indices", C.c_int64),
                ("sorted_pos", C.c_void_p), ("uniq_rows", C.c_void_p), ("seg_offsets", C.c_void_p),
                ("table_uniq_offsets", C.c_void_p), ("num_unique", C.c_void_p), ("workspace", C.c_void_p),
                ("max_table_lookups", C.c_int32)]


MAX_DEDUPE_BATCHES = 8


class dqrm_segsum_batch_t(C.Structure):
    _fields_ = [("num_indices", C.c_int64), ("grad_out", C.c_void_p), ("values", C.c_void_p), ("g_absmax", C.c_void_p),
                ("workspace", C.c_void_p)]


class dqrm_quant_block_t(C.Structure):
    _fields_ = [("capacity", C.c_int64), ("values", C.c_void_p), ("table_uniq_offsets", C.c_void_p),
                ("g_absmax", C.c_void_p), ("gq", C.c_void_p), ("g_scale", C.c_void_p)]


class dqrm_dense_model_t(C.Structure):
    _fields_ = [("num_dense", C.c_int32), ("num_tables", C.c_int32), ("dim", C.c_int32), ("bot_layers", C.c_int32),
                ("bot_dims", C.c_void_p), ("bot_w", C.c_void_p), ("bot_b", C.c_void_p), ("top_layers", C.c_int32),
                ("top_dims", C.c_void_p), ("top_w", C.c_void_p), ("top_b", C.c_void_p)]


class dqrm_dense_quant_t(C.Structure):
    _fields_ = [("weight_bits", C.c_int32), ("grad_bits", C.c_int32), ("grad_error", C.c_void_p),
                ("grad_scale", C.c_void_p), ("grad_codes", C.c_void_p), ("grads", C.c_void_p), ("wq", C.c_void_p),
                ("grad_buffer", C.c_void_p), ("buffer_add", C.c_int32), ("buffer_update", C.c_int32)]


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """The loaded C-ABI library.  Builds it only if no built library is present."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build_library(force=True)
        L = C.CDLL(path)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        tp = C.POINTER(dqrm_tables_t)
        L.dqrm_find_scale.argtypes = [tp, vp]
        L.dqrm_pack_int4.argtypes = [tp, vp]
        L.dqrm_embbag_fwd.argtypes = [tp, vp, vp, i32, i64, i32, vp, vp, vp]
        L.dqrm_embbag_bwd_workspace_bytes.argtypes = [i32, i32, i32, i64]
        L.dqrm_embbag_bwd_workspace_bytes.restype = sz
        L.dqrm_embbag_bwd.argtypes = [tp, vp, vp, i32, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.dqrm_embbag_bwd_noalloc.argtypes = [tp, vp, vp, i32, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.dqrm_embbag_bwd_noalloc.restype = i32
        L.dqrm_dedupe.argtypes = [tp, vp, vp, i32, i64, vp, vp, vp, vp, vp, vp, sz, vp]
        L.dqrm_dedupe_multi.argtypes = [tp, i32, i32, C.POINTER(dqrm_dedupe_batch_t), sz, vp]
        L.dqrm_dedupe_multi.restype = i32
        L.dqrm_segment_sum.argtypes = [tp, i32, i64, vp, vp, vp, vp, sz, vp]
        L.dqrm_segment_sum_multi.argtypes = [tp, i32, i32, C.POINTER(dqrm_segsum_batch_t), sz, vp]
        L.dqrm_segment_sum_multi.restype = i32
        L.dqrm_grad_quant_int8_multi.argtypes = [i32, i32, i32, C.POINTER(dqrm_quant_block_t), vp]
        L.dqrm_grad_quant_int8_multi.restype = i32
        L.dqrm_quant_update.argtypes = [tp, i64, i64, vp, vp, vp, vp, vp, vp, C.c_float, vp, sz, vp]
        L.dqrm_grad_quant_int8.argtypes = [i32, i32, i64, vp, vp, vp, vp, vp, vp]
        L.dqrm_sparse_update.argtypes = [tp, i64, vp, vp, vp, vp, C.c_float, vp]
        L.dqrm_sparse_update_sums.argtypes = [tp, i64, vp, vp, vp, vp, C.c_float, vp]
        L.dqrm_sparse_update_sums.restype = i32
        L.dqrm_sparse_merge_workspace_bytes.argtypes = [i32, i32, i32, i64]
        L.dqrm_sparse_merge_workspace_bytes.restype = sz
        L.dqrm_sparse_merge.argtypes = [tp, i32, C.POINTER(dqrm_sparse_block_t), i64, vp, vp, vp, vp, vp, sz, vp]
        L.dqrm_sparse_merge.restype = i32
        dp = C.POINTER(dqrm_dense_model_t)
        L.dqrm_dense_workspace_bytes.argtypes = [dp, i32]
        L.dqrm_dense_workspace_bytes.restype = sz
        L.dqrm_dense_step.argtypes = [dp, i32, vp, vp, vp, C.c_float, vp, vp, vp, sz, vp]
        L.dqrm_dense_step.restype = i32
        L.dqrm_dense_param_count.argtypes = [dp]
        L.dqrm_dense_param_count.restype = i64
        L.dqrm_dense_step_quant.argtypes = [dp, C.POINTER(dqrm_dense_quant_t), i32, vp, vp, vp, C.c_float, vp, vp, vp,
                                            sz, vp]
        L.dqrm_dense_step_quant.restype = i32
        L.dqrm_check_status.argtypes = [vp, C.POINTER(i32), C.POINTER(i64)]
        for n in ("dqrm_find_scale", "dqrm_pack_int4", "dqrm_embbag_fwd", "dqrm_embbag_bwd", "dqrm_dedupe", "dqrm_segment_sum",
                  "dqrm_quant_update", "dqrm_grad_quant_int8", "dqrm_sparse_update", "dqrm_check_status"):
            getattr(L, n).restype = i32
        L.dqrm_last_hip_error.restype = C.c_char_p
        L.dqrm_version.restype = C.c_char_p
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "DQRM buffers must be contiguous"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(rc: int, where: str) -> None:
    if rc != OK:
        detail = lib().dqrm_last_hip_error().decode() if rc == ERR_HIP else ""
        raise DqrmError(rc, where, detail)


class Tables:
    """Owns the device buffers of the embedding layer and the C descriptor."""

    def __init__(self, row_offsets: np.ndarray, dim: int, master: torch.Tensor, packed: Optional[torch.Tensor] = None,
                 w_scale: Optional[torch.Tensor] = None):
        self.row_offsets_host = np.ascontiguousarray(row_offsets, dtype=np.int64)
        self.T = len(self.row_offsets_host) - 1
        self.D = int(dim)
        self.R = int(self.row_offsets_host[-1])
        dev = master.device
        assert master.dtype == torch.float32 and tuple(master.shape) == (self.R, self.D)
        self.master = master
        self.packed = packed
        if packed is not None:
            assert packed.dtype == torch.uint8 and tuple(packed.shape) == (self.R, self.D // 2)
        self.w_scale = w_scale if w_scale is not None else torch.ones(self.T, dtype=torch.float32, device=dev)
        self.row_offsets_dev = torch.from_numpy(self.row_offsets_host).to(dev)
        self.c = dqrm_tables_t(self.T, self.D, self.row_offsets_host.ctypes.data, _ptr(self.row_offsets_dev),
                               _ptr(self.master), _ptr(self.packed), _ptr(self.w_scale))

    @property
    def ref(self):
        return C.byref(self.c)


def dqrm_version() -> str:
    return lib().dqrm_version().decode()


def dqrm_find_scale(tables: Tables, stream=None) -> None:
    _check(lib().dqrm_find_scale(tables.ref, _stream(stream)), "dqrm_find_scale")


def dqrm_pack_int4(tables: Tables, stream=None) -> None:
    _check(lib().dqrm_pack_int4(tables.ref, _stream(stream)), "dqrm_pack_int4")


def dqrm_embbag_fwd(tables: Tables, indices: torch.Tensor, offsets: torch.Tensor, batch: int, mode: int,
                    out: torch.Tensor, codes_dbg: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(lib().dqrm_embbag_fwd(tables.ref, _ptr(indices), _ptr(offsets), batch, indices.numel(), mode, _ptr(out),
                                 _ptr(codes_dbg), _stream(stream)), "dqrm_embbag_fwd")


def dqrm_embbag_bwd_workspace_bytes(num_tables: int, dim: int, batch: int, num_indices: int) -> int:
    return int(lib().dqrm_embbag_bwd_workspace_bytes(num_tables, dim, batch, num_indices))


def dqrm_embbag_bwd(tables: Tables, indices: torch.Tensor, offsets: torch.Tensor, batch: int, grad_out: torch.Tensor,
                    sorted_pos: torch.Tensor, uniq_rows: torch.Tensor, seg_offsets: torch.Tensor,
                    table_uniq_offsets: torch.Tensor, num_unique: torch.Tensor, values: torch.Tensor,
                    g_absmax: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    _check(lib().dqrm_embbag_bwd(tables.ref, _ptr(indices), _ptr(offsets), batch, indices.numel(), _ptr(grad_out),
                                 _ptr(sorted_pos), _ptr(uniq_rows), _ptr(seg_offsets), _ptr(table_uniq_offsets),
                                 _ptr(num_unique), _ptr(values), _ptr(g_absmax), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream)), "dqrm_embbag_bwd")


def dqrm_embbag_bwd_noalloc(tables: Tables, indices: torch.Tensor, offsets: torch.Tensor, batch: int,
                            grad_out: torch.Tensor, sorted_pos: torch.Tensor, uniq_rows: torch.Tensor,
                            seg_offsets: torch.Tensor, table_uniq_offsets: torch.Tensor, num_unique: torch.Tensor,
                            values: torch.Tensor, g_absmax: torch.Tensor, stream=None) -> None:
    rc = lib().dqrm_embbag_bwd_noalloc(tables.ref, _ptr(indices), _ptr(offsets), batch, indices.numel(), _ptr(grad_out),
                                       _ptr(sorted_pos), _ptr(uniq_rows), _ptr(seg_offsets), _ptr(table_uniq_offsets),
                                       _ptr(num_unique), _ptr(values), _ptr(g_absmax), _stream(stream))
    if rc == ERR_SCRATCH_LIMIT:
        raise DqrmError(rc, "dqrm_embbag_bwd_noalloc", lib().dqrm_last_hip_error().decode())
    _check(rc, "dqrm_embbag_bwd_noalloc")


def dqrm_dedupe(tables: Tables, indices: torch.Tensor, offsets: torch.Tensor, batch: int, sorted_pos: torch.Tensor,
                uniq_rows: torch.Tensor, seg_offsets: torch.Tensor, table_uniq_offsets: torch.Tensor,
                num_unique: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    _check(lib().dqrm_dedupe(tables.ref, _ptr(indices), _ptr(offsets), batch, indices.numel(), _ptr(sorted_pos),
                             _ptr(uniq_rows), _ptr(seg_offsets), _ptr(table_uniq_offsets), _ptr(num_unique),
                             _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "dqrm_dedupe")


def dqrm_dedupe_multi(tables: Tables, batch: int, batches, stream=None, max_table_lookups: int = 0) -> None:
    """``batches``: sequence of tuples (indices, offsets, sorted_pos, uniq_rows, seg_offsets, table_uniq_offsets,
    num_unique, workspace) of device tensors, one per batch (at most MAX_DEDUPE_BATCHES).  ``max_table_lookups``:
    the caller's bound on the lookups of any one table in any of the batches, 0 if none is known."""
    arr = (dqrm_dedupe_batch_t * len(batches))()
    ws_bytes = None
    for i, (ix, of, sp, ur, so, tuo, nu, ws) in enumerate(batches):
        arr[i] = dqrm_dedupe_batch_t(_ptr(ix), _ptr(of), ix.numel(), _ptr(sp), _ptr(ur), _ptr(so), _ptr(tuo), _ptr(nu),
                                     _ptr(ws), max_table_lookups)
        nb = ws.numel() * ws.element_size()
        ws_bytes = nb if ws_bytes is None else min(ws_bytes, nb)
    _check(lib().dqrm_dedupe_multi(tables.ref, batch, len(batches), arr, ws_bytes or 0, _stream(stream)),
           "dqrm_dedupe_multi")


def dqrm_segment_sum(tables: Tables, batch: int, num_indices: int, grad_out: torch.Tensor, values: torch.Tensor,
                     g_absmax: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    _check(lib().dqrm_segment_sum(tables.ref, batch, num_indices, _ptr(grad_out), _ptr(values), _ptr(g_absmax),
                                  _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "dqrm_segment_sum")


def dqrm_segment_sum_multi(tables: Tables, batch: int, batches, stream=None) -> None:
    """``batches``: sequence of tuples (num_indices, grad_out, values, g_absmax or None, workspace) of device tensors,
    one per batch (at most MAX_DEDUPE_BATCHES)."""
    arr = (dqrm_segsum_batch_t * len(batches))()
    ws_bytes = None
    for i, (n, g, v, am, ws) in enumerate(batches):
        arr[i] = dqrm_segsum_batch_t(int(n), _ptr(g), _ptr(v), _ptr(am), _ptr(ws))
        nb = ws.numel() * ws.element_size()
        ws_bytes = nb if ws_bytes is None else min(ws_bytes, nb)
    _check(lib().dqrm_segment_sum_multi(tables.ref, batch, len(batches), arr, ws_bytes or 0, _stream(stream)),
           "dqrm_segment_sum_multi")


def dqrm_grad_quant_int8_multi(num_tables: int, dim: int, blocks, stream=None) -> None:
    """``blocks``: sequence of tuples (values, table_uniq_offsets, g_absmax, gq, g_scale) of device tensors, one per
    block (at most MAX_DEDUPE_BATCHES); the capacity of a block is the smaller first dimension of values and gq."""
    arr = (dqrm_quant_block_t * len(blocks))()
    for i, (v, tuo, am, gq, gs) in enumerate(blocks):
        arr[i] = dqrm_quant_block_t(min(v.shape[0], gq.shape[0]), _ptr(v), _ptr(tuo), _ptr(am), _ptr(gq), _ptr(gs))
    _check(lib().dqrm_grad_quant_int8_multi(num_tables, dim, len(blocks), arr, _stream(stream)),
           "dqrm_grad_quant_int8_multi")


def dqrm_grad_quant_int8(num_tables: int, dim: int, capacity: int, values: torch.Tensor,
                         table_uniq_offsets: torch.Tensor, g_absmax: torch.Tensor, gq: torch.Tensor,
                         g_scale: torch.Tensor, stream=None) -> None:
    _check(lib().dqrm_grad_quant_int8(num_tables, dim, capacity, _ptr(values), _ptr(table_uniq_offsets),
                                      _ptr(g_absmax), _ptr(gq), _ptr(g_scale), _stream(stream)),
           "dqrm_grad_quant_int8")


def dqrm_sparse_merge_workspace_bytes(num_tables: int, dim: int, num_blocks: int, max_total: int) -> int:
    return int(lib().dqrm_sparse_merge_workspace_bytes(num_tables, dim, num_blocks, max_total))


def dqrm_sparse_merge(tables: Tables, blocks, uniq_rows: torch.Tensor, table_uniq_offsets: torch.Tensor,
                      num_unique: torch.Tensor, sums: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    """``blocks``: sequence of tuples (uniq_rows, table_uniq_offsets, gq) of device tensors, one per micro-batch
    (at most MAX_DEDUPE_BATCHES).  The outputs' first dimension is the capacity ``max_total``."""
    arr = (dqrm_sparse_block_t * len(blocks))()
    for i, (ur, tuo, gq) in enumerate(blocks):
        arr[i] = dqrm_sparse_block_t(_ptr(ur), _ptr(tuo), _ptr(gq), min(ur.shape[0], gq.shape[0]))
    _check(lib().dqrm_sparse_merge(tables.ref, len(blocks), arr, min(uniq_rows.shape[0], sums.shape[0]), _ptr(uniq_rows),
                                   _ptr(table_uniq_offsets), _ptr(num_unique), _ptr(sums), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream)), "dqrm_sparse_merge")


def dqrm_sparse_update_sums(tables: Tables, capacity: int, uniq_rows: torch.Tensor, table_uniq_offsets: torch.Tensor,
                            sums: torch.Tensor, g_scale: torch.Tensor, lr: float, stream=None) -> None:
    _check(lib().dqrm_sparse_update_sums(tables.ref, capacity, _ptr(uniq_rows), _ptr(table_uniq_offsets), _ptr(sums),
                                         _ptr(g_scale), lr, _stream(stream)), "dqrm_sparse_update_sums")


def dqrm_sparse_update(tables: Tables, capacity: int, uniq_rows: torch.Tensor, table_uniq_offsets: torch.Tensor,
                       gq: torch.Tensor, g_scale: torch.Tensor, lr: float, stream=None) -> None:
    _check(lib().dqrm_sparse_update(tables.ref, capacity, _ptr(uniq_rows), _ptr(table_uniq_offsets), _ptr(gq),
                                    _ptr(g_scale), lr, _stream(stream)), "dqrm_sparse_update")


def dqrm_quant_update(tables: Tables, capacity: int, num_indices: int, values: torch.Tensor, uniq_rows: torch.Tensor,
                      table_uniq_offsets: torch.Tensor, g_absmax: torch.Tensor, gq: torch.Tensor,
                      g_scale: torch.Tensor, lr: float, workspace: torch.Tensor, stream=None) -> None:
    _check(lib().dqrm_quant_update(tables.ref, capacity, num_indices, _ptr(values), _ptr(uniq_rows),
                                   _ptr(table_uniq_offsets), _ptr(g_absmax), _ptr(gq), _ptr(g_scale), lr,
                                   _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "dqrm_quant_update")


class DenseModel:
    """Device copies of the MLP parameters and the C descriptor of the dense part of the model."""

    def __init__(self, num_tables: int, dim: int, bot_dims, bot_w, bot_b, top_dims, top_w, top_b, device):
        to_dev = lambda lst: [torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(device) for a in lst]
        self.bot_w, self.bot_b, self.top_w, self.top_b = to_dev(bot_w), to_dev(bot_b), to_dev(top_w), to_dev(top_b)
        self.bot_dims = np.ascontiguousarray(bot_dims, np.int32)
        self.top_dims = np.ascontiguousarray(top_dims, np.int32)
        ptrs = lambda lst: (C.c_void_p * len(lst))(*[t.data_ptr() for t in lst])
        self._pw = [ptrs(self.bot_w), ptrs(self.bot_b), ptrs(self.top_w), ptrs(self.top_b)]
        addr = lambda a: C.cast(a, C.c_void_p).value
        self.c = dqrm_dense_model_t(int(self.bot_dims[0]), num_tables, dim, len(self.bot_w),
                                    self.bot_dims.ctypes.data, addr(self._pw[0]), addr(self._pw[1]),
                                    len(self.top_w), self.top_dims.ctypes.data, addr(self._pw[2]), addr(self._pw[3]))
        self.num_tables, self.dim = num_tables, dim

    @property
    def ref(self):
        return C.byref(self.c)


def dqrm_dense_workspace_bytes(model: DenseModel, batch: int) -> int:
    return int(lib().dqrm_dense_workspace_bytes(model.ref, batch))


def dqrm_dense_step(model: DenseModel, batch: int, dense_x: torch.Tensor, emb_out: torch.Tensor,
                    labels: torch.Tensor, lr: float, loss: torch.Tensor, grad_emb: torch.Tensor,
                    workspace: torch.Tensor, stream=None) -> None:
    _check(lib().dqrm_dense_step(model.ref, batch, _ptr(dense_x), _ptr(emb_out), _ptr(labels), lr, _ptr(loss),
                                 _ptr(grad_emb), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                 _stream(stream)), "dqrm_dense_step")


def dqrm_dense_param_count(model: DenseModel) -> int:
    return int(lib().dqrm_dense_param_count(model.ref))


class DenseQuant:
    """Descriptor of the quantised variants of the dense step; the tensors (device) stay owned by the caller."""

    def __init__(self, weight_bits: int = 0, grad_bits: int = 0, grad_error: Optional[torch.Tensor] = None,
                 grad_scale: Optional[torch.Tensor] = None, grad_codes: Optional[torch.Tensor] = None,
                 grads: Optional[torch.Tensor] = None, wq: Optional[torch.Tensor] = None,
                 grad_buffer: Optional[torch.Tensor] = None, buffer_add: bool = False, buffer_update: bool = False):
        self._keep = (grad_error, grad_scale, grad_codes, grads, wq, grad_buffer)
        p = lambda t: t.data_ptr() if t is not None else None
        self.c = dqrm_dense_quant_t(weight_bits, grad_bits, p(grad_error), p(grad_scale), p(grad_codes), p(grads), p(wq),
                                    p(grad_buffer), int(buffer_add), int(buffer_update))

    @property
    def ref(self):
        return C.byref(self.c)


def dqrm_dense_step_quant(model: DenseModel, quant: Optional[DenseQuant], batch: int, dense_x: torch.Tensor,
                          emb_out: torch.Tensor, labels: torch.Tensor, lr: float, loss: torch.Tensor,
                          grad_emb: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    _check(lib().dqrm_dense_step_quant(model.ref, quant.ref if quant is not None else None, batch, _ptr(dense_x),
                                       _ptr(emb_out), _ptr(labels), lr, _ptr(loss), _ptr(grad_emb), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream)),
           "dqrm_dense_step_quant")


def dqrm_check_status(stream=None) -> Tuple[int, int, int]:
    """(code, table, value); code 0 = no data-dependent problem since the last call.  Synchronises."""
    t, v = C.c_int32(-1), C.c_int64(-1)
    rc = lib().dqrm_check_status(_stream(stream), C.byref(t), C.byref(v))
    if rc == ERR_HIP:
        _check(rc, "dqrm_check_status")
    return int(rc), int(t.value), int(v.value)


class StepBuffers:
    """Device buffers one training step needs, allocated once (the library itself allocates nothing)."""

    def __init__(self, T: int, D: int, B: int, N: int, device, want_codes: bool = False):
        cap = max(N, 1)
        i32, i64, f32 = torch.int32, torch.int64, torch.float32
        self.T, self.D, self.B, self.N, self.cap = T, D, B, N, cap
        self.out = torch.empty((B, T, D), dtype=f32, device=device)
        self.codes = torch.empty((cap, D), dtype=torch.int8, device=device) if want_codes else None
        self.sorted_pos = torch.empty(cap, dtype=i32, device=device)
        self.uniq_rows = torch.empty(cap, dtype=i64, device=device)
        self.seg_offsets = torch.empty(cap + 1, dtype=i32, device=device)
        self.table_uniq_offsets = torch.empty(T + 1, dtype=i32, device=device)
        self.num_unique = torch.empty(1, dtype=i32, device=device)
        self.values = torch.empty((cap, D), dtype=f32, device=device)
        self.g_absmax = torch.empty(T, dtype=f32, device=device)
        self.gq = torch.empty((cap, D), dtype=torch.int8, device=device)
        self.g_scale = torch.empty(T, dtype=f32, device=device)
        nbytes = dqrm_embbag_bwd_workspace_bytes(T, D, B, N)
        if nbytes == 0:
            raise DqrmError(ERR_UNSUPPORTED, "dqrm_embbag_bwd_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)


def dqrm_fwd_bwd_step(tables: Tables, bufs: StepBuffers, indices: torch.Tensor, offsets: torch.Tensor,
                      grad_out: torch.Tensor, lr: float, mode: int = FWD_MASTER, stream=None) -> None:
    """One pass of the whole hot path: the five per-step C calls in order, on one stream, no host sync."""
    dqrm_embbag_fwd(tables, indices, offsets, bufs.B, mode, bufs.out, bufs.codes, stream)
    dqrm_embbag_bwd(tables, indices, offsets, bufs.B, grad_out, bufs.sorted_pos, bufs.uniq_rows, bufs.seg_offsets,
                    bufs.table_uniq_offsets, bufs.num_unique, bufs.values, bufs.g_absmax, bufs.workspace, stream)
    dqrm_grad_quant_int8(bufs.T, bufs.D, bufs.cap, bufs.values, bufs.table_uniq_offsets, bufs.g_absmax, bufs.gq,
                         bufs.g_scale, stream)
    dqrm_sparse_update(tables, bufs.cap, bufs.uniq_rows, bufs.table_uniq_offsets, bufs.gq, bufs.g_scale, lr, stream)
