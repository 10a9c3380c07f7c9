"""ctypes front end of the CPU oracle (``dqrm_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  The product package never imports this.
All arrays are host numpy arrays; nothing here touches a GPU.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dqrm_oracle.c")
_SRC_DENSE = os.path.join(_HERE, "dqrm_dense_oracle.c")
# DQRM_ORACLE_SANITIZE=1 in the environment: a second build with AddressSanitizer and
# UndefinedBehaviorSanitizer (the process must then have libasan preloaded; tests/test_oracle_sanitizers.py
# starts such a process and runs the pin tests in it)
_SANITIZE = os.environ.get("DQRM_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libdqrm_oracle_san.so" if _SANITIZE else "libdqrm_oracle.so")
_lib: Optional[C.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (one rounding per operation: no contraction)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_DENSE))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
               "-fno-sanitize-recover=undefined"] if _SANITIZE else ["-O2"]
        cmd = ["gcc"] + opt + ["-ffp-contract=off", "-fno-fast-math", "-std=c11", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, _SRC_DENSE, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _p(a: Optional[np.ndarray], ct):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"], "oracle arrays must be contiguous"
    return a.ctypes.data_as(C.POINTER(ct))


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_quantize_code.restype = C.c_int
        _lib.oracle_quantize_code.argtypes = [C.c_float, C.c_float, C.c_int]
        _lib.oracle_scale_from_absmax.restype = C.c_float
        _lib.oracle_scale_from_absmax.argtypes = [C.c_float, C.c_int]
        _lib.oracle_seg_chunk.restype = C.c_int
        _lib.oracle_embbag_bwd.restype = C.c_int64
        _lib.oracle_dense_step.restype = C.c_double
        _lib.oracle_dense_step_ex.restype = C.c_double
        _lib.oracle_mlp_grad_quant_ec.restype = C.c_float
    return _lib


def quantize_code(x: float, scale: float, bits: int) -> int:
    return int(lib().oracle_quantize_code(x, scale, bits))


def scale_from_absmax(absmax: float, bits: int) -> float:
    return float(lib().oracle_scale_from_absmax(absmax, bits))


def seg_chunk() -> int:
    return int(lib().oracle_seg_chunk())


def find_scale(W: np.ndarray, row_offsets: np.ndarray) -> np.ndarray:
    T = len(row_offsets) - 1
    D = W.shape[1]
    s = np.empty(T, np.float32)
    lib().oracle_find_scale(_p(W, C.c_float), _p(row_offsets, C.c_int64), C.c_int(T), C.c_int(D),
                            _p(s, C.c_float))
    return s


def pack_int4(W: np.ndarray, row_offsets: np.ndarray, w_scale: np.ndarray) -> np.ndarray:
    T = len(row_offsets) - 1
    R, D = W.shape
    packed = np.empty((R, D // 2), np.uint8)
    lib().oracle_pack_int4(_p(W, C.c_float), _p(row_offsets, C.c_int64), C.c_int(T), C.c_int(D),
                           _p(w_scale, C.c_float), _p(packed, C.c_uint8))
    return packed


def unpack_int4(packed: np.ndarray) -> np.ndarray:
    R, half = packed.shape
    codes = np.empty((R, 2 * half), np.int8)
    lib().oracle_unpack_int4(_p(packed, C.c_uint8), C.c_int64(R), C.c_int(2 * half), _p(codes, C.c_int8))
    return codes


def embbag_fwd(W: Optional[np.ndarray], packed: Optional[np.ndarray], row_offsets: np.ndarray,
               w_scale: Optional[np.ndarray], B: int, indices: np.ndarray, offsets: np.ndarray,
               mode: int = 0, quantise: bool = True, want_codes: bool = True
               ) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    T = len(row_offsets) - 1
    D = W.shape[1] if W is not None else packed.shape[1] * 2
    N = len(indices)
    out = np.empty((B, T, D), np.float32)
    codes = np.zeros((N, D), np.int8) if want_codes else None
    lib().oracle_embbag_fwd(_p(W, C.c_float), _p(packed, C.c_uint8), _p(row_offsets, C.c_int64),
                            _p(w_scale, C.c_float), C.c_int(T), C.c_int(D), C.c_int(B),
                            _p(indices, C.c_int64), _p(offsets, C.c_int64), C.c_int(mode),
                            C.c_int(1 if quantise else 0), _p(out, C.c_float), _p(codes, C.c_int8))
    return out, codes


def embbag_bwd(T: int, D: int, B: int, indices: np.ndarray, offsets: np.ndarray, grad_out: np.ndarray):
    """Returns dict with sorted_pos, uniq_rows, seg_offsets, table_uniq_offsets, values, g_absmax, U
    (arrays trimmed to U)."""
    N = len(indices)
    sorted_pos = np.empty(N, np.int32)
    uniq_rows = np.empty(max(N, 1), np.int64)
    seg_offsets = np.empty(N + 1, np.int32)
    tuo = np.empty(T + 1, np.int32)
    values = np.empty((max(N, 1), D), np.float32)
    g_absmax = np.empty(T, np.float32)
    U = lib().oracle_embbag_bwd(C.c_int(T), C.c_int(D), C.c_int(B), _p(indices, C.c_int64),
                                _p(offsets, C.c_int64), _p(grad_out, C.c_float), _p(sorted_pos, C.c_int32),
                                _p(uniq_rows, C.c_int64), _p(seg_offsets, C.c_int32), _p(tuo, C.c_int32),
                                _p(values, C.c_float), _p(g_absmax, C.c_float))
    U = int(U)
    return dict(U=U, sorted_pos=sorted_pos, uniq_rows=uniq_rows[:U].copy(), seg_offsets=seg_offsets[:U + 1].copy(),
                table_uniq_offsets=tuo, values=values[:U].copy(), g_absmax=g_absmax)


def grad_quant_int8(T: int, D: int, values: np.ndarray, table_uniq_offsets: np.ndarray, g_absmax: np.ndarray):
    U = values.shape[0]
    gq = np.empty((max(U, 1), D), np.int8)
    g_scale = np.empty(T, np.float32)
    lib().oracle_grad_quant_int8(C.c_int(T), C.c_int(D), _p(values, C.c_float), _p(table_uniq_offsets, C.c_int32),
                                 _p(g_absmax, C.c_float), _p(gq, C.c_int8), _p(g_scale, C.c_float))
    return gq[:U], g_scale


def sparse_update(W: np.ndarray, packed: Optional[np.ndarray], row_offsets: np.ndarray, w_scale: np.ndarray,
                  uniq_rows: np.ndarray, table_uniq_offsets: np.ndarray, gq: np.ndarray, g_scale: np.ndarray,
                  lr: float) -> None:
    """In place on W (and packed)."""
    T = len(row_offsets) - 1
    D = W.shape[1]
    gq = np.ascontiguousarray(gq)
    lib().oracle_sparse_update(_p(W, C.c_float), _p(packed, C.c_uint8), _p(row_offsets, C.c_int64),
                               _p(w_scale, C.c_float), C.c_int(T), C.c_int(D), _p(uniq_rows, C.c_int64),
                               _p(table_uniq_offsets, C.c_int32), _p(gq, C.c_int8), _p(g_scale, C.c_float),
                               C.c_float(lr))


class SimulatedDP:
    """Simulated data parallelism on one device for the embedding tables (appendix "Simulated Data
    Parallelism Environment", Algorithm 1; INT8 gradients as in the distributed-training appendix).

    Micro-batches come in groups of ``simulated_nodes``; micro-batch j sits at place ``j % simulated_nodes`` of
    its group.  A group owns one accumulator of integer gradient codes: the group's first micro-batch starts it
    from zero and fixes the quantisation scale, every micro-batch adds the codes of its sparse gradient, and the
    group's last micro-batch applies the accumulated gradient to the weights once.  Reading: a group is complete
    after every ``simulated_nodes``-th micro-batch, (j + 1) % simulated_nodes == 0 (as printed, with j counted
    from 0, the very first group would be a single micro-batch; the steady state is the same).  The accumulator is
    dense, [rows][D] int32 over all tables: small tables only."""

    def __init__(self, W, packed, row_offsets, w_scale, simulated_nodes: int, lr: float):
        self.W, self.packed, self.row_offsets, self.w_scale = W, packed, row_offsets, w_scale
        self.n, self.lr = int(simulated_nodes), float(lr)
        self.T, self.D = len(row_offsets) - 1, W.shape[1]
        self.buffer = np.zeros(W.shape, np.int32)
        self.touched = np.zeros(W.shape[0], np.uint8)
        self.group_absmax = None  # the per-table maxima of the group's first micro-batch
        self.g_scale = None
        self.blocks = []          # this group's (uniq_rows, table_uniq_offsets, gq), for inspection

    def _start_group(self, first_absmax):
        self.buffer[:] = 0
        self.touched[:] = 0
        self.blocks = []
        self.group_absmax = first_absmax.copy()

    def _apply_group(self):
        lib().oracle_simdp_weight_update(_p(self.W, C.c_float), _p(self.packed, C.c_uint8),
                                         _p(self.row_offsets, C.c_int64), _p(self.w_scale, C.c_float),
                                         C.c_int(self.T), C.c_int(self.D), _p(self.buffer, C.c_int32),
                                         _p(self.touched, C.c_uint8), _p(self.g_scale, C.c_float), C.c_float(self.lr))

    def micro_batch(self, j: int, B: int, indices: np.ndarray, offsets: np.ndarray, grad_out: np.ndarray) -> bool:
        """Returns True if this micro-batch completed a group (the weights were updated)."""
        place = j % self.n
        sparse = embbag_bwd(self.T, self.D, B, indices, offsets, grad_out)
        if place == 0:
            self._start_group(sparse["g_absmax"])
        gq, self.g_scale = grad_quant_int8(self.T, self.D, sparse["values"], sparse["table_uniq_offsets"],
                                           self.group_absmax)
        gq = np.ascontiguousarray(gq)
        self.blocks.append((sparse["uniq_rows"], sparse["table_uniq_offsets"], gq))
        lib().oracle_simdp_accumulate(C.c_int(self.T), C.c_int(self.D), _p(self.row_offsets, C.c_int64),
                                      _p(sparse["uniq_rows"], C.c_int64), _p(sparse["table_uniq_offsets"], C.c_int32),
                                      _p(gq, C.c_int8), _p(self.buffer, C.c_int32), _p(self.touched, C.c_uint8))
        completes = place == self.n - 1
        if completes:
            self._apply_group()
        return completes


def dense_step(bot_dims, bot_w, bot_b, top_dims, top_w, top_b, dense_x, emb, labels, lr):
    """The dense part of one train step in float64.  bot_w / bot_b / top_w / top_b: lists of float64 arrays
    (updated IN PLACE by the SGD step).  dense_x [B][num_dense], emb [B][T][D], labels [B] (any float dtype).
    Returns (loss, grad_emb [B][T][D] float64)."""
    B, T, D = emb.shape
    f64 = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    x, e, y = f64(dense_x), f64(emb), f64(labels)
    for a in list(bot_w) + list(bot_b) + list(top_w) + list(top_b):
        assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    bd = np.ascontiguousarray(bot_dims, dtype=np.int32)
    td = np.ascontiguousarray(top_dims, dtype=np.int32)
    PP = C.POINTER(C.c_double)
    arr = lambda lst: (PP * len(lst))(*[a.ctypes.data_as(PP) for a in lst])
    grad = np.empty((B, T, D), np.float64)
    loss = lib().oracle_dense_step(C.c_int(B), C.c_int(x.shape[1]), C.c_int(T), C.c_int(D), C.c_int(len(bot_w)),
                                   _p(bd, C.c_int32), arr(bot_w), arr(bot_b), C.c_int(len(top_w)), _p(td, C.c_int32),
                                   arr(top_w), arr(top_b), _p(x, C.c_double), _p(e, C.c_double), _p(y, C.c_double),
                                   C.c_double(lr), _p(grad, C.c_double))
    return float(loss), grad


def dense_step_ex(bot_dims, bot_w, bot_b, top_dims, top_w, top_b, dense_x, emb, labels, lr, bot_wf=None, top_wf=None,
                  apply_sgd=True, want_grads=False):
    """The general dense step in float64: ``bot_wf`` / ``top_wf`` (lists of float64 arrays or None) are the
    weights the forward and the input gradients use; the master weights take the step iff ``apply_sgd``.
    Returns (loss, grad_emb[, (bot_gw, bot_gb, top_gw, top_gb)])."""
    B, T, D = emb.shape
    f64 = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    x, e, y = f64(dense_x), f64(emb), f64(labels)
    for a in list(bot_w) + list(bot_b) + list(top_w) + list(top_b) + list(bot_wf or []) + list(top_wf or []):
        assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    bd = np.ascontiguousarray(bot_dims, dtype=np.int32)
    td = np.ascontiguousarray(top_dims, dtype=np.int32)
    PP = C.POINTER(C.c_double)
    arr = lambda lst: (PP * len(lst))(*[a.ctypes.data_as(PP) for a in lst]) if lst is not None else None
    grads = None
    if want_grads:
        grads = tuple([np.zeros_like(a) for a in lst] for lst in (bot_w, bot_b, top_w, top_b))
    grad = np.empty((B, T, D), np.float64)
    loss = lib().oracle_dense_step_ex(
        C.c_int(B), C.c_int(x.shape[1]), C.c_int(T), C.c_int(D), C.c_int(len(bot_w)), _p(bd, C.c_int32), arr(bot_w),
        arr(bot_b), C.c_int(len(top_w)), _p(td, C.c_int32), arr(top_w), arr(top_b), _p(x, C.c_double),
        _p(e, C.c_double), _p(y, C.c_double), C.c_double(lr), _p(grad, C.c_double), arr(bot_wf), arr(top_wf),
        C.c_int(1 if apply_sgd else 0), arr(grads[0]) if grads else None, arr(grads[1]) if grads else None,
        arr(grads[2]) if grads else None, arr(grads[3]) if grads else None)
    return (float(loss), grad, grads) if want_grads else (float(loss), grad)


class SimulatedDPDense:
    """Simulated data parallelism for the MLPs (appendix "Simulated Data Parallelism Environment", Algorithm 1),
    FP32 gradients.  Micro-batch j sits at place ``j % simulated_nodes`` of its group; a group owns one gradient
    accumulator per parameter tensor (of the tensor's shape).  The group's first micro-batch starts the
    accumulators from zero, every micro-batch adds its gradient (forward and backward on the weights the group
    started with, mean loss over the micro-batch), and the group's last micro-batch takes ``p <- p - lr *
    accumulator`` once.  Float64, on the lists of arrays given (updated in place)."""

    def __init__(self, bot_dims, bot_w, bot_b, top_dims, top_w, top_b, simulated_nodes: int, lr: float):
        self.model = (bot_dims, bot_w, bot_b, top_dims, top_w, top_b)
        self.n, self.lr = int(simulated_nodes), float(lr)
        self.buffers = tuple([np.zeros_like(a) for a in lst] for lst in (bot_w, bot_b, top_w, top_b))

    def micro_batch(self, j: int, dense_x, emb, labels):
        """Returns (loss, grad_emb, completed_group)."""
        bot_dims, bot_w, bot_b, top_dims, top_w, top_b = self.model
        place = j % self.n
        loss, grad_emb, grads = dense_step_ex(bot_dims, bot_w, bot_b, top_dims, top_w, top_b, dense_x, emb, labels,
                                              self.lr, apply_sgd=False, want_grads=True)
        for acc_list, grad_list in zip(self.buffers, grads):
            for acc, g in zip(acc_list, grad_list):
                if place == 0:
                    acc[:] = g
                else:
                    acc += g
        completes = place == self.n - 1
        if completes:
            for params, acc_list in zip((bot_w, bot_b, top_w, top_b), self.buffers):
                for p_, acc in zip(params, acc_list):
                    p_ -= self.lr * acc
        return loss, grad_emb, completes


def mlp_fake_quant(W: np.ndarray, bits: int):
    """Channel-wise fake quantisation of W [out][in] (float32).  Returns (Wq float32, row_scale float32, codes int8)."""
    assert W.dtype == np.float32 and W.flags["C_CONTIGUOUS"] and W.ndim == 2
    out, inn = W.shape
    Wq = np.empty_like(W)
    scale = np.empty(out, np.float32)
    codes = np.empty((out, inn), np.int8)
    lib().oracle_mlp_fake_quant(_p(W, C.c_float), C.c_int(out), C.c_int(inn), C.c_int(bits), _p(Wq, C.c_float),
                                _p(scale, C.c_float), _p(codes, C.c_int8))
    return Wq, scale, codes


def mlp_grad_quant_ec(g: np.ndarray, err: Optional[np.ndarray], param: np.ndarray, lr: float):
    """INT8 + error compensation on one tensor, IN PLACE on ``err`` (may be None) and ``param`` (float32, any
    shape, contiguous).  Returns (scale, codes int8 of g's shape)."""
    for a in (g, param) + ((err,) if err is not None else ()):
        assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    codes = np.empty(g.shape, np.int8)
    s = lib().oracle_mlp_grad_quant_ec(C.c_int64(g.size), _p(g, C.c_float), _p(err, C.c_float) if err is not None else None,
                                       _p(param, C.c_float), C.c_float(lr), _p(codes, C.c_int8))
    return float(np.float32(s)), codes
