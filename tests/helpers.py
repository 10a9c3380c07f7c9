"""Shared plumbing of the GPU parity tests: run the HIP path through the C ABI, run
the oracle on the same host arrays, compare to the stated bar.

Bar: bit-exact for INT4 / INT8 codes, packed bytes, sorted positions, unique rows,
segment and table offsets, counts; floats within |a-b| <= 1e-6 + 1e-5*|b|.
"""
from __future__ import annotations

import numpy as np

RTOL = 1e-5
ATOL = 1e-6


def assert_float_close(got: np.ndarray, exp: np.ndarray, what: str) -> None:
    got = np.asarray(got, np.float64)
    exp = np.asarray(exp, np.float64)
    assert got.shape == exp.shape, (what, got.shape, exp.shape)
    bad = np.abs(got - exp) > ATOL + RTOL * np.abs(exp)
    if bad.any():
        k = np.argwhere(bad)[0]
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} outside tolerance, first at {tuple(k)}: "
                             f"got {got[tuple(k)]!r} expected {exp[tuple(k)]!r}")


def assert_exact(got: np.ndarray, exp: np.ndarray, what: str) -> None:
    got = np.asarray(got)
    exp = np.asarray(exp)
    assert got.shape == exp.shape, (what, got.shape, exp.shape)
    if not np.array_equal(got, exp):
        k = np.argwhere(got != exp)[0]
        raise AssertionError(f"{what}: {(got != exp).sum()} of {got.size} differ, first at {tuple(k)}: "
                             f"got {got[tuple(k)]!r} expected {exp[tuple(k)]!r}")


class GpuRun:
    """Device copies of one workload + the per-step buffers, driven only through the C ABI binding."""

    def __init__(self, row_offsets, D, W, B, N, with_packed=True, want_codes=True, device="cuda:0"):
        import torch
        import paper_2410_20046_amd as dq

        self.torch, self.dq = torch, dq
        self.dev = torch.device(device)
        T = len(row_offsets) - 1
        R = W.shape[0]
        self.master = torch.from_numpy(W).to(self.dev)
        self.packed = torch.zeros((R, D // 2), dtype=torch.uint8, device=self.dev) if with_packed else None
        self.tables = dq.Tables(row_offsets, D, self.master, self.packed)
        self.bufs = dq.StepBuffers(T, D, B, N, self.dev, want_codes=want_codes)
        self.T, self.D, self.B, self.N = T, D, B, N

    def upload_batch(self, idx, off, grad=None):
        t = self.torch
        self.idx = t.from_numpy(idx).to(self.dev)
        self.off = t.from_numpy(off).to(self.dev)
        self.grad = t.from_numpy(grad).to(self.dev) if grad is not None else None

    def status(self):
        return self.dq.dqrm_check_status()

    def find_scale(self):
        self.dq.dqrm_find_scale(self.tables)
        return self.tables.w_scale.cpu().numpy()

    def set_scale(self, s):
        self.tables.w_scale.copy_(self.torch.from_numpy(np.ascontiguousarray(s, np.float32)))

    def pack(self):
        self.dq.dqrm_pack_int4(self.tables)
        return self.packed.cpu().numpy()

    def fwd(self, mode):
        b = self.bufs
        self.dq.dqrm_embbag_fwd(self.tables, self.idx, self.off, self.B, mode, b.out, b.codes)
        return b.out.cpu().numpy(), (b.codes.cpu().numpy()[: self.N] if b.codes is not None else None)

    def bwd(self):
        b = self.bufs
        self.dq.dqrm_embbag_bwd(self.tables, self.idx, self.off, self.B, self.grad, b.sorted_pos, b.uniq_rows,
                                b.seg_offsets, b.table_uniq_offsets, b.num_unique, b.values, b.g_absmax, b.workspace)
        U = int(b.num_unique.cpu().item())
        return dict(U=U, sorted_pos=b.sorted_pos.cpu().numpy()[: self.N], uniq_rows=b.uniq_rows.cpu().numpy()[:U],
                    seg_offsets=b.seg_offsets.cpu().numpy()[: U + 1],
                    table_uniq_offsets=b.table_uniq_offsets.cpu().numpy(), values=b.values.cpu().numpy()[:U],
                    g_absmax=b.g_absmax.cpu().numpy())

    def quant(self):
        b = self.bufs
        self.dq.dqrm_grad_quant_int8(self.T, self.D, b.cap, b.values, b.table_uniq_offsets, b.g_absmax, b.gq,
                                     b.g_scale)
        U = int(b.num_unique.cpu().item())
        return b.gq.cpu().numpy()[:U], b.g_scale.cpu().numpy()

    def update(self, lr):
        b = self.bufs
        self.dq.dqrm_sparse_update(self.tables, b.cap, b.uniq_rows, b.table_uniq_offsets, b.gq, b.g_scale, lr)

    def master_np(self):
        return self.master.cpu().numpy()

    def packed_np(self):
        return self.packed.cpu().numpy()


def compare_bwd(g, o, what=""):
    assert g["U"] == o["U"], (what, g["U"], o["U"])
    assert_exact(g["table_uniq_offsets"], o["table_uniq_offsets"], what + " table_uniq_offsets")
    assert_exact(g["sorted_pos"], o["sorted_pos"], what + " sorted_pos")
    assert_exact(g["uniq_rows"], o["uniq_rows"], what + " uniq_rows")
    assert_exact(g["seg_offsets"], o["seg_offsets"], what + " seg_offsets")
    assert_float_close(g["values"], o["values"], what + " values")
    assert_float_close(g["g_absmax"], o["g_absmax"], what + " g_absmax")


def full_step_parity(oracle, wl, W, idx, off, grad, lr=0.1, stale=None, check_bits=True, what=""):
    """Runs S0, S1, F (both modes), B1-B5 on the GPU and in the oracle on the same inputs and compares
    every output.  Returns the GpuRun for further checks."""
    N = len(idx)
    run = GpuRun(wl.row_offsets, wl.D, W, wl.B, N)
    run.upload_batch(idx, off, grad)
    Wo = W.copy()

    s_gpu = run.find_scale()
    s_or = oracle.find_scale(Wo, wl.row_offsets)
    assert_exact(s_gpu.view(np.uint32), s_or.view(np.uint32), what + " w_scale bits")
    if stale is not None:
        s_or = (s_or * np.float32(stale)).astype(np.float32)
        run.set_scale(s_or)

    p_gpu = run.pack()
    p_or = oracle.pack_int4(Wo, wl.row_offsets, s_or)
    assert_exact(p_gpu, p_or, what + " packed bytes")

    out_or, codes_or = oracle.embbag_fwd(Wo, None, wl.row_offsets, s_or, wl.B, idx, off, mode=0)
    for mode in (0, 1):
        out_g, codes_g = run.fwd(mode)
        assert_exact(codes_g, codes_or, what + f" INT4 codes mode {mode}")
        assert_float_close(out_g, out_or, what + f" out mode {mode}")
        if check_bits:
            assert_exact(out_g.view(np.uint32), out_or.view(np.uint32), what + f" out bits mode {mode}")

    g = run.bwd()
    o = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, grad)
    compare_bwd(g, o, what)
    if check_bits:
        assert_exact(g["values"].view(np.uint32), o["values"].view(np.uint32), what + " values bits")

    gq_g, gs_g = run.quant()
    # stage-isolated: the oracle quantises the GPU's own values (bit-identical inputs)
    gq_iso, gs_iso = oracle.grad_quant_int8(wl.T, wl.D, g["values"], g["table_uniq_offsets"], g["g_absmax"])
    assert_exact(gq_g, gq_iso, what + " INT8 codes (stage-isolated)")
    assert_exact(gs_g.view(np.uint32), gs_iso.view(np.uint32), what + " g_scale bits (stage-isolated)")
    # chained: the oracle's own chain
    gq_or, gs_or = oracle.grad_quant_int8(wl.T, wl.D, o["values"], o["table_uniq_offsets"], o["g_absmax"])
    assert_float_close(gs_g, gs_or, what + " g_scale")
    if check_bits:
        assert_exact(gq_g, gq_or, what + " INT8 codes (chained)")
    assert gq_g.min(initial=0) >= -128 and gq_g.max(initial=0) <= 127

    run.update(lr)
    oracle.sparse_update(Wo, p_or, wl.row_offsets, s_or, o["uniq_rows"], o["table_uniq_offsets"], gq_or, gs_or, lr)
    Wg = run.master_np()
    assert_float_close(Wg, Wo, what + " master after update")
    if check_bits:
        assert_exact(Wg.view(np.uint32), Wo.view(np.uint32), what + " master bits after update")
        assert_exact(run.packed_np(), p_or, what + " packed after update")
    code, tb, val = run.status()
    assert code == 0, (what, "device status", code, tb, val)
    return run
