"""CPU-only checks of the boundary: the library loads, exports every symbol the header
declares, and every host-side validation error is returned before anything is launched
(so none of these calls needs a GPU)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2410_20046_amd as dq
from paper_2410_20046_amd.binding import dqrm_tables_t

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000  # a non-null, aligned address that is never dereferenced (validation fails first)


def _tables(T=2, D=16, rows=(5, 7), master=FAKE, packed=FAKE, w_scale=FAKE, ro_dev=FAKE):
    ro = np.concatenate([[0], np.cumsum(rows)]).astype(np.int64)
    t = dqrm_tables_t(T, D, ro.ctypes.data, ro_dev, master, packed, w_scale)
    t._keep = ro
    return t


def test_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "dqrm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(dqrm_[a-z0-9_]+)\s*\(", text))
    assert {"dqrm_embbag_fwd", "dqrm_embbag_bwd", "dqrm_grad_quant_int8", "dqrm_sparse_update", "dqrm_pack_int4",
            "dqrm_find_scale"} <= declared
    L = dq.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert set(dq.EXPORTS) == declared


def test_header_constants_match_binding():
    text = open(os.path.join(ROOT, "include", "dqrm.h")).read()
    defs = dict(re.findall(r"#define\s+(DQRM_[A-Z_0-9]+)\s+\(?(-?\d+)", text))
    assert int(defs["DQRM_SEG_CHUNK"]) == dq.SEG_CHUNK == 32
    assert int(defs["DQRM_MAX_TABLE_LOOKUPS"]) == dq.MAX_TABLE_LOOKUPS
    assert int(defs["DQRM_MAX_TABLES"]) == dq.MAX_TABLES and int(defs["DQRM_MAX_DIM"]) == dq.MAX_DIM
    assert int(defs["DQRM_MAX_DEDUPE_BATCHES"]) == dq.MAX_DEDUPE_BATCHES
    for n in ("INVALID_ARG", "UNSUPPORTED", "WORKSPACE_TOO_SMALL", "INDEX_OUT_OF_RANGE", "CAPACITY", "BAD_OFFSETS"):
        assert int(defs["DQRM_ERR_" + n]) == getattr(dq, "ERR_" + n)
    assert int(defs["DQRM_ERR_HIP"]) == dq.ERR_HIP
    assert int(defs["DQRM_ERR_SCRATCH_LIMIT"]) == dq.ERR_SCRATCH_LIMIT
    m = re.search(r"#define\s+DQRM_NOALLOC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", text)
    assert int(m.group(1)) << int(m.group(2)) == dq.NOALLOC_SCRATCH_BYTES


def test_workspace_bytes():
    f = dq.dqrm_embbag_bwd_workspace_bytes
    a = f(26, 64, 8192, 212992)
    assert 0 < a < 64 << 20
    assert f(26, 64, 8192, 2 * 212992) > a
    assert f(0, 64, 8192, 10) == 0 and f(26, 12, 8192, 10) == 0 and f(26, 512, 8, 10) == 0
    assert f(26, 64, 0, 10) == 0 and f(26, 64, 8, -1) == 0 and f(2000, 64, 8, 10) == 0
    assert f(1, 8, 1, 0) > 0


def test_validation_errors_before_any_launch():
    L = dq.lib()
    S = None  # stream: never used, validation fails first
    ok = _tables()
    r = C.byref
    # tables descriptor
    assert L.dqrm_find_scale(None, S) == dq.ERR_INVALID_ARG
    assert L.dqrm_find_scale(r(_tables(master=None)), S) == dq.ERR_INVALID_ARG
    assert L.dqrm_find_scale(r(_tables(w_scale=None)), S) == dq.ERR_INVALID_ARG
    assert L.dqrm_find_scale(r(_tables(ro_dev=None)), S) == dq.ERR_INVALID_ARG
    assert L.dqrm_find_scale(r(_tables(D=12)), S) == dq.ERR_UNSUPPORTED
    assert L.dqrm_find_scale(r(_tables(D=264)), S) == dq.ERR_UNSUPPORTED
    assert L.dqrm_find_scale(r(_tables(D=0)), S) == dq.ERR_INVALID_ARG
    assert L.dqrm_find_scale(r(_tables(master=FAKE + 4)), S) == dq.ERR_INVALID_ARG  # misaligned
    bad = _tables()
    bad._keep[1] = 9
    bad._keep[2] = 3  # row offsets decrease
    assert L.dqrm_find_scale(r(bad), S) == dq.ERR_INVALID_ARG
    big = _tables(rows=(5, 2 ** 31))
    assert L.dqrm_find_scale(r(big), S) == dq.ERR_UNSUPPORTED
    many = dqrm_tables_t(5000, 16, ok._keep.ctypes.data, FAKE, FAKE, FAKE, FAKE)
    assert L.dqrm_find_scale(r(many), S) == dq.ERR_UNSUPPORTED
    assert L.dqrm_pack_int4(r(_tables(packed=None)), S) == dq.ERR_INVALID_ARG
    # forward
    fwd = lambda tb=ok, idx=FAKE, off=FAKE, B=4, N=8, mode=0, out=FAKE, codes=None: L.dqrm_embbag_fwd(
        r(tb), idx, off, B, N, mode, out, codes, S)
    assert fwd(mode=2) == dq.ERR_INVALID_ARG
    assert fwd(off=None) == dq.ERR_INVALID_ARG
    assert fwd(idx=None) == dq.ERR_INVALID_ARG
    assert fwd(B=0) == dq.ERR_INVALID_ARG
    assert fwd(N=-1) == dq.ERR_INVALID_ARG
    assert fwd(out=None) == dq.ERR_INVALID_ARG
    assert fwd(out=FAKE + 8) == dq.ERR_INVALID_ARG
    assert fwd(mode=1, tb=_tables(packed=None)) == dq.ERR_INVALID_ARG
    assert fwd(N=2 ** 31) == dq.ERR_UNSUPPORTED
    # backward
    def bwd(tb=ok, N=8, ws=FAKE, ws_bytes=1 << 30, grad=FAKE, nu=FAKE, values=FAKE):
        return L.dqrm_embbag_bwd(r(tb), FAKE, FAKE, 4, N, grad, FAKE, FAKE, FAKE, FAKE, nu, values, FAKE, ws,
                                 ws_bytes, S)
    assert bwd(ws_bytes=16) == dq.ERR_WORKSPACE_TOO_SMALL
    assert bwd(ws_bytes=dq.dqrm_embbag_bwd_workspace_bytes(2, 16, 4, 8) - 1) == dq.ERR_WORKSPACE_TOO_SMALL
    assert bwd(ws=None) == dq.ERR_INVALID_ARG
    assert bwd(ws=FAKE + 64) == dq.ERR_INVALID_ARG
    assert bwd(grad=None) == dq.ERR_INVALID_ARG
    assert bwd(nu=None) == dq.ERR_INVALID_ARG
    assert bwd(values=FAKE + 4) == dq.ERR_INVALID_ARG
    assert bwd(tb=_tables(D=20)) == dq.ERR_UNSUPPORTED
    # the variant with the built-in scratch array: shapes beyond the array are refused on the host
    def bwd_na(tb=ok, B=4, N=8, grad=FAKE):
        return L.dqrm_embbag_bwd_noalloc(r(tb), FAKE, FAKE, B, N, grad, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, S)
    wide = _tables(D=64)
    assert dq.dqrm_embbag_bwd_workspace_bytes(2, 64, 8192, 2 * 8192 * 8) > dq.NOALLOC_SCRATCH_BYTES
    assert bwd_na(tb=wide, B=8192, N=2 * 8192 * 8) == dq.ERR_SCRATCH_LIMIT
    assert b"scratch" in L.dqrm_last_hip_error()
    assert L.dqrm_embbag_bwd_noalloc(None, FAKE, FAKE, 4, 8, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, S) == dq.ERR_INVALID_ARG
    assert bwd_na(N=-1) == dq.ERR_INVALID_ARG
    assert bwd_na(tb=_tables(D=20)) == dq.ERR_UNSUPPORTED
    # several batches in one dedupe launch
    from paper_2410_20046_amd.binding import dqrm_dedupe_batch_t

    def dd(n=2, bound=0, sp=FAKE, ws=FAKE, ws_bytes=1 << 30, arr="ok"):
        a = (dqrm_dedupe_batch_t * 8)()
        for k in range(8):
            a[k] = dqrm_dedupe_batch_t(FAKE, FAKE, 8, sp, FAKE, FAKE, FAKE, FAKE, ws, bound)
        return L.dqrm_dedupe_multi(r(ok), 4, n, a if arr == "ok" else None, ws_bytes, S)
    assert dd(arr=None) == dq.ERR_INVALID_ARG
    assert dd(n=0) == dq.ERR_INVALID_ARG
    assert dd(n=dq.MAX_DEDUPE_BATCHES + 1) == dq.ERR_UNSUPPORTED
    assert dd(sp=None) == dq.ERR_INVALID_ARG
    assert dd(ws=FAKE + 64) == dq.ERR_INVALID_ARG
    assert dd(bound=-1) == dq.ERR_INVALID_ARG
    assert dd(ws_bytes=16) == dq.ERR_WORKSPACE_TOO_SMALL
    from paper_2410_20046_amd.binding import dqrm_segsum_batch_t, dqrm_quant_block_t

    def ssm(n=2, N=8, grad=FAKE, values=FAKE, ws=FAKE, ws_bytes=1 << 30, arr="ok", tb=ok):
        a = (dqrm_segsum_batch_t * 8)()
        for k in range(8):
            a[k] = dqrm_segsum_batch_t(N, grad, values, None, ws)
        return L.dqrm_segment_sum_multi(r(tb), 4, n, a if arr == "ok" else None, ws_bytes, S)
    assert ssm(arr=None) == dq.ERR_INVALID_ARG
    assert ssm(n=0) == dq.ERR_INVALID_ARG
    assert ssm(n=dq.MAX_DEDUPE_BATCHES + 1) == dq.ERR_UNSUPPORTED
    assert ssm(N=-1) == dq.ERR_INVALID_ARG
    assert ssm(grad=None) == dq.ERR_INVALID_ARG
    assert ssm(values=FAKE + 4) == dq.ERR_INVALID_ARG
    assert ssm(ws=FAKE + 64) == dq.ERR_INVALID_ARG
    assert ssm(ws_bytes=16) == dq.ERR_WORKSPACE_TOO_SMALL
    assert ssm(tb=_tables(D=20)) == dq.ERR_UNSUPPORTED

    def gqm(n=2, T=2, D=16, cap=8, v=FAKE, q=FAKE, am=FAKE, arr="ok"):
        a = (dqrm_quant_block_t * 8)()
        for k in range(8):
            a[k] = dqrm_quant_block_t(cap, v, FAKE, am, q, FAKE)
        return L.dqrm_grad_quant_int8_multi(T, D, n, a if arr == "ok" else None, S)
    assert gqm(arr=None) == dq.ERR_INVALID_ARG
    assert gqm(n=0) == dq.ERR_INVALID_ARG
    assert gqm(n=dq.MAX_DEDUPE_BATCHES + 1) == dq.ERR_UNSUPPORTED
    assert gqm(cap=-1) == dq.ERR_INVALID_ARG
    assert gqm(v=None) == dq.ERR_INVALID_ARG
    assert gqm(am=None) == dq.ERR_INVALID_ARG
    assert gqm(q=FAKE + 2) == dq.ERR_INVALID_ARG
    assert gqm(D=12) == dq.ERR_UNSUPPORTED
    assert gqm(T=0) == dq.ERR_INVALID_ARG
    # quantise / update
    gq = lambda T=2, D=16, cap=8, v=FAKE, tuo=FAKE, am=FAKE, q=FAKE, gs=FAKE: L.dqrm_grad_quant_int8(
        T, D, cap, v, tuo, am, q, gs, S)
    assert gq(v=None) == dq.ERR_INVALID_ARG
    assert gq(q=None) == dq.ERR_INVALID_ARG
    assert gq(cap=-1) == dq.ERR_INVALID_ARG
    assert gq(D=12) == dq.ERR_UNSUPPORTED
    assert gq(T=0) == dq.ERR_INVALID_ARG
    up = lambda tb=ok, cap=8, ur=FAKE, tuo=FAKE, q=FAKE, gs=FAKE: L.dqrm_sparse_update(r(tb), cap, ur, tuo, q, gs,
                                                                                      0.1, S)
    assert up(ur=None) == dq.ERR_INVALID_ARG
    assert up(gs=None) == dq.ERR_INVALID_ARG
    assert up(cap=-5) == dq.ERR_INVALID_ARG
    assert up(tb=_tables(D=4)) == dq.ERR_UNSUPPORTED
    # merging sparse blocks, update from integer sums
    ups = lambda tb=ok, cap=8, ur=FAKE, tuo=FAKE, sm=FAKE, gs=FAKE: L.dqrm_sparse_update_sums(r(tb), cap, ur, tuo, sm,
                                                                                               gs, 0.1, S)
    assert ups(sm=None) == dq.ERR_INVALID_ARG
    assert ups(sm=FAKE + 4) == dq.ERR_INVALID_ARG
    assert ups(ur=None) == dq.ERR_INVALID_ARG
    assert ups(cap=-1) == dq.ERR_INVALID_ARG
    from paper_2410_20046_amd.binding import dqrm_sparse_block_t

    def merge(n=2, blocks="ok", max_total=64, ur=FAKE, tuo=FAKE, nu=FAKE, sm=FAKE, ws=FAKE, ws_bytes=1 << 30, tb=ok,
              cap=16, gq=FAKE):
        arr = (dqrm_sparse_block_t * 8)()
        for k in range(8):
            arr[k] = dqrm_sparse_block_t(FAKE, FAKE, gq, cap)
        return L.dqrm_sparse_merge(r(tb), n, arr if blocks == "ok" else None, max_total, ur, tuo, nu, sm, ws, ws_bytes, S)

    assert merge(blocks=None) == dq.ERR_INVALID_ARG
    assert merge(n=0) == dq.ERR_INVALID_ARG
    assert merge(n=dq.MAX_DEDUPE_BATCHES + 1) == dq.ERR_UNSUPPORTED
    assert merge(max_total=-1) == dq.ERR_INVALID_ARG
    assert merge(sm=None) == dq.ERR_INVALID_ARG
    assert merge(sm=FAKE + 8) == dq.ERR_INVALID_ARG
    assert merge(ws=FAKE + 16) == dq.ERR_INVALID_ARG
    assert merge(gq=None) == dq.ERR_INVALID_ARG
    assert merge(cap=1 << 28) == dq.ERR_UNSUPPORTED
    assert merge(ws_bytes=dq.dqrm_sparse_merge_workspace_bytes(2, 16, 2, 64) - 1) == dq.ERR_WORKSPACE_TOO_SMALL
    f = dq.dqrm_sparse_merge_workspace_bytes
    assert 0 < f(26, 64, 8, 212992) < 16 << 20 and f(26, 64, 8, 2 * 212992) > f(26, 64, 8, 212992)
    assert f(26, 64, 9, 10) == 0 and f(26, 12, 2, 10) == 0 and f(0, 16, 2, 10) == 0 and f(2, 16, 2, -1) == 0


def test_product_never_touches_the_oracle():
    """the HIP path and its binding share nothing with oracle/: no import, include, link or path."""
    pkg = os.path.join(ROOT, "paper_2410_20046_amd")
    pat = re.compile(r"import\s+oracle|from\s+oracle|oracle/|dqrm_oracle|oracle\.")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                assert not pat.search(open(os.path.join(dirpath, f)).read()), f
    assert not pat.search(open(os.path.join(ROOT, "include", "dqrm.h")).read())
