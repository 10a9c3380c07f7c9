"""Pins of the CPU oracle against things other than itself (CPU only).

Each test names the mistake it would catch.  Sources of truth used here:
hand-worked values (tests/golden), the sizes the paper prints, numpy / torch-CPU
library routines for the special cases that reduce to them, brute force on tiny
inputs, and integer closed forms.
"""
import os

import numpy as np
import pytest
import torch

from gen import make_workload, Workload

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(path):
    with open(os.path.join(GOLD, path)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


# --------------------------------------------------------------------------
# quantiser
# --------------------------------------------------------------------------
def test_quantizer_hand_example(oracle):
    """wrong rounding mode (half-away), missing clamp, asymmetric range, reciprocal sign slip."""
    for bits, s, x, q in _rows("quantizer_hand_example.txt"):
        assert oracle.quantize_code(float(x), float(s), int(bits)) == int(q), (bits, s, x, q)


def test_scale_closed_form(oracle):
    """scale = absmax / (2^(b-1)-1): 7 for INT4, 127 for INT8; floor for an all-zero tensor."""
    assert oracle.scale_from_absmax(1.75, 4) == 0.25
    assert oracle.scale_from_absmax(63.5, 8) == 0.5
    assert oracle.scale_from_absmax(0.0, 4) == np.float32(1e-8)
    assert oracle.scale_from_absmax(0.0, 8) == np.float32(1e-8)
    # fresh scale: the largest magnitude maps to exactly +-7 / +-127, nothing clamps to -8 / -128
    rng = np.random.default_rng(0)
    for bits, qmax in ((4, 7), (8, 127)):
        x = rng.standard_normal(1000).astype(np.float32)
        s = oracle.scale_from_absmax(float(np.abs(x).max()), bits)
        q = np.array([oracle.quantize_code(float(v), s, bits) for v in x])
        assert q.max() <= qmax and q.min() >= -qmax
        assert abs(q[np.argmax(np.abs(x))]) == qmax


def test_quantizer_invariants(oracle):
    """range, |x - s*q| <= s/2 when unclipped, idempotence q(s*q) = q."""
    rng = np.random.default_rng(1)
    for bits in (4, 8):
        lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
        for s in (np.float32(0.013), np.float32(1e-8), np.float32(3.7)):
            x = (rng.standard_normal(2000) * float(s) * hi * 0.6).astype(np.float32)
            q = np.array([oracle.quantize_code(float(v), float(s), bits) for v in x])
            assert q.min() >= lo and q.max() <= hi
            unclipped = np.abs(x.astype(np.float64)) <= (hi + 0.5) * float(s)
            err = np.abs(x.astype(np.float64) - float(s) * q)
            assert np.all(err[unclipped] <= 0.5 * float(s) * (1 + 1e-6))
            deq = (np.float32(s) * q.astype(np.float32)).astype(np.float32)
            q2 = np.array([oracle.quantize_code(float(v), float(s), bits) for v in deq])
            assert np.array_equal(q, q2)


def test_find_scale_matches_numpy(oracle):
    """wrong table boundaries, max instead of absmax, per-row instead of per-table."""
    wl = make_workload("tiny")
    W = wl.tables(threads=1)
    W[1234, 3] = -0.9  # the extreme is negative in table 1
    s = oracle.find_scale(W, wl.row_offsets)
    for t in range(wl.T):
        a = np.abs(W[wl.row_offsets[t]:wl.row_offsets[t + 1]]).max()
        assert s[t] == np.float32(a) / np.float32(7.0)
    assert s[1] == np.float32(0.9) / np.float32(7.0)


# --------------------------------------------------------------------------
# packed INT4 storage
# --------------------------------------------------------------------------
def test_packed_size_matches_paper(oracle):
    """bytes = rows * dim / 2; the synthetic shapes reproduce the paper's printed sizes."""
    for name, D, fp32_gb, int4_gb in _rows("paper_model_sizes.txt"):
        wl = make_workload(name)
        assert wl.D == int(D)
        assert abs(wl.R * wl.D * 4 / 1e9 - float(fp32_gb)) < 2e-3
        assert abs(wl.R * wl.D / 2 / 1e9 - float(int4_gb)) < 1e-3
    wl = make_workload("tiny")
    W = wl.tables(threads=1)
    packed = oracle.pack_int4(W, wl.row_offsets, oracle.find_scale(W, wl.row_offsets))
    assert packed.nbytes == wl.R * wl.D // 2 and packed.dtype == np.uint8


def test_pack_layout_and_roundtrip(oracle):
    """nibble order (even element low), two's complement, every code value survives."""
    # one table, 2 rows x 8: codes chosen directly by using scale 1 and integer weights
    W = np.array([[-8, -7, -1, 0, 1, 7, 3, -4], [0, 1, 2, 3, 4, 5, 6, 7]], np.float32)
    ro = np.array([0, 2], np.int64)
    packed = oracle.pack_int4(W, ro, np.array([1.0], np.float32))
    # hand-packed: low nibble = even element, high nibble = odd element
    exp0 = [(-8 & 15) | ((-7 & 15) << 4), (-1 & 15) | (0 << 4), 1 | (7 << 4), 3 | ((-4 & 15) << 4)]
    assert packed[0].tolist() == exp0 == [0x98, 0x0F, 0x71, 0xC3]
    assert packed[1].tolist() == [0x10, 0x32, 0x54, 0x76]
    assert np.array_equal(oracle.unpack_int4(packed), W.astype(np.int8))


def test_packed_forward_equals_master_forward(oracle):
    wl = make_workload("tiny")
    W = wl.tables(threads=1)
    s = oracle.find_scale(W, wl.row_offsets)
    packed = oracle.pack_int4(W, wl.row_offsets, s)
    idx, off = wl.batch(0, pooling="ragged", max_len=5)
    o0, c0 = oracle.embbag_fwd(W, None, wl.row_offsets, s, wl.B, idx, off, mode=0)
    o1, c1 = oracle.embbag_fwd(None, packed, wl.row_offsets, s, wl.B, idx, off, mode=1)
    assert np.array_equal(c0, c1)
    assert np.array_equal(o0.view(np.uint32), o1.view(np.uint32))


# --------------------------------------------------------------------------
# forward: gather + fake-quant + sum pooling
# --------------------------------------------------------------------------
@pytest.mark.parametrize("pooling", ["one", "ragged"])
def test_forward_identity_quantizer_is_embedding_bag(oracle, pooling):
    """wrong table base, wrong bag->(b,t) output slot, off-by-one in offsets, empty bags."""
    wl = make_workload("tiny")
    W = wl.tables(threads=1)
    idx, off = wl.batch(3, pooling=pooling, max_len=6)
    out, _ = oracle.embbag_fwd(W, None, wl.row_offsets, None, wl.B, idx, off, quantise=False, want_codes=False)
    for t in range(wl.T):
        lo, hi = off[t * wl.B], off[(t + 1) * wl.B]
        ref = torch.nn.functional.embedding_bag(
            torch.from_numpy(idx[lo:hi]), torch.from_numpy(W[wl.row_offsets[t]:wl.row_offsets[t + 1]]),
            torch.from_numpy(off[t * wl.B:(t + 1) * wl.B] - lo), mode="sum")
        np.testing.assert_allclose(out[:, t, :], ref.numpy(), rtol=1e-6, atol=1e-7)


def test_forward_quantized_explicit_loop(oracle):
    """bag sums reproduced by an explicit loop over numpy float32 scalars; codes within [-8, 7];
    stale scale clamps."""
    wl = make_workload("tiny")
    W = wl.tables(threads=1)
    s = oracle.find_scale(W, wl.row_offsets)
    s[2] *= np.float32(0.4)  # stale scale: table 2 has out-of-range weights -> clamping
    idx, off = wl.batch(1, pooling="ragged", max_len=3)
    out, codes = oracle.embbag_fwd(W, None, wl.row_offsets, s, wl.B, idx, off)
    assert codes.min() >= -8 and codes.max() <= 7
    assert codes.min() == -8 and codes.max() == 7  # the stale table saturates both ways
    exp = np.zeros_like(out)
    for t in range(wl.T):
        for b in range(wl.B):
            acc = np.zeros(wl.D, np.float32)
            for i in range(off[t * wl.B + b], off[t * wl.B + b + 1]):
                w = W[wl.row_offsets[t] + idx[i]]
                q = np.clip(np.rint(w / s[t]), -8, 7).astype(np.float32)  # numpy: fp32 divide, half-even
                assert np.array_equal(q.astype(np.int8), codes[i])
                acc = acc + s[t] * q
            exp[b, t] = acc
    assert np.array_equal(out.view(np.uint32), exp.view(np.uint32))


# --------------------------------------------------------------------------
# backward: dedupe + segment sums ("specified sparsity", lossless)
# --------------------------------------------------------------------------
def _dense_gradient_bruteforce(wl: Workload, idx, off, g, dtype):
    """G_t[r] = sum_i [idx_i == r] g[bag(i)]  by the O(N * rows) double loop of the definition."""
    G = [np.zeros((int(c), wl.D), dtype) for c in wl.cards]
    for t in range(wl.T):
        for r in range(int(wl.cards[t])):
            for b in range(wl.B):
                for i in range(off[t * wl.B + b], off[t * wl.B + b + 1]):
                    if idx[i] == r:
                        G[t][r] += g[b, t].astype(dtype)
    return G


def test_sparse_gradient_equals_dense_bruteforce(oracle):
    """lossless: scattering (uniq_rows, values) into zeros IS the dense gradient.  Exact on dyadic
    inputs (integer closed form), to tolerance on general floats (fp64 brute force)."""
    wl = make_workload("tiny", T=3, B=48, fixed_card=40, rows=120)
    for pooling in ("one", "ragged"):
        idx, off = wl.batch(5, pooling=pooling, max_len=4)
        for kind in ("dyadic", "normal"):
            g = wl.grad_dyadic(0) if kind == "dyadic" else wl.grad_normal(0)
            r = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, g)
            G = _dense_gradient_bruteforce(wl, idx, off, g, np.float64)
            tuo = r["table_uniq_offsets"]
            touched = 0
            for t in range(wl.T):
                S = np.zeros_like(G[t])
                rows = r["uniq_rows"][tuo[t]:tuo[t + 1]]
                S[rows] = r["values"][tuo[t]:tuo[t + 1]]
                lo, hi = off[t * wl.B], off[(t + 1) * wl.B]
                assert set(rows.tolist()) == set(idx[lo:hi].tolist())  # exactly the touched rows
                touched += len(rows)
                if kind == "dyadic":
                    assert np.array_equal(S, G[t])  # fp64 brute force is exact here
                    m = np.rint(G[t] * 2.0 ** 24).astype(np.int64)  # integer closed form
                    assert np.array_equal(np.rint(S.astype(np.float64) * 2.0 ** 24).astype(np.int64), m)
                else:
                    np.testing.assert_allclose(S, G[t], rtol=1e-5, atol=1e-9)
                assert r["g_absmax"][t] == (np.abs(r["values"][tuo[t]:tuo[t + 1]]).max() if len(rows) else 0.0)
            assert touched == r["U"]


def test_dedupe_matches_numpy_unique(oracle):
    """uniq_rows ascending per table == numpy.unique; segment lengths == counts; sorted_pos is a
    stable permutation; seg_offsets global and ending at N."""
    wl = make_workload("tiny", B=300, fixed_card=37, rows=4 * 37)
    idx, off = wl.batch(2, pooling="ragged", max_len=3)
    N = len(idx)
    r = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, wl.grad_dyadic(0))
    sp, so, tuo = r["sorted_pos"], r["seg_offsets"], r["table_uniq_offsets"]
    assert sorted(sp.tolist()) == list(range(N))
    assert so[-1] == N and tuo[0] == 0 and tuo[-1] == r["U"]
    for t in range(wl.T):
        lo, hi = off[t * wl.B], off[(t + 1) * wl.B]
        vals, cnt = np.unique(idx[lo:hi], return_counts=True)
        assert np.array_equal(r["uniq_rows"][tuo[t]:tuo[t + 1]], vals)
        assert np.array_equal(np.diff(so[tuo[t]:tuo[t + 1] + 1]), cnt)
        if len(vals):
            assert so[tuo[t]] == lo
        # stable: equals numpy's stable argsort of the table's rows
        assert np.array_equal(sp[lo:hi], lo + np.argsort(idx[lo:hi], kind="stable"))


def test_sparse_gradient_is_torch_coalesce(oracle):
    """the paper's own baseline op: sparse COO of per-lookup gradients, coalesced."""
    wl = make_workload("tiny")
    idx, off = wl.batch(4)
    g = wl.grad_normal(1)
    r = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, g)
    tuo = r["table_uniq_offsets"]
    for t in range(wl.T):
        rows = torch.from_numpy(idx[t * wl.B:(t + 1) * wl.B])
        sp = torch.sparse_coo_tensor(rows[None, :], torch.from_numpy(g[:, t, :].copy()),
                                     (int(wl.cards[t]), wl.D)).coalesce()
        assert np.array_equal(sp.indices()[0].numpy(), r["uniq_rows"][tuo[t]:tuo[t + 1]])
        np.testing.assert_allclose(r["values"][tuo[t]:tuo[t + 1]], sp.values().numpy(), rtol=1e-5, atol=1e-9)


def test_segment_sum_order(oracle):
    """the documented order: chunks of seg_chunk() left to right, then chunk sums left to right.
    (A regression check of the stated reading; the order itself is not fixed by the paper.)"""
    ch = oracle.seg_chunk()
    assert ch == 32
    T, D, B = 1, 8, 100
    idx = np.zeros(B, np.int64)  # one segment of length 100
    idx[70:] = 1  # and one of length 30
    off = np.arange(B + 1, dtype=np.int64)
    rng = np.random.default_rng(7)
    g = (rng.standard_normal((B, T, D)) * 10.0 ** rng.integers(-6, 3, (B, T, D))).astype(np.float32)
    r = oracle.embbag_bwd(T, D, B, idx, off, g)
    for seg, (lo, hi) in enumerate(((0, 70), (70, 100))):
        total = None
        for c in range(lo, hi, ch):
            part = g[c, 0].copy()
            for k in range(c + 1, min(c + ch, hi)):
                part = part + g[k, 0]
            total = part if total is None else total + part
        assert np.array_equal(r["values"][seg].view(np.uint32), total.view(np.uint32))
    # and the order matters on these inputs (otherwise the check above proves nothing)
    plain = g[0, 0].copy()
    for k in range(1, 70):
        plain = plain + g[k, 0]  # one left-to-right fp32 sum over the whole segment, no chunks
    assert not np.array_equal(r["values"][0].view(np.uint32), plain.view(np.uint32))


# --------------------------------------------------------------------------
# INT8 gradient quantisation and the sparse update
# --------------------------------------------------------------------------
def test_grad_quant_closed_form(oracle):
    """scale = absmax/127 per table; codes in [-128,127] (in fact [-127,127] with a fresh scale);
    only values are quantised; an all-zero table gives zero codes."""
    wl = make_workload("tiny")
    idx, off = wl.batch(6)
    g = wl.grad_normal(2)
    g[:, 3, :] = 0.0  # table 3: all-zero gradient
    r = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, g)
    rows_before = r["uniq_rows"].copy()
    gq, gs = oracle.grad_quant_int8(wl.T, wl.D, r["values"], r["table_uniq_offsets"], r["g_absmax"])
    assert np.array_equal(rows_before, r["uniq_rows"])
    tuo = r["table_uniq_offsets"]
    for t in range(wl.T):
        v = r["values"][tuo[t]:tuo[t + 1]]
        if t == 3:
            assert gs[t] == np.float32(1e-8) and not gq[tuo[t]:tuo[t + 1]].any()
            continue
        assert gs[t] == np.abs(v).max() / np.float32(127.0)
        exp = np.clip(np.rint(v / gs[t]), -128, 127).astype(np.int8)
        assert np.array_equal(gq[tuo[t]:tuo[t + 1]], exp)
        assert np.abs(exp).max() == 127
        assert np.all(np.abs(v.astype(np.float64) - float(gs[t]) * exp) <= 0.5 * float(gs[t]) * (1 + 1e-6))


def test_sparse_update_pins(oracle):
    """zero codes leave rows bit-identical; untouched rows never change; one-row hand example;
    packed mirror re-encoded with the cached weight scale."""
    # hand example: 1 table, 3 rows x 8, update row 1 with codes, g_scale 0.5, lr 0.25:
    #   step = 0.25 * (0.5 * code) = code / 8  (exact)
    W = np.arange(24, dtype=np.float32).reshape(3, 8) / 4.0
    W0 = W.copy()
    ro = np.array([0, 3], np.int64)
    ws = np.array([1.0], np.float32)
    packed = oracle.pack_int4(W, ro, ws)
    p0 = packed.copy()
    gq = np.array([[8, -8, 16, 0, 127, -128, 1, -1]], np.int8)
    oracle.sparse_update(W, packed, ro, ws, np.array([1], np.int64), np.array([0, 1], np.int32), gq,
                         np.array([0.5], np.float32), 0.25)
    assert np.array_equal(W[0], W0[0]) and np.array_equal(W[2], W0[2])
    assert np.array_equal(packed[0], p0[0]) and np.array_equal(packed[2], p0[2])
    assert np.array_equal(W[1], W0[1] - gq[0].astype(np.float32) / 8.0)
    exp_codes = np.clip(np.rint(W[1]), -8, 7).astype(np.int8)
    assert np.array_equal(oracle.unpack_int4(packed)[1], exp_codes)
    # zero codes: bit-identical
    W1 = W.copy()
    oracle.sparse_update(W, None, ro, ws, np.array([0, 2], np.int64), np.array([0, 2], np.int32),
                         np.zeros((2, 8), np.int8), np.array([123.0], np.float32), 0.1)
    assert np.array_equal(W.view(np.uint32), W1.view(np.uint32))


def test_full_step_chain_tiny(oracle):
    """fwd -> bwd -> quant -> update on the tiny config: everything stays consistent."""
    wl = make_workload("tiny")
    W = wl.tables(threads=1)
    W0 = W.copy()
    s = oracle.find_scale(W, wl.row_offsets)
    packed = oracle.pack_int4(W, wl.row_offsets, s)
    idx, off = wl.batch(0)
    g = wl.grad_normal(0)
    r = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, g)
    gq, gs = oracle.grad_quant_int8(wl.T, wl.D, r["values"], r["table_uniq_offsets"], r["g_absmax"])
    oracle.sparse_update(W, packed, wl.row_offsets, s, r["uniq_rows"], r["table_uniq_offsets"], gq, gs, 0.1)
    touched = np.zeros(wl.R, bool)
    tuo = r["table_uniq_offsets"]
    for t in range(wl.T):
        touched[wl.row_offsets[t] + r["uniq_rows"][tuo[t]:tuo[t + 1]]] = True
    assert np.array_equal(W[~touched], W0[~touched])
    assert touched.sum() == r["U"]
    # the update is -lr * dequantised gradient, within INT8 resolution of the true gradient
    for t in range(wl.T):
        rows = wl.row_offsets[t] + r["uniq_rows"][tuo[t]:tuo[t + 1]]
        v = r["values"][tuo[t]:tuo[t + 1]].astype(np.float64)
        np.testing.assert_allclose((W0[rows].astype(np.float64) - W[rows]) / 0.1, v, atol=0.51 * gs[t] + 1e-7)
    # packed mirror stays in sync with the master under the cached scale
    assert np.array_equal(packed, oracle.pack_int4(W, wl.row_offsets, s))
