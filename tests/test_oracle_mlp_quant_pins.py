"""Pins of the oracle's quantised dense-part routines (CPU only).

* ``mlp_fake_quant`` (channel-wise INT4 / INT8 weights) against: the hand-worked example, the scalar quantiser
  that the embedding pins already fix (``quantize_code`` / ``scale_from_absmax``), the table-wise
  ``find_scale`` on the same matrix read as one-row tables, closed-form invariants, idempotence.
* ``mlp_grad_quant_ec`` (INT8 gradient + error compensation) against: the hand-worked example, the
  table-wise ``grad_quant_int8`` + ``sparse_update`` pair when no residual is carried, the telescoping
  identity of error feedback, the residual bound.
* ``dense_step_ex`` against torch autograd (float64) with a straight-through weight.
Mistakes these catch: a matrix-wise instead of row-wise scale, a transposed matrix, truncation instead of
round-half-even, the residual subtracted instead of added or taken before the clamp, the residual of the wrong
step, a step taken with the unquantised gradient, input gradients through the master instead of the
quantised weights."""
import os

import numpy as np
import pytest
import torch

from gen import make_dense_model, dense_batch

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


# ---------------------------------------------------------------- channel-wise weights
def test_fake_quant_hand_example(oracle):
    rows, scales, cur = [], [], None
    for tok in _rows("mlp_channelwise_hand_example.txt"):
        if tok[0] == "row":
            scales.append(float(tok[3]))
            cur = []
            rows.append(cur)
        else:
            cur.append((float(tok[0]), int(tok[1]), float(tok[2])))
    W = np.array([[e[0] for e in r] for r in rows], np.float32)
    Wq, s, codes = oracle.mlp_fake_quant(W, 4)
    assert s.tolist() == scales
    assert codes.tolist() == [[e[1] for e in r] for r in rows]
    assert Wq.tolist() == [[e[2] for e in r] for r in rows]


@pytest.mark.parametrize("bits", [4, 8])
def test_fake_quant_is_the_pinned_scalar_quantiser_row_by_row(oracle, bits):
    rng = np.random.default_rng(11)
    W = (rng.standard_normal((9, 13)) * rng.uniform(0.01, 3.0, size=(9, 1))).astype(np.float32)
    W[4] = 0.0  # an all-zero row: scale floor, all codes 0
    Wq, s, codes = oracle.mlp_fake_quant(W, bits)
    for o in range(W.shape[0]):
        so = oracle.scale_from_absmax(float(np.abs(W[o]).max()), bits)
        assert np.float32(so) == s[o]
        for i in range(W.shape[1]):
            c = oracle.quantize_code(float(W[o, i]), so, bits)
            assert c == codes[o, i]
            assert np.float32(np.float32(so) * np.float32(c)) == Wq[o, i]
    assert s[4] == np.float32(1e-8) and not codes[4].any()


def test_fake_quant_rows_are_one_row_tables(oracle):
    """The embedding oracle's per-table scale of a layer read as `out` tables of one row each."""
    rng = np.random.default_rng(12)
    W = rng.standard_normal((6, 16)).astype(np.float32)
    _, s, _ = oracle.mlp_fake_quant(W, 4)
    s_tab = oracle.find_scale(W, np.arange(7, dtype=np.int64))
    assert np.array_equal(s.view(np.uint32), s_tab.view(np.uint32))


@pytest.mark.parametrize("bits", [4, 8])
def test_fake_quant_invariants(oracle, bits):
    rng = np.random.default_rng(13)
    W = (rng.standard_normal((32, 40)) * rng.uniform(1e-3, 10.0, size=(32, 1))).astype(np.float32)
    Wq, s, codes = oracle.mlp_fake_quant(W, bits)
    qmax = 2 ** (bits - 1) - 1
    assert codes.min() >= -qmax - 1 and codes.max() <= qmax
    # a fresh scale never clips: error at most half a step (plus rounding slack)
    assert np.all(np.abs(Wq.astype(np.float64) - W) <= 0.5 * s[:, None].astype(np.float64) * (1 + 1e-6))
    # the row's largest element sits on the last code
    rows = np.arange(W.shape[0])
    top = np.abs(W).argmax(axis=1)
    assert np.all(np.abs(codes[rows, top]) == qmax)
    # idempotent, row by row independent
    Wq2, s2, codes2 = oracle.mlp_fake_quant(Wq, bits)
    assert np.array_equal(codes2, codes)
    W2 = W.copy()
    W2[5] *= 3.0
    Wq3, _, _ = oracle.mlp_fake_quant(W2, bits)
    keep = np.arange(W.shape[0]) != 5
    assert np.array_equal(Wq3[keep], Wq[keep]) and not np.array_equal(Wq3[5], Wq[5])
    # a matrix-wise scale would differ
    assert len(np.unique(s)) > 1


# ---------------------------------------------------------------- INT8 gradients with error compensation
def test_grad_ec_hand_example(oracle):
    u = np.float32(2.0 ** -10)
    t = np.array([[float(x) for x in r] for r in _rows("mlp_grad_error_compensation_hand_example.txt")])
    g = (t[:, 0] * u).astype(np.float32)
    e = (t[:, 1] * u).astype(np.float32)
    p = t[:, 2].astype(np.float32)
    s, codes = oracle.mlp_grad_quant_ec(g, e, p, 0.5)
    assert s == float(u)
    assert codes.tolist() == t[:, 3].astype(int).tolist()
    assert (e / u).tolist() == t[:, 4].tolist()
    assert ((p.astype(np.float64) - 1.0) / float(u)).tolist() == t[:, 5].tolist()


def test_grad_ec_without_residual_is_the_table_wise_int8_path(oracle):
    """No residual kept: the same codes, scale and updated values as the embedding oracle's
    grad_quant_int8 + sparse_update on the tensor read as one table whose every row is touched."""
    rng = np.random.default_rng(21)
    n_rows, D = 37, 8
    g = (rng.standard_normal((n_rows, D)) * 1e-3).astype(np.float32)
    p = rng.standard_normal((n_rows, D)).astype(np.float32)
    p1 = p.copy()
    s, codes = oracle.mlp_grad_quant_ec(g, None, p1, 0.1)
    tuo = np.array([0, n_rows], np.int32)
    absmax = np.array([np.abs(g).max()], np.float32)
    gq, gs = oracle.grad_quant_int8(1, D, g, tuo, absmax)
    assert np.array_equal(gq, codes) and float(gs[0]) == s
    p2 = p.copy()
    oracle.sparse_update(p2, None, np.array([0, n_rows], np.int64), np.ones(1, np.float32),
                         np.arange(n_rows, dtype=np.int64), tuo, gq, gs, 0.1)
    assert np.array_equal(p1.view(np.uint32), p2.view(np.uint32))


def test_grad_ec_telescopes(oracle):
    """Error feedback's defining identity: over K steps the applied updates sum to lr * (sum of the true
    gradients + e_0 - e_K), i.e. nothing is lost but the last residual; and the residual stays within half a
    quantisation step."""
    rng = np.random.default_rng(22)
    n, K, lr = 500, 12, 0.05
    p0 = rng.standard_normal(n).astype(np.float32)
    p, e = p0.copy(), np.zeros(n, np.float32)
    gsum = np.zeros(n, np.float64)
    plain = p0.copy()  # INT8 without compensation, for contrast
    for k in range(K):
        g = (rng.standard_normal(n) * 10.0 ** rng.uniform(-4, -2)).astype(np.float32)
        g[::7] *= 0.01  # many values far below one step: they only get through thanks to the residual
        gsum += g
        s, codes = oracle.mlp_grad_quant_ec(g, e, p, lr)
        assert np.all(np.abs(e) <= 0.5 * s * (1 + 1e-5))
        oracle.mlp_grad_quant_ec(g, None, plain, lr)
    applied = p0.astype(np.float64) - p
    assert np.allclose(applied, lr * (gsum - e), rtol=0, atol=5e-6)
    # and the compensated run tracks the exact SGD trajectory more closely than the uncompensated one
    exact = p0 - lr * gsum
    assert np.abs(p - exact).sum() < 0.5 * np.abs(plain - exact).sum()


def test_grad_ec_sign_and_order_of_the_residual(oracle):
    """One element, two steps, by hand: g = 0.4 s then 0.4 s with the scale pinned by a second element at 127 s."""
    s = np.float32(2.0 ** -8)
    p = np.zeros(2, np.float32)
    e = np.zeros(2, np.float32)
    g = np.array([127 * s, 0.375 * s], np.float32)
    _, c1 = oracle.mlp_grad_quant_ec(g, e, p, 1.0)
    assert c1.tolist() == [127, 0] and e.tolist() == [0.0, 0.375 * s]
    _, c2 = oracle.mlp_grad_quant_ec(g, e, p, 1.0)
    assert c2.tolist() == [127, 1] and e.tolist() == [0.0, -0.25 * s]  # 0.75 s -> code 1, residual -0.25 s
    assert p.tolist() == [-254 * s, -1 * s]


# ---------------------------------------------------------------- the dense step with a straight-through weight
def _torch_ste_reference(bot_w, bot_b, top_w, top_b, bot_wq, top_wq, x, emb, y):
    t64 = lambda a: torch.tensor(np.asarray(a, np.float64), dtype=torch.float64, requires_grad=True)
    BW, BB, TW, TB = [list(map(t64, l)) for l in (bot_w, bot_b, top_w, top_b)]
    ste = lambda W, Wq: W + (torch.tensor(np.asarray(Wq, np.float64)) - W).detach()  # value Wq, gradient to W
    X = torch.tensor(np.asarray(x, np.float64))
    E = t64(emb)
    Y = torch.tensor(np.asarray(y, np.float64))
    h = X
    for W, Wq, b in zip(BW, bot_wq, BB):
        h = torch.relu(torch.nn.functional.linear(h, ste(W, Wq), b))
    B, T, D = E.shape
    Z = torch.cat([h[:, None, :], E], dim=1)
    G = torch.bmm(Z, Z.transpose(1, 2))
    li, lj = np.tril_indices(T + 1, k=-1)
    t = torch.cat([h, G[:, li, lj]], dim=1)
    for k, (W, Wq, b) in enumerate(zip(TW, top_wq, TB)):
        t = torch.nn.functional.linear(t, ste(W, Wq), b)
        if k + 1 < len(TW):
            t = torch.relu(t)
    loss = torch.nn.functional.binary_cross_entropy(torch.sigmoid(t[:, 0]), Y, reduction="mean")
    loss.backward()
    gr = lambda ps: [p.grad.numpy() for p in ps]
    return float(loss), E.grad.numpy(), gr(BW), gr(BB), gr(TW), gr(TB)


@pytest.mark.parametrize("bits", [0, 4])
def test_dense_step_ex_matches_torch_with_straight_through_weights(oracle, bits):
    T, D, B = 3, 16, 11
    bot_dims, bw, bb, top_dims, tw, tb = make_dense_model("small", T, D, seed=9)
    x, y = dense_batch(B, bot_dims[0], seed=9, k=1)
    emb = (np.random.default_rng(4).standard_normal((B, T, D)) * 0.3).astype(np.float32)
    f64 = lambda l: [np.ascontiguousarray(a, np.float64) for a in l]
    fq = (lambda l: [oracle.mlp_fake_quant(np.ascontiguousarray(a, np.float32), bits)[0] for a in l]) if bits else (lambda l: l)
    bwq, twq = fq(bw), fq(tw)
    if bits:
        assert any(not np.array_equal(a, b) for a, b in zip(bwq + twq, bw + tw))
    ref = _torch_ste_reference(bw, bb, tw, tb, bwq, twq, x, emb, y)
    BW, BB, TW, TB = f64(bw), f64(bb), f64(tw), f64(tb)
    keep = [a.copy() for a in BW + BB + TW + TB]
    loss, grad, (gbw, gbb, gtw, gtb) = oracle.dense_step_ex(bot_dims, BW, BB, top_dims, TW, TB, x, emb, y, 0.1,
                                                            bot_wf=f64(bwq), top_wf=f64(twq), apply_sgd=False,
                                                            want_grads=True)
    assert abs(loss - ref[0]) < 1e-12
    np.testing.assert_allclose(grad, ref[1], rtol=1e-10, atol=1e-14)
    for got, exp in zip(gbw + gbb + gtw + gtb, ref[2] + ref[3] + ref[4] + ref[5]):
        np.testing.assert_allclose(got, exp, rtol=1e-10, atol=1e-14)
    assert all(np.array_equal(a, b) for a, b in zip(BW + BB + TW + TB, keep))  # apply_sgd=False: untouched
    # with the step: master weights move by -lr * those gradients
    oracle.dense_step_ex(bot_dims, BW, BB, top_dims, TW, TB, x, emb, y, 0.1, bot_wf=f64(bwq), top_wf=f64(twq))
    for got, k0, g in zip(BW + BB + TW + TB, keep, gbw + gbb + gtw + gtb):
        np.testing.assert_allclose(got, k0 - 0.1 * g, rtol=1e-12, atol=1e-15)
