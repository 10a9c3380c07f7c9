"""Pins of the oracle's simulated data parallelism for the embedding tables (CPU only).

``oracle.SimulatedDP`` follows the appendix algorithm micro-batch by micro-batch with a dense integer buffer.
It is pinned against: the hand-worked example; the single step the other pins already fix (one simulated node);
``torch.sparse_coo_tensor(...).coalesce()`` of the micro-batches' integer gradients; a lossless case where the
group must equal ONE plain SGD step on the whole batch with the brute-force dense gradient; clipping under the
reused scale; a fresh buffer for every group.
Mistakes these catch: a block dropped or added twice, rows of one table landing in another, a per-block instead
of the first block's scale, a buffer that is not cleared, an update that averages or that touches other rows,
an update after the wrong micro-batch."""
import os

import numpy as np
import pytest
import torch

from gen import make_workload, split_batch, make_dense_model, dense_batch

GOLD = os.path.join(os.path.dirname(__file__), "golden")
U7 = np.float32(2.0 ** -7)


def _gold():
    mbs, buf, w, scale = {}, {}, {}, None
    with open(os.path.join(GOLD, "simulated_dp_hand_example.txt")) as f:
        for line in f:
            tok = line.split()
            if not tok or tok[0].startswith("#"):
                continue
            if tok[0] == "mb":
                mbs.setdefault(int(tok[1]), []).append((int(tok[2]), float(tok[3]), float(tok[4])))
            elif tok[0] == "buffer":
                buf[int(tok[1])] = (int(tok[2]), int(tok[3]), int(tok[4]))
            elif tok[0] == "scale":
                scale = float(tok[1])
            elif tok[0] == "weight":
                w[int(tok[1])] = (float(tok[2]), float(tok[3]))
    return mbs, buf, scale, w


def test_hand_example(oracle):
    mbs, buf, scale, w = _gold()
    W = np.ones((4, 2), np.float32)
    ro = np.array([0, 4], np.int64)
    sim = oracle.SimulatedDP(W, None, ro, np.ones(1, np.float32), simulated_nodes=2, lr=0.5)
    for k in sorted(mbs):
        idx = np.array([s[0] for s in mbs[k]], np.int64)
        off = np.arange(len(idx) + 1, dtype=np.int64)
        g = np.array([[[s[1], s[2]]] for s in mbs[k]], np.float32) * U7  # [B][T=1][D]
        ended = sim.micro_batch(k, len(idx), idx, off, np.ascontiguousarray(g))
        assert ended == (k == 1)
    assert sim.g_scale[0] == np.float32(scale) * U7
    for r in range(4):
        assert tuple(sim.buffer[r]) == buf[r][:2] and int(sim.touched[r]) == buf[r][2]
        assert W[r, 0] == np.float32(1.0) + np.float32(w[r][0]) * U7
        assert W[r, 1] == np.float32(1.0) + np.float32(w[r][1]) * U7


def _tiny(seed=77, B=64):
    wl = make_workload("tiny", B=B, seed=seed)
    return wl, wl.tables(threads=1)


def test_one_node_is_the_plain_quantised_step(oracle):
    wl, W0 = _tiny()
    idx, off = wl.batch(3)
    g = wl.grad_normal(3)
    ws = oracle.find_scale(W0, wl.row_offsets)
    Wa, Wb = W0.copy(), W0.copy()
    pa, pb = oracle.pack_int4(Wa, wl.row_offsets, ws), oracle.pack_int4(Wb, wl.row_offsets, ws)
    sim = oracle.SimulatedDP(Wa, pa, wl.row_offsets, ws, simulated_nodes=1, lr=0.1)
    assert sim.micro_batch(0, wl.B, idx, off, g)
    bw = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, g)
    gq, gs = oracle.grad_quant_int8(wl.T, wl.D, bw["values"], bw["table_uniq_offsets"], bw["g_absmax"])
    oracle.sparse_update(Wb, pb, wl.row_offsets, ws, bw["uniq_rows"], bw["table_uniq_offsets"], gq, gs, 0.1)
    assert np.array_equal(Wa.view(np.uint32), Wb.view(np.uint32)) and np.array_equal(pa, pb)
    assert not np.array_equal(Wa, W0)


@pytest.mark.parametrize("nodes", [2, 4, 8])
def test_buffer_is_the_coalesced_sum_of_the_blocks(oracle, nodes):
    wl, W = _tiny(seed=78)
    idx, off = wl.batch(0)
    g = wl.grad_normal(0)
    sim = oracle.SimulatedDP(W, None, wl.row_offsets, np.ones(wl.T, np.float32), simulated_nodes=nodes, lr=0.0)
    Bm = wl.B // nodes
    for k, (ik, ok) in enumerate(split_batch(idx, off, wl.T, wl.B, nodes)):
        sim.micro_batch(k, Bm, ik, ok, np.ascontiguousarray(g[k * Bm:(k + 1) * Bm]))
    assert len(sim.blocks) == nodes
    rows, vals = [], []
    for ur, tuo, gq in sim.blocks:
        for t in range(wl.T):
            rows.append(wl.row_offsets[t] + ur[tuo[t]:tuo[t + 1]])
            vals.append(gq[tuo[t]:tuo[t + 1]].astype(np.int64))
    rows, vals = np.concatenate(rows), np.concatenate(vals)
    sp = torch.sparse_coo_tensor(torch.from_numpy(rows)[None, :], torch.from_numpy(vals), (wl.R, wl.D)).coalesce()
    dense = sp.to_dense().numpy()
    assert np.array_equal(dense, sim.buffer.astype(np.int64))
    assert np.array_equal(np.flatnonzero(sim.touched), np.unique(rows))
    # every block used the FIRST block's scale
    ur0, tuo0, gq0 = sim.blocks[0]
    bw0 = oracle.embbag_bwd(wl.T, wl.D, Bm, *split_batch(idx, off, wl.T, wl.B, nodes)[0], np.ascontiguousarray(g[:Bm]))
    _, gs0 = oracle.grad_quant_int8(wl.T, wl.D, bw0["values"], bw0["table_uniq_offsets"], bw0["g_absmax"])
    assert np.array_equal(sim.g_scale, gs0)


def test_lossless_group_equals_one_plain_step_on_the_whole_batch(oracle):
    """Upstream gradients m * 2^-10 with small integers m, and one sample per micro-batch 0 and table that
    carries 127 * 2^-10: the scale is 2^-10 exactly, nothing clips (a row is hit by few samples), every code is the
    integer m-sum, and the group's update is w - lr * (whole-batch gradient), the dense gradient by brute force."""
    nodes, s = 4, np.float32(2.0 ** -10)
    wl, W = _tiny(seed=79, B=32)
    idx, off = wl.batch(1)
    rng = np.random.default_rng(5)
    m = rng.integers(-3, 4, size=(wl.B, wl.T, wl.D)).astype(np.float32)
    m[0, :, 0] = 127.0
    # keep the coalesced sums of micro-batch 0 inside the scale's range: the row of sample 0 gets no other sample there
    Bm = wl.B // nodes
    for t in range(wl.T):
        same = np.flatnonzero(idx[t * wl.B: t * wl.B + Bm] == idx[t * wl.B])
        m[same[1:], t, :] = 0.0
    g = np.ascontiguousarray(m * s)
    W0 = W.copy()
    sim = oracle.SimulatedDP(W, None, wl.row_offsets, np.ones(wl.T, np.float32), simulated_nodes=nodes, lr=0.25)
    for k, (ik, ok) in enumerate(split_batch(idx, off, wl.T, wl.B, nodes)):
        sim.micro_batch(k, Bm, ik, ok, np.ascontiguousarray(g[k * Bm:(k + 1) * Bm]))
    assert np.all(sim.g_scale == s)
    dense = np.zeros((wl.R, wl.D), np.float64)
    for t in range(wl.T):
        for b in range(wl.B):
            dense[wl.row_offsets[t] + idx[t * wl.B + b]] += g[b, t].astype(np.float64)
    expect = (W0.astype(np.float64) - 0.25 * dense).astype(np.float32)  # exact: dyadic, few bits
    assert np.array_equal(W, expect)
    assert np.array_equal(sim.buffer.astype(np.float64) * float(s), dense)


def test_reused_scale_clips_later_micro_batches(oracle):
    W = np.zeros((8, 4), np.float32)
    ro = np.array([0, 8], np.int64)
    sim = oracle.SimulatedDP(W, None, ro, np.ones(1, np.float32), simulated_nodes=2, lr=1.0)
    one = np.arange(2, dtype=np.int64)
    g0 = np.zeros((1, 1, 4), np.float32); g0[0, 0] = [1.0, -0.5, 0.25, 0.0]
    g1 = np.zeros((1, 1, 4), np.float32); g1[0, 0] = [4.0, -4.0, 0.5, 1.0 / 127.0]
    sim.micro_batch(0, 1, np.array([2], np.int64), one, g0)
    sim.micro_batch(1, 1, np.array([5], np.int64), one, g1)
    s = np.float32(1.0) / np.float32(127.0)
    assert sim.g_scale[0] == s
    assert sim.buffer[2].tolist() == [127, -64, 32, 0]     # -63.5 -> -64 and 31.75 -> 32 (nearest)
    assert sim.buffer[5].tolist() == [127, -128, 64, 1]    # clipped at both ends; 63.5 -> 64 (half to even)
    assert W[5].tolist() == [float(-(s * np.float32(c))) for c in (127, -128, 64, 1)]


def test_every_group_starts_from_a_cleared_buffer(oracle):
    wl, W = _tiny(seed=80)
    nodes, Bm = 2, wl.B // 2
    ones = np.ones(wl.T, np.float32)
    batches = [(wl.batch(k), wl.grad_normal(k)) for k in range(2)]
    Wa = W.copy()
    sim = oracle.SimulatedDP(Wa, None, wl.row_offsets, ones, simulated_nodes=nodes, lr=0.05)
    j = 0
    for (idx, off), g in batches:
        for k, (ik, ok) in enumerate(split_batch(idx, off, wl.T, wl.B, nodes)):
            sim.micro_batch(j, Bm, ik, ok, np.ascontiguousarray(g[k * Bm:(k + 1) * Bm]))
            j += 1
    # the same two groups, each with an object of its own
    Wb = W.copy()
    for (idx, off), g in batches:
        fresh = oracle.SimulatedDP(Wb, None, wl.row_offsets, ones, simulated_nodes=nodes, lr=0.05)
        for k, (ik, ok) in enumerate(split_batch(idx, off, wl.T, wl.B, nodes)):
            fresh.micro_batch(k, Bm, ik, ok, np.ascontiguousarray(g[k * Bm:(k + 1) * Bm]))
    assert np.array_equal(Wa.view(np.uint32), Wb.view(np.uint32))
    assert np.array_equal(sim.buffer, fresh.buffer)


# ---------------------------------------------------------------- the MLPs' gradient buffers
@pytest.mark.parametrize("nodes", [2, 4])
def test_dense_group_equals_one_plain_step_with_lr_times_nodes(oracle, nodes):
    """Micro-batches of equal size, mean loss each: the sum of their gradients is `nodes` times the gradient of
    the whole batch's mean loss, so a group with step size lr must equal ONE plain step (the routine pinned against
    torch autograd) on the whole batch with step size lr * nodes; the embedding gradients are the whole batch's
    times `nodes`, slice by slice; the mean of the micro-batch losses is the whole batch's loss."""
    T, D, B, lr = 3, 16, 48, 0.05
    bot_dims, bw, bb, top_dims, tw, tb = make_dense_model("small", T, D, seed=31)
    x, y = dense_batch(B, bot_dims[0], seed=31, k=0)
    emb = (np.random.default_rng(7).standard_normal((B, T, D)) * 0.25).astype(np.float32)
    f64 = lambda l: [np.ascontiguousarray(a, np.float64) for a in l]
    A, Bp = (f64(bw), f64(bb), f64(tw), f64(tb)), (f64(bw), f64(bb), f64(tw), f64(tb))
    sim = oracle.SimulatedDPDense(bot_dims, A[0], A[1], top_dims, A[2], A[3], simulated_nodes=nodes, lr=lr)
    Bm = B // nodes
    losses, gemb = [], []
    for k in range(nodes):
        sl = slice(k * Bm, (k + 1) * Bm)
        before = [a.copy() for a in A[2]]
        loss, ge, ended = sim.micro_batch(k, x[sl], emb[sl], y[sl])
        assert ended == (k == nodes - 1)
        if not ended:
            assert all(np.array_equal(a, b) for a, b in zip(A[2], before))  # weights untouched inside a group
        losses.append(loss)
        gemb.append(ge)
    loss_w, ge_w = oracle.dense_step(bot_dims, Bp[0], Bp[1], top_dims, Bp[2], Bp[3], x, emb, y, lr * nodes)
    assert abs(np.mean(losses) - loss_w) <= 1e-12 * abs(loss_w)
    assert np.allclose(np.concatenate(gemb), ge_w * nodes, rtol=1e-10, atol=1e-14)
    for got, exp in zip(A, Bp):
        for g, e in zip(got, exp):
            assert np.allclose(g, e, rtol=1e-10, atol=1e-13)
    assert not np.allclose(A[2][0], np.asarray(tw[0], np.float64))


def test_dense_buffers_are_cleared_between_groups(oracle):
    T, D, B, lr, nodes = 3, 16, 24, 0.05, 2
    bot_dims, bw, bb, top_dims, tw, tb = make_dense_model("small", T, D, seed=32)
    f64 = lambda l: [np.ascontiguousarray(a, np.float64) for a in l]
    A, Bp = (f64(bw), f64(bb), f64(tw), f64(tb)), (f64(bw), f64(bb), f64(tw), f64(tb))
    sim = oracle.SimulatedDPDense(bot_dims, A[0], A[1], top_dims, A[2], A[3], simulated_nodes=nodes, lr=lr)
    rng = np.random.default_rng(9)
    j = 0
    for grp in range(2):
        x, y = dense_batch(B, bot_dims[0], seed=32, k=grp)
        emb = (rng.standard_normal((B, T, D)) * 0.25).astype(np.float32)
        fresh = oracle.SimulatedDPDense(bot_dims, Bp[0], Bp[1], top_dims, Bp[2], Bp[3], simulated_nodes=nodes, lr=lr)
        for k in range(nodes):
            sl = slice(k * (B // nodes), (k + 1) * (B // nodes))
            sim.micro_batch(j, x[sl], emb[sl], y[sl])
            fresh.micro_batch(k, x[sl], emb[sl], y[sl])
            j += 1
    for got, exp in zip(A, Bp):
        for g, e in zip(got, exp):
            assert np.array_equal(g, e)
