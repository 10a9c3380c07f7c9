"""GPU parity of simulated data parallelism for the embedding tables: micro-batch backward, INT8 codes with
the first micro-batch's scale, dqrm_sparse_merge, dqrm_sparse_update_sums, against oracle.SimulatedDP.
Everything is integer or bit-comparable: exact equality throughout."""
import sys

import numpy as np
import pytest

from gen import make_workload, split_batch
from helpers import GpuRun, assert_exact

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[simdp] {msg}", flush=True)
    sys.stdout.flush()


class Group:
    """Device-side driver of one group of micro-batches through the C ABI."""

    def __init__(self, wl, W, nodes, Bm, N_cap, with_packed=True):
        import torch
        import paper_2410_20046_amd as dq

        self.torch, self.dq, self.wl, self.nodes, self.Bm = torch, dq, wl, nodes, Bm
        self.run = GpuRun(wl.row_offsets, wl.D, W, Bm, N_cap, with_packed=with_packed, want_codes=False)
        dev = self.run.dev
        self.cap_total = nodes * N_cap
        self.m_rows = torch.empty(max(self.cap_total, 1), dtype=torch.int64, device=dev)
        self.m_tuo = torch.empty(wl.T + 1, dtype=torch.int32, device=dev)
        self.m_nu = torch.zeros(1, dtype=torch.int32, device=dev)
        self.m_sums = torch.empty((max(self.cap_total, 1), wl.D), dtype=torch.int32, device=dev)
        nbytes = dq.dqrm_sparse_merge_workspace_bytes(wl.T, wl.D, nodes, max(self.cap_total, 1))
        assert nbytes > 0
        self.m_ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def micro_batches(self, parts, grads):
        """Backward + quantisation of every micro-batch; returns the device blocks and their host copies."""
        run, b, dq = self.run, self.run.bufs, self.dq
        blocks, host = [], []
        absmax0 = None
        for k, ((ik, ok), gk) in enumerate(zip(parts, grads)):
            run.N = len(ik)
            run.upload_batch(ik, ok, np.ascontiguousarray(gk))
            g = run.bwd()
            if absmax0 is None:
                absmax0 = b.g_absmax.clone()
            dq.dqrm_grad_quant_int8(run.T, run.D, b.cap, b.values, b.table_uniq_offsets, absmax0, b.gq, b.g_scale)
            blocks.append((b.uniq_rows.clone(), b.table_uniq_offsets.clone(), b.gq.clone()))
            host.append((g["uniq_rows"], g["table_uniq_offsets"], b.gq.cpu().numpy()[: g["U"]], g["values"]))
        self.g_scale = b.g_scale.clone()
        return blocks, host

    def merge(self, blocks):
        self.dq.dqrm_sparse_merge(self.run.tables, blocks, self.m_rows, self.m_tuo, self.m_nu, self.m_sums, self.m_ws)
        U = int(self.m_nu.cpu().item())
        return U, self.m_rows.cpu().numpy()[:U], self.m_tuo.cpu().numpy(), self.m_sums.cpu().numpy()[:U]

    def update(self, lr):
        self.dq.dqrm_sparse_update_sums(self.run.tables, self.cap_total, self.m_rows, self.m_tuo, self.m_sums,
                                        self.g_scale, lr)


def _check_group(oracle, wl, W, Wo, po, s_w, grp, idx, off, grad, nodes, lr, j0, sim, what):
    Bm = wl.B // nodes
    parts = split_batch(idx, off, wl.T, wl.B, nodes)
    grads = [grad[k * Bm:(k + 1) * Bm] for k in range(nodes)]
    for k in range(nodes):
        sim.micro_batch(j0 + k, Bm, parts[k][0], parts[k][1], np.ascontiguousarray(grads[k]))
    blocks, host = grp.micro_batches(parts, grads)
    for k, ((ur, tuo, gq, _), (our, otuo, ogq)) in enumerate(zip(host, sim.blocks)):
        assert_exact(ur, our, f"{what} block {k} uniq_rows")
        assert_exact(tuo, otuo, f"{what} block {k} table_uniq_offsets")
        assert_exact(gq, ogq, f"{what} block {k} INT8 codes")
    assert_exact(grp.g_scale.cpu().numpy().view(np.uint32), sim.g_scale.view(np.uint32), what + " g_scale bits")
    U, rows, tuo, sums = grp.merge(blocks)
    # the merged list is the oracle's dense buffer, sparse: rows ascending inside each table, nothing else touched
    touched = np.flatnonzero(sim.touched)
    glob = np.concatenate([wl.row_offsets[t] + rows[tuo[t]:tuo[t + 1]] for t in range(wl.T)]) if U else np.empty(0, np.int64)
    assert tuo[0] == 0 and tuo[wl.T] == U
    assert_exact(glob, touched, what + " merged rows")
    assert_exact(sums, sim.buffer[touched], what + " merged integer sums")
    grp.update(lr)
    assert_exact(grp.run.master_np().view(np.uint32), Wo.view(np.uint32), what + " master bits after the group")
    if po is not None:
        assert_exact(grp.run.packed_np(), po, what + " packed after the group")
    code, tb, val = grp.run.status()
    assert code == 0, (what, "device status", code, tb, val)


def _setup(oracle, wl, nodes, N_cap=None):
    W = wl.tables(threads=1) if wl.R < 10_000_000 else wl.tables()
    Wo = W.copy()
    s_w = oracle.find_scale(Wo, wl.row_offsets)
    po = oracle.pack_int4(Wo, wl.row_offsets, s_w)
    Bm = wl.B // nodes
    grp = Group(wl, W, nodes, Bm, N_cap if N_cap is not None else wl.T * Bm)
    grp.run.find_scale()
    grp.run.pack()
    return W, Wo, po, s_w, grp


@pytest.mark.parametrize("nodes", [1, 2, 4, 8])
def test_groups_tiny(oracle, nodes):
    wl = make_workload("tiny", seed=1201)
    _say(f"tiny, {nodes} simulated nodes, two groups in a row")
    W, Wo, po, s_w, grp = _setup(oracle, wl, nodes)
    sim = oracle.SimulatedDP(Wo, po, wl.row_offsets, s_w, simulated_nodes=nodes, lr=0.1)
    for step in range(2):  # the second group meets the first one's leftovers in every buffer
        idx, off = wl.batch(step)
        _check_group(oracle, wl, W, Wo, po, s_w, grp, idx, off, wl.grad_normal(step), nodes, 0.1, step * nodes, sim,
                     f"tiny n={nodes} group {step}")


@pytest.mark.parametrize("D", [8, 24, 64, 128])
def test_dims_and_ragged_bags(oracle, D):
    wl = make_workload("tiny", D=D, B=96, seed=1202 + D)
    nodes = 4
    _say(f"ragged bags, D={D}, {nodes} nodes")
    idx, off = wl.batch(0, pooling="ragged", max_len=5)
    W, Wo, po, s_w, grp = _setup(oracle, wl, nodes, N_cap=len(idx))
    sim = oracle.SimulatedDP(Wo, po, wl.row_offsets, s_w, simulated_nodes=nodes, lr=0.05)
    _check_group(oracle, wl, W, Wo, po, s_w, grp, idx, off, wl.grad_normal(0), nodes, 0.05, 0, sim, f"ragged D={D}")


def test_hot_rows_shared_by_every_block_and_an_empty_block(oracle):
    """Zipf indices on a small table: most rows occur in every micro-batch; micro-batch 2 has only empty bags."""
    wl = make_workload("single", B=1024, fixed_card=300, rows=300, seed=1203)
    nodes = 4
    _say("hot rows + an empty micro-batch")
    idx, off = wl.batch(0)
    Bm = wl.B // nodes
    lens = np.diff(off).copy()
    lens[2 * Bm:3 * Bm] = 0
    keep = np.ones(len(idx), bool)
    keep[2 * Bm:3 * Bm] = False
    idx, off = np.ascontiguousarray(idx[keep]), np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    W, Wo, po, s_w, grp = _setup(oracle, wl, nodes)
    sim = oracle.SimulatedDP(Wo, po, wl.row_offsets, s_w, simulated_nodes=nodes, lr=0.1)
    _check_group(oracle, wl, W, Wo, po, s_w, grp, idx, off, wl.grad_normal(0), nodes, 0.1, 0, sim, "hot rows")
    assert sim.blocks[2][0].size == 0


def test_later_micro_batches_clip_under_the_first_scale(oracle):
    wl = make_workload("tiny", seed=1204)
    nodes = 2
    _say("clipping under the reused scale")
    idx, off = wl.batch(0)
    grad = wl.grad_normal(0).copy()
    grad[wl.B // 2:] *= np.float32(5.0)  # the second micro-batch exceeds the first one's range
    W, Wo, po, s_w, grp = _setup(oracle, wl, nodes)
    sim = oracle.SimulatedDP(Wo, po, wl.row_offsets, s_w, simulated_nodes=nodes, lr=0.1)
    _check_group(oracle, wl, W, Wo, po, s_w, grp, idx, off, grad, nodes, 0.1, 0, sim, "clipping")
    assert (np.abs(sim.blocks[1][2].astype(np.int32)) >= 127).sum() > 10


def test_bad_blocks_are_reported_not_used(oracle):
    import torch

    wl = make_workload("tiny", seed=1205)
    nodes = 2
    _say("a block with decreasing offsets; outputs too small")
    idx, off = wl.batch(0)
    W, Wo, po, s_w, grp = _setup(oracle, wl, nodes)
    Bm = wl.B // nodes
    parts = split_batch(idx, off, wl.T, wl.B, nodes)
    grad = wl.grad_normal(0)
    blocks, host = grp.micro_batches(parts, [grad[:Bm], grad[Bm:]])
    bad_tuo = blocks[1][1].clone()
    bad_tuo[2] = bad_tuo[1] - 1  # table 1 ends before it starts; table 2 then starts before table 1's begin
    U, rows, tuo, sums = grp.merge([blocks[0], (blocks[1][0], bad_tuo, blocks[1][2])])
    code, tb, val = grp.run.status()
    assert code == grp.dq.ERR_BAD_OFFSETS, (code, tb, val)
    # the outputs cannot hold both blocks
    small_rows = torch.empty(host[0][0].size + 3, dtype=torch.int64, device=grp.run.dev)
    small_sums = torch.empty((host[0][0].size + 3, wl.D), dtype=torch.int32, device=grp.run.dev)
    grp.dq.dqrm_sparse_merge(grp.run.tables, blocks, small_rows, grp.m_tuo, grp.m_nu, small_sums, grp.m_ws)
    code, tb, val = grp.run.status()
    assert code == grp.dq.ERR_CAPACITY, (code, tb, val)
    assert int(grp.m_nu.cpu().item()) <= host[0][0].size + 3
    # and a good call afterwards is clean
    U, rows, tuo, sums = grp.merge(blocks)
    assert grp.run.status()[0] == 0
    assert U == np.unique(np.concatenate([wl.row_offsets[t] + h[0][h[1][t]:h[1][t + 1]] for h in host for t in range(wl.T)])).size


def test_merge_of_random_blocks(oracle):
    """dqrm_sparse_merge alone on blocks built directly (random ascending rows per table, random codes): empty
    tables, tables present in one block only, rows shared by all blocks, single rows, and a table whose union is
    far larger than one workgroup's sort would hold; against the oracle's dense buffer."""
    import ctypes as C
    import torch
    import paper_2410_20046_amd as dq

    dev = torch.device("cuda:0")
    rng = np.random.default_rng(4242)
    for case in range(24):
        T = int(rng.integers(1, 9))
        D = int(rng.choice([8, 16, 40, 64]))
        n = int(rng.integers(1, 9))
        cards = rng.choice([1, 2, 7, 100, 5000, 200000], size=T).astype(np.int64)
        if case == 0:
            T, n, cards = 3, 4, np.array([5, 400000, 64], np.int64)  # 4 x 30000 rows of one table
        ro = np.concatenate([[0], np.cumsum(cards)]).astype(np.int64)
        R = int(ro[-1])
        _say(f"random blocks case {case}: T={T} D={D} n={n} cards={cards.tolist()}")
        blocks_h = []
        for k in range(n):
            rows, tuo = [], [0]
            for t in range(T):
                c = int(cards[t])
                want = 30000 if (case == 0 and t == 1) else int(rng.choice([0, 1, 3, min(c, 50), min(c, 700)]))
                r = np.sort(rng.choice(c, size=min(want, c), replace=False)).astype(np.int64)
                rows.append(r)
                tuo.append(tuo[-1] + len(r))
            rows = np.concatenate(rows) if rows else np.empty(0, np.int64)
            gq = rng.integers(-128, 128, size=(max(len(rows), 1), D)).astype(np.int8)
            blocks_h.append((rows, np.array(tuo, np.int32), gq))
        buffer = np.zeros((R, D), np.int32)
        touched = np.zeros(R, np.uint8)
        for rows, tuo, gq in blocks_h:
            oracle.lib().oracle_simdp_accumulate(
                C.c_int(T), C.c_int(D), ro.ctypes.data_as(C.POINTER(C.c_int64)), rows.ctypes.data_as(C.POINTER(C.c_int64)),
                tuo.ctypes.data_as(C.POINTER(C.c_int32)), gq.ctypes.data_as(C.POINTER(C.c_int8)),
                buffer.ctypes.data_as(C.POINTER(C.c_int32)), touched.ctypes.data_as(C.POINTER(C.c_uint8)))
        master = torch.zeros((R, D), dtype=torch.float32, device=dev)
        tables = dq.Tables(ro, D, master, None)
        blocks_d = []
        for rows, tuo, gq in blocks_h:
            cap = max(len(rows), 1) + int(rng.integers(0, 5))  # some slack behind the rows
            rd = torch.zeros(cap, dtype=torch.int64, device=dev)
            rd[: len(rows)] = torch.from_numpy(rows).to(dev)
            gd = torch.zeros((cap, D), dtype=torch.int8, device=dev)
            gd[: gq.shape[0]] = torch.from_numpy(gq).to(dev)
            blocks_d.append((rd, torch.from_numpy(tuo).to(dev), gd))
        total = sum(len(b[0]) for b in blocks_h)
        cap_total = max(total, 1)
        m_rows = torch.full((cap_total,), -7, dtype=torch.int64, device=dev)
        m_tuo = torch.empty(T + 1, dtype=torch.int32, device=dev)
        m_nu = torch.zeros(1, dtype=torch.int32, device=dev)
        m_sums = torch.zeros((cap_total, D), dtype=torch.int32, device=dev)
        ws = torch.empty(dq.dqrm_sparse_merge_workspace_bytes(T, D, n, cap_total), dtype=torch.uint8, device=dev)
        dq.dqrm_sparse_merge(tables, blocks_d, m_rows, m_tuo, m_nu, m_sums, ws)
        code, tb, val = dq.dqrm_check_status()
        assert code == 0, (case, code, tb, val)
        U = int(m_nu.cpu().item())
        tuo_g, rows_g, sums_g = m_tuo.cpu().numpy(), m_rows.cpu().numpy()[:U], m_sums.cpu().numpy()[:U]
        want = np.flatnonzero(touched)
        assert U == want.size and tuo_g[0] == 0 and tuo_g[T] == U, (case, U, want.size)
        glob = np.concatenate([ro[t] + rows_g[tuo_g[t]:tuo_g[t + 1]] for t in range(T)]) if U else np.empty(0, np.int64)
        assert_exact(glob, want, f"case {case} merged rows")
        assert_exact(sums_g, buffer[want], f"case {case} merged sums")


def test_terabyte_full_size_eight_nodes(oracle):
    """The benchmark workload at full size, its batch of 8192 split over 8 simulated nodes."""
    wl = make_workload("terabyte")
    nodes = 8
    _say(f"terabyte-shaped full size, {nodes} simulated nodes")
    W, Wo, po, s_w, grp = _setup(oracle, wl, nodes)
    sim = oracle.SimulatedDP(Wo, po, wl.row_offsets, s_w, simulated_nodes=nodes, lr=0.1)
    idx, off = wl.batch(0)
    _check_group(oracle, wl, W, Wo, po, s_w, grp, idx, off, wl.grad_normal(0), nodes, 0.1, 0, sim, "terabyte n=8")


@pytest.mark.parametrize("D,nodes,ragged", [(64, 8, False), (16, 4, True), (24, 3, True)])
def test_micro_batches_in_one_launch_each(oracle, D, nodes, ragged):
    """dqrm_dedupe_multi -> dqrm_segment_sum_multi -> dqrm_grad_quant_int8_multi over the micro-batches of a group ==
    the oracle's backward and quantisation of each micro-batch (values and maxima bit for bit, codes and index
    outputs exactly), with the first micro-batch's maxima for every block; one batch asks for no maxima."""
    import torch
    import paper_2410_20046_amd as dq
    from gen import Workload

    cards = np.array([9, 700, 120000, 33, 5000], np.int64)
    wl = Workload(name="multi", T=5, D=D, B=384 * nodes, alpha=1.1, seed=600 + D, cards=cards)
    Bm = wl.B // nodes
    idx, off = wl.batch(0, pooling="ragged", max_len=4) if ragged else wl.batch(0)
    grad = wl.grad_normal(0)
    parts = split_batch(idx, off, wl.T, wl.B, nodes)
    dev = torch.device("cuda:0")
    W = np.zeros((wl.R, wl.D), np.float32)
    tables = dq.Tables(wl.row_offsets, wl.D, torch.from_numpy(W).to(dev), None)
    cap = max(len(i) for i, _ in parts)
    bufs = [dq.StepBuffers(wl.T, wl.D, Bm, cap, dev) for _ in range(nodes)]
    di = [torch.from_numpy(i).to(dev) for i, _ in parts]
    do = [torch.from_numpy(o).to(dev) for _, o in parts]
    dg = [torch.from_numpy(np.ascontiguousarray(grad[k * Bm:(k + 1) * Bm])).to(dev) for k in range(nodes)]
    _say(f"multi launches: D={D}, {nodes} micro-batches of {Bm}, up to {cap} lookups")
    dq.dqrm_dedupe_multi(tables, Bm, [(di[k], do[k], b.sorted_pos, b.uniq_rows, b.seg_offsets, b.table_uniq_offsets,
                                       b.num_unique, b.workspace) for k, b in enumerate(bufs)])
    skip = nodes - 1  # this micro-batch asks for no maxima
    for b in bufs:
        b.g_absmax.fill_(-1.0)
    dq.dqrm_segment_sum_multi(tables, Bm, [(di[k].numel(), dg[k], b.values, None if k == skip else b.g_absmax, b.workspace)
                                           for k, b in enumerate(bufs)])
    dq.dqrm_grad_quant_int8_multi(wl.T, wl.D, [(b.values, b.table_uniq_offsets, bufs[0].g_absmax, b.gq, b.g_scale)
                                               for b in bufs])
    code, tb, val = dq.dqrm_check_status()
    assert code == 0, (code, tb, val)
    absmax0 = None
    for k, b in enumerate(bufs):
        o = oracle.embbag_bwd(wl.T, wl.D, Bm, parts[k][0], parts[k][1], np.ascontiguousarray(grad[k * Bm:(k + 1) * Bm]))
        U = int(b.num_unique.cpu().item())
        what = f"multi D={D} micro-batch {k}"
        assert U == len(o["uniq_rows"]), what
        assert_exact(b.uniq_rows.cpu().numpy()[:U], o["uniq_rows"], what + " uniq_rows")
        assert_exact(b.table_uniq_offsets.cpu().numpy(), o["table_uniq_offsets"], what + " table_uniq_offsets")
        assert_exact(b.values.cpu().numpy()[:U].view(np.uint32), o["values"].view(np.uint32), what + " values bits")
        if k == skip:
            assert (b.g_absmax.cpu().numpy() == -1.0).all(), what + ": maxima written though not asked for"
        else:
            assert_exact(b.g_absmax.cpu().numpy().view(np.uint32), o["g_absmax"].view(np.uint32), what + " g_absmax bits")
        if absmax0 is None:
            absmax0 = o["g_absmax"]
        ogq, ogs = oracle.grad_quant_int8(wl.T, wl.D, o["values"], o["table_uniq_offsets"], absmax0)
        assert_exact(b.gq.cpu().numpy()[:U], ogq, what + " INT8 codes")
        assert_exact(b.g_scale.cpu().numpy().view(np.uint32), ogs.view(np.uint32), what + " g_scale bits")
