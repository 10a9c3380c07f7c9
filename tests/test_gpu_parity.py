"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Bit-exact on codes / indices / offsets / packed bytes; floats to
|a-b| <= 1e-6 + 1e-5*|b| (and, because both sides use the same documented summation order and
one rounding per operation, the float outputs are also expected to agree bit for bit)."""
import numpy as np
import pytest

from gen import make_workload, Workload
from helpers import GpuRun, assert_exact, assert_float_close, compare_bwd, full_step_parity

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


# --------------------------------------------------------------------------
# the benchmark configurations
# --------------------------------------------------------------------------
@pytest.mark.parametrize("grad", ["dyadic", "normal"])
def test_config_tiny(oracle, grad):
    wl = make_workload("tiny")
    _say(f"tiny grad={grad}")
    W = wl.tables(threads=1)
    idx, off = wl.batch(0)
    g = wl.grad_dyadic(0) if grad == "dyadic" else wl.grad_normal(0)
    full_step_parity(oracle, wl, W, idx, off, g, what=f"tiny/{grad}")


def test_config_single_table(oracle):
    wl = make_workload("single")
    _say("single table 1M x 16, batch 2048, Zipf 1.05")
    W = wl.tables()
    idx, off = wl.batch(0)
    full_step_parity(oracle, wl, W, idx, off, wl.grad_normal(0), what="single")


def test_config_kaggle_full_size(oracle):
    wl = make_workload("kaggle")
    _say(f"kaggle-shaped full size: R={wl.R}")
    W = wl.tables()
    idx, off = wl.batch(0)
    full_step_parity(oracle, wl, W, idx, off, wl.grad_normal(0), what="kaggle")


def test_config_terabyte_full_size(oracle):
    """The benchmark workload at full size through the five-call path (dqrm_embbag_bwd, dqrm_grad_quant_int8,
    dqrm_sparse_update).  The launch sequence bench.py times is checked by test_gpu_bench_path.py."""
    wl = make_workload("terabyte")
    _say(f"terabyte-shaped full size: R={wl.R} ({wl.R * wl.D * 4 / 1e9:.2f} GB fp32)")
    W = wl.tables()
    idx, off = wl.batch(0)
    run = full_step_parity(oracle, wl, W, idx, off, wl.grad_normal(0), what="terabyte")
    del run


# --------------------------------------------------------------------------
# shapes that span several tiles, ragged tails, degenerate cases
# --------------------------------------------------------------------------
@pytest.mark.parametrize("D", [8, 16, 24, 64, 128, 256])
def test_dims_ragged_bags(oracle, D):
    """every lane-group width, bags of 0..5 lookups (empty bags included), a stale weight scale."""
    wl = make_workload("tiny", T=5, D=D, B=333, fixed_card=211, rows=5 * 211)
    wl.seed += D
    _say(f"ragged D={D}")
    W = wl.tables(threads=1)
    idx, off = wl.batch(1, pooling="ragged", max_len=5)
    full_step_parity(oracle, wl, W, idx, off, wl.grad_normal(1), stale=0.5, what=f"ragged D={D}")


@pytest.mark.parametrize("T,D,B", [(100, 16, 48), (1024, 8, 16)])
def test_many_tables(oracle, T, D, B):
    """More tables than a forward tile holds (32), up to the limit of 1024: several table tiles per sample tile in the
    forward, a sorting workgroup per table, per-table lists and maxima of the backward at their largest."""
    import paper_2410_20046_amd as dq

    assert T <= dq.MAX_TABLES
    rng = np.random.default_rng(T)
    cards = rng.integers(1, 400, size=T).astype(np.int64)
    wl = Workload(name=f"tables{T}", T=T, D=D, B=B, alpha=1.05, seed=900 + T, cards=cards)
    idx, off = wl.batch(0, pooling="ragged", max_len=3)
    _say(f"{T} tables: {len(idx)} lookups")
    full_step_parity(oracle, wl, wl.tables(threads=1), idx, off, wl.grad_normal(0), stale=0.7, what=f"tables{T}")


@pytest.mark.parametrize("L", [20, 40])
def test_pooling_factor(oracle, L):
    """Every bag holds L lookups.  A forward tile (16 samples x 8 tables) then has 2560 lookups (their row
    offsets are staged in LDS, 4096 fit) or 5120 (they are not: one lookup at a time); packed and master mode,
    debug codes on."""
    cards = np.array([7, 900, 50000, 33, 4000, 120, 60000, 15], np.int64)
    wl = Workload(name=f"pool{L}", T=8, D=16, B=64, alpha=1.05, seed=300 + L, cards=cards)
    idx, off = wl.batch(0, pooling="fixed", max_len=L)
    assert len(idx) == 8 * 64 * L
    _say(f"pooling factor {L}: {len(idx)} lookups")
    full_step_parity(oracle, wl, wl.tables(threads=1), idx, off, wl.grad_normal(0), what=f"pool{L}")


@pytest.mark.parametrize("B,L", [(8192, 8), (2500, 7)])
def test_large_tables(oracle, B, L):
    """More lookups per table than one workgroup sorts in LDS (16384): pooling factor 8 at batch 8192 = 65536
    lookups in every table (four full tiles), and 17500 (one full tile and a short one).  Tiny tables (every row
    hot: segments of thousands of lookups across tile borders) next to large ones (mostly singles)."""
    cards = np.array([7, 50000, 2000000, 33], np.int64)
    wl = Workload(name=f"large{B}x{L}", T=4, D=64, B=B, alpha=1.1, seed=500 + L, cards=cards)
    idx, off = wl.batch(0, pooling="fixed", max_len=L)
    assert len(idx) == 4 * B * L
    _say(f"large tables: {B * L} lookups per table")
    full_step_parity(oracle, wl, wl.tables(threads=1), idx, off, wl.grad_normal(0), what=f"large{B}x{L}")


@pytest.mark.parametrize("D", [8, 24, 32, 40, 48, 56, 72, 96, 136, 200, 256])
def test_hot_rows_at_every_row_width(oracle, D):
    """Segments of hundreds of lookups (many chunks, the combine of parked chunk sums) at every lane-group width and at
    widths that are not a power of two; rows narrower than a wave share the wave in the combine, wider ones loop."""
    rng = np.random.default_rng(D)
    cards = np.concatenate([rng.integers(2, 40, size=4), [3000 + D, 250000]]).astype(np.int64)
    B = int(rng.integers(1200, 2600))
    wl = Workload(name=f"hot{D}", T=len(cards), D=D, B=B, alpha=1.15, seed=1000 + D, cards=cards)
    idx, off = wl.batch(0, pooling="ragged", max_len=3)
    _say(f"hot rows D={D}: batch {B}, {len(idx)} lookups")
    full_step_parity(oracle, wl, wl.tables(threads=1), idx, off, wl.grad_normal(0), what=f"hot D={D}")


def test_hot_segments_long_chunks(oracle):
    """tiny tables: segments of several hundred to several thousand lookups (many chunks per segment,
    the last-arrival combine), next to a table with no duplicates at all."""
    cards = np.array([3, 1, 17, 5000, 40], np.int64)
    wl = Workload(name="hot", T=5, D=64, B=4096, alpha=1.2, seed=77, cards=cards)
    _say("hot segments")
    W = wl.tables(threads=1)
    idx, off = wl.batch(0)
    run = full_step_parity(oracle, wl, W, idx, off, wl.grad_normal(0), what="hot")
    # the same call again on the same workspace: the self-resetting counters must be ready
    g1 = run.bwd()
    o = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, wl.grad_normal(0))
    compare_bwd(g1, o, "hot/second call")
    assert_exact(g1["values"].view(np.uint32), o["values"].view(np.uint32), "hot/second call values bits")


def test_max_table_lookups(oracle):
    """a table that receives exactly the maximum number of lookups a batch may bring to one table (65536: four
    tiles of the in-LDS sort, merged by the large-table path), with bags of two, next to an empty table (no
    lookups) and a small one."""
    import paper_2410_20046_amd as dq

    B = dq.MAX_TABLE_LOOKUPS // 2
    cards = np.array([100000, 50, 9], np.int64)
    wl = Workload(name="cap", T=3, D=16, B=B, alpha=1.05, seed=5, cards=cards)
    rng = np.random.default_rng(3)
    lens = np.concatenate([np.full(B, 2), np.zeros(B, np.int64), (np.arange(B) % 3 == 0).astype(np.int64)])
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = np.concatenate([rng.integers(0, 100000, 2 * B), rng.integers(0, 9, int(lens[2 * B:].sum()))]).astype(np.int64)
    _say(f"capacity case N={len(idx)}")
    W = wl.tables(threads=1)
    full_step_parity(oracle, wl, W, idx, off, wl.grad_dyadic(0), what="cap")


def test_zero_lookups_and_single_table(oracle):
    wl = make_workload("tiny", T=1, B=7, fixed_card=5, rows=5)
    W = wl.tables(threads=1)
    off = np.zeros(wl.T * wl.B + 1, np.int64)
    idx = np.zeros(0, np.int64)
    _say("empty batch")
    full_step_parity(oracle, wl, W, idx, off, wl.grad_normal(0), what="empty")


def test_all_zero_gradient_and_all_zero_table(oracle):
    """the scale floor: an all-zero table and an all-zero gradient give all-zero codes."""
    wl = make_workload("tiny")
    W = wl.tables(threads=1)
    W[wl.row_offsets[1]:wl.row_offsets[2]] = 0.0
    g = wl.grad_normal(0)
    g[:, 2, :] = 0.0
    idx, off = wl.batch(2)
    _say("zero table / zero gradient")
    run = full_step_parity(oracle, wl, W, idx, off, g, what="zeros")
    assert run.tables.w_scale.cpu().numpy()[1] == np.float32(1e-8)
    assert run.bufs.g_scale.cpu().numpy()[2] == np.float32(1e-8)


# --------------------------------------------------------------------------
# properties that hold at any size (checked on the benchmark-shaped dimension)
# --------------------------------------------------------------------------
def test_dyadic_integer_closed_form(oracle):
    """on the dyadic grid every summation order is exact: GPU values == int64 closed form."""
    cards = np.array([13, 900, 30000], np.int64)
    wl = Workload(name="dy", T=3, D=64, B=8192, alpha=1.1, seed=11, cards=cards)
    idx, off = wl.batch(0)
    g = wl.grad_dyadic(0)
    _say("dyadic closed form")
    W = np.zeros((wl.R, wl.D), np.float32)
    run = GpuRun(wl.row_offsets, wl.D, W, wl.B, len(idx), with_packed=False, want_codes=False)
    run.upload_batch(idx, off, g)
    r = run.bwd()
    m = np.rint(g.astype(np.float64) * 2.0 ** 24).astype(np.int64)  # [B, T, D] integers
    tuo = r["table_uniq_offsets"]
    for t in range(wl.T):
        dense = np.zeros((int(cards[t]), wl.D), np.int64)
        np.add.at(dense, idx[t * wl.B:(t + 1) * wl.B], m[:, t, :])
        rows = r["uniq_rows"][tuo[t]:tuo[t + 1]]
        got = np.rint(r["values"][tuo[t]:tuo[t + 1]].astype(np.float64) * 2.0 ** 24).astype(np.int64)
        assert_exact(got, dense[rows], f"dyadic table {t}")
        assert set(rows.tolist()) == set(idx[t * wl.B:(t + 1) * wl.B].tolist())
    assert run.status()[0] == 0


def test_determinism(oracle):
    """same inputs, repeated launches: byte-identical outputs (no dependence on scheduling)."""
    cards = np.array([7, 300, 100000, 2], np.int64)
    wl = Workload(name="det", T=4, D=64, B=8192, alpha=1.1, seed=21, cards=cards)
    idx, off = wl.batch(0)
    W = wl.tables(threads=1)
    run = GpuRun(wl.row_offsets, wl.D, W, wl.B, len(idx), with_packed=False, want_codes=False)
    run.upload_batch(idx, off, wl.grad_normal(0))
    _say("determinism")
    first = run.bwd()
    gq0, gs0 = run.quant()
    for _ in range(20):
        r = run.bwd()
        gq, gs = run.quant()
        for k in ("sorted_pos", "uniq_rows", "seg_offsets", "table_uniq_offsets"):
            assert_exact(r[k], first[k], k)
        assert_exact(r["values"].view(np.uint32), first["values"].view(np.uint32), "values bits")
        assert_exact(r["g_absmax"].view(np.uint32), first["g_absmax"].view(np.uint32), "g_absmax bits")
        assert_exact(gq, gq0, "gq")
    assert run.status()[0] == 0


def test_split_backward_on_two_streams(oracle):
    """dqrm_dedupe on a side stream (it needs only the indices), dqrm_segment_sum on the main stream
    after an event, twice on the same dedupe result with different gradients: same outputs as the
    one-call backward / the oracle."""
    import torch
    import paper_2410_20046_amd as dq

    cards = np.array([5, 2000, 300000, 64], np.int64)
    wl = Workload(name="split", T=4, D=64, B=4096, alpha=1.1, seed=31, cards=cards)
    idx, off = wl.batch(0)
    W = np.zeros((wl.R, wl.D), np.float32)
    run = GpuRun(wl.row_offsets, wl.D, W, wl.B, len(idx), with_packed=False, want_codes=False)
    _say("split backward")
    b = run.bufs
    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    run.upload_batch(idx, off, wl.grad_normal(0))
    side.wait_stream(main)
    dq.dqrm_dedupe(run.tables, run.idx, run.off, wl.B, b.sorted_pos, b.uniq_rows, b.seg_offsets,
                   b.table_uniq_offsets, b.num_unique, b.workspace, stream=side)
    ev = torch.cuda.Event()
    ev.record(side)
    main.wait_event(ev)
    for k in (0, 1):
        g = wl.grad_normal(k)
        gd = torch.from_numpy(g).to(run.dev)
        dq.dqrm_segment_sum(run.tables, wl.B, len(idx), gd, b.values, b.g_absmax, b.workspace)
        U = int(b.num_unique.cpu().item())
        got = dict(U=U, sorted_pos=b.sorted_pos.cpu().numpy(), uniq_rows=b.uniq_rows.cpu().numpy()[:U],
                   seg_offsets=b.seg_offsets.cpu().numpy()[:U + 1],
                   table_uniq_offsets=b.table_uniq_offsets.cpu().numpy(), values=b.values.cpu().numpy()[:U],
                   g_absmax=b.g_absmax.cpu().numpy())
        o = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, g)
        compare_bwd(got, o, f"split/{k}")
        assert_exact(got["values"].view(np.uint32), o["values"].view(np.uint32), f"split/{k} values bits")
        assert_exact(got["g_absmax"].view(np.uint32), o["g_absmax"].view(np.uint32), f"split/{k} g_absmax bits")
    assert run.status()[0] == 0


def test_dedupe_multi_equals_single(oracle):
    """three batches deduped by one dqrm_dedupe_multi launch == the oracle's dedupe of each batch, and the
    segment sums that follow use each batch's own workspace."""
    import torch
    import paper_2410_20046_amd as dq

    cards = np.array([11, 5000, 250000], np.int64)
    wl = Workload(name="multi", T=3, D=16, B=2048, alpha=1.05, seed=51, cards=cards)
    W = np.zeros((wl.R, wl.D), np.float32)
    _say("multi-batch dedupe")
    runs, batches = [], []
    host = [wl.batch(k, pooling="ragged" if k == 1 else "one", max_len=3) for k in range(3)]
    cap = max(len(i) for i, _ in host)  # every batch gets buffers and a workspace sized for the largest
    for k in range(3):
        idx, off = host[k]
        r = GpuRun(wl.row_offsets, wl.D, W, wl.B, cap, with_packed=False, want_codes=False)
        r.upload_batch(idx, off, wl.grad_normal(k))
        runs.append((r, idx, off))
        b = r.bufs
        batches.append((r.idx, r.off, b.sorted_pos, b.uniq_rows, b.seg_offsets, b.table_uniq_offsets, b.num_unique,
                        b.workspace))
    dq.dqrm_dedupe_multi(runs[0][0].tables, wl.B, batches)
    for k, (r, idx, off) in enumerate(runs):
        b = r.bufs
        dq.dqrm_segment_sum(r.tables, wl.B, len(idx), r.grad, b.values, b.g_absmax, b.workspace)
        U = int(b.num_unique.cpu().item())
        got = dict(U=U, sorted_pos=b.sorted_pos.cpu().numpy()[:len(idx)], uniq_rows=b.uniq_rows.cpu().numpy()[:U],
                   seg_offsets=b.seg_offsets.cpu().numpy()[:U + 1],
                   table_uniq_offsets=b.table_uniq_offsets.cpu().numpy(), values=b.values.cpu().numpy()[:U],
                   g_absmax=b.g_absmax.cpu().numpy())
        o = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, wl.grad_normal(k))
        compare_bwd(got, o, f"multi/{k}")
        assert_exact(got["values"].view(np.uint32), o["values"].view(np.uint32), f"multi/{k} values bits")
    assert runs[0][0].status()[0] == 0


def test_dedupe_with_a_promised_bound_on_table_lookups(oracle):
    """A caller's bound on the lookups of one table (dqrm_dedupe_batch_t.max_table_lookups): with a true bound the
    results are the oracle's; a table beyond a stated bound is skipped and reported like one beyond the limit."""
    import paper_2410_20046_amd as dq

    cards = np.array([7, 3000, 400000], np.int64)
    wl = Workload(name="bound", T=3, D=32, B=8192, alpha=1.05, seed=77, cards=cards)  # 24576 lookups, 8192 a table
    W = np.zeros((wl.R, wl.D), np.float32)
    idx, off = wl.batch(0)
    g = wl.grad_normal(0)
    o = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, g)
    for bound, ok in ((wl.B, True), (dq.MAX_TABLE_LOOKUPS, True), (wl.B - 1, False)):
        _say(f"promised bound {bound}")
        r = GpuRun(wl.row_offsets, wl.D, W, wl.B, len(idx), with_packed=False, want_codes=False)
        r.upload_batch(idx, off, g)
        b = r.bufs
        dq.dqrm_dedupe_multi(r.tables, wl.B, [(r.idx, r.off, b.sorted_pos, b.uniq_rows, b.seg_offsets,
                                               b.table_uniq_offsets, b.num_unique, b.workspace)], max_table_lookups=bound)
        dq.dqrm_segment_sum(r.tables, wl.B, len(idx), r.grad, b.values, b.g_absmax, b.workspace)
        code, tb, val = r.status()
        U = int(b.num_unique.cpu().item())
        if not ok:
            assert code == dq.ERR_CAPACITY and val == wl.B and U == 0
            continue
        assert code == 0
        got = dict(U=U, sorted_pos=b.sorted_pos.cpu().numpy()[:len(idx)], uniq_rows=b.uniq_rows.cpu().numpy()[:U],
                   seg_offsets=b.seg_offsets.cpu().numpy()[:U + 1],
                   table_uniq_offsets=b.table_uniq_offsets.cpu().numpy(), values=b.values.cpu().numpy()[:U],
                   g_absmax=b.g_absmax.cpu().numpy())
        compare_bwd(got, o, f"bound {bound}")
        assert_exact(got["values"].view(np.uint32), o["values"].view(np.uint32), f"bound {bound} values bits")


def test_fused_quant_update_matches_two_call_path(oracle):
    """dqrm_segment_sum(g_absmax=NULL) + dqrm_quant_update == segment_sum + grad_quant_int8 + sparse_update
    == the oracle, bit for bit (codes, scales, absmax, master, packed)."""
    import torch
    import paper_2410_20046_amd as dq

    cards = np.array([9, 700, 120000, 33], np.int64)
    wl = Workload(name="fused", T=4, D=64, B=4096, alpha=1.1, seed=41, cards=cards)
    idx, off = wl.batch(0)
    g = wl.grad_normal(0)
    W = wl.tables(threads=1)
    _say("fused quant+update")
    run = GpuRun(wl.row_offsets, wl.D, W, wl.B, len(idx), want_codes=False)
    run.upload_batch(idx, off, g)
    s = run.find_scale()
    run.pack()
    b = run.bufs
    dq.dqrm_dedupe(run.tables, run.idx, run.off, wl.B, b.sorted_pos, b.uniq_rows, b.seg_offsets,
                   b.table_uniq_offsets, b.num_unique, b.workspace)
    dq.dqrm_segment_sum(run.tables, wl.B, len(idx), run.grad, b.values, None, b.workspace)
    dq.dqrm_quant_update(run.tables, b.cap, len(idx), b.values, b.uniq_rows, b.table_uniq_offsets, b.g_absmax, b.gq,
                         b.g_scale, 0.1, b.workspace)
    U = int(b.num_unique.cpu().item())
    Wo = W.copy()
    po = oracle.pack_int4(Wo, wl.row_offsets, s)
    o = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, g)
    gq_o, gs_o = oracle.grad_quant_int8(wl.T, wl.D, o["values"], o["table_uniq_offsets"], o["g_absmax"])
    oracle.sparse_update(Wo, po, wl.row_offsets, s, o["uniq_rows"], o["table_uniq_offsets"], gq_o, gs_o, 0.1)
    assert U == o["U"]
    assert_exact(b.g_absmax.cpu().numpy().view(np.uint32), o["g_absmax"].view(np.uint32), "fused g_absmax bits")
    assert_exact(b.g_scale.cpu().numpy().view(np.uint32), gs_o.view(np.uint32), "fused g_scale bits")
    # (the rows of segments of more than one chunk are written by dqrm_quant_update in this mode)
    assert_exact(b.values.cpu().numpy()[:U].view(np.uint32), o["values"].view(np.uint32), "fused values bits")
    assert_exact(b.gq.cpu().numpy()[:U], gq_o, "fused INT8 codes")
    assert_exact(run.master_np().view(np.uint32), Wo.view(np.uint32), "fused master bits")
    assert_exact(run.packed_np(), po, "fused packed bytes")
    assert run.status()[0] == 0


def test_training_loop_with_periodic_scale_refresh(oracle):
    """Several train steps in a row, the per-table scale recomputed from the whole master table every
    `period` steps and stale in between (Sec. 3.2, Sec. 4.1): after every step the master rows, the packed
    mirror and the scales equal the oracle's, bit for bit.  The learning rate is large so that rows move
    by several quantisation steps and the refreshed scale differs from the stale one."""
    import paper_2410_20046_amd as dq

    cards = np.array([5, 300, 60000, 2000], np.int64)
    wl = Workload(name="loop", T=4, D=32, B=1024, alpha=1.1, seed=77, cards=cards)
    W = wl.tables(threads=1)
    Wo = W.copy()
    N = wl.T * wl.B
    run = GpuRun(wl.row_offsets, wl.D, W, wl.B, N, want_codes=False)
    b = run.bufs
    period, lr = 3, 4.0
    s_o, p_o = None, None
    scales_seen = []
    for k in range(7):
        _say(f"loop step {k}")
        idx, off = wl.batch(k)
        g = wl.grad_normal(k)
        run.upload_batch(idx, off, g)
        if k % period == 0:
            s_g = run.find_scale()
            s_o = oracle.find_scale(Wo, wl.row_offsets)
            assert_exact(s_g.view(np.uint32), s_o.view(np.uint32), f"loop/{k} refreshed w_scale bits")
            p_o = oracle.pack_int4(Wo, wl.row_offsets, s_o)
            assert_exact(run.pack(), p_o, f"loop/{k} re-encoded packed bytes")
            scales_seen.append(s_o.copy())
        for mode in (0, 1):
            out_g, _ = run.fwd(mode)
            out_o, _ = oracle.embbag_fwd(Wo, None, wl.row_offsets, s_o, wl.B, idx, off, mode=0, want_codes=False)
            assert_exact(out_g.view(np.uint32), out_o.view(np.uint32), f"loop/{k} out bits mode {mode}")
        dq.dqrm_dedupe(run.tables, run.idx, run.off, wl.B, b.sorted_pos, b.uniq_rows, b.seg_offsets,
                       b.table_uniq_offsets, b.num_unique, b.workspace)
        dq.dqrm_segment_sum(run.tables, wl.B, N, run.grad, b.values, None, b.workspace)
        dq.dqrm_quant_update(run.tables, b.cap, N, b.values, b.uniq_rows, b.table_uniq_offsets, b.g_absmax, b.gq,
                             b.g_scale, lr, b.workspace)
        o = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, g)
        gq_o, gs_o = oracle.grad_quant_int8(wl.T, wl.D, o["values"], o["table_uniq_offsets"], o["g_absmax"])
        oracle.sparse_update(Wo, p_o, wl.row_offsets, s_o, o["uniq_rows"], o["table_uniq_offsets"], gq_o, gs_o, lr)
        assert_exact(run.master_np().view(np.uint32), Wo.view(np.uint32), f"loop/{k} master bits")
        assert_exact(run.packed_np(), p_o, f"loop/{k} packed bytes")
        assert_exact(run.tables.w_scale.cpu().numpy().view(np.uint32), s_o.view(np.uint32), f"loop/{k} scale kept")
    assert len(scales_seen) == 3 and not np.array_equal(scales_seen[0], scales_seen[1]), \
        "the refresh never changed a scale: the case does not exercise staleness"
    assert run.status()[0] == 0


# --------------------------------------------------------------------------
# data-dependent errors: reported, never acted upon
# --------------------------------------------------------------------------
def test_out_of_range_index_is_reported_not_used(oracle):
    import paper_2410_20046_amd as dq

    wl = make_workload("tiny")
    W = wl.tables(threads=1)
    idx, off = wl.batch(0)
    bad = idx.copy()
    bad[200] = 1000  # table 1 has rows 0..999
    bad[300] = -1
    _say("out-of-range index")
    run = GpuRun(wl.row_offsets, wl.D, W, wl.B, len(idx))
    run.upload_batch(bad, off, wl.grad_normal(0))
    run.find_scale()
    out, _ = run.fwd(0)
    code, tb, val = run.status()
    assert code == dq.ERR_INDEX_OUT_OF_RANGE and tb in (1, 2) and val in (1000, -1)
    # the bad lookups were skipped: their bags are empty, everything else is as with valid input
    s = oracle.find_scale(W, wl.row_offsets)
    good_out, _ = oracle.embbag_fwd(W, None, wl.row_offsets, s, wl.B, idx, off)
    good_out[200 - 128, 1] = 0.0
    good_out[300 - 256, 2] = 0.0
    assert_exact(out.view(np.uint32), good_out.view(np.uint32), "out with skipped lookups")
    r = run.bwd()
    code, tb, val = run.status()
    assert code == dq.ERR_INDEX_OUT_OF_RANGE
    exp_u = 0
    for t in range(wl.T):
        rows = bad[t * wl.B:(t + 1) * wl.B]
        exp_u += len(np.unique(rows[(rows >= 0) & (rows < wl.cards[t])]))
    assert r["U"] == exp_u
    assert run.status()[0] == 0  # cleared by the read


def test_capacity_overflow_is_reported(oracle):
    import paper_2410_20046_amd as dq

    B = dq.MAX_TABLE_LOOKUPS + 1
    wl = make_workload("tiny", T=2, B=B, fixed_card=50, rows=100)
    W = wl.tables(threads=1)
    idx, off = wl.batch(0)
    _say("capacity overflow")
    run = GpuRun(wl.row_offsets, wl.D, W, wl.B, len(idx), with_packed=False, want_codes=False)
    run.upload_batch(idx, off, wl.grad_normal(0))
    r = run.bwd()
    code, tb, val = run.status()
    assert code == dq.ERR_CAPACITY and val == B
    assert r["U"] == 0
