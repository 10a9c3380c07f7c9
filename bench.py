#!/usr/bin/env python3
"""Benchmark of the DQRM embedding hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic batch, all through the C ABI:
  dqrm_embbag_fwd (gather -> INT4 fake-quant -> sum-pool) ->
  dqrm_embbag_bwd (dedupe -> segment-sum)                 ->
  dqrm_grad_quant_int8 -> dqrm_sparse_update (SGD on master rows + packed re-encode).
Workload: the Terabyte-shaped embedding layer (26 tables, ~49.12 M rows, dim 64, batch 8192,
one Zipf(1.1) index per table per sample), tables and batches resident in HBM before timing.
Prints ONE JSON line.  The CPU oracle is used only for the "cpu_baseline" leg.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, vendor figure


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(T, D, B, N, U, packed_fwd, packed_mirror):
    """Bytes the method itself has to move per step (duplicates of a row within a step count once)."""
    bags = T * B
    b = {
        "fwd": 8 * N + (D // 2 if packed_fwd else 4 * D) * U + 4 * D * bags,
        "dedupe": 64 * N,
        "segsum": 4 * D * bags + (8 + 4 * D) * U,
        "quant": (4 * D + D) * U,
        "update": (D + 8 * D) * U + (D // 2 * U if packed_mirror else 0),
    }
    b["step"] = sum(b.values())
    return b


def read_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, "profiles", "terabyte_pmc_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        p = line.split()
        if len(p) >= 3 and p[0] == "traffic_bytes_per_launch" and p[1] == kernel:
            return float(p[2])
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1920)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="terabyte", choices=["terabyte", "kaggle", "single", "tiny"])
    ap.add_argument("--mode", default="packed", choices=["packed", "master"])
    ap.add_argument("--pool", type=int, default=64, help="distinct index batches cycled")
    ap.add_argument("--grad-pool", type=int, default=8, help="distinct grad_out buffers cycled")
    ap.add_argument("--lr", type=float, default=0.1)
    ap.add_argument("--pooling", type=int, default=1,
                    help="indices per bag (pooling factor; the paper-shaped workloads have 1).  A table may have at "
                         "most 16384 lookups per batch: lower --batch accordingly")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--mlp-weight-bits", type=int, default=0, choices=[0, 4, 8],
                    help="with --dense: channel-wise fake quantisation of the MLP weights (dqrm_dense_step_quant)")
    ap.add_argument("--mlp-grad-bits", type=int, default=0, choices=[0, 8],
                    help="with --dense: INT8 MLP gradients with error compensation (dqrm_dense_step_quant)")
    ap.add_argument("--refresh-period", type=int, default=0,
                    help="P > 0: every P steps the per-table weight scale is recomputed from the whole master table "
                         "(dqrm_find_scale) and the packed mirror re-encoded (dqrm_pack_int4), in line, inside the timed "
                         "region -- the paper's periodic scale update; 0 = never (the scale stays cached)")
    ap.add_argument("--dense", action="store_true",
                    help="full DQRM train step (use with --workload kaggle): dqrm_dense_step (MLPs 13-512-256-64-16 / "
                         "367-512-256-1, interaction, BCE, backward, SGD) runs between the tables' forward and "
                         "backward and produces grad_out")
    ap.add_argument("--overlap", default="ahead", choices=["none", "fwd", "pipeline", "pipeline2", "ahead", "group"],
                    help="where dqrm_dedupe (needs only the indices) runs: none = in line on the one stream; "
                         "fwd = on a second stream beside the same step's forward; pipeline = on a second stream, "
                         "one step ahead (double-buffered workspace); pipeline2 = two steps ahead, alternating between two "
                         "side streams; ahead = in line on the one stream, but for the "
                         "next --ahead batches in one dqrm_dedupe_multi launch (a table's sort fills one CU, so several "
                         "batches fill the chip; the data loader has their indices already); group = that launch on the "
                         "second stream, one group of --ahead batches ahead, so the streams meet once per group")
    ap.add_argument("--ahead", type=int, default=8, help="batches per dqrm_dedupe_multi launch with --overlap ahead / group")
    ap.add_argument("--side-multi", action="store_true",
                    help="with --overlap group: the side stream uses one dqrm_dedupe_multi launch per group instead "
                         "of one dqrm_dedupe per batch")
    ap.add_argument("--two-call-update", dest="fused", action="store_false",
                    help="dqrm_grad_quant_int8 + dqrm_sparse_update (and the absmax fold inside dqrm_segment_sum) "
                         "instead of the one-pass dqrm_quant_update")
    ap.add_argument("--no-graph", dest="graph", action="store_false",
                    help="launch every kernel from the host instead of replaying a captured HIP graph of `pool` steps")
    ap.add_argument("--simulated-nodes", type=int, default=1,
                    help="simulated data parallelism: the batch is cut into this many micro-batches (forward, backward "
                         "and INT8 codes each, with the first one's scale), their integer gradients are merged "
                         "(dqrm_sparse_merge) and the tables are updated once per step; all calls in line on one stream")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1. "
                 "The repository's design notes say how the path would shard.")

    import numpy as np
    import torch

    import paper_2410_20046_amd as dq
    from gen import make_workload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    dq.lib()  # fail loudly if the HIP library is missing

    wl = make_workload(args.workload, **({"B": args.batch} if args.batch else {}))
    T, D, B = wl.T, wl.D, wl.B
    t0 = time.time()
    W = wl.tables(threads=16)
    log(f"[bench] {args.workload}: T={T} D={D} B={B} R={wl.R} ({W.nbytes / 1e9:.2f} GB fp32), tables in {time.time() - t0:.1f}s")
    master = torch.from_numpy(W).to(dev)
    packed = torch.empty((wl.R, D // 2), dtype=torch.uint8, device=dev)
    tables = dq.Tables(wl.row_offsets, D, master, packed)

    t0 = time.time()
    pool = [wl.batch(k) if args.pooling == 1 else wl.batch(k, pooling="fixed", max_len=args.pooling)
            for k in range(args.pool)]
    N = len(pool[0][0])
    idx_d = [torch.from_numpy(i).to(dev) for i, _ in pool]
    off_d = [torch.from_numpy(o).to(dev) for _, o in pool]
    grads = [wl.grad_normal(k) for k in range(args.grad_pool)]
    grad_d = [torch.from_numpy(g).to(dev) for g in grads]
    log(f"[bench] {args.pool} batches of {N} lookups + {args.grad_pool} grad_out in {time.time() - t0:.1f}s")

    bufs = dq.StepBuffers(T, D, B, N, dev, want_codes=False)
    mode = dq.FWD_PACKED if args.mode == "packed" else dq.FWD_MASTER
    dq.dqrm_find_scale(tables)
    dq.dqrm_pack_int4(tables)
    torch.cuda.synchronize()

    side = torch.cuda.Stream()  # default priority
    nbuf = {"pipeline": 2, "pipeline2": 4, "ahead": args.ahead, "group": 2 * args.ahead}.get(args.overlap, 1)
    dup = lambda x: [x] + [torch.empty_like(x) for _ in range(nbuf - 1)]
    wss, sps, urs, sos = dup(bufs.workspace), dup(bufs.sorted_pos), dup(bufs.uniq_rows), dup(bufs.seg_offsets)
    tuos, nus = dup(bufs.table_uniq_offsets), dup(bufs.num_unique)
    ev_dedupe = [torch.cuda.Event() for _ in range(nbuf)]   # dedupe into buffer i finished
    ev_update = [torch.cuda.Event() for _ in range(nbuf)]   # last reader (the update) of buffer i finished
    batch_of = lambda k: (idx_d[k % args.pool], off_d[k % args.pool])

    side2 = torch.cuda.Stream()  # default priority; pipeline2 alternates between the two side streams

    def dedupe_on_side(k, stream=None):
        stream = stream or side
        i = k % nbuf
        stream.wait_event(ev_update[i])  # the buffer's previous reader (no-op before the first record)
        ix, of = batch_of(k)
        dq.dqrm_dedupe(tables, ix, of, B, sps[i], urs[i], sos[i], tuos[i], nus[i], wss[i], stream=stream)
        ev_dedupe[i].record(stream)

    nodes = args.simulated_nodes
    if nodes > 1:
        from gen import split_batch
        assert B % nodes == 0 and nodes <= dq.MAX_DEDUPE_BATCHES and not args.dense
        Bm = B // nodes
        parts = [split_batch(i, o, T, B, nodes) for i, o in pool]
        mb_idx = [[torch.from_numpy(i).to(dev) for i, _ in p] for p in parts]
        mb_off = [[torch.from_numpy(o).to(dev) for _, o in p] for p in parts]
        Nm = max(len(i) for p in parts for i, _ in p)
        mb = [dq.StepBuffers(T, D, Bm, Nm, dev, want_codes=False) for _ in range(nodes)]
        m_cap = nodes * Nm
        m_rows = torch.empty(m_cap, dtype=torch.int64, device=dev)
        m_tuo = torch.empty(T + 1, dtype=torch.int32, device=dev)
        m_nu = torch.zeros(1, dtype=torch.int32, device=dev)
        m_sums = torch.empty((m_cap, D), dtype=torch.int32, device=dev)
        m_ws = torch.empty(dq.dqrm_sparse_merge_workspace_bytes(T, D, nodes, m_cap), dtype=torch.uint8, device=dev)

    def simulated_step(k):
        """One weight update from `nodes` micro-batches (appendix on simulated data parallelism)."""
        p, g = k % args.pool, grad_d[k % args.grad_pool]
        # the micro-batches' indices are all there: one sort launch for all of them (26 x nodes workgroups)
        dq.dqrm_dedupe_multi(tables, Bm, [(mb_idx[p][j], mb_off[p][j], b.sorted_pos, b.uniq_rows, b.seg_offsets,
                                           b.table_uniq_offsets, b.num_unique, b.workspace) for j, b in enumerate(mb)])
        # the weights do not change inside a group and bags are independent: the micro-batches' forwards are one
        # call on the whole batch
        dq.dqrm_embbag_fwd(tables, idx_d[p], off_d[p], B, mode, bufs.out, None)
        for j in range(nodes):
            b, ix, of = mb[j], mb_idx[p][j], mb_off[p][j]
            # (only the first micro-batch's maxima are used: its scale serves the whole group)
            dq.dqrm_segment_sum(tables, Bm, ix.numel(), g[j * Bm:(j + 1) * Bm], b.values, b.g_absmax, b.workspace)
            dq.dqrm_grad_quant_int8(T, D, b.cap, b.values, b.table_uniq_offsets, mb[0].g_absmax, b.gq, b.g_scale)
        dq.dqrm_sparse_merge(tables, [(b.uniq_rows, b.table_uniq_offsets, b.gq) for b in mb], m_rows, m_tuo, m_nu,
                             m_sums, m_ws)
        dq.dqrm_sparse_update_sums(tables, m_cap, m_rows, m_tuo, m_sums, mb[0].g_scale, args.lr)

    dense = None
    if args.dense:
        from gen import make_dense_model, dense_batch
        bd, bw, bb, td, tw, tb = make_dense_model("kaggle", T, D, wl.seed)
        dense = dq.DenseModel(T, D, bd, bw, bb, td, tw, tb, dev)
        dense_ws = torch.empty(dq.dqrm_dense_workspace_bytes(dense, B), dtype=torch.uint8, device=dev)
        dense_in = [dense_batch(B, bd[0], wl.seed, k) for k in range(args.grad_pool)]
        dense_x = [torch.from_numpy(x).to(dev) for x, _ in dense_in]
        dense_y = [torch.from_numpy(y).to(dev) for _, y in dense_in]
        loss_d = torch.zeros(1, dtype=torch.float32, device=dev)
        grad_live = torch.empty((B, T, D), dtype=torch.float32, device=dev)
        dense_quant = None
        if args.mlp_weight_bits or args.mlp_grad_bits:
            P = dq.dqrm_dense_param_count(dense)
            dense_quant = dq.DenseQuant(
                weight_bits=args.mlp_weight_bits, grad_bits=args.mlp_grad_bits,
                grad_error=torch.zeros(P, dtype=torch.float32, device=dev) if args.mlp_grad_bits else None,
                grad_scale=torch.zeros(2 * (len(bw) + len(tw)), dtype=torch.float32, device=dev) if args.mlp_grad_bits else None,
                grad_codes=torch.zeros(P, dtype=torch.int8, device=dev) if args.mlp_grad_bits else None)

    def refresh_scale():
        """Sec. 3.2: recompute the per-table scale from the whole master table, re-encode the packed mirror."""
        dq.dqrm_find_scale(tables)
        dq.dqrm_pack_int4(tables)

    refresh_in_steps = [args.refresh_period > 0]  # False while a graph handles the refresh between replays

    def forward(k, ix, of):
        if refresh_in_steps[0] and (k - args.warmup) % args.refresh_period == 0:
            refresh_scale()
        dq.dqrm_embbag_fwd(tables, ix, of, B, mode, bufs.out, None)
        if dense is not None:
            j = k % args.grad_pool
            dq.dqrm_dense_step_quant(dense, dense_quant, B, dense_x[j], bufs.out, dense_y[j], args.lr, loss_d, grad_live,
                                     dense_ws)

    def rest_of_step(k, i):
        """B3-B5 on the current stream, from the dedupe result in buffer i."""
        g = grad_live if dense is not None else grad_d[k % args.grad_pool]
        if args.fused:
            dq.dqrm_segment_sum(tables, B, N, g, bufs.values, None, wss[i])
            dq.dqrm_quant_update(tables, bufs.cap, N, bufs.values, urs[i], tuos[i], bufs.g_absmax, bufs.gq,
                                 bufs.g_scale, args.lr, wss[i])
        else:
            dq.dqrm_segment_sum(tables, B, N, g, bufs.values, bufs.g_absmax, wss[i])
            dq.dqrm_grad_quant_int8(T, D, bufs.cap, bufs.values, tuos[i], bufs.g_absmax, bufs.gq, bufs.g_scale)
            dq.dqrm_sparse_update(tables, bufs.cap, urs[i], tuos[i], bufs.gq, bufs.g_scale, args.lr)

    def run_steps(k0, n):
        """n consecutive steps starting with batch k0, all launches on the current stream (+ the side
        stream for dqrm_dedupe when overlapping).  Self-contained: the side stream is joined at the end."""
        main = torch.cuda.current_stream()
        if nodes > 1:
            for k in range(k0, k0 + n):
                simulated_step(k)
            return
        if args.overlap == "ahead":
            for k in range(k0, k0 + n):
                if (k - k0) % nbuf == 0:  # dedupe of this and the next nbuf-1 batches, in one launch pair
                    group = range(k, min(k + nbuf, k0 + n))
                    dq.dqrm_dedupe_multi(tables, B, [batch_of(j) + (sps[j % nbuf], urs[j % nbuf], sos[j % nbuf],
                                                                    tuos[j % nbuf], nus[j % nbuf], wss[j % nbuf])
                                                     for j in group])
                ix, of = batch_of(k)
                forward(k, ix, of)
                rest_of_step(k, k % nbuf)
            return
        if args.overlap == "group":
            # dqrm_dedupe_multi of the NEXT group of --ahead batches runs on the side stream while the main
            # stream works through the current group: the two streams meet once per group, not once per step
            A = args.ahead
            groups = [range(s, min(s + A, k0 + n)) for s in range(k0, k0 + n, A)]
            slot = lambda gi, k: (gi % 2) * A + (k - groups[gi][0])
            def dedupe_group(gi, stream):
                if stream is side and not args.side_multi:
                    # one batch at a time: 26 workgroups take 26 CUs from the main stream's kernels, 208 would
                    # take most of the chip
                    for k in groups[gi]:
                        j = slot(gi, k)
                        dq.dqrm_dedupe(tables, *batch_of(k), B, sps[j], urs[j], sos[j], tuos[j], nus[j], wss[j],
                                       stream=side)
                    return
                dq.dqrm_dedupe_multi(tables, B, [batch_of(k) + (sps[slot(gi, k)], urs[slot(gi, k)], sos[slot(gi, k)],
                                                                tuos[slot(gi, k)], nus[slot(gi, k)], wss[slot(gi, k)])
                                                 for k in groups[gi]], stream=stream)
            side.wait_stream(main)
            dedupe_group(0, main)  # the first group in line
            for gi, grp in enumerate(groups):
                if gi + 1 < len(groups):
                    if gi >= 1:
                        side.wait_event(ev_update[(gi - 1) % 2])  # readers of that half of the buffers are done
                    dedupe_group(gi + 1, side)
                    ev_dedupe[(gi + 1) % 2].record(side)
                if gi >= 1:
                    main.wait_event(ev_dedupe[gi % 2])
                for k in grp:
                    ix, of = batch_of(k)
                    forward(k, ix, of)
                    rest_of_step(k, slot(gi, k))
                ev_update[gi % 2].record(main)
            main.wait_stream(side)
            return
        if args.overlap == "none":
            for k in range(k0, k0 + n):
                ix, of = batch_of(k)
                forward(k, ix, of)
                dq.dqrm_dedupe(tables, ix, of, B, sps[0], urs[0], sos[0], tuos[0], nus[0], wss[0])
                rest_of_step(k, 0)
            return
        if args.overlap == "pipeline2":
            # two steps ahead, alternating between two side streams: a dedupe has two step times to finish
            sides = [side, side2]
            side.wait_stream(main)
            side2.wait_stream(main)
            dedupe_on_side(k0, sides[k0 % 2])
            if n > 1:
                dedupe_on_side(k0 + 1, sides[(k0 + 1) % 2])
            for k in range(k0, k0 + n):
                ix, of = batch_of(k)
                i = k % nbuf
                forward(k, ix, of)
                if k + 2 < k0 + n:
                    dedupe_on_side(k + 2, sides[k % 2])
                main.wait_event(ev_dedupe[i])
                rest_of_step(k, i)
                ev_update[i].record(main)
            main.wait_stream(side)
            main.wait_stream(side2)
            return
        side.wait_stream(main)  # everything enqueued so far is visible to the side stream
        if args.overlap == "pipeline":
            dedupe_on_side(k0)
        for k in range(k0, k0 + n):
            ix, of = batch_of(k)
            i = k % nbuf
            if args.overlap == "fwd":
                dedupe_on_side(k)  # beside this step's forward
            forward(k, ix, of)
            if args.overlap == "pipeline" and k + 1 < k0 + n:
                dedupe_on_side(k + 1)  # one step ahead: the next batch's indices are already here
            main.wait_event(ev_dedupe[i])
            rest_of_step(k, i)
            ev_update[i].record(main)

    # ---- warm-up (eager), optional capture of `graph_steps` steps into one HIP graph ----
    run_steps(0, args.warmup)
    torch.cuda.synchronize()
    graph, graph_steps = None, 0
    if args.graph:
        graph_steps = min(args.pool, args.steps)
        P = args.refresh_period
        if P > graph_steps:
            assert P % graph_steps == 0, "--refresh-period must be a multiple (or a divisor) of the graph's steps"
            refresh_in_steps[0] = False  # refreshed eagerly before every (P / graph_steps)-th replay
        elif P > 0:
            assert graph_steps % P == 0, "--refresh-period must be a multiple (or a divisor) of the graph's steps"
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run_steps(args.warmup, graph_steps)
        graph.replay()  # one untimed replay
        torch.cuda.synchronize()

    # ---- the timed region: exactly K steps, no host synchronisation inside ----
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_start = time.perf_counter()
    e0.record()
    if graph is not None:
        for rep in range(args.steps // graph_steps):
            if args.refresh_period > graph_steps and (rep * graph_steps) % args.refresh_period == 0:
                refresh_scale()
            graph.replay()
        if args.steps % graph_steps:
            run_steps(args.warmup, args.steps % graph_steps)
    else:
        run_steps(args.warmup, args.steps)
    e1.record()
    t_issued = time.perf_counter() - t_start
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = wall * 1e3 / args.steps
    code, tb, val = dq.dqrm_check_status()
    assert code == 0, f"device status {code} (table {tb}, value {val})"
    log(f"[bench] timed {args.steps} steps: wall {wall * 1e3:.2f} ms, events {ev_ms:.2f} ms, {ms_per_step * 1e3:.1f} us/step "
        f"(host issued them in {t_issued * 1e3:.2f} ms = {t_issued * 1e6 / args.steps:.1f} us/step)")

    # ---- unique rows per batch (for the algorithmic byte counts) ----
    us = []
    for k in range(min(args.pool, 16)):
        dq.dqrm_embbag_bwd(tables, idx_d[k], off_d[k], B, grad_d[0], bufs.sorted_pos, bufs.uniq_rows,
                           bufs.seg_offsets, bufs.table_uniq_offsets, bufs.num_unique, bufs.values, bufs.g_absmax,
                           bufs.workspace)
        us.append(int(bufs.num_unique.cpu().item()))
    U = float(np.mean(us))
    ab = algorithmic_bytes(T, D, B, N, U, packed_fwd=(mode == dq.FWD_PACKED), packed_mirror=True)

    # ---- per-call HIP-event timing, one stream, events on the launch stream ----
    stages = ["fwd", "dedupe", "segment_sum", "quant", "update", "quant_update"]
    calls = {
        "fwd": lambda k: dq.dqrm_embbag_fwd(tables, idx_d[k % args.pool], off_d[k % args.pool], B, mode, bufs.out, None),
        "dedupe": lambda k: dq.dqrm_dedupe(tables, idx_d[k % args.pool], off_d[k % args.pool], B, bufs.sorted_pos,
                                           bufs.uniq_rows, bufs.seg_offsets, bufs.table_uniq_offsets,
                                           bufs.num_unique, bufs.workspace),
        "segment_sum": lambda k: dq.dqrm_segment_sum(tables, B, N, grad_d[k % args.grad_pool], bufs.values,
                                                     bufs.g_absmax, bufs.workspace),
        "quant": lambda k: dq.dqrm_grad_quant_int8(T, D, bufs.cap, bufs.values, bufs.table_uniq_offsets,
                                                   bufs.g_absmax, bufs.gq, bufs.g_scale),
        "update": lambda k: dq.dqrm_sparse_update(tables, bufs.cap, bufs.uniq_rows, bufs.table_uniq_offsets, bufs.gq,
                                                  bufs.g_scale, args.lr),
        "quant_update": lambda k: dq.dqrm_quant_update(tables, bufs.cap, N, bufs.values, bufs.uniq_rows,
                                                       bufs.table_uniq_offsets, bufs.g_absmax, bufs.gq, bufs.g_scale,
                                                       args.lr, bufs.workspace),
    }
    # Each call is timed on its own: `reps` back-to-back launches of the same call (cycling through the
    # batches) between two events, so that the cost of recording an event is not charged to a 5-20 us kernel.
    # The calls are launched in path order first, so every call finds valid inputs.
    if nodes > 1:
        simulated_step(args.warmup)  # valid blocks for the two calls below
        stages += ["sparse_merge", "update_sums"]
        calls["sparse_merge"] = lambda k: dq.dqrm_sparse_merge(
            tables, [(b.uniq_rows, b.table_uniq_offsets, b.gq) for b in mb], m_rows, m_tuo, m_nu, m_sums, m_ws)
        calls["update_sums"] = lambda k: dq.dqrm_sparse_update_sums(tables, m_cap, m_rows, m_tuo, m_sums, mb[0].g_scale,
                                                                   args.lr)
    for name in stages:
        calls[name](args.warmup)
    reps = max(10, min(args.steps, 200))
    stage_us = {}
    for name in stages:
        for k in range(3):
            calls[name](args.warmup + k)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for k in range(reps):
            calls[name](args.warmup + k)
        ev1.record()
        torch.cuda.synchronize()
        stage_us[name] = 1e3 * ev0.elapsed_time(ev1) / reps
    log("[bench] per-call HIP-event time (us): " + ", ".join(f"{k}={v:.1f}" for k, v in stage_us.items()))
    stage_bytes = {"fwd": ab["fwd"], "dedupe": ab["dedupe"], "segment_sum": ab["segsum"], "quant": ab["quant"],
                   "update": ab["update"], "quant_update": ab["quant"] + ab["update"] - D * U}
    if nodes > 1:
        Um = int(m_nu.cpu().item())
        blocks_rows = sum(int(b.num_unique.cpu().item()) for b in mb)
        # merge: every block row's id (8 B) and codes (D B) in, the union's ids and 32-bit sums out
        stage_bytes["sparse_merge"] = blocks_rows * (8 + D) + Um * (8 + 4 * D)
        # update from sums: id + sums + master row read and written + packed row written
        stage_bytes["update_sums"] = Um * (8 + 4 * D + 8 * D + D // 2)
        log(f"[bench] simulated nodes {nodes}: {blocks_rows} block rows merge into {Um}")
    stage_gbs = {k: stage_bytes[k] / (stage_us[k] * 1e-6) / 1e9 for k in stages}

    # The dominant kernel of the step's critical path: dqrm_embbag_fwd is exactly one kernel launch
    # (embbag_fwd_kernel), so its event time is that kernel's average launch duration.
    dom, dom_kernel = "fwd", "embbag_fwd_kernel"
    dom_bytes, dom_gbs = stage_bytes[dom], stage_gbs[dom]
    roofline = {"bound": "hbm", "kernel": dom_kernel, "achieved": round(dom_gbs, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(dom_gbs / HBM_PEAK_GBS, 4), "traffic": read_traffic(dom_kernel),
                "algorithmic_bytes_per_launch": int(dom_bytes), "avg_launch_us": round(stage_us[dom], 2)}

    # ---- device-to-device copy bandwidth, for context ----
    a = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    b = torch.empty_like(a)
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(10):
        b.copy_(a)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 10 * 2 * a.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del a, b
    roofline["frac_of_copy_bw"] = round(dom_gbs / copy_gbs, 4)  # against what a plain copy reaches on this machine

    lookups_per_s = N * args.steps / wall
    step_gbs = ab["step"] / (ms_per_step * 1e-3) / 1e9

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        oracle.build()
        Wo = W  # the oracle updates the host copy in place, as the GPU does on the device
        s = oracle.find_scale(Wo, wl.row_offsets)  # the cached scale is an input of a step: not timed
        # packed mirror: only the rows a step touches are re-encoded, so an empty mirror gives the same work
        pk = np.zeros((wl.R, D // 2), np.uint8)
        done, t_cpu = 0, 0.0
        while t_cpu < args.cpu_seconds and done < 8 * args.pool:
            idx, off = pool[done % args.pool]
            g = grads[done % args.grad_pool]
            t1 = time.perf_counter()
            oracle.embbag_fwd(Wo, None, wl.row_offsets, s, B, idx, off, mode=0, want_codes=False)
            r = oracle.embbag_bwd(T, D, B, idx, off, g)
            gq, gs = oracle.grad_quant_int8(T, D, r["values"], r["table_uniq_offsets"], r["g_absmax"])
            oracle.sparse_update(Wo, pk, wl.row_offsets, s, r["uniq_rows"], r["table_uniq_offsets"], gq, gs, args.lr)
            t_cpu += time.perf_counter() - t1
            done += 1
        cpu = {"value": round(N * done / t_cpu, 1), "unit": "lookups/s", "cores": 1, "kind": "oracle",
               "sample": f"{done} steps of the same {args.workload} workload (its {args.pool} batches in turn), "
                         f"{t_cpu:.1f} s of single-threaded C oracle (fwd master mode + bwd + quant + update)"}
        log(f"[bench] oracle: {done} steps in {t_cpu:.1f}s")

    out = {
        "metric": "embedding lookups/s for INT4-QAT fwd+bwd; achieved HBM GB/s vs peak",
        "value": round(lookups_per_s, 1),
        "unit": "lookups/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}-shaped embedding layer: {T} tables, {wl.R} rows, dim {D}, batch {B}, "
                               f"1 Zipf index per table per sample, {args.mode}-mode forward, INT8 sparse grads, "
                               f"SGD lr {args.lr}, dedupe overlap: {args.overlap}"
                               + (f", {nodes} simulated nodes (micro-batches of {B // nodes}, one update per step)" if nodes > 1 else ""),
                   "lookups_per_step": N, "unique_rows_per_step": round(U, 1), "fwd_mode": args.mode, "overlap": args.overlap, "scale_refresh_period": args.refresh_period, "pooling": args.pooling, "dense_part": bool(args.dense), "mlp_weight_bits": args.mlp_weight_bits, "mlp_grad_bits": args.mlp_grad_bits, "simulated_nodes": nodes,
                   "update": ("dqrm_quant_update (one pass)" if args.fused else "dqrm_grad_quant_int8 + dqrm_sparse_update"),
                   "launch": (f"HIP graph of {graph_steps} steps replayed" if graph is not None else "eager launches")},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "step_algorithmic_bytes": int(ab["step"]),
        "step_hbm_gbs": round(step_gbs, 1),
        "step_hbm_frac_of_peak": round(step_gbs / HBM_PEAK_GBS, 4),
        "call_us": {k: round(v, 2) for k, v in stage_us.items()},
        "call_algorithmic_gbs": {k: round(v, 1) for k, v in stage_gbs.items()},
        "event_ms_per_step": round(ev_ms / args.steps, 5),
        "copy_bw_gbs": round(copy_gbs, 1),
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
