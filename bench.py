#!/usr/bin/env python3
"""Benchmark of the DQRM embedding hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic batch, all through the C ABI:
  dqrm_embbag_fwd (gather -> INT4 fake-quant -> sum-pool)                          ->
  dqrm_dedupe[_multi] + dqrm_segment_sum (dedupe -> segment-sum = sparse gradient) ->
  dqrm_quant_update (INT8 codes of the gradient values, SGD on the master rows, packed re-encode).
Workload: the Terabyte-shaped embedding layer (26 tables, ~49.12 M rows, dim 64, batch 8192,
one Zipf(1.1) index per table per sample), tables and batches resident in HBM before timing.
Prints ONE JSON line.  The CPU oracle is used only for the "cpu_baseline" leg.

`HotPath` holds the device state and the launch sequence; tests/test_gpu_bench_path.py drives the
very same object against the oracle.
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


class HotPath:
    """Device state of one workload plus the launch sequence of the timed step.

    overlap: where dqrm_dedupe (needs only the indices) runs --
      "none"     in line on the one stream, every step;
      "pipeline" on a second stream, one step ahead (double-buffered workspace);
      "ahead"    in line, but for the next `ahead` batches in one dqrm_dedupe_multi launch (a table's sort
                 fills one CU, so several batches fill the chip; a data loader has their indices already).
    fused: dqrm_quant_update instead of dqrm_grad_quant_int8 + dqrm_sparse_update.
    """

    def __init__(self, wl, W, pool, grads, dev, mode="packed", overlap="ahead", ahead=8, fused=True, lr=0.1,
                 dense_args=None, refresh_period=0):
        import numpy as np
        import torch
        import paper_2410_20046_amd as dq

        self.torch, self.dq, self.dev = torch, dq, dev
        self.wl, self.T, self.D, self.B = wl, wl.T, wl.D, wl.B
        self.lr, self.fused, self.overlap = lr, fused, overlap
        self.mode = dq.FWD_PACKED if mode == "packed" else dq.FWD_MASTER
        self.master = torch.from_numpy(W).to(dev)
        self.packed = torch.empty((wl.R, wl.D // 2), dtype=torch.uint8, device=dev)
        self.tables = dq.Tables(wl.row_offsets, wl.D, self.master, self.packed)
        self.pool = len(pool)
        self.N = len(pool[0][0])
        # a bound the data loader knows: bags per table x the longest bag of any batch in the pool
        self.max_table_lookups = int(self.B * max(int(np.diff(o).max()) for _, o in pool))
        self.idx_d = [torch.from_numpy(i).to(dev) for i, _ in pool]
        self.off_d = [torch.from_numpy(o).to(dev) for _, o in pool]
        self.grad_d = [torch.from_numpy(g).to(dev) for g in grads]
        self.bufs = dq.StepBuffers(self.T, self.D, self.B, self.N, dev, want_codes=False)
        self.nbuf = {"pipeline": 2, "ahead": ahead}.get(overlap, 1)
        b = self.bufs
        dup = lambda x: [x] + [torch.empty_like(x) for _ in range(self.nbuf - 1)]
        self.wss, self.sps, self.urs, self.sos = dup(b.workspace), dup(b.sorted_pos), dup(b.uniq_rows), dup(b.seg_offsets)
        self.tuos, self.nus = dup(b.table_uniq_offsets), dup(b.num_unique)
        self.side = torch.cuda.Stream()  # default priority
        self.ev_dedupe = [torch.cuda.Event() for _ in range(self.nbuf)]  # dedupe into buffer i finished
        self.ev_update = [torch.cuda.Event() for _ in range(self.nbuf)]  # last reader (the update) of buffer i finished
        self.refresh_period = refresh_period
        self.refresh_in_steps = refresh_period > 0  # False while the caller refreshes between graph replays
        self.step0 = 0                              # step number that counts as 0 for the refresh period
        self.dense = None
        if dense_args is not None:
            self._init_dense(**dense_args)
        self.probe = None  # list that collects (name, event) pairs while timing calls in sequence

    # ---- set-up ----------------------------------------------------------------------------------
    def prepare(self):
        """Sec. 3.2: the per-table scale from the whole master table, then the packed mirror."""
        self.dq.dqrm_find_scale(self.tables)
        self.dq.dqrm_pack_int4(self.tables)

    def _init_dense(self, weight_bits, grad_bits, grad_pool):
        torch, dq, dev = self.torch, self.dq, self.dev
        from gen import make_dense_model, dense_batch

        bd, bw, bb, td, tw, tb = make_dense_model("kaggle", self.T, self.D, self.wl.seed)
        self.dense = dq.DenseModel(self.T, self.D, bd, bw, bb, td, tw, tb, dev)
        self.dense_ws = torch.empty(dq.dqrm_dense_workspace_bytes(self.dense, self.B), dtype=torch.uint8, device=dev)
        dense_in = [dense_batch(self.B, bd[0], self.wl.seed, k) for k in range(grad_pool)]
        self.dense_x = [torch.from_numpy(x).to(dev) for x, _ in dense_in]
        self.dense_y = [torch.from_numpy(y).to(dev) for _, y in dense_in]
        self.loss_d = torch.zeros(1, dtype=torch.float32, device=dev)
        self.grad_live = torch.empty((self.B, self.T, self.D), dtype=torch.float32, device=dev)
        self.dense_quant = None
        if weight_bits or grad_bits:
            P = dq.dqrm_dense_param_count(self.dense)
            self.dense_quant = dq.DenseQuant(
                weight_bits=weight_bits, grad_bits=grad_bits,
                grad_error=torch.zeros(P, dtype=torch.float32, device=dev) if grad_bits else None,
                grad_scale=torch.zeros(2 * (len(bw) + len(tw)), dtype=torch.float32, device=dev) if grad_bits else None,
                grad_codes=torch.zeros(P, dtype=torch.int8, device=dev) if grad_bits else None)

    # ---- the calls of one step -------------------------------------------------------------------
    def batch_of(self, k):
        return self.idx_d[k % self.pool], self.off_d[k % self.pool]

    def _mark(self, name):
        if self.probe is not None:
            ev = self.torch.cuda.Event(enable_timing=True)
            ev.record()
            self.probe.append((name, ev))

    def refresh_scale(self):
        self.dq.dqrm_find_scale(self.tables)
        self.dq.dqrm_pack_int4(self.tables)

    def forward(self, k):
        dq = self.dq
        if self.refresh_in_steps and (k - self.step0) % self.refresh_period == 0:
            self.refresh_scale()
            self._mark("refresh")
        ix, of = self.batch_of(k)
        dq.dqrm_embbag_fwd(self.tables, ix, of, self.B, self.mode, self.bufs.out, None)
        self._mark("fwd")
        if self.dense is not None:
            j = k % len(self.dense_x)
            dq.dqrm_dense_step_quant(self.dense, self.dense_quant, self.B, self.dense_x[j], self.bufs.out, self.dense_y[j],
                                     self.lr, self.loss_d, self.grad_live, self.dense_ws)
            self._mark("dense")

    def dedupe(self, k, i, stream=None):
        ix, of = self.batch_of(k)
        # (one batch through the multi-batch entry point: it takes the bound on a table's lookups)
        self.dq.dqrm_dedupe_multi(self.tables, self.B, [(ix, of, self.sps[i], self.urs[i], self.sos[i], self.tuos[i],
                                                         self.nus[i], self.wss[i])], stream=stream,
                                  max_table_lookups=self.max_table_lookups)

    def dedupe_group(self, ks):
        """dqrm_dedupe_multi for the batches `ks` into the buffers k % nbuf."""
        n = self.nbuf
        self.dq.dqrm_dedupe_multi(self.tables, self.B, [self.batch_of(j) + (self.sps[j % n], self.urs[j % n], self.sos[j % n],
                                                                           self.tuos[j % n], self.nus[j % n], self.wss[j % n])
                                                       for j in ks], max_table_lookups=self.max_table_lookups)
        self._mark("dedupe_multi")

    def rest_of_step(self, k, i):
        """B3-B5 on the current stream, from the dedupe result in buffer i."""
        dq, b = self.dq, self.bufs
        g = self.grad_live if self.dense is not None else self.grad_d[k % len(self.grad_d)]
        if self.fused:
            dq.dqrm_segment_sum(self.tables, self.B, self.N, g, b.values, None, self.wss[i])
            self._mark("segment_sum")
            dq.dqrm_quant_update(self.tables, b.cap, self.N, b.values, self.urs[i], self.tuos[i], b.g_absmax, b.gq,
                                 b.g_scale, self.lr, self.wss[i])
            self._mark("quant_update")
        else:
            dq.dqrm_segment_sum(self.tables, self.B, self.N, g, b.values, b.g_absmax, self.wss[i])
            self._mark("segment_sum")
            dq.dqrm_grad_quant_int8(self.T, self.D, b.cap, b.values, self.tuos[i], b.g_absmax, b.gq, b.g_scale)
            self._mark("quant")
            dq.dqrm_sparse_update(self.tables, b.cap, self.urs[i], self.tuos[i], b.gq, b.g_scale, self.lr)
            self._mark("update")

    def run_steps(self, k0, n):
        """n consecutive steps starting with batch k0, all launches on the current stream (+ the side stream
        for dqrm_dedupe with overlap = "pipeline").  Self-contained: the side stream is joined at the end."""
        torch = self.torch
        main = torch.cuda.current_stream()
        if self.overlap == "ahead":
            for k in range(k0, k0 + n):
                if (k - k0) % self.nbuf == 0:  # dedupe of this and the next nbuf-1 batches, in one launch pair
                    self.dedupe_group(range(k, min(k + self.nbuf, k0 + n)))
                self.forward(k)
                self.rest_of_step(k, k % self.nbuf)
            return
        if self.overlap == "none":
            for k in range(k0, k0 + n):
                self.forward(k)
                self.dedupe(k, 0)
                self._mark("dedupe")
                self.rest_of_step(k, 0)
            return
        # "pipeline": dqrm_dedupe on the side stream, one step ahead
        side = self.side
        side.wait_stream(main)  # everything enqueued so far is visible to the side stream

        def dedupe_on_side(k):
            i = k % self.nbuf
            side.wait_event(self.ev_update[i])  # the buffer's previous reader (no-op before the first record)
            self.dedupe(k, i, stream=side)
            self.ev_dedupe[i].record(side)

        dedupe_on_side(k0)
        for k in range(k0, k0 + n):
            i = k % self.nbuf
            self.forward(k)
            if k + 1 < k0 + n:
                dedupe_on_side(k + 1)  # the next batch's indices are already here
            main.wait_event(self.ev_dedupe[i])
            self.rest_of_step(k, i)
            self.ev_update[i].record(main)
        main.wait_stream(side)

    def capture(self, k0, n):
        """The steps k0 .. k0+n-1 as one HIP graph (the library only launches kernels: no memset nodes)."""
        g = self.torch.cuda.CUDAGraph()
        with self.torch.cuda.graph(g):
            self.run_steps(k0, n)
        return g

    # ---- per-call times inside the step sequence -------------------------------------------------
    def time_calls_in_sequence(self, k0, n):
        """Runs n steps eagerly with one HIP event between consecutive calls, all recorded on the launch stream,
        and returns ({call: median microseconds between the events around it, corrected for the cost of an event
        pair itself}, {call: times it ran}, that cost).  The GPU is kept busy with large copies while the host
        enqueues, so the steps then run back to back as in the timed region and no interval holds host time."""
        torch = self.torch
        a = torch.empty(1 << 28, dtype=torch.float32, device=self.dev)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        for _ in range(40):  # ~15 ms of device-to-device copies: longer than the host needs to enqueue n steps
            b.copy_(a)
        self.probe = []
        self._mark("start")
        self.run_steps(k0, n)
        for _ in range(16):  # adjacent events with nothing in between
            self._mark("cal")
        probe, self.probe = self.probe, None
        torch.cuda.synchronize()
        del a, b
        spans = {}
        for (_, e0), (name, e1) in zip(probe[:-1], probe[1:]):
            spans.setdefault(name, []).append(1e3 * e0.elapsed_time(e1))
        # medians: an interval in which the GPU waited for the host (a step with many launches can outrun the gating
        # copies) is far out and must not count
        med = lambda v: sorted(v)[len(v) // 2]
        base = med(spans.pop("cal"))
        return {k: max(med(v) - base, 0.0) for k, v in spans.items()}, {k: len(v) for k, v in spans.items()}, base


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
                         "most 65536 lookups per batch (pooling 8 at the default batch)")
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
    ap.add_argument("--overlap", default="ahead", choices=["none", "pipeline", "ahead"],
                    help="where dqrm_dedupe (needs only the indices) runs: none = in line on the one stream; "
                         "pipeline = on a second stream, one step ahead (double-buffered workspace); ahead = in line on "
                         "the one stream, but for the next --ahead batches in one dqrm_dedupe_multi launch")
    ap.add_argument("--ahead", type=int, default=8, help="batches per dqrm_dedupe_multi launch with --overlap ahead")
    ap.add_argument("--two-call-update", dest="fused", action="store_false",
                    help="dqrm_grad_quant_int8 + dqrm_sparse_update (and the absmax fold inside dqrm_segment_sum) "
                         "instead of the one-pass dqrm_quant_update")
    ap.add_argument("--no-graph", dest="graph", action="store_false",
                    help="launch every kernel from the host instead of replaying a captured HIP graph")
    ap.add_argument("--simulated-nodes", type=int, default=1,
                    help="simulated data parallelism: the batch is cut into this many micro-batches (forward, backward "
                         "and INT8 codes each, with the first one's scale), their integer gradients are merged "
                         "(dqrm_sparse_merge) and the tables are updated once per step; all calls in line on one stream")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-master-leg", action="store_true", help="skip the short master-mode run reported beside the headline")
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
    t0 = time.time()
    pool = [wl.batch(k) if args.pooling == 1 else wl.batch(k, pooling="fixed", max_len=args.pooling)
            for k in range(args.pool)]
    grads = [wl.grad_normal(k) for k in range(args.grad_pool)]
    dense_args = dict(weight_bits=args.mlp_weight_bits, grad_bits=args.mlp_grad_bits, grad_pool=args.grad_pool) if args.dense else None
    hp = HotPath(wl, W, pool, grads, dev, mode=args.mode, overlap=args.overlap, ahead=args.ahead, fused=args.fused,
                 lr=args.lr, dense_args=dense_args, refresh_period=args.refresh_period)
    N = hp.N
    log(f"[bench] {args.pool} batches of {N} lookups + {args.grad_pool} grad_out in {time.time() - t0:.1f}s")
    hp.prepare()
    torch.cuda.synchronize()
    hp.step0 = args.warmup
    bufs, tables = hp.bufs, hp.tables

    nodes = args.simulated_nodes
    if nodes > 1:
        from gen import split_batch
        assert B % nodes == 0 and nodes <= dq.MAX_DEDUPE_BATCHES and not args.dense
        Bm = B // nodes
        parts = [split_batch(i, o, T, B, nodes) for i, o in pool]
        mb_idx = [[torch.from_numpy(i).to(dev) for i, _ in p] for p in parts]
        mb_off = [[torch.from_numpy(o).to(dev) for _, o in p] for p in parts]
        Nm = max(len(i) for p in parts for i, _ in p)
        mb_bound = int(Bm * max(int(np.diff(o).max()) for p in parts for _, o in p))  # lookups of one table, at most
        mb = [dq.StepBuffers(T, D, Bm, Nm, dev, want_codes=False) for _ in range(nodes)]
        m_cap = nodes * Nm
        m_rows = torch.empty(m_cap, dtype=torch.int64, device=dev)
        m_tuo = torch.empty(T + 1, dtype=torch.int32, device=dev)
        m_nu = torch.zeros(1, dtype=torch.int32, device=dev)
        m_sums = torch.empty((m_cap, D), dtype=torch.int32, device=dev)
        m_ws = torch.empty(dq.dqrm_sparse_merge_workspace_bytes(T, D, nodes, m_cap), dtype=torch.uint8, device=dev)

        def simulated_step(k):
            """One weight update from `nodes` micro-batches (appendix on simulated data parallelism)."""
            p, g = k % args.pool, hp.grad_d[k % args.grad_pool]
            # the micro-batches' indices are all there: one sort launch for all of them (26 x nodes workgroups)
            dq.dqrm_dedupe_multi(tables, Bm, [(mb_idx[p][j], mb_off[p][j], b.sorted_pos, b.uniq_rows, b.seg_offsets,
                                               b.table_uniq_offsets, b.num_unique, b.workspace) for j, b in enumerate(mb)],
                                 max_table_lookups=mb_bound)
            # the weights do not change inside a group and bags are independent: the micro-batches' forwards are one
            # call on the whole batch
            dq.dqrm_embbag_fwd(tables, hp.idx_d[p], hp.off_d[p], B, hp.mode, bufs.out, None)
            # segment sums and INT8 codes of all micro-batches in one launch each; only the first micro-batch's maxima
            # are used (its scale serves the whole group): the others ask for none
            dq.dqrm_segment_sum_multi(tables, Bm, [(mb_idx[p][j].numel(), g[j * Bm:(j + 1) * Bm], b.values,
                                                    b.g_absmax if j == 0 else None, b.workspace) for j, b in enumerate(mb)])
            dq.dqrm_grad_quant_int8_multi(T, D, [(b.values, b.table_uniq_offsets, mb[0].g_absmax, b.gq, b.g_scale) for b in mb])
            dq.dqrm_sparse_merge(tables, [(b.uniq_rows, b.table_uniq_offsets, b.gq) for b in mb], m_rows, m_tuo, m_nu,
                                 m_sums, m_ws)
            dq.dqrm_sparse_update_sums(tables, m_cap, m_rows, m_tuo, m_sums, mb[0].g_scale, args.lr)

        def run_steps(k0, n):
            for k in range(k0, k0 + n):
                simulated_step(k)
    else:
        run_steps = hp.run_steps

    # ---- warm-up (eager), optional capture of `graph_steps` steps into one HIP graph ----
    run_steps(0, args.warmup)
    torch.cuda.synchronize()
    graph, graph_steps = None, 0
    P = args.refresh_period
    if args.graph:
        graph_steps = min(args.pool, args.steps)
        if P > graph_steps:
            # the refresh runs eagerly before every (P / graph_steps)-th replay: the graph's length divides P
            graph_steps = max(d for d in range(1, graph_steps + 1) if P % d == 0)
            hp.refresh_in_steps = False
        elif P > 0:
            graph_steps = graph_steps // P * P
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
            if P > graph_steps and (rep * graph_steps) % P == 0:
                hp.refresh_scale()
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
    hp.refresh_in_steps = False  # the measurements below leave the scale alone

    # ---- unique rows per batch (for the algorithmic byte counts) ----
    us = []
    for k in range(min(args.pool, 16)):
        dq.dqrm_embbag_bwd(tables, hp.idx_d[k], hp.off_d[k], B, hp.grad_d[0], bufs.sorted_pos, bufs.uniq_rows,
                           bufs.seg_offsets, bufs.table_uniq_offsets, bufs.num_unique, bufs.values, bufs.g_absmax,
                           bufs.workspace)
        us.append(int(bufs.num_unique.cpu().item()))
    U = float(np.mean(us))
    packed_fwd = hp.mode == dq.FWD_PACKED
    ab = algorithmic_bytes(T, D, B, N, U, packed_fwd=packed_fwd, packed_mirror=True)

    # ---- every call's time INSIDE the step sequence (HIP events on the launch stream between the calls) ----
    kernels, roofline = [], None
    if nodes == 1:
        n_probe = 8 * max(args.ahead, 1) if args.overlap == "ahead" else 32
        call_us, call_n, ev_cost = hp.time_calls_in_sequence(args.warmup, n_probe)
        per_step = {k: call_us[k] * call_n[k] / n_probe for k in call_us}  # dedupe_multi runs once per --ahead steps
        log(f"[bench] per call, in sequence (us; an event pair costs {ev_cost:.2f}): "
            + ", ".join(f"{k}={call_us[k]:.2f}" + (f" (x{call_n[k]}/{n_probe} steps)" if call_n[k] != n_probe else "")
                        for k in call_us))
        G = 1
        while G < D // 4:
            G *= 2
        # which kernel(s) a call launches, and the algorithmic bytes of one launch
        dd = "dedupe_kernel + " + ("dedupe_merge_kernel + dedupe_large_kernel + " if N > 16384 and hp.max_table_lookups > 16384 else "") + "dedupe_finish_kernel"
        call_kernels = {
            "fwd": (f"embbag_fwd_kernel<{G},{'packed' if packed_fwd else 'master'}>", ab["fwd"]),
            "segment_sum": (f"segment_sum_kernel<{G}>" + ("" if args.fused else " + absmax_finalize_kernel"), ab["segsum"]),
            "quant_update": ("quant_update_kernel", ab["quant"] + ab["update"] - D * U),
            "quant": ("grad_quant_kernel", ab["quant"]),
            "update": ("sparse_update_kernel", ab["update"]),
            "dedupe": (dd, ab["dedupe"]),
            "dedupe_multi": (dd, ab["dedupe"] * max(args.ahead, 1)),
        }
        # The events between the calls take the dispatch gap that precedes every kernel out of the intervals (their own
        # cost, measured on adjacent events, is subtracted): the calls' times add up to less than the step.  A kernel
        # trace counts that gap as part of the kernel.  So does the roofline here: the step's time beyond the sum of
        # the calls, shared equally among the step's launches, is added to every launch.
        launches = lambda name: call_kernels[name][0].count("+") + 1
        gap_us = 0.0
        if all(k in call_kernels for k in call_us) and args.refresh_period == 0:
            per_step_launches = sum(launches(k) * call_n[k] / n_probe for k in call_us)
            gap_us = max(0.0, (ms_per_step * 1e3 - sum(per_step.values())) / per_step_launches)
        for name, us_events in call_us.items():
            if name not in call_kernels:
                continue
            kname, nbytes = call_kernels[name]
            us_call = us_events + gap_us * launches(name)
            gbs = nbytes / (us_call * 1e-6) / 1e9 if us_call > 0 else 0.0
            kernels.append({"call": name, "kernel": kname, "algorithmic_bytes_per_launch": int(nbytes),
                            "avg_launch_us": round(us_call, 2), "between_events_us": round(us_events, 2),
                            "us_per_step": round(us_call * call_n[name] / n_probe, 2),
                            "achieved_gbs": round(gbs, 1), "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4)})
        # the dominant kernel: the single-kernel call with the largest share of the step
        single = [k for k in kernels if "+" not in k["kernel"]]
        dom = max(single, key=lambda k: k["us_per_step"])
        roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["achieved_gbs"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": dom["frac_of_peak"], "traffic": read_traffic(dom["kernel"].split("<")[0]),
                    "algorithmic_bytes_per_launch": dom["algorithmic_bytes_per_launch"],
                    "avg_launch_us": dom["avg_launch_us"], "dispatch_gap_us": round(gap_us, 2),
                    "share_of_step": round(dom["us_per_step"] / sum(k["us_per_step"] for k in kernels), 4),
                    "how": "HIP events on the launch stream between consecutive calls of the step sequence, plus the "
                           "dispatch gap per launch (step time beyond the sum of the calls / launches per step), "
                           "which a kernel trace counts inside the kernel"}
        log(f"[bench] dispatch gap {gap_us:.2f} us per launch; dominant kernel {dom['kernel']}: {dom['avg_launch_us']:.2f} us, "
            f"{dom['achieved_gbs']:.0f} GB/s = {dom['frac_of_peak']:.3f} of peak")

    # ---- the master-mode forward beside the packed headline: a short run of the same steps ----
    master_leg = None
    if packed_fwd and nodes == 1 and not args.no_master_leg and not args.dense:
        hp.mode = dq.FWD_MASTER
        n_m = min(args.pool, args.steps, 64)
        gm = hp.capture(args.warmup, n_m) if args.graph else None
        (gm.replay() if gm is not None else hp.run_steps(args.warmup, n_m))
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        reps = max(1, min(args.steps, 640) // n_m)
        for _ in range(reps):
            (gm.replay() if gm is not None else hp.run_steps(args.warmup, n_m))
        torch.cuda.synchronize()
        ms_m = (time.perf_counter() - t1) * 1e3 / (reps * n_m)
        abm = algorithmic_bytes(T, D, B, N, U, packed_fwd=False, packed_mirror=True)
        master_leg = {"fwd_mode": "master", "steps": reps * n_m, "ms_per_step": round(ms_m, 5),
                      "value": round(N / (ms_m * 1e-3), 1), "unit": "lookups/s",
                      "step_algorithmic_bytes": int(abm["step"]),
                      "step_hbm_frac_of_peak": round(abm["step"] / (ms_m * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        hp.mode = dq.FWD_PACKED
        log(f"[bench] master-mode forward, same steps: {ms_m * 1e3:.1f} us/step")

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
    if roofline is not None:
        roofline["frac_of_copy_bw"] = round(roofline["achieved"] / copy_gbs, 4)  # against what a plain copy reaches here

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
                   "lookups_per_step": N, "unique_rows_per_step": round(U, 1), "fwd_mode": args.mode, "overlap": args.overlap,
                   "scale_refresh_period": args.refresh_period, "pooling": args.pooling, "dense_part": bool(args.dense),
                   "mlp_weight_bits": args.mlp_weight_bits, "mlp_grad_bits": args.mlp_grad_bits, "simulated_nodes": nodes,
                   "update": ("dqrm_quant_update (one pass)" if args.fused else "dqrm_grad_quant_int8 + dqrm_sparse_update"),
                   "launch": (f"HIP graph of {graph_steps} steps replayed" if graph is not None else "eager launches")},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "step_algorithmic_bytes": int(ab["step"]),
        "step_hbm_gbs": round(step_gbs, 1),
        "step_hbm_frac_of_peak": round(step_gbs / HBM_PEAK_GBS, 4),
        "kernels": kernels,
        "master_mode": master_leg,
        "event_ms_per_step": round(ev_ms / args.steps, 5),
        "copy_bw_gbs": round(copy_gbs, 1),
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
