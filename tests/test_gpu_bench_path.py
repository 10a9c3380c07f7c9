"""The launch sequence bench.py times, at the benchmark's full size, against the oracle.

bench.HotPath is the object the benchmark drives: Terabyte-shaped tables, packed-mode forward,
dqrm_dedupe_multi for the next 8 batches in one launch, then per step dqrm_embbag_fwd ->
dqrm_segment_sum(g_absmax = NULL) -> dqrm_quant_update, captured into one HIP graph and replayed.
Here a graph of 16 steps is replayed twice (the second replay starts from the tables the first one
left, with the program's own copies and synchronisations in between); after each replay the master
table, the packed mirror, the last step's forward output, INT8 codes, scales, maxima and unique rows
must equal the oracle's after the same steps, bit for bit."""
import numpy as np
import pytest

from gen import make_workload
from helpers import assert_exact

pytestmark = pytest.mark.gpu

STEPS = 16  # two dqrm_dedupe_multi groups of 8


def test_benchmark_launch_sequence_at_full_size(oracle):
    import torch
    import bench

    wl = make_workload("terabyte")
    print(f"bench path: terabyte-shaped, R={wl.R}, {STEPS} steps per graph replay", flush=True)
    W = wl.tables()
    pool = [wl.batch(k) for k in range(STEPS)]
    grads = [wl.grad_normal(k) for k in range(3)]  # (cycled with another period than the batches)
    dev = torch.device("cuda:0")
    hp = bench.HotPath(wl, W, pool, grads, dev, mode="packed", overlap="ahead", ahead=8, fused=True, lr=0.1)
    hp.prepare()
    graph = hp.capture(0, STEPS)  # capturing launches nothing
    torch.cuda.synchronize()

    Wo = W  # the oracle steps the host copy in place
    s = oracle.find_scale(Wo, wl.row_offsets)
    po = oracle.pack_int4(Wo, wl.row_offsets, s)
    assert_exact(hp.tables.w_scale.cpu().numpy().view(np.uint32), s.view(np.uint32), "w_scale bits")

    b = hp.bufs
    for replay in range(2):
        graph.replay()
        torch.cuda.synchronize()
        for k in range(STEPS):
            idx, off = pool[k]
            g = grads[k % len(grads)]
            out_o, _ = oracle.embbag_fwd(Wo, po, wl.row_offsets, s, wl.B, idx, off, mode=1, want_codes=False)
            o = oracle.embbag_bwd(wl.T, wl.D, wl.B, idx, off, g)
            gq_o, gs_o = oracle.grad_quant_int8(wl.T, wl.D, o["values"], o["table_uniq_offsets"], o["g_absmax"])
            oracle.sparse_update(Wo, po, wl.row_offsets, s, o["uniq_rows"], o["table_uniq_offsets"], gq_o, gs_o, 0.1)
        what = f"replay {replay}"
        # the last step's outputs (the dedupe results of step k live in buffer k % 8)
        i = (STEPS - 1) % hp.nbuf
        U = int(hp.nus[i].cpu().item())
        assert U == o["U"], (what, U, o["U"])
        assert_exact(hp.urs[i].cpu().numpy()[:U], o["uniq_rows"], what + " uniq_rows")
        assert_exact(hp.tuos[i].cpu().numpy(), o["table_uniq_offsets"], what + " table_uniq_offsets")
        assert_exact(hp.sos[i].cpu().numpy()[:U + 1], o["seg_offsets"], what + " seg_offsets")
        assert_exact(b.out.cpu().numpy().view(np.uint32), out_o.view(np.uint32), what + " out bits")
        assert_exact(b.values.cpu().numpy()[:U].view(np.uint32), o["values"].view(np.uint32), what + " values bits")
        assert_exact(b.g_absmax.cpu().numpy().view(np.uint32), o["g_absmax"].view(np.uint32), what + " g_absmax bits")
        assert_exact(b.g_scale.cpu().numpy().view(np.uint32), gs_o.view(np.uint32), what + " g_scale bits")
        assert_exact(b.gq.cpu().numpy()[:U], gq_o, what + " INT8 codes")
        # the state all 16 steps built
        assert_exact(hp.packed.cpu().numpy(), po, what + " packed bytes")
        Wg = hp.master.cpu().numpy()
        assert_exact(Wg.view(np.uint32), Wo.view(np.uint32), what + " master bits")
        del Wg
    code, tb, val = hp.dq.dqrm_check_status()
    assert code == 0, (code, tb, val)
