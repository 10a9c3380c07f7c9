"""dqrm_embbag_bwd_noalloc (the entry point for callers that cannot allocate: its scratch is an array
built into the library) against dqrm_embbag_bwd on a caller-provided workspace: every output bit for
bit, on two calls in a row, the second with a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest

from gen import Workload
from helpers import assert_exact

pytestmark = pytest.mark.gpu


def _outputs(b, N):
    U = int(b.num_unique.cpu().item())
    return dict(U=np.array([U]), sorted_pos=b.sorted_pos.cpu().numpy()[:N], uniq_rows=b.uniq_rows.cpu().numpy()[:U],
                seg_offsets=b.seg_offsets.cpu().numpy()[:U + 1], table_uniq_offsets=b.table_uniq_offsets.cpu().numpy(),
                values=b.values.cpu().numpy()[:U].view(np.uint32), g_absmax=b.g_absmax.cpu().numpy().view(np.uint32))


def _both_ways(wl, idx, off, grad, what):
    import torch
    import paper_2410_20046_amd as dq

    dev = torch.device("cuda:0")
    N = len(idx)
    W = wl.tables(threads=1)
    tables = dq.Tables(wl.row_offsets, wl.D, torch.from_numpy(W).to(dev))
    ix, of, g = (torch.from_numpy(a).to(dev) for a in (idx, off, grad))
    assert dq.dqrm_embbag_bwd_workspace_bytes(wl.T, wl.D, wl.B, N) <= dq.NOALLOC_SCRATCH_BYTES
    ref, got = dq.StepBuffers(wl.T, wl.D, wl.B, N, dev), dq.StepBuffers(wl.T, wl.D, wl.B, N, dev)
    print(f"{what}: T={wl.T} D={wl.D} B={wl.B} N={N}", flush=True)
    dq.dqrm_embbag_bwd(tables, ix, of, wl.B, g, ref.sorted_pos, ref.uniq_rows, ref.seg_offsets, ref.table_uniq_offsets,
                       ref.num_unique, ref.values, ref.g_absmax, ref.workspace)
    dq.dqrm_embbag_bwd_noalloc(tables, ix, of, wl.B, g, got.sorted_pos, got.uniq_rows, got.seg_offsets,
                               got.table_uniq_offsets, got.num_unique, got.values, got.g_absmax)
    torch.cuda.synchronize()
    r, o = _outputs(ref, N), _outputs(got, N)
    assert r["U"][0] > 0
    for k in r:
        assert_exact(o[k], r[k], f"{what} {k}")
    code, tb, val = dq.dqrm_check_status()
    assert code == 0, (what, code, tb, val)


def test_noalloc_matches_workspace_entry_point_twice():
    # first call: hot rows (segments of many chunks) next to large tables, several tiles, ragged bags
    cards = np.array([3, 17, 5000, 40, 250000, 1], np.int64)
    big = Workload(name="noalloc-a", T=6, D=64, B=2048, alpha=1.2, seed=91, cards=cards)
    idx, off = big.batch(0, pooling="ragged", max_len=3)
    _both_ways(big, idx, off, big.grad_normal(0), "first call")
    # second call, smaller input, other dim: the array still holds the first call's lists
    small = Workload(name="noalloc-b", T=3, D=24, B=333, alpha=1.05, seed=92, cards=np.array([211, 9, 4000], np.int64))
    idx, off = small.batch(1)
    _both_ways(small, idx, off, small.grad_normal(1), "second call")
