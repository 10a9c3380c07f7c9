"""Pin of the dense-part oracle (CPU only): the same network written with torch float64 tensors and
autograd -- an independent library implementation of linear layers, ReLU, batched dot products, sigmoid
and binary cross-entropy -- must give the same loss, the same gradient w.r.t. the pooled embeddings and the
same parameters after one SGD step.  Mistakes this catches: a transposed weight, a missing ReLU mask, the
wrong triangle or order of the interaction, a wrong sign or 1/B factor, weights updated before use."""
import numpy as np
import pytest
import torch

from gen import make_dense_model, dense_batch


def _torch_reference(bot_w, bot_b, top_w, top_b, x, emb, y, lr):
    t64 = lambda a: torch.tensor(np.asarray(a, np.float64), dtype=torch.float64, requires_grad=True)
    BW, BB, TW, TB = [list(map(t64, l)) for l in (bot_w, bot_b, top_w, top_b)]
    X = torch.tensor(np.asarray(x, np.float64))
    E = t64(emb)
    Y = torch.tensor(np.asarray(y, np.float64))
    h = X
    for W, b in zip(BW, BB):
        h = torch.relu(torch.nn.functional.linear(h, W, b))
    B, T, D = E.shape
    Z = torch.cat([h[:, None, :], E], dim=1)  # [B, V, D]
    G = torch.bmm(Z, Z.transpose(1, 2))  # all pairwise dots
    li, lj = np.tril_indices(T + 1, k=-1)  # strictly lower triangle, row-major
    R = torch.cat([h, G[:, li, lj]], dim=1)
    t = R
    for k, (W, b) in enumerate(zip(TW, TB)):
        t = torch.nn.functional.linear(t, W, b)
        if k + 1 < len(TW):
            t = torch.relu(t)
    loss = torch.nn.functional.binary_cross_entropy(torch.sigmoid(t[:, 0]), Y, reduction="mean")
    loss.backward()
    upd = lambda ps: [(p - lr * p.grad).detach().numpy() for p in ps]
    return float(loss), E.grad.numpy(), upd(BW), upd(BB), upd(TW), upd(TB)


@pytest.mark.parametrize("T,D,B", [(3, 16, 9), (5, 8, 33)])
def test_dense_oracle_matches_torch_autograd(oracle, T, D, B):
    bot_dims, bw, bb, top_dims, tw, tb = make_dense_model("small" if D == 16 else "small8", T, D, seed=7)
    x, y = dense_batch(B, bot_dims[0], seed=7, k=0)
    rng = np.random.default_rng(3)
    emb = (rng.standard_normal((B, T, D)) * 0.3).astype(np.float32)
    lr = 0.1
    ref = _torch_reference(bw, bb, tw, tb, x, emb, y, lr)
    f64 = lambda l: [np.ascontiguousarray(a, np.float64) for a in l]
    BW, BB, TW, TB = f64(bw), f64(bb), f64(tw), f64(tb)
    loss, grad = oracle.dense_step(bot_dims, BW, BB, top_dims, TW, TB, x, emb, y, lr)
    assert abs(loss - ref[0]) < 1e-12
    np.testing.assert_allclose(grad, ref[1], rtol=1e-10, atol=1e-14)
    for got, exp in zip(BW + BB + TW + TB, ref[2] + ref[3] + ref[4] + ref[5]):
        np.testing.assert_allclose(got, exp, rtol=1e-10, atol=1e-14)
    assert np.abs(grad).max() > 0  # the check is not vacuous


def test_interaction_width_matches_paper(oracle):
    """26 tables of width 16 -> 16 + 27*26/2 = 367 inputs to the top MLP (the paper's Kaggle top MLP takes
    the 367-wide interaction output)."""
    bot_dims, bw, bb, top_dims, tw, tb = make_dense_model("kaggle", 26, 16, seed=1005)
    assert top_dims == [367, 512, 256, 1] and bot_dims == [13, 512, 256, 64, 16]
    n_params = sum(w.size for w in bw + tw) + sum(b.size for b in bb + tb)
    assert n_params == 475985  # ~1.90 MB of fp32: 95 % of the paper's 2.01 MB sparse-gradient message
