"""Pins for the oracle's loading step, GraphSAGE forward and backward.

  * gather == table[ids] (an independent library routine);
  * mean aggregation == D^-1 A H with a dense block adjacency matrix;
  * the whole forward == an independent dense expression on GLOBAL vertex ids (no frontiers, no
    relabelling, no shuffle index) built from the sampled edge list;
  * split-parallel logits and weight gradients == the unsplit mini-batch's (the paper's "no
    algorithmic bias" claim);
  * backward == central finite differences of the loss, and == torch.autograd on the dense
    expression;
  * bfloat16 rounding == torch's conversion."""
import numpy as np
import pytest
import torch

import workloads
from oracle import reference as R


def _np(t):
    return t.cpu().numpy()


@pytest.fixture(scope="module")
def small():
    w = workloads.custom(600, 6000, dims=[12, 10, 9, 5], fanouts=[4, 3, 2], batch=40, n_splits=3,
                         name="sage-small")
    ip, ix, pm = _np(w.indptr).astype(np.int64), _np(w.indices), _np(w.pmap)
    tg = _np(w.targets(0))
    b = R.sp_sample(ip, ix, pm, 3, w.fanouts, tg, seed=21, it=1)
    u = R.sp_sample(ip, ix, np.zeros_like(pm), 1, w.fanouts, tg, seed=21, it=1)
    p = R.SageParams([_np(x) for x in w.w_self], [_np(x) for x in w.w_neigh], [_np(x) for x in w.bias])
    return w, ip, ix, pm, tg, b, u, p


def test_gather_is_index_select(small):
    w, *_ = small
    table = _np(w.feat)
    ids = np.array([5, 0, 599, 5, 17], np.int32)
    assert (R.gather_rows(table, ids) == table[ids]).all()
    t16 = w.feat.to(torch.bfloat16).view(torch.int16).numpy()
    assert (R.gather_rows(t16, ids) == t16[ids]).all()
    assert R.gather_rows(table, np.empty(0, np.int32)).shape == (0, table.shape[1])


def test_mean_aggregate_is_normalised_adjacency_product(small):
    w, ip, ix, pm, tg, b, u, p = small
    rng = np.random.default_rng(0)
    for blk in (b.blocks[0][1], b.blocks[2][0], u.blocks[1][0]):
        n_dst, n_src = blk.dst.shape[0], blk.mixed_front.shape[0]
        H = rng.standard_normal((n_src, 7))
        A = np.zeros((n_dst, n_src))
        for i in range(n_dst):
            for e in range(blk.blk_indptr[i], blk.blk_indptr[i + 1]):
                A[i, blk.blk_src[e]] += 1.0
        deg = A.sum(1, keepdims=True)
        want = np.where(deg > 0, A / np.maximum(deg, 1), 0.0) @ H
        got = R.mean_aggregate(blk.blk_indptr, blk.blk_src, H)
        assert np.allclose(got, want, rtol=1e-13, atol=1e-13)
        # adjoint: <A H, G> == <H, A^T G>
        G = rng.standard_normal(got.shape)
        adj = R.mean_aggregate_adjoint(blk.blk_indptr, blk.blk_src, G, n_src)
        assert np.isclose((got * G).sum(), (H * adj).sum(), rtol=1e-12)


def _global_edges(batch, l):
    out = []
    for blk in batch.blocks[l]:
        out.append(np.stack([np.repeat(blk.dst, blk.cnt), blk.mixed_front[blk.blk_src]], 1))
    return np.concatenate(out)


def _dense_forward_torch(n_vertices, batch, feat, params, tg):
    """GraphSAGE on global ids with dense [V x V] operators: no frontier bookkeeping at all."""
    L = batch.n_layers
    H = torch.zeros((n_vertices, feat.shape[1]), dtype=torch.float64)
    H[:] = torch.from_numpy(feat.astype(np.float64))
    Ws = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in params.w_self]
    Wn = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in params.w_neigh]
    B = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in params.bias]
    for l in range(L):
        e = _global_edges(batch, l)
        A = torch.zeros((n_vertices, n_vertices), dtype=torch.float64)
        A.index_put_((torch.from_numpy(e[:, 0]).long(), torch.from_numpy(e[:, 1]).long()),
                     torch.ones(e.shape[0], dtype=torch.float64), accumulate=True)
        deg = A.sum(1, keepdim=True)
        M = (A / deg.clamp(min=1)) @ H
        Z = H @ Ws[l] + M @ Wn[l] + B[l]
        H = Z if l == L - 1 else torch.relu(Z)
    return H[torch.from_numpy(tg).long()], Ws, Wn, B


def test_forward_backward_match_dense_autograd(small):
    w, ip, ix, pm, tg, b, u, p = small
    feat = _np(w.feat)
    lab = _np(w.labels)
    fwd = R.sp_forward(b, R.gather_rows(feat, b.local_cat(0)), p)
    order = tg[b.target_perm]
    logits_t, Ws, Wn, B = _dense_forward_torch(w.n_vertices, b, feat, p, order)
    assert np.allclose(fwd.logits, logits_t.detach().numpy(), rtol=1e-11, atol=1e-12)
    loss, g = R.softmax_xent(fwd.logits, lab[order])
    loss_t = torch.nn.functional.cross_entropy(logits_t, torch.from_numpy(lab[order]))
    assert np.isclose(loss, float(loss_t.detach()), rtol=1e-12)
    loss_t.backward()
    bwd = R.sp_backward(b, fwd, p, g)
    for l in range(w.n_layers):
        assert np.allclose(bwd.gw_self[l], Ws[l].grad.numpy(), rtol=1e-9, atol=1e-13)
        assert np.allclose(bwd.gw_neigh[l], Wn[l].grad.numpy(), rtol=1e-9, atol=1e-13)
        assert np.allclose(bwd.gbias[l], B[l].grad.numpy(), rtol=1e-9, atol=1e-13)


def test_split_equals_unsplit(small):
    w, ip, ix, pm, tg, b, u, p = small
    feat, lab = _np(w.feat), _np(w.labels)
    fs = R.sp_forward(b, R.gather_rows(feat, b.local_cat(0)), p)
    fu = R.sp_forward(u, R.gather_rows(feat, u.local_cat(0)), p)
    # bring both back to the caller's target order
    ls = np.empty_like(fs.logits); ls[b.target_perm] = fs.logits
    lu = np.empty_like(fu.logits); lu[u.target_perm] = fu.logits
    assert np.allclose(ls, lu, rtol=1e-12, atol=1e-13)
    _, g = R.softmax_xent(lu, lab[tg])
    bs = R.sp_backward(b, fs, p, g[b.target_perm])
    bu = R.sp_backward(u, fu, p, g[u.target_perm])
    for l in range(w.n_layers):
        assert np.allclose(bs.gw_self[l], bu.gw_self[l], rtol=1e-10, atol=1e-14)
        assert np.allclose(bs.gw_neigh[l], bu.gw_neigh[l], rtol=1e-10, atol=1e-14)
        assert np.allclose(bs.gbias[l], bu.gbias[l], rtol=1e-10, atol=1e-14)


def test_backward_matches_finite_differences(small):
    w, ip, ix, pm, tg, b, u, p = small
    feat, lab = _np(w.feat), _np(w.labels)
    x0 = R.gather_rows(feat, b.local_cat(0))
    y = lab[tg[b.target_perm]]

    def loss_of(params):
        return R.softmax_xent(R.sp_forward(b, x0, params).logits, y)[0]

    fwd = R.sp_forward(b, x0, p)
    bwd = R.sp_backward(b, fwd, p, R.softmax_xent(fwd.logits, y)[1])
    rng = np.random.default_rng(3)
    eps = 1e-6
    for l in range(w.n_layers):
        for name, grads in (("w_self", bwd.gw_self), ("w_neigh", bwd.gw_neigh), ("bias", bwd.gbias)):
            arr = getattr(p, name)[l]
            for _ in range(4):
                idx = tuple(rng.integers(0, n) for n in arr.shape)
                q = R.SageParams([a.astype(np.float64).copy() for a in p.w_self],
                                 [a.astype(np.float64).copy() for a in p.w_neigh],
                                 [a.astype(np.float64).copy() for a in p.bias])
                getattr(q, name)[l][idx] += eps
                up = loss_of(q)
                getattr(q, name)[l][idx] -= 2 * eps
                dn = loss_of(q)
                fd = (up - dn) / (2 * eps)
                assert abs(fd - grads[l][idx]) <= 1e-6 * max(1.0, abs(fd)) + 1e-8, (name, l, idx)


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(5000).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 5000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38], np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert (R.to_bf16_rne(x).view(np.uint32) == want.view(np.uint32)).all()


def test_bf16_storage_forward_close_to_fp32(small):
    w, ip, ix, pm, tg, b, u, p = small
    x0 = R.gather_rows(_np(w.feat), b.local_cat(0))
    a = R.sp_forward(b, x0, p).logits
    c = R.sp_forward(b, x0, p, store_bf16=True).logits
    err = np.abs(c - a).max() / np.abs(a).max()      # bf16 keeps 8 significant bits
    assert 0 < err < 2e-2


def test_relu_decision_slack_bounds_a_flipped_decision(small):
    """The slack must cover what flipping the most nearly undecided ReLU does to the gradients,
    and must vanish when no pre-activation is near zero."""
    w, ip, ix, pm, tg, b, u, p = small
    feat, lab = _np(w.feat), _np(w.labels)
    x0 = R.gather_rows(feat, b.local_cat(0))
    y = lab[tg[b.target_perm]]
    fwd = R.sp_forward(b, x0, p)
    g = R.softmax_xent(fwd.logits, y)[1]
    bwd = R.sp_backward(b, fwd, p, g)
    sws, swn, sb, n0 = R.relu_decision_slack(b, fwd, p, bwd, rel_tau=0.0)
    assert n0 == 0 and all(float(x.max()) == 0.0 for x in sws + swn + sb)
    # flip the decision of the entry of layer 0 closest to zero and recompute the gradients
    l, s = 0, 1
    z = fwd.z[l][s]
    i, c = np.unravel_index(np.abs(z).argmin(), z.shape)
    tau = float(np.abs(z[i, c])) / max(float(np.abs(zz).max()) for zz in fwd.z[l]) * 1.0001
    sws, swn, sb, n1 = R.relu_decision_slack(b, fwd, p, bwd, rel_tau=tau)
    assert n1 >= 1
    flipped = R.Forward(fwd.logits, fwd.hidden, fwd.mixed, fwd.mean, [[zz.copy() for zz in row] for row in fwd.z])
    flipped.z[l][s][i, c] = -z[i, c]
    bwd2 = R.sp_backward(b, flipped, p, g)
    for k in range(w.n_layers):
        assert (np.abs(bwd2.gw_self[k] - bwd.gw_self[k]) <= sws[k] * (1 + 1e-9) + 1e-18).all()
        assert (np.abs(bwd2.gw_neigh[k] - bwd.gw_neigh[k]) <= swn[k] * (1 + 1e-9) + 1e-18).all()
        assert (np.abs(bwd2.gbias[k] - bwd.gbias[k]) <= sb[k] * (1 + 1e-9) + 1e-18).all()
    assert np.abs(bwd2.gw_self[0] - bwd.gw_self[0]).max() > 0
