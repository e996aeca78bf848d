"""Pins for the oracle's loading step, GraphSAGE forward and backward.

  * gather == table[ids] (an independent library routine);
  * mean aggregation == D^-1 A H with a dense block adjacency matrix;
  * the whole forward == an independent dense expression on GLOBAL vertex ids (no frontiers, no
    relabelling, no shuffle index) built from the sampled edge list;
  * split-parallel logits and weight gradients == the unsplit mini-batch's (the paper's "no
    algorithmic bias" claim);
  * backward == central finite differences of the loss, and == torch.autograd on the dense
    expression;
  * bfloat16 rounding == torch's conversion; the bf16-storage forward/backward == the dense
    expression under torch.autograd with the same rounding points;
  * ReLU decisions conditioned on a device's stored activations: taken from the device only inside
    the rounding band, counted as errors outside it; a planted 1 % error in a bottom-layer weight
    gradient is caught."""
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


def _fwd_bwd(small):
    w, ip, ix, pm, tg, b, u, p = small
    feat, lab = _np(w.feat), _np(w.labels)
    x0 = R.gather_rows(feat, b.local_cat(0))
    y = lab[tg[b.target_perm]]
    fwd = R.sp_forward(b, x0, p)
    g = R.softmax_xent(fwd.logits, y)[1]
    return fwd, g, R.sp_backward(b, fwd, p, g)


def test_conditioned_relu_masks_take_the_device_decision_only_inside_the_band(small):
    """The gradient check that replaces any tolerance for undecidable ReLU decisions: the oracle's
    backward pass takes the device's decision where |z| is below the forward pass's rounding
    noise and its own everywhere else, and counts disagreements outside the band."""
    w, ip, ix, pm, tg, b, u, p = small
    fwd, g, bwd = _fwd_bwd(small)
    L = w.n_layers
    # a device that stores exactly the oracle's activations: same decisions, same gradients
    act = [None] + [fwd.hidden[l].astype(np.float32) for l in range(1, L)]
    masks, rep = R.conditioned_relu_masks(b, fwd, act, rel_tau=1e-5)
    assert masks[L - 1] is None and all(r[1] == 0 and r[2] == 0 for r in rep)
    same = R.sp_backward(b, fwd, p, g, relu_mask=masks)
    for k in range(L):
        assert np.array_equal(same.gw_self[k], bwd.gw_self[k]) and np.array_equal(same.gbias[k], bwd.gbias[k])
    # the device decides the entry of layer 0 closest to zero the other way
    l, s = 0, 1
    z = fwd.z[l][s]
    i, c = np.unravel_index(np.abs(z).argmin(), z.shape)
    zmax = max(float(np.abs(zz).max()) for zz in fwd.z[l])
    tau = float(np.abs(z[i, c])) / zmax * 1.0001
    row = int(b.local_off(l + 1)[s]) + int(i)
    dev = [None if a is None else a.copy() for a in act]
    dev[l + 1][row, c] = 0.0 if z[i, c] > 0 else 1.0
    masks, rep = R.conditioned_relu_masks(b, fwd, dev, rel_tau=tau)
    assert rep[l][0] >= 1 and rep[l][1] == 1 and rep[l][2] == 0
    got = R.sp_backward(b, fwd, p, g, relu_mask=masks)
    flipped = R.Forward(fwd.logits, fwd.hidden, fwd.mixed, fwd.mean, [[zz.copy() for zz in r] for r in fwd.z])
    flipped.z[l][s][i, c] = -z[i, c] if z[i, c] != 0 else 1.0
    want = R.sp_backward(b, flipped, p, g)
    for k in range(L):
        assert np.array_equal(got.gw_self[k], want.gw_self[k])
        assert np.array_equal(got.gw_neigh[k], want.gw_neigh[k])
        assert np.array_equal(got.gbias[k], want.gbias[k])
    assert np.abs(got.gw_self[0] - bwd.gw_self[0]).max() > 0        # the decision matters
    # with a band too narrow to hold that entry the same disagreement is an error, not an excuse
    masks, rep = R.conditioned_relu_masks(b, fwd, dev, rel_tau=tau * 0.5)
    assert rep[l][2] == 1
    still = R.sp_backward(b, fwd, p, g, relu_mask=masks)
    assert np.array_equal(still.gw_self[0], bwd.gw_self[0])


def test_a_one_percent_error_in_a_bottom_layer_weight_gradient_is_caught(small):
    """What the elementwise 1e-4 check with no allowance must catch: 1 % on a single entry of the
    bottom layer's weight gradient (planted in the oracle's result, on the CPU)."""
    w, *_ = small
    fwd, g, bwd = _fwd_bwd(small)
    o = bwd.gw_self[0]
    assert R.max_rel_err(o.astype(np.float32), o) < 1e-6        # float32 storage alone passes
    big = np.unravel_index(np.abs(o).argmax(), o.shape)
    typical = np.unravel_index(np.argsort(np.abs(o).reshape(-1))[o.size // 2], o.shape)
    for idx in (big, typical):
        bad = o.copy()
        bad[idx] *= 1.01
        assert R.max_rel_err(bad, o) > 1e-4 or abs(o[idx]) < 1e-2 * np.abs(o).max()
    bad = o.copy()
    bad[big] *= 1.01
    assert R.max_rel_err(bad, o) > 50 * 1e-4
    bad = o.copy()
    bad[typical] += 0.01 * np.abs(o).max() * 0.011               # 1.1 % of the floor: just over 1e-4
    assert R.max_rel_err(bad, o) > 1e-4


class _RoundValue(torch.autograd.Function):
    """bfloat16 rounding of a stored value; the gradient passes unchanged."""
    @staticmethod
    def forward(ctx, x):
        return x.to(torch.float32).to(torch.bfloat16).to(torch.float64)

    @staticmethod
    def backward(ctx, gr):
        return gr


class _RoundGradient(torch.autograd.Function):
    """Identity whose incoming gradient is rounded to bfloat16 (dZ as a bf16 product operand)."""
    @staticmethod
    def forward(ctx, x):
        return x.view_as(x)

    @staticmethod
    def backward(ctx, gr):
        return gr.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def test_bf16_backward_matches_dense_autograd_with_the_same_rounding_points(small):
    """sp_forward / sp_backward(store_bf16=True) against an independent route: the dense global-id
    expression of the model under torch.autograd in float64, with bfloat16 rounding applied where
    the bf16 storage scheme stores a value (features, weights, the neighbourhood mean, activations
    between layers: value rounded, gradient passed through) and where a gradient becomes an
    operand of a bf16 product (dZ of every layer: rounded on the way back, so the weight, bias and
    input gradients all see the rounded dZ).  torch's own float32 -> bfloat16 conversion does the
    rounding here."""
    w, ip, ix, pm, tg, b, u, p = small
    feat, lab = _np(w.feat), _np(w.labels)
    L = w.n_layers
    order = tg[b.target_perm]
    rv, rg = _RoundValue.apply, _RoundGradient.apply
    H = rv(torch.from_numpy(feat.astype(np.float64)))
    Ws = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in p.w_self]
    Wn = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in p.w_neigh]
    B = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in p.bias]
    n = w.n_vertices
    for l in range(L):
        e = _global_edges(b, l)
        A = torch.zeros((n, n), dtype=torch.float64)
        A.index_put_((torch.from_numpy(e[:, 0]).long(), torch.from_numpy(e[:, 1]).long()),
                     torch.ones(e.shape[0], dtype=torch.float64), accumulate=True)
        M = rv((A / A.sum(1, keepdim=True).clamp(min=1)) @ H)
        Z = rg(H @ rv(Ws[l]) + M @ rv(Wn[l]) + B[l])
        H = Z if l == L - 1 else rv(torch.relu(Z))
    logits_t = H[torch.from_numpy(order).long()]
    fwd = R.sp_forward(b, R.gather_rows(feat, b.local_cat(0)), p, store_bf16=True)
    assert np.allclose(fwd.logits, logits_t.detach().numpy(), rtol=1e-11, atol=1e-12)
    _, g = R.softmax_xent(fwd.logits, lab[order])
    logits_t.backward(torch.from_numpy(g))
    bwd = R.sp_backward(b, fwd, p, g, store_bf16=True)
    plain = R.sp_backward(b, fwd, p, g)
    for l in range(L):
        assert np.allclose(bwd.gw_self[l], Ws[l].grad.numpy(), rtol=1e-9, atol=1e-13)
        assert np.allclose(bwd.gw_neigh[l], Wn[l].grad.numpy(), rtol=1e-9, atol=1e-13)
        assert np.allclose(bwd.gbias[l], B[l].grad.numpy(), rtol=1e-9, atol=1e-13)
    # the rounding of dZ is not a no-op on this batch: the pin distinguishes the two backward passes
    assert max(np.abs(bwd.gw_self[l] - plain.gw_self[l]).max() for l in range(L)) > 0
