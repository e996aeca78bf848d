"""Pins of the GAT oracle (the layer of Velickovic et al. that the paper's section 7.1 names, run
per split as Algorithm 2 prescribes): a hand-computed example, the uniform-attention special case,
finite differences for every parameter gradient, and split == unsplit."""
import numpy as np
import pytest

import workloads
from oracle import reference as R
from oracle import gat as G


def _params(rng, dims, heads, scale=0.4):
    L = len(heads)
    w, a_s, a_d, b = [], [], [], []
    for l in range(L):
        last = l == L - 1
        width = heads[l] * (dims[l + 1] if last else dims[l + 1] // heads[l])
        w.append(rng.standard_normal((dims[l], width)) * scale)
        a_s.append(rng.standard_normal(width) * scale)
        a_d.append(rng.standard_normal(width) * scale)
        b.append(rng.standard_normal(dims[l + 1]) * 0.1)
    return G.GatParams(list(heads), w, a_s, a_d, b)


def _batch(S=3, seed=1, it=0, pmap=None):
    w = workloads.custom(800, 9000, dims=[12, 8, 6], fanouts=[4, 3], batch=40, n_splits=S, name="gat-pin")
    pm = w.pmap.numpy() if pmap is None else pmap
    b = R.sp_sample(w.indptr.numpy(), w.indices.numpy(), pm, S, w.fanouts, w.targets(it).numpy(), seed, it)
    x0 = R.gather_rows(w.feat.numpy().astype(np.float64), b.local_cat(0))
    return w, b, x0


def test_hand_computed_single_edge():
    """One destination (vertex 0) with one sampled neighbour (vertex 1), one head, one feature:
    z_0 = 1, z_1 = 3, a_dst = 2, a_src = -1.  e_00 = LeakyReLU(2*1 - 1*1) = 1,
    e_01 = LeakyReLU(2*1 - 1*3) = -0.2, alpha = softmax(1, -0.2), out = alpha_0 * 1 + alpha_1 * 3."""
    indptr = np.array([0, 1, 1], np.int64)
    indices = np.array([1], np.int32)
    pmap = np.zeros(2, np.uint8)
    b = R.sp_sample(indptr, indices, pmap, 1, [5], np.array([0], np.int32), 3, 0)
    x0 = np.array([[1.0], [3.0]])[b.local_cat(0)]
    P = G.GatParams([1], [np.array([[1.0]])], [np.array([-1.0])], [np.array([2.0])], [np.array([0.25])])
    f = G.gat_forward(b, x0, P)
    a0 = np.exp(1.0) / (np.exp(1.0) + np.exp(-0.2))
    assert abs(f.logits[0, 0] - (a0 * 1.0 + (1 - a0) * 3.0 + 0.25)) < 1e-12


def test_zero_attention_vectors_give_the_mean_over_self_and_neighbours():
    rng = np.random.default_rng(3)
    w, b, x0 = _batch()
    P = _params(rng, [12, 8, 6], [2, 1])
    P.a_src = [np.zeros_like(a) for a in P.a_src]
    P.a_dst = [np.zeros_like(a) for a in P.a_dst]
    f = G.gat_forward(b, x0, P)
    # layer 0 recomputed from the definition of a neighbourhood mean, straight from the blocks
    for s in range(b.n_splits):
        blk = b.blocks[0][s]
        mixed = x0[blk.shuffle_src_row]
        for i in range(blk.dst.shape[0]):
            rows = [i] + list(blk.blk_src[blk.blk_indptr[i]:blk.blk_indptr[i + 1]])
            want = mixed[rows].mean(0) @ P.w[0] + P.bias[0]
            assert np.allclose(f.pre[0][s][i], want, atol=1e-12)


@pytest.mark.parametrize("heads", [[2, 1], [4, 3]])
def test_gradients_match_finite_differences(heads):
    rng = np.random.default_rng(11)
    w, b, x0 = _batch()
    P = _params(rng, [12, 8, 6], heads)
    g = rng.standard_normal((b.local_cat(2).shape[0], 6))
    f = G.gat_forward(b, x0, P)
    bw = G.gat_backward(b, f, P, g)
    loss = lambda: float((G.gat_forward(b, x0, P).logits * g).sum())
    eps = 1e-6
    for name, arrs, grads in (("w", P.w, bw.gw), ("a_src", P.a_src, bw.ga_src), ("a_dst", P.a_dst, bw.ga_dst),
                              ("bias", P.bias, bw.gbias)):
        for l in range(2):
            flat = arrs[l].reshape(-1)
            for idx in rng.choice(flat.shape[0], size=min(5, flat.shape[0]), replace=False):
                old = flat[idx]
                flat[idx] = old + eps; lp = loss()
                flat[idx] = old - eps; lm = loss()
                flat[idx] = old
                num = (lp - lm) / (2 * eps)
                ana = grads[l].reshape(-1)[idx]
                assert abs(num - ana) <= 1e-6 * max(1.0, abs(ana)), (name, l, idx, num, ana)


def test_split_equals_unsplit():
    rng = np.random.default_rng(5)
    P = _params(rng, [12, 8, 6], [2, 2])
    res = []
    for S in (1, 4):
        w, b, x0 = _batch(S=S, pmap=None if S == 4 else np.zeros(800, np.uint8))
        f = G.gat_forward(b, x0, P)
        order = np.argsort(b.local_cat(2), kind="stable")           # rows by vertex id
        g = np.sin(np.arange(f.logits.size)).reshape(f.logits.shape)[np.argsort(order)]   # same per vertex
        bw = G.gat_backward(b, f, P, g)
        res.append((f.logits[order], bw))
    assert np.allclose(res[0][0], res[1][0], atol=1e-10)
    for l in range(2):
        assert np.allclose(res[0][1].gw[l], res[1][1].gw[l], atol=1e-9)
        assert np.allclose(res[0][1].ga_src[l], res[1][1].ga_src[l], atol=1e-9)
        assert np.allclose(res[0][1].ga_dst[l], res[1][1].ga_dst[l], atol=1e-9)
        assert np.allclose(res[0][1].gbias[l], res[1][1].gbias[l], atol=1e-9)


def _local_terms(b, f, p, l):
    """What a device stores per row of local_cat[l]: a_src . z and a_dst . z per head, in float32."""
    K = p.heads[l]
    W = np.asarray(p.w[l], np.float64)
    F = W.shape[1] // K
    z = (f.hidden[l] @ W).reshape(-1, K, F)
    src = (z * np.asarray(p.a_src[l]).reshape(K, F)).sum(2).astype(np.float32)
    dst = (z * np.asarray(p.a_dst[l]).reshape(K, F)).sum(2).astype(np.float32)
    return src, dst


def test_conditioned_slopes_and_gradient_term_magnitudes():
    """The two things the GPU tests take from the oracle besides its results.  (i) LeakyReLU slope
    decisions conditioned on a device's stored score terms: with the oracle's own terms nothing
    changes; a score inside the band that the device puts on the other side of zero takes the
    device's slope (the gradients then equal those of a run whose score has that sign); outside the
    band the same disagreement is counted as an error.  Hand example: scores 2*1 - 1*1 = 1 and
    2*1 + a_src*3, which a_src = -2/3 puts at zero.  (ii) The term magnitudes bound the attention
    gradients entry by entry and are not a loose bound where nothing cancels."""
    rng = np.random.default_rng(5)
    w, b, x0 = _batch()
    p = _params(rng, w.dims, [2, 1])
    f = G.gat_forward(b, x0, p)
    g = rng.standard_normal(f.logits.shape)
    bw = G.gat_backward(b, f, p, g)
    terms = [_local_terms(b, f, p, l) for l in range(2)]
    slopes, rep = G.conditioned_slopes(b, f, p, terms, rel_tau=1e-6)
    assert all(r[1] == 0 and r[2] == 0 for r in rep)
    same = G.gat_backward(b, f, p, g, slope_positive=slopes)
    for l in range(2):
        assert np.array_equal(same.gw[l], bw.gw[l]) and np.array_equal(same.ga_src[l], bw.ga_src[l])
    # the device's dst term of one destination is shifted so that its smallest score changes sign
    l, s = 0, 0
    blk = b.blocks[l][s]
    K = p.heads[l]
    F = np.shape(p.w[l])[1] // K
    z = f.z[l][s]
    e_src = (z * np.asarray(p.a_src[l]).reshape(K, F)).sum(2)
    e_dst = (z * np.asarray(p.a_dst[l]).reshape(K, F)).sum(2)
    i = int(np.argmax(blk.cnt))          # a destination with several neighbours: its softmax has a gradient
    assert blk.cnt[i] >= 2
    nbrs = np.concatenate([[i], blk.blk_src[blk.blk_indptr[i]:blk.blk_indptr[i + 1]]]).astype(np.int64)
    raw = e_dst[i][None, :] + e_src[nbrs]
    j, k = np.unravel_index(np.abs(raw).argmin(), raw.shape)
    dev = [(t[0].copy(), t[1].copy()) for t in terms]
    dev[l][1][blk.shuffle_src_row[i], k] -= np.float32(2.0 * raw[j, k])
    slopes, rep = G.conditioned_slopes(b, f, p, dev, rel_tau=1.0)     # band = everything: the device decides
    assert rep[l][1] >= 1 and rep[l][2] == 0
    assert bool(slopes[l][s][i][j, k]) == (not raw[j, k] > 0.0)
    got = G.gat_backward(b, f, p, g, slope_positive=slopes)
    assert np.abs(got.ga_src[l] - bw.ga_src[l]).max() > 0
    slopes0, rep0 = G.conditioned_slopes(b, f, p, dev, rel_tau=0.0)   # no band: every disagreement is an error
    assert rep0[l][2] >= 1 and bool(slopes0[l][s][i][j, k]) == bool(raw[j, k] > 0.0)
    # hand example: with a_src = -2/3 the second score is 2 - 2 = 0; a device that computed +1e-9 there
    indptr = np.array([0, 1, 1], np.int64)
    indices = np.array([1], np.int32)
    hb = R.sp_sample(indptr, indices, np.zeros(2, np.uint8), 1, [5], np.array([0], np.int32), 3, 0)
    hx = np.array([[1.0], [3.0]])[hb.local_cat(0)]
    hp = G.GatParams([1], [np.array([[1.0]])], [np.array([-2.0 / 3.0])], [np.array([2.0])], [np.array([0.0])])
    hf = G.gat_forward(hb, hx, hp)
    rows = {int(v): r for r, v in enumerate(hb.local_cat(0))}
    src = np.zeros((2, 1), np.float32); dst = np.zeros((2, 1), np.float32)
    src[rows[0]], src[rows[1]] = -2.0 / 3.0, -2.0
    dst[rows[0]], dst[rows[1]] = 2.0, 6.0
    src[rows[1]] = np.float32(-2.0) + np.float32(1e-6)
    hs, hrep = G.conditioned_slopes(hb, hf, hp, [(src, dst)], rel_tau=1e-5)
    assert hrep[0] == (1, 1, 0)
    assert hs[0][0][0].reshape(-1).tolist() == [True, True]
    g1 = np.array([[1.0]])
    own = G.gat_backward(hb, hf, hp, g1)
    cond = G.gat_backward(hb, hf, hp, g1, slope_positive=hs)
    # slope 1 instead of 0.2 on the neighbour's score: its share of d a_src grows fivefold
    a = hf.alpha[0][0][0][:, 0]
    da = np.array([1.0, 3.0]) * 1.0
    de = a * (da - (a * da).sum())
    assert np.isclose(own.ga_src[0][0], de[0] * 1.0 * 1.0 + de[1] * 0.2 * 3.0)
    assert np.isclose(cond.ga_src[0][0], de[0] * 1.0 * 1.0 + de[1] * 1.0 * 3.0)
    for l in range(2):
        t = bw.ga_terms[l].reshape(-1)
        assert np.all(np.abs(bw.ga_src[l].reshape(-1)) <= t * (1 + 1e-12))
        assert np.all(np.abs(bw.ga_dst[l].reshape(-1)) <= t * (1 + 1e-12))
        assert np.abs(bw.ga_src[l]).max() > 1e-3 * t.max()
