"""Pins of the oracle's pre-sampling stage (section 4: k_v counts appearances at layers l > 0, k_e
counts sampled edges; analysis after Eq. 2: E[X_i] = L_i, E[Y] = sum of k_e / N over the cut)."""
import numpy as np
import pytest

from oracle import reference as R


def _ring_lattice(n, half):
    """Every vertex v is adjacent to v +- 1 .. v +- half (mod n): degree 2 * half, sorted rows."""
    rows = []
    for v in range(n):
        rows.append(sorted({(v + d) % n for d in range(-half, half + 1) if d != 0}))
    indptr = np.zeros(n + 1, np.int64)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    return indptr, np.array([u for r in rows for u in r], np.int32), rows


def test_all_neighbours_kept_gives_breadth_first_balls():
    """Fanout >= degree: no randomness.  Level l is the ball of radius L - l around the targets, so
    k_v = number of levels 1..L whose ball holds v and an edge of row u is counted once for every
    level 1..L whose ball holds u.  A wrong layer convention (counting level 0, skipping the
    targets, off-by-one in the radius) changes these numbers."""
    n, half, L = 60, 2, 3
    indptr, indices, rows = _ring_lattice(n, half)
    fanouts = [7, 5, 4]                                       # all >= degree 4
    targets = np.array([3, 30], np.int32)
    k_v, k_e = R.presample_counts(indptr, indices, fanouts, [targets], seed=1, iters=[0])
    dist = np.full(n, 10**9)
    for t in targets:
        d = np.minimum(np.abs(np.arange(n) - t), n - np.abs(np.arange(n) - t))
        dist = np.minimum(dist, (d + half - 1) // half)      # hops on the lattice
    want_v = np.zeros(n, np.int64)
    want_rows = np.zeros(n, np.int64)
    for level in range(1, L + 1):
        ball = dist <= L - level
        want_v += ball
        want_rows += ball                                     # level >= 1 frontiers are the sampled rows
    assert np.array_equal(k_v, want_v)
    assert np.array_equal(k_e, np.repeat(want_rows, np.diff(indptr)))
    # level 0 (radius 3 ball) is larger than anything counted: it must not contribute
    assert k_v[(dist == L)].sum() == 0 and (dist == L).any()


def test_counts_are_conserved_and_bounded():
    import workloads
    w = workloads.tiny()
    ip, ix = w.indptr.numpy(), w.indices.numpy()
    batches = [w.targets(i).numpy() for i in range(6)]
    k_v, k_e = R.presample_counts(ip, ix, w.fanouts, batches, seed=9, iters=list(range(6)))
    # the same samples through Algorithm 1 with one split: frontier sizes and edge totals
    pm = np.zeros(ip.shape[0] - 1, np.uint8)
    tot_v = tot_e = 0
    for i, tg in enumerate(batches):
        b = R.sp_sample(ip, ix, pm, 1, w.fanouts, tg, 9, i)
        tot_v += sum(b.local_front[l][0].shape[0] for l in range(1, b.n_layers + 1))
        tot_e += sum(int(b.blocks[l][0].cnt.sum()) for l in range(b.n_layers))
    assert k_v.sum() == tot_v and k_e.sum() == tot_e
    L = len(w.fanouts)
    assert k_v.max() <= len(batches) * L and k_e.max() <= len(batches) * L
    # an edge is only sampled from a row that appeared at a level > 0
    row_of_edge = np.repeat(np.arange(ip.shape[0] - 1), np.diff(ip))
    assert (k_v[row_of_edge[k_e > 0]] > 0).all()


def test_edge_of_a_wide_row_is_kept_with_probability_fanout_over_degree():
    """A star: the hub has degree 200, fanout 10, and is the only target.  Each hub edge is kept in a
    sample with probability 10 / 200; over N samples k_e / N must be near 0.05 for every edge
    (binomial, 6 sigma) and the hub's row total is exactly 10 per sample."""
    deg, fan, N = 200, 10, 4000
    indptr = np.zeros(deg + 2, np.int64)
    indptr[1] = deg
    indptr[2:] = deg + np.arange(1, deg + 1)                  # leaf v lists the hub
    indices = np.concatenate([np.arange(1, deg + 1), np.zeros(deg)]).astype(np.int32)
    batches = [np.array([0], np.int32)] * N
    k_v, k_e = R.presample_counts(indptr, indices, [fan], batches, seed=123, iters=list(range(N)))
    hub = k_e[:deg]
    assert hub.sum() == fan * N and k_e[deg:].sum() == 0
    p = fan / deg
    sigma = np.sqrt(N * p * (1 - p))
    assert np.abs(hub - N * p).max() < 6 * sigma
    assert k_v[0] == N and k_v[1:].sum() == 0                 # one layer: only the target level counts


def test_expected_load_and_cut_match_the_weights():
    """E[X_i] = L_i and E[Y] = sum over the cut of k_e / N: loads and cross edges of fresh batches
    against the weights of a separate pre-sampling run."""
    import workloads
    w = workloads.tiny()
    ip, ix = w.indptr.numpy(), w.indices.numpy()
    S, n_pre, n_new = 4, 40, 40
    k_v, k_e = R.presample_counts(ip, ix, w.fanouts, [w.targets(i).numpy() for i in range(n_pre)], 5,
                                  list(range(n_pre)))
    w_v, w_e = R.presample_weights(k_v, k_e, n_pre)
    pm = w.pmap.numpy()
    load = np.array([w_v[pm == s].sum() for s in range(S)])
    row_of_edge = np.repeat(np.arange(ip.shape[0] - 1), np.diff(ip))
    cut = w_e[pm[row_of_edge] != pm[ix]].sum()
    xs, ys = np.zeros(S), 0.0
    for i in range(n_pre, n_pre + n_new):
        b = R.sp_sample(ip, ix, pm, S, w.fanouts, w.targets(i).numpy(), 5, i)
        for s in range(S):
            xs[s] += sum(b.local_front[l][s].shape[0] for l in range(1, b.n_layers + 1))
        q = R.split_quality(b, pm)
        ys += q["cross_edge_fraction"] * q["edges"]
    xs /= n_new
    ys /= n_new
    assert np.abs(xs - load).max() / load.max() < 0.03
    assert abs(ys - cut) / cut < 0.03
