"""Pins of the oracle's feature-cache functions: the sampling-frequency count of the input layer,
the f_G-aligned selection of what each split caches, and the loading step that takes a row from
the cache when its split holds it and from the host table otherwise (paper sections 3, 4, 7.1)."""
import numpy as np
import pytest

import workloads
from oracle import reference as R


def _csr(n, pairs):
    adj = [set() for _ in range(n)]
    for a, b in pairs:
        a, b = int(a), int(b)
        if a != b:
            adj[a].add(b); adj[b].add(a)
    indptr = np.zeros(n + 1, np.int64)
    for v in range(n):
        indptr[v + 1] = indptr[v] + len(adj[v])
    return indptr, np.array([u for v in range(n) for u in sorted(adj[v])], np.int32), adj


def test_input_counts_equal_ball_membership_when_every_neighbour_is_kept():
    rng = np.random.default_rng(4)
    n, L = 250, 2
    ip, ix, adj = _csr(n, rng.integers(0, n, (500, 2)))
    fan = [int((ip[1:] - ip[:-1]).max())] * L
    batches = [rng.choice(n, 5, replace=False).astype(np.int32) for _ in range(6)]
    k_in = R.input_counts(ip, ix, fan, batches, 9, list(range(6)))
    want = np.zeros(n, np.int64)
    for tg in batches:
        ball = set(int(v) for v in tg)
        for _ in range(L):
            ball |= {u for v in ball for u in adj[v]}
        want[list(ball)] += 1
    assert np.array_equal(k_in, want)


def test_input_counts_are_conserved_against_algorithm_1():
    w = workloads.tiny()
    ip, ix, pm = w.indptr.numpy(), w.indices.numpy(), w.pmap.numpy()
    batches = [w.targets(i).numpy() for i in range(3)]
    k_in = R.input_counts(ip, ix, w.fanouts, batches, 21, [0, 1, 2])
    total = 0
    seen = np.zeros(ip.shape[0] - 1, np.int64)
    for i, tg in enumerate(batches):
        b = R.sp_sample(ip, ix, pm, w.n_splits, w.fanouts, tg, 21, i)
        total += b.local_cat(0).shape[0]
        seen[b.local_cat(0)] += 1
    assert int(k_in.sum()) == total and np.array_equal(k_in, seen)


def test_cache_select_by_hand_and_by_properties():
    #           v: 0  1  2  3  4  5  6  7
    k = np.array([5, 0, 7, 7, 1, 9, 0, 3])
    pm = np.array([0, 0, 0, 1, 1, 1, 0, 0], np.uint8)
    got = R.cache_select(k, pm, 2, [3, 2])
    assert got[0].tolist() == [2, 0, 7] and got[1].tolist() == [5, 3]      # 1 and 6 were never sampled
    assert R.cache_select(k, pm, 2, [10, 0])[0].tolist() == [2, 0, 7] and R.cache_select(k, pm, 2, [10, 0])[1].size == 0
    k2 = np.array([4, 4, 4, 4])                                               # ties: smaller id first
    assert R.cache_select(k2, np.zeros(4, np.uint8), 1, [2])[0].tolist() == [0, 1]
    rng = np.random.default_rng(2)
    k3 = rng.integers(0, 6, 500)
    pm3 = rng.integers(0, 4, 500).astype(np.uint8)
    sel = R.cache_select(k3, pm3, 4, [30, 0, 1000, 7])
    for s, ids in enumerate(sel):
        assert ids.shape[0] == min([30, 0, 1000, 7][s], int(((pm3 == s) & (k3 > 0)).sum()))
        assert (pm3[ids] == s).all() and len(set(ids.tolist())) == ids.shape[0]
        rest = np.setdiff1d(np.nonzero((pm3 == s) & (k3 > 0))[0], ids)
        if ids.size and rest.size:
            assert k3[rest].max() <= k3[ids].min()                           # nothing hotter was left out


@pytest.fixture(scope="module")
def tiny_cache():
    w = workloads.tiny()
    ip, ix, pm = w.indptr.numpy(), w.indices.numpy(), w.pmap.numpy()
    k_in = R.input_counts(ip, ix, w.fanouts, [w.targets(100 + i).numpy() for i in range(8)], 5, list(range(100, 108)))
    return w, ip, ix, pm, k_in


def test_cached_gather_returns_the_table_rows_and_counts_every_row_once(tiny_cache):
    w, ip, ix, pm, k_in = tiny_cache
    table = w.feat.numpy()
    b = R.sp_sample(ip, ix, pm, w.n_splits, w.fanouts, w.targets(0).numpy(), 5, 0)
    n_local0 = np.array([b.local_front[0][s].shape[0] for s in range(w.n_splits)])
    for cap in ([0] * 4, [200] * 4, [10 ** 9] * 4, [0, 50, 10 ** 9, 3]):
        ids = R.cache_select(np.maximum(k_in, 1) if cap[0] == 10 ** 9 else k_in, pm, w.n_splits, cap)
        rows = [table[i] for i in ids]
        out, hits, misses = R.cached_gather(table, ids, rows, b)
        assert np.array_equal(out.view(np.int32), table[b.local_cat(0)].view(np.int32))
        assert np.array_equal(hits + misses, n_local0)
        if cap == [0] * 4:
            assert hits.sum() == 0
        if cap == [10 ** 9] * 4:
            assert misses.sum() == 0                       # every vertex cached by its owner
        if cap == [0, 50, 10 ** 9, 3]:
            assert hits[0] == 0 and hits[1] <= 50 and hits[3] <= 3
            assert misses[2] == int((k_in[b.local_front[0][2]] == 0).sum())   # only never-sampled vertices miss


def test_hits_come_from_the_cache_and_misses_from_the_host_table(tiny_cache):
    w, ip, ix, pm, k_in = tiny_cache
    table = w.feat.numpy()
    ids = R.cache_select(k_in, pm, w.n_splits, [300] * 4)
    rows = [table[i].copy() for i in ids]
    later = table + 1.0                                    # the host table changes after the cache was filled
    b = R.sp_sample(ip, ix, pm, w.n_splits, w.fanouts, w.targets(1).numpy(), 5, 1)
    out, hits, misses = R.cached_gather(later, ids, rows, b)
    cached = np.zeros(table.shape[0], bool)
    cached[np.concatenate(ids)] = True
    v = b.local_cat(0)
    assert hits.sum() > 0 and misses.sum() > 0
    assert np.array_equal(out[cached[v]], table[v[cached[v]]])
    assert np.array_equal(out[~cached[v]], later[v[~cached[v]]])


def test_a_frequency_ranked_cache_hits_far_more_often_than_its_share_of_the_vertices(tiny_cache):
    """Static caches are filled with frequently accessed input features (section 2): on a power-law
    graph the hottest 10 % of each split's vertices serve well over 10 % of the loads."""
    w, ip, ix, pm, k_in = tiny_cache
    table = w.feat.numpy()
    n = table.shape[0]
    cap = [int(0.1 * (pm == s).sum()) for s in range(w.n_splits)]
    ids = R.cache_select(k_in, pm, w.n_splits, cap)
    b = R.sp_sample(ip, ix, pm, w.n_splits, w.fanouts, w.targets(2).numpy(), 5, 2)     # a held-out batch
    _, hits, misses = R.cached_gather(table, ids, [table[i] for i in ids], b)
    rate = hits.sum() / (hits.sum() + misses.sum())
    assert rate > 0.25
