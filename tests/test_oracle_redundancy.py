"""Pins of the oracle's split statistics (workload imbalance and cross-edge share, paper section
7.3) and of the data-parallel micro-batch counters behind Table 1 (section 2)."""
import numpy as np
import pytest

import workloads
from oracle import reference as R


def _csr(n, pairs):
    """Symmetric CSR (int64 indptr, int32 indices, sorted rows) from undirected pairs."""
    adj = [set() for _ in range(n)]
    for a, b in pairs:
        if a != b:
            adj[a].add(b); adj[b].add(a)
    indptr = np.zeros(n + 1, np.int64)
    for v in range(n):
        indptr[v + 1] = indptr[v] + len(adj[v])
    indices = np.array([u for v in range(n) for u in sorted(adj[v])], np.int32)
    return indptr, indices, adj


@pytest.fixture(scope="module")
def tiny():
    w = workloads.tiny()
    ip, ix, pm = w.indptr.numpy(), w.indices.numpy(), w.pmap.numpy()
    tg = w.targets(0).numpy()
    return w, ip, ix, pm, tg


def test_stats_agree_with_the_relabelled_route_and_with_the_papers_random_map_figure(tiny):
    w, ip, ix, pm, tg = tiny
    b = R.sp_sample(ip, ix, pm, w.n_splits, w.fanouts, tg, 7, 0)
    edges, cross = R.batch_stats(b, pm)                    # from nbr / cnt, global ids
    q = R.split_quality(b, pm)                             # from blk_src through the mixed frontier
    assert int(edges.sum()) == q["edges"]
    q2 = R.quality_from_stats(edges, cross)
    assert abs(q2["cross_edge_fraction"] - q["cross_edge_fraction"]) < 1e-15
    assert abs(q2["workload_imbalance"] - q["workload_imbalance"]) < 1e-15
    # section 7.3: a random map has 75 % of the edges crossing with four splits
    assert abs(q2["cross_edge_fraction"] - 0.75) < 0.02
    for l in range(w.n_layers):
        for s in range(w.n_splits):
            assert edges[l, s] == int(b.blocks[l][s].cnt.sum())


def test_one_split_has_no_cross_edges_and_no_imbalance(tiny):
    w, ip, ix, pm, tg = tiny
    b = R.sp_sample(ip, ix, np.zeros_like(pm), 1, w.fanouts, tg, 7, 0)
    edges, cross = R.batch_stats(b, np.zeros_like(pm))
    assert cross.sum() == 0 and edges.sum() > 0
    assert R.quality_from_stats(edges, cross) == {"workload_imbalance": 1.0, "cross_edge_fraction": 0.0}


def test_bipartite_graph_split_by_side_crosses_every_edge_and_by_component_none():
    rng = np.random.default_rng(5)
    n = 400
    pairs = [(2 * int(a), 2 * int(b) + 1) for a, b in rng.integers(0, n // 2, (3000, 2))]
    ip, ix, _ = _csr(n, pairs)
    tg = rng.choice(n, 40, replace=False).astype(np.int32)
    side = (np.arange(n) % 2).astype(np.uint8)
    b = R.sp_sample(ip, ix, side, 2, [4, 3], tg, 1, 0)
    edges, cross = R.batch_stats(b, side)
    assert edges.sum() > 0 and (cross == edges).all()
    # two disjoint copies of the graph, one per split: nothing crosses
    ip2 = np.concatenate([ip, ip[1:] + ip[-1]])
    ix2 = np.concatenate([ix, ix + n]).astype(np.int32)
    comp = (np.arange(2 * n) >= n).astype(np.uint8)
    tg2 = np.concatenate([tg[:20], tg[20:] + n]).astype(np.int32)
    b2 = R.sp_sample(ip2, ix2, comp, 2, [4, 3], tg2, 1, 0)
    e2, c2 = R.batch_stats(b2, comp)
    assert e2.sum() > 0 and c2.sum() == 0


def _balls(adj, seeds, hops):
    """levels[h] = vertices within h hops of the seeds (every neighbour kept)."""
    levels = [set(int(v) for v in seeds)]
    for _ in range(hops):
        cur = levels[-1]
        levels.append(cur | {u for v in cur for u in adj[v]})
    return levels


def test_counts_equal_breadth_first_balls_when_every_neighbour_is_kept():
    """With fanout >= max degree sampling keeps all neighbours, so a batch of L layers reads the
    L-hop ball of its targets and computes, at the layer that expands the h-hop ball, the degree
    sum of that ball: brute force with Python sets, for the mini-batch and for each micro-batch."""
    rng = np.random.default_rng(9)
    n = 300
    ip, ix, adj = _csr(n, rng.integers(0, n, (700, 2)))
    maxdeg = int((ip[1:] - ip[:-1]).max())
    fan = [maxdeg, maxdeg + 1, maxdeg]
    tg = rng.choice(n, 24, replace=False).astype(np.int32)
    S = 4
    pm = rng.integers(0, S, n).astype(np.uint8)
    mini = R.sp_sample(ip, ix, pm, S, fan, tg, 3, 2)
    micro = R.micro_batches(ip, ix, fan, tg, S, 3, 2)
    got = R.redundancy_counts(mini, micro)
    deg = lambda vs: sum(len(adj[v]) for v in vs)
    lv = _balls(adj, tg, 3)
    assert got["features_mini"] == len(lv[3])
    assert got["edges_mini"] == deg(lv[0]) + deg(lv[1]) + deg(lv[2])
    f = e = 0
    for m in range(S):
        lm = _balls(adj, tg[6 * m:6 * m + 6], 3)
        f += len(lm[3]); e += deg(lm[0]) + deg(lm[1]) + deg(lm[2])
    assert got["features_micro"] == f and got["edges_micro"] == e
    assert f >= got["features_mini"] and e >= got["edges_mini"]


def test_complete_graph_closed_form_and_disjoint_cliques_have_no_redundancy():
    n, S, B = 12, 4, 8
    pairs = [(a, b) for a in range(n) for b in range(a + 1, n)]
    ip, ix, _ = _csr(n, pairs)
    tg = np.arange(B, dtype=np.int32)
    pm = (np.arange(n) % S).astype(np.uint8)
    fan = [n, n]                                           # keeps all n - 1 neighbours
    got = R.redundancy_counts(R.sp_sample(ip, ix, pm, S, fan, tg, 1, 0), R.micro_batches(ip, ix, fan, tg, S, 1, 0))
    # every micro-batch reaches all n vertices after one hop
    assert got["features_mini"] == n and got["features_micro"] == S * n
    assert got["edges_mini"] == B * (n - 1) + n * (n - 1)
    assert got["edges_micro"] == B * (n - 1) + S * n * (n - 1)
    # S disjoint cliques, micro-batch m's targets inside clique m: nothing is shared
    c = 6
    pairs = [(m * c + a, m * c + b) for m in range(S) for a in range(c) for b in range(a + 1, c)]
    ip, ix, _ = _csr(S * c, pairs)
    tg = np.array([m * c + j for m in range(S) for j in range(2)], np.int32)
    pm = (np.arange(S * c) // c).astype(np.uint8)
    got = R.redundancy_counts(R.sp_sample(ip, ix, pm, S, [c, c], tg, 1, 0), R.micro_batches(ip, ix, [c, c], tg, S, 1, 0))
    assert got["features_micro"] == got["features_mini"] == S * c
    assert got["edges_micro"] == got["edges_mini"]


def test_mini_batch_counts_do_not_depend_on_the_splits_and_micro_batches_overlap(tiny):
    w, ip, ix, pm, tg = tiny
    one = R.sp_sample(ip, ix, np.zeros_like(pm), 1, w.fanouts, tg, 11, 3)
    four = R.sp_sample(ip, ix, pm, 4, w.fanouts, tg, 11, 3)
    micro = R.micro_batches(ip, ix, w.fanouts, tg, 4, 11, 3)
    a, b = R.redundancy_counts(one, micro), R.redundancy_counts(four, micro)
    assert a == b                                          # splitting creates no redundancy
    assert sum(m.local_cat(w.n_layers).shape[0] for m in micro) == tg.shape[0]
    # Table 1's direction: more feature rows loaded and at least as many edges computed
    assert a["features_micro"] > 1.05 * a["features_mini"]
    assert a["edges_micro"] >= a["edges_mini"]
