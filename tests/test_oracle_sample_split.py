"""Pins for the oracle's sampling, splitting, dedup/relabel and shuffle index.

  * invariants the paper's definitions fix: sampled edges exist, no repeated neighbour, the count
    is min(degree, fanout); splits are disjoint, every member is owned by its split, their union is
    the unsplit mini-batch frontier, the multiset of global edges is the unsplit one;
  * brute force: with fanout >= max degree sampling is deterministic and each layer must be the
    exact k-hop ball computed by an independent set-based BFS;
  * the worked example of the paper's training-pipeline section (tests/golden/fig3_example.txt);
  * the closed form for a uniform-random partition map: a fraction 1 - 1/S of edges cross splits
    (the paper reports 75 % for 4 splits)."""
import os

import numpy as np
import pytest

import workloads
from conftest import GOLDEN
from oracle import reference as R


def _np(t):
    return t.cpu().numpy()


def _graph(w):
    return _np(w.indptr).astype(np.int64), _np(w.indices), _np(w.pmap)


@pytest.fixture(scope="module")
def tiny_batch(tiny_workload):
    w = tiny_workload
    ip, ix, pm = _graph(w)
    tg = _np(w.targets(0))
    return w, ip, ix, pm, tg, R.sp_sample(ip, ix, pm, w.n_splits, w.fanouts, tg, seed=11, it=3)


def test_sample_layer_invariants(tiny_workload):
    w = tiny_workload
    ip, ix, _ = _graph(w)
    front = _np(w.targets(5))
    for fan in (1, 5, 10, 64):
        nbr, cnt = R.sample_layer(ip, ix, front, fan, 1, 7, 0)
        for i, v in enumerate(front):
            row = ix[ip[v]:ip[v + 1]]
            got = nbr[i, :cnt[i]]
            assert cnt[i] == min(len(row), fan)
            assert (nbr[i, cnt[i]:] == -1).all()
            assert len(set(got.tolist())) == cnt[i]
            assert set(got.tolist()) <= set(row.tolist())
            if len(row) <= fan:
                assert got.tolist() == row.tolist()       # CSR order, no randomness


def test_sampling_depends_on_vertex_not_on_position(tiny_workload):
    w = tiny_workload
    ip, ix, _ = _graph(w)
    front = _np(w.targets(1))[:200]
    nbr, cnt = R.sample_layer(ip, ix, front, 5, 0, 3, 9)
    perm = np.random.default_rng(0).permutation(front.shape[0])
    nbr2, cnt2 = R.sample_layer(ip, ix, front[perm], 5, 0, 3, 9)
    assert (nbr2 == nbr[perm]).all() and (cnt2 == cnt[perm]).all()
    nbr3, _ = R.sample_layer(ip, ix, front, 5, 0, 3, 10)
    assert (nbr3 != nbr).any()


def _khop_sets(ip, ix, targets, hops):
    """Independent brute force: layer sets by set-based expansion (self included)."""
    layers = [set(targets.tolist())]
    for _ in range(hops):
        nxt = set(layers[-1])
        for v in layers[-1]:
            nxt.update(ix[ip[v]:ip[v + 1]].tolist())
        layers.append(nxt)
    return layers


def test_full_khop_when_fanout_covers_degree():
    w = workloads.custom(300, 1800, dims=[8, 8, 4], fanouts=[1, 1], batch=12, n_splits=3,
                         name="khop")
    ip, ix, pm = _graph(w)
    maxdeg = int((ip[1:] - ip[:-1]).max())
    tg = _np(w.targets(0))
    b = R.sp_sample(ip, ix, pm, 3, [maxdeg, maxdeg + 3], tg, seed=1, it=0)
    want = _khop_sets(ip, ix, tg, 2)
    for hop, l in enumerate((2, 1, 0)):
        got = set(np.concatenate(b.local_front[l]).tolist())
        assert got == want[hop]
    # edges of each layer = every CSR edge leaving the layer above
    for hop, l in enumerate((1, 0)):
        got = set()
        for s in range(3):
            blk = b.blocks[l][s]
            for i, v in enumerate(blk.dst):
                for e in range(blk.blk_indptr[i], blk.blk_indptr[i + 1]):
                    got.add((int(v), int(blk.mixed_front[blk.blk_src[e]])))
        full = {(v, int(u)) for v in want[hop] for u in ix[ip[v]:ip[v + 1]]}
        assert got == full


def test_split_invariants_and_equivalence_to_unsplit(tiny_batch):
    w, ip, ix, pm, tg, b = tiny_batch
    S, L = w.n_splits, w.n_layers
    u = R.sp_sample(ip, ix, np.zeros_like(pm), 1, w.fanouts, tg, seed=11, it=3)
    for l in range(L + 1):
        fronts = b.local_front[l]
        allv = np.concatenate(fronts)
        assert np.unique(allv).shape[0] == allv.shape[0]                   # disjoint, no dups
        for s in range(S):
            assert (pm[fronts[s]] == s).all()                              # owned by its split
        assert set(allv.tolist()) == set(u.local_front[l][0].tolist())     # union = unsplit
    for l in range(L):
        def edges(batch, n_s):
            out = []
            for s in range(n_s):
                blk = batch.blocks[l][s]
                dst = np.repeat(blk.dst, blk.cnt)
                src = blk.mixed_front[blk.blk_src]
                out.append(np.stack([dst, src], 1))
            e = np.concatenate(out)
            return e[np.lexsort((e[:, 1], e[:, 0]))]
        assert (edges(b, S) == edges(u, 1)).all()                          # same multiset of edges


def test_relabel_and_shuffle_index_round_trip(tiny_batch):
    w, ip, ix, pm, tg, b = tiny_batch
    for l in range(w.n_layers):
        cat = b.local_cat(l)
        for s in range(w.n_splits):
            blk = b.blocks[l][s]
            n_dst = blk.dst.shape[0]
            assert (blk.mixed_front[:n_dst] == blk.dst).all()              # self prefix
            assert np.unique(blk.mixed_front).shape[0] == blk.mixed_front.shape[0]
            assert (cat[blk.shuffle_src_row] == blk.mixed_front).all()     # gather index is right
            # block rows mapped back to global ids give the sampled slots, in slot order
            for i in range(0, n_dst, 37):
                a, e = blk.blk_indptr[i], blk.blk_indptr[i + 1]
                assert (blk.mixed_front[blk.blk_src[a:e]] == blk.nbr[i, :blk.cnt[i]]).all()
            # first-occurrence order: scanning dst then slots, new ids appear in mixed order
            seq = np.concatenate([blk.dst, R.slot_stream(blk.nbr, blk.cnt)])
            _, first = np.unique(seq, return_index=True)
            assert (seq[np.sort(first)] == blk.mixed_front).all()
    assert (tg[b.target_perm] == b.local_cat(w.n_layers)).all()


def test_buckets_are_stable_and_route_to_owner(tiny_batch):
    w, ip, ix, pm, tg, b = tiny_batch
    for l in range(w.n_layers):
        for s in range(w.n_splits):
            blk = b.blocks[l][s]
            sampled_part = blk.mixed_front[blk.dst.shape[0]:]
            for t in range(w.n_splits):
                assert (blk.buckets[t] == sampled_part[pm[sampled_part] == t]).all()
        for t in range(w.n_splits):
            recv = np.concatenate([b.blocks[l][s].buckets[t] for s in range(w.n_splits)])
            seq = np.concatenate([b.local_front[l + 1][t], recv])
            _, first = np.unique(seq, return_index=True)
            assert (seq[np.sort(first)] == b.local_front[l][t]).all()


def test_random_map_cross_edge_fraction(tiny_batch):
    w, ip, ix, pm, tg, b = tiny_batch
    q = R.split_quality(b, pm)
    assert abs(q["cross_edge_fraction"] - (1 - 1 / w.n_splits)) < 0.02    # paper: 75 % for 4 splits
    assert 1.0 <= q["workload_imbalance"] < 1.2


def _fig3():
    sets, adj = {}, {}
    with open(os.path.join(GOLDEN, "fig3_example.txt")) as f:
        for line in f:
            if line.startswith("#") or "=" not in line:
                continue
            k, v = [x.strip() for x in line.split("=")]
            if k.startswith("chosen.adj."):
                adj[k.split(".")[-1]] = v.split()
            else:
                sets[k] = set(v.split())
    return sets, adj


def test_paper_worked_example():
    sets, adj = _fig3()
    names = "abcdefghijklmnop"
    idx = {c: i for i, c in enumerate(names)}
    ip = np.zeros(len(names) + 1, np.int64)
    cols = []
    for i, c in enumerate(names):
        row = sorted(idx[u] for u in adj.get(c, []))
        cols += row
        ip[i + 1] = ip[i] + len(row)
    ix = np.array(cols, np.int32)
    pm = np.zeros(len(names), np.uint8)
    for c in sets["paper.owner.gpu2"]:
        pm[idx[c]] = 1
    tg = np.array([idx[c] for c in "abcd"], np.int32)
    b = R.sp_sample(ip, ix, pm, 2, [4, 4], tg, seed=0, it=0)
    nm = lambda arr: {names[i] for i in np.asarray(arr).tolist()}
    G = ("gpu1", "gpu2")
    for s in range(2):
        assert nm(b.local_front[2][s]) == sets[f"paper.targets.{G[s]}"]
        top = b.blocks[1][s]
        n_dst = top.dst.shape[0]
        # sampled mixed frontier and new local frontier, without the destination vertices themselves
        assert nm(top.mixed_front[n_dst:]) == sets[f"paper.layer1.mixed.{G[s]}"]
        assert nm(b.local_front[1][s]) - nm(b.local_front[2][s]) == sets[f"paper.layer1.local.{G[s]}"]
        assert nm(b.local_front[1][s]) - nm(b.local_front[2][s]) | nm(top.mixed_front[n_dst:]) \
            == sets[f"paper.layer1.next.{G[s]}"]
        # layer 0: what is new below layer 1
        assert nm(b.local_front[0][s]) - nm(b.local_front[1][s]) == sets[f"paper.layer0.local.{G[s]}"]
    upper = nm(np.concatenate(b.local_front[1]))
    assert nm(b.blocks[0][0].mixed_front) - upper == sets["paper.layer0.mixed.gpu1"]
    # training shuffles = rows of a mixed frontier owned by the other split
    def remote(l, s):
        mf = b.blocks[l][s].mixed_front
        return nm(mf[pm[mf] != s])
    assert remote(0, 1) - upper == sets["paper.layer0.send.gpu1_to_gpu2"]
    assert remote(0, 0) - upper == sets["paper.layer0.recv.gpu1"]
    assert remote(1, 1) == sets["paper.layer1.send.gpu1_to_gpu2"]
    assert remote(1, 0) == sets["paper.layer1.recv.gpu1"]


def test_edge_cases():
    # isolated targets, a split that owns nothing, empty target list
    ip = np.array([0, 0, 2, 3, 3, 4], np.int64)
    ix = np.array([2, 4, 1, 1], np.int32)
    pm = np.array([0, 1, 1, 2, 1], np.uint8)
    b = R.sp_sample(ip, ix, pm, 4, [2, 1], np.array([0, 3], np.int32), 5, 5)
    assert [f.tolist() for f in b.local_front[0]] == [[0], [], [3], []]
    assert all(blk.blk_indptr[-1] == 0 for row in b.blocks for blk in row)
    b = R.sp_sample(ip, ix, pm, 4, [2, 1], np.array([], np.int32), 5, 5)
    assert all(f.shape[0] == 0 for f in b.local_front[0])
    b = R.sp_sample(ip, ix, pm, 4, [2, 2], np.array([1], np.int32), 5, 5)
    assert sorted(np.concatenate(b.local_front[0]).tolist()) == [1, 2, 4]
    with pytest.raises(AssertionError):
        R.sp_sample(ip, ix, pm, 4, [2], np.array([1, 1], np.int32), 0, 0)
