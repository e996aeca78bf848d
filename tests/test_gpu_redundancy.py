"""GPU parity of the split statistics (gsplit_batch_stats) and of the data-parallel micro-batch
mode (contexts with one split, one per micro-batch, the same kernels) against the oracle:
every count bit-exact."""
import numpy as np
import pytest
import torch

import workloads
from oracle import reference as R
from test_gpu_parity import assert_batch_equal

pytestmark = pytest.mark.gpu


def _dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


CASES = {
    "tiny-S4": lambda: workloads.tiny(),
    "ragged-S3": lambda: workloads.custom(3001, 41000, dims=[20, 12, 6], fanouts=[7, 3], batch=257, n_splits=3,
                                          name="ragged"),
    "int64-S8-fan33": lambda: workloads.custom(5000, 200000, dims=[8, 8, 8, 4], fanouts=[33, 20, 17], batch=100,
                                               n_splits=8, index64=True, name="wide"),
    "S1": lambda: workloads.custom(2000, 30000, dims=[16, 16, 4], fanouts=[5, 5], batch=300, n_splits=1, name="s1"),
    "range-map-deep": lambda: workloads.custom(20000, 600000, dims=[8, 8, 8, 8, 4], fanouts=[4, 3, 3, 2], batch=500,
                                               n_splits=4, pmap_kind="range", name="deep"),
}


@pytest.mark.parametrize("name", list(CASES))
def test_batch_stats_bit_exact_and_accumulating(name):
    from paper_2303_13775_amd import Context
    dev = _dev()
    w = CASES[name]()
    L, S = w.n_layers, w.n_splits
    ctx = Context(w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev), S, w.fanouts, w.batch)
    edges = torch.zeros(L * S, dtype=torch.int64, device=dev)
    cross = torch.zeros(L * S, dtype=torch.int64, device=dev)
    want_e = np.zeros((L, S), np.int64)
    want_c = np.zeros((L, S), np.int64)
    for it in (0, 1):
        tg = w.targets(it)
        ctx.gsplit_sample_split(tg.to(dev), 99, it)
        ctx.gsplit_batch_stats(edges, cross)
        ob = R.sp_sample(w.indptr.numpy(), w.indices.numpy(), w.pmap.numpy(), S, w.fanouts, tg.numpy(), 99, it)
        e, c = R.batch_stats(ob, w.pmap.numpy())
        want_e += e; want_c += c
        assert np.array_equal(edges.cpu().numpy().reshape(L, S), want_e), it
        assert np.array_equal(cross.cpu().numpy().reshape(L, S), want_c), it
    # the edge counts are also what gsplit_batch_sizes reports for the last batch
    _, _, n_edges, _ = ctx.gsplit_batch_sizes()
    assert np.array_equal(np.asarray(n_edges), e)
    ctx.close()


@pytest.mark.parametrize("name", ["tiny-S4", "int64-S8-fan33", "ragged-S3"])
def test_micro_batch_mode_counts_match_the_oracle(name):
    """Table 1: the mini-batch once, split S ways, and the same targets as S micro-batches."""
    from paper_2303_13775_amd import Context
    dev = _dev()
    w = CASES[name]()
    L, S = w.n_layers, w.n_splits
    ip, ix, pm = w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev)
    mini_ctx = Context(ip, ix, pm, S, w.fanouts, w.batch)
    micro_ctx = Context(ip, ix, torch.zeros_like(pm), 1, w.fanouts, (w.batch + S - 1) // S)
    for it in (0, 3):
        tg = w.targets(it)
        mini_ctx.gsplit_sample_split(tg.to(dev), 5, it)
        n_local, _, n_edges, _ = mini_ctx.gsplit_batch_sizes()
        got = {"edges_mini": int(np.sum(n_edges)), "features_mini": int(np.sum(n_local[0])), "edges_micro": 0,
               "features_micro": 0}
        micro_o = R.micro_batches(w.indptr.numpy(), w.indices.numpy(), w.fanouts, tg.numpy(), S, 5, it)
        for m, part in enumerate(workloads.micro_batch_parts(tg, S)):
            micro_ctx.gsplit_sample_split(part.to(dev), 5, it * S + m)
            nl, _, ne, _ = micro_ctx.gsplit_batch_sizes()
            got["edges_micro"] += int(np.sum(ne)); got["features_micro"] += int(np.sum(nl[0]))
            assert_batch_equal(micro_ctx.fetch_batch(), micro_o[m], 1, L)
        mini_o = R.sp_sample(w.indptr.numpy(), w.indices.numpy(), w.pmap.numpy(), S, w.fanouts, tg.numpy(), 5, it)
        assert got == R.redundancy_counts(mini_o, micro_o)
    mini_ctx.close(); micro_ctx.close()


def test_batch_stats_error_paths():
    from paper_2303_13775_amd import Context, GsplitError
    dev = _dev()
    w = workloads.tiny()
    ctx = Context(w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev), w.n_splits, w.fanouts, w.batch)
    e = torch.zeros(w.n_layers * w.n_splits, dtype=torch.int64, device=dev)
    with pytest.raises(GsplitError):      # no batch yet
        ctx.gsplit_batch_stats(e, e.clone())
    ctx.gsplit_sample_split(torch.empty(0, dtype=torch.int32, device=dev), 1, 0)
    ctx.gsplit_batch_stats(e, e)          # an empty batch adds nothing
    assert int(e.sum()) == 0
    ctx.close()
