"""gsplit_sample_split_noalloc (the entry point for callers that cannot allocate: all working memory
in a static device array) against gsplit_sample_split on a context: every output bit for bit, on two
calls in a row that share the array, the second with a smaller input (fewer targets, another graph,
fewer splits and layers), then the first again; and the capacity error."""
import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu


def _outputs(w, dev, fill):
    from paper_2303_13775_amd import noalloc_output_sizes
    sizes = noalloc_output_sizes(w.n_vertices, w.n_splits, w.fanouts, w.batch)
    mk = lambda n: torch.full((n,), fill, dtype=torch.int32, device=dev)
    return {k: [mk(n) for n in v] if isinstance(v, list) else mk(v) for k, v in sizes.items()}


def _compare(w, dev, targets, seed, it, fill, check_free=True):
    """One call of each entry point on the same inputs; returns the number of compared entries.
    check_free: the amount of free device memory must be the same after the call (not on the very
    first launch out of the library, when the runtime loads its code and the static array)."""
    from paper_2303_13775_amd import Context, gsplit_sample_split_noalloc
    S, L = w.n_splits, w.n_layers
    gi, gx, gp = w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev)
    tg = targets.to(dev)
    out = _outputs(w, dev, fill)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    gsplit_sample_split_noalloc(gi, gx, gp, S, w.fanouts, w.batch, tg, seed, it, out)
    torch.cuda.synchronize()
    assert not check_free or torch.cuda.mem_get_info()[0] == free_before, "the call changed the amount of free device memory"
    ctx = Context(gi, gx, gp, S, w.fanouts, w.batch)
    ctx.gsplit_sample_split(tg, seed, it)
    ref = ctx.fetch_batch()
    n = 0
    for l in range(L + 1):
        off = [0] + list(np.cumsum(ref["n_local"][l]))
        assert out["local_off"][l * (S + 1):(l + 1) * (S + 1)].tolist() == off, ("local_off", l)
        cat = torch.cat(ref["local_front"][l]) if S else torch.empty(0)
        assert torch.equal(out["local_cat"][l][:off[-1]], cat), ("local_cat", l)
        assert bool((out["local_cat"][l][off[-1]:] == fill).all()), ("rows past the live size were written", l)
        n += off[-1]
    for l in range(L):
        lay = ref["layers"][l]
        n_dst, nnz = sum(ref["n_local"][l + 1]), sum(ref["n_edges"][l])
        moff = [0] + list(np.cumsum(ref["n_mixed"][l]))
        assert out["mixed_off"][l * (S + 1):(l + 1) * (S + 1)].tolist() == moff, ("mixed_off", l)
        assert out["recv_off"][l * (S + 1):(l + 1) * (S + 1)].tolist() == lay["recv_off"].tolist(), ("recv_off", l)
        for name, want in (("nbr", lay["nbr"].reshape(-1)), ("cnt", lay["cnt"]), ("mixed_cat", torch.cat(lay["mixed"])),
                           ("blk_indptr", lay["blk_indptr"]), ("blk_src", lay["blk_src"]),
                           ("shuffle_src_row", torch.cat(lay["shuffle_src_row"])), ("recv_cat", lay["recv"])):
            assert torch.equal(out[name][l][:want.numel()], want), (name, l)
            n += want.numel()
        assert lay["blk_indptr"].numel() == n_dst + 1 and lay["blk_src"].numel() == nnz
    ctx.close()
    return n


def test_noalloc_entry_point_equals_the_context_path_on_consecutive_calls():
    assert torch.cuda.is_available(), "needs the MI355X"
    dev = torch.device("cuda:0")
    big = workloads.tiny()                         # 1024 targets, fanouts [10, 5], 4 splits: 8 MiB of the array
    small = workloads.custom(3001, 41000, dims=[8, 8, 4], fanouts=[7], batch=257, n_splits=1, index64=True,
                             name="noalloc-small")
    n1 = _compare(big, dev, big.targets(0), 1234, 0, fill=-7, check_free=False)
    n2 = _compare(small, dev, small.targets(1)[:100], 99, 1, fill=-9)      # smaller in every respect
    n3 = _compare(big, dev, big.targets(2), 1235, 2, fill=-11)             # and the large one again
    n4 = _compare(small, dev, small.targets(3)[:0], 5, 3, fill=-13)        # an empty batch
    assert n1 > 50000 and 0 < n2 < n1 and n3 > 50000 and n4 == 1      # (an empty batch still has blk_indptr[0])


def test_noalloc_entry_point_rejects_what_does_not_fit():
    from paper_2303_13775_amd import GsplitError, gsplit_sample_split_noalloc
    dev = torch.device("cuda:0")
    w = workloads.custom(60000, 1500000, dims=[8, 8, 8, 4], fanouts=[15, 10, 5], batch=1024, n_splits=4, name="too-big")
    out = _outputs(w, dev, 0)
    with pytest.raises(GsplitError) as e:
        gsplit_sample_split_noalloc(w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev), 4, w.fanouts, w.batch,
                                    w.targets(0).to(dev), 1, 0, out)
    assert e.value.code == -3 and "KiB" in str(e.value)
    with pytest.raises(GsplitError) as e:           # more targets than max_targets
        gsplit_sample_split_noalloc(w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev), 4, [3, 2], 16,
                                    w.targets(0).to(dev), 1, 0, _outputs(workloads.custom(
                                        60000, 1500000, dims=[8, 8, 4], fanouts=[3, 2], batch=16, n_splits=4), dev, 0))
    assert e.value.code == -3
