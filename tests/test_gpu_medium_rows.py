"""The rows built on top of the hot path, at the size and in the configuration bench.py times them:
the medium workload (2.4M vertices, about 131M edges, fanouts [15,10,5], 100-256-256-47).  GAT
forward/backward (heads 4-4-1), the split statistics and the micro-batch counters (4096 targets as
4 x 1024), the cached loading step with the table in pinned host memory, the pre-sampling counts and the
bf16 path, all against the
oracle on the same batch."""
import numpy as np
import pytest
import torch

import workloads
from oracle import reference as R
from oracle import gat as G
from test_gpu_parity import assert_batch_equal, check_sage, TOL_F32
import sage_check as SC
from test_gpu_gat import attention_grad_err, conditioned_gat_backward

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def medium():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    dev = torch.device("cuda:0")
    w = workloads.medium(device=dev)
    host = dict(indptr=w.indptr.cpu().numpy(), indices=w.indices.cpu().numpy(), pmap=w.pmap.cpu().numpy())
    return w, dev, host


def test_gat_medium_full_size(medium):
    from paper_2303_13775_amd import Context, GatParams
    w, dev, host = medium
    heads = [4, 4, 1]
    ctx = Context(w.indptr, w.indices, w.pmap, w.n_splits, w.fanouts, w.batch, gat_index=True)
    wt, a_s, a_d, b = workloads.gat_weights(w.dims, heads, seed=w.seed, device=dev)
    params = GatParams(w.dims, heads, wt, a_s, a_d, b)
    op = G.GatParams(heads, *[[t.cpu().numpy() for t in lst] for lst in (wt, a_s, a_d, b)])
    x0 = torch.empty((ctx.gsplit_max_rows(0), w.dims[0]), device=dev)
    logits = torch.empty((w.batch, w.dims[-1]), device=dev)
    glog = torch.empty_like(logits)
    grads = [[torch.empty_like(t) for t in lst] for lst in (wt, a_s, a_d, b)]
    tg = w.targets(3)
    ctx.gsplit_sample_split(tg, 99, 3)
    ctx.gsplit_gather_features(w.feat, x0)
    ctx.gsplit_gat_fwd(params, x0, logits)
    ctx.gsplit_softmax_xent(logits, w.labels, glog)
    ctx.gsplit_gat_bwd(params, x0, glog, *grads)
    ob = R.sp_sample(host["indptr"], host["indices"], host["pmap"], w.n_splits, w.fanouts, tg.cpu().numpy(), 99, 3)
    ids = torch.from_numpy(ob.local_cat(0)).long().to(dev)
    of = G.gat_forward(ob, w.feat[ids].cpu().numpy(), op)
    y = w.labels[torch.from_numpy(tg.cpu().numpy()[ob.target_perm]).to(dev).long()].cpu().numpy()
    _, g = R.softmax_xent(of.logits, y)
    obw, _ = conditioned_gat_backward(ctx, ob, of, op, g, heads, who="gat")
    assert R.max_rel_err(logits.cpu().numpy(), of.logits) < TOL_F32
    for l in range(w.n_layers):
        for name, got, want in (("gw", grads[0][l], obw.gw[l]), ("gbias", grads[3][l], obw.gbias[l])):
            assert R.max_rel_err(got.cpu().numpy().reshape(-1), np.asarray(want).reshape(-1)) < TOL_F32, (name, l)
        for name, got, want in (("ga_src", grads[1][l], obw.ga_src[l]), ("ga_dst", grads[2][l], obw.ga_dst[l])):
            assert attention_grad_err(got.cpu().numpy(), want, obw.ga_src[l], obw.ga_dst[l], obw.ga_terms[l]) < TOL_F32, (name, l)
    ctx.close()


def test_stats_and_micro_batches_medium_full_size(medium):
    from paper_2303_13775_amd import Context
    w, dev, host = medium
    S, L = w.n_splits, w.n_layers
    batch = w.batch * S
    mini = Context(w.indptr, w.indices, w.pmap, S, w.fanouts, batch)
    micro = Context(w.indptr, w.indices, torch.zeros_like(w.pmap), 1, w.fanouts, w.batch)
    tg = workloads.draw_targets(w.n_vertices, batch, seed=w.seed, it=1, device=dev)
    mini.gsplit_sample_split(tg, 7, 1)
    edges = torch.zeros(L * S, dtype=torch.int64, device=dev)
    cross = torch.zeros(L * S, dtype=torch.int64, device=dev)
    mini.gsplit_batch_stats(edges, cross)
    ob = R.sp_sample(host["indptr"], host["indices"], host["pmap"], S, w.fanouts, tg.cpu().numpy(), 7, 1)
    we, wc = R.batch_stats(ob, host["pmap"])
    assert np.array_equal(edges.cpu().numpy().reshape(L, S), we)
    assert np.array_equal(cross.cpu().numpy().reshape(L, S), wc)
    n_local, _, n_edges, _ = mini.gsplit_batch_sizes()
    got = {"edges_mini": int(np.sum(n_edges)), "features_mini": int(np.sum(n_local[0])), "edges_micro": 0,
           "features_micro": 0}
    mo = R.micro_batches(host["indptr"], host["indices"], w.fanouts, tg.cpu().numpy(), S, 7, 1)
    for m, part in enumerate(workloads.micro_batch_parts(tg, S)):
        micro.gsplit_sample_split(part, 7, 1 * S + m)
        nl, _, ne, _ = micro.gsplit_batch_sizes()
        got["edges_micro"] += int(np.sum(ne)); got["features_micro"] += int(np.sum(nl[0]))
        if m == 0:
            assert_batch_equal(micro.fetch_batch(), mo[m], 1, L)
    assert got == R.redundancy_counts(ob, mo)
    mini.close(); micro.close()


def test_cached_loading_medium_full_size(medium):
    from paper_2303_13775_amd import Context
    w, dev, host = medium
    S = w.n_splits
    ctx = Context(w.indptr, w.indices, w.pmap, S, w.fanouts, w.batch)
    table = torch.empty(w.feat.shape, dtype=w.feat.dtype, pin_memory=True)
    table.copy_(w.feat)
    cnt = torch.zeros(w.n_vertices, dtype=torch.int32, device=dev)
    pre = [w.targets(1000 + i) for i in range(12)]
    for i, t in enumerate(pre):
        ctx.gsplit_sample_split(t, 31, 1000 + i)
        ctx.gsplit_input_counts_accumulate(cnt)
    k_in = R.input_counts(host["indptr"], host["indices"], w.fanouts, [t.cpu().numpy() for t in pre], 31,
                          [1000 + i for i in range(12)])
    assert np.array_equal(cnt.cpu().numpy().astype(np.int64), k_in)
    own = [int((host["pmap"] == s).sum()) for s in range(S)]
    sel = R.cache_select(k_in, host["pmap"], S, [own[s] // 4 for s in range(S)])
    ctx.gsplit_cache_build(table, torch.from_numpy(np.concatenate(sel)).to(dev), [x.shape[0] for x in sel])
    tg = w.targets(2)
    ctx.gsplit_sample_split(tg, 31, 2)
    out = torch.empty((ctx.gsplit_max_rows(0), w.dims[0]), device=dev)
    hits = torch.zeros(S, dtype=torch.int64, device=dev)
    misses = torch.zeros(S, dtype=torch.int64, device=dev)
    ctx.gsplit_gather_features_cached(out, hits, misses)
    ob = R.sp_sample(host["indptr"], host["indices"], host["pmap"], S, w.fanouts, tg.cpu().numpy(), 31, 2)
    tab = table.numpy()
    want, wh, wm = R.cached_gather(tab, sel, [tab[i] for i in sel], ob)
    assert np.array_equal(out[:want.shape[0]].cpu().numpy().view(np.int32), want.view(np.int32))
    assert np.array_equal(hits.cpu().numpy(), wh) and np.array_equal(misses.cpu().numpy(), wm)
    assert wh.sum() > 0 and wm.sum() > 0
    ctx.close()


def test_bf16_path_medium_full_size(medium):
    """`bench.py --dtype bf16` on the benchmark workload: bf16 features, activations and stacked
    weights, bf16 MFMA products with float accumulation, against the oracle that rounds the same
    stored values to bf16."""
    from paper_2303_13775_amd import Context, SageParams, GSPLIT_BF16
    w, dev, host = medium
    ctx = Context(w.indptr, w.indices, w.pmap, w.n_splits, w.fanouts, w.batch)
    table = w.feat.to(torch.bfloat16)
    params = SageParams(w.dims, w.w_self, w.w_neigh, w.bias, dtype=GSPLIT_BF16)
    op = R.SageParams([t.cpu().numpy() for t in w.w_self], [t.cpu().numpy() for t in w.w_neigh],
                      [t.cpu().numpy() for t in w.bias])
    x0 = torch.empty((ctx.gsplit_max_rows(0), w.dims[0]), dtype=torch.bfloat16, device=dev)
    logits = torch.empty((w.batch, w.dims[-1]), device=dev)
    glog = torch.empty_like(logits)
    gws = [torch.empty_like(t) for t in w.w_self]
    gwn = [torch.empty_like(t) for t in w.w_neigh]
    gb = [torch.empty_like(t) for t in w.bias]
    it = 3
    tg = w.targets(it)
    ctx.gsplit_sample_split(tg, 99, it)
    ctx.gsplit_gather_features(table, x0)
    ctx.gsplit_sage_fwd(params, x0, logits)
    ob = R.sp_sample(host["indptr"], host["indices"], host["pmap"], w.n_splits, w.fanouts, tg.cpu().numpy(), 99, it)
    ids = torch.from_numpy(ob.local_cat(0)).long().to(dev)
    assert torch.equal(x0[:ids.numel()].view(torch.int16), table[ids].view(torch.int16))
    of = R.sp_forward(ob, table[ids].float().cpu().numpy(), op, store_bf16=True)
    y = w.labels[torch.from_numpy(tg.cpu().numpy()[ob.target_perm]).to(dev).long()].cpu().numpy()
    _, g = R.softmax_xent(of.logits, y)
    ctx.gsplit_sage_bwd(params, torch.from_numpy(g.astype(np.float32)).to(dev), gws, gwn, gb)
    torch.cuda.synchronize()
    rows = table[ids].float().cpu().numpy()
    r = dict(logits=logits.cpu().numpy(), gws=[t.cpu().numpy() for t in gws], gwn=[t.cpu().numpy() for t in gwn],
             gb=[t.cpu().numpy() for t in gb], of=of, batch=ob, op=op, rows=rows, g=g,
             act=SC.device_activations(ctx, w.dims, True))
    r["ob"], r["report"] = SC.conditioned_backward(ob, of, op, g, r["act"], SC.TAU_BF16_ROUNDED, store_bf16=True,
                                                   who="medium bf16")
    check_sage(r, w.n_layers, bf16=True, tag="medium")
    ctx.close()


def test_presample_counts_medium_full_size(medium):
    """`bench.py --presample` on the benchmark workload: vertex and edge counts of three sampled
    batches bit-exact, weights as count / N."""
    from paper_2303_13775_amd import Context
    w, dev, host = medium
    ctx = Context(w.indptr, w.indices, w.pmap, w.n_splits, w.fanouts, w.batch, keep_edge_ids=True)
    k_v = torch.zeros(w.n_vertices, dtype=torch.int32, device=dev)
    k_e = torch.zeros(w.indices.numel(), dtype=torch.int32, device=dev)
    its = [0, 1, 2]
    batches = [w.targets(i) for i in its]
    for i, tg in zip(its, batches):
        ctx.gsplit_sample_split(tg, 4242, i)
        ctx.gsplit_presample_accumulate(k_v, k_e)
    ov, oe = R.presample_counts(host["indptr"], host["indices"], w.fanouts, [b.cpu().numpy() for b in batches],
                                4242, its)
    assert np.array_equal(k_v.cpu().numpy().astype(np.int64), ov)
    assert np.array_equal(k_e.cpu().numpy().astype(np.int64), oe)
    w_v = torch.empty(w.n_vertices, dtype=torch.float32, device=dev)
    ctx.gsplit_presample_weights(k_v, len(its), w_v)
    want_v, _ = R.presample_weights(ov, oe, len(its))
    assert np.abs(w_v.cpu().numpy() - want_v).max() <= 1e-6 * max(1.0, want_v.max())
    ctx.close()
