"""Parity at the sizes of the large configurations (111M-vertex / 1.6B-edge graph, int64 indptr,
57 GB feature table resident in HBM; 65M-vertex / 3.6B-edge skewed graph).  The graphs are generated
on the GPU in a few seconds each and the whole file runs in about half a minute; it needs about
80 GB of HBM and 10 GB of host memory.  GSPLIT_SKIP_BIG=1 leaves it out.  The tests print their
progress.  (The file name puts them last in the GPU suite: they are the tests that depend most
on what else is using the machine.)"""
import os
import time

import numpy as np
import pytest
import torch

import workloads
from oracle import reference as R
from test_gpu_parity import assert_batch_equal, check_sage, TOL_F32
import sage_check as SC

pytestmark = [pytest.mark.gpu,
              pytest.mark.skipif(os.environ.get("GSPLIT_SKIP_BIG") == "1", reason="GSPLIT_SKIP_BIG=1")]


def say(msg):
    print(f"[big {time.strftime('%H:%M:%S')}] {msg}", flush=True)


def _run(w, dev, iters=(0, 1)):
    from paper_2303_13775_amd import Context, SageParams
    ctx = Context(w.indptr, w.indices, w.pmap, w.n_splits, w.fanouts, w.batch)
    say("context created; copying the CSR to the host for the oracle")
    host = dict(indptr=w.indptr.cpu().numpy(), indices=w.indices.cpu().numpy(), pmap=w.pmap.cpu().numpy())
    params = SageParams(w.dims, w.w_self, w.w_neigh, w.bias)
    op = R.SageParams([t.cpu().numpy() for t in w.w_self], [t.cpu().numpy() for t in w.w_neigh],
                      [t.cpu().numpy() for t in w.bias])
    x0 = torch.empty((ctx.gsplit_max_rows(0), w.dims[0]), dtype=w.feat.dtype, device=dev)
    logits = torch.empty((w.batch, w.dims[-1]), device=dev)
    glog = torch.empty_like(logits)
    gws = [torch.empty_like(t) for t in w.w_self]
    gwn = [torch.empty_like(t) for t in w.w_neigh]
    gb = [torch.empty_like(t) for t in w.bias]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    for it in iters:
        tg = w.targets(it)
        torch.cuda.synchronize()
        ev[0].record(); ctx.gsplit_sample_split(tg, 4242, it)
        ev[1].record(); ctx.gsplit_gather_features(w.feat, x0)
        ev[2].record(); ctx.gsplit_sage_fwd(params, x0, logits)
        ev[3].record(); ctx.gsplit_softmax_xent(logits, w.labels, glog)
        ev[4].record(); ctx.gsplit_sage_bwd(params, glog, gws, gwn, gb)
        ev[5].record(); torch.cuda.synchronize()
        ms = [ev[k].elapsed_time(ev[k + 1]) for k in range(5)]
        n_local, n_mixed, n_edges, _ = ctx.gsplit_batch_sizes()
        rows0 = sum(n_local[0])
        gbs = rows0 * (2 * w.dims[0] * w.feat.element_size() + 4) / (ms[1] * 1e-3) / 1e9
        say(f"iter {it}: sample_split {ms[0]:.3f} ms, gather {ms[1]:.3f} ms ({gbs:.0f} GB/s), fwd {ms[2]:.3f}, "
            f"loss {ms[3]:.3f}, bwd {ms[4]:.3f}; rows/level {[sum(x) for x in n_local]}, "
            f"edges/layer {[sum(x) for x in n_edges]}")
        t0 = time.time()
        ob = R.sp_sample(host["indptr"], host["indices"], host["pmap"], w.n_splits, w.fanouts,
                         tg.cpu().numpy(), 4242, it)
        say(f"oracle sampled the batch in {time.time() - t0:.1f} s; comparing every integer output")
        assert_batch_equal(ctx.fetch_batch(), ob, w.n_splits, w.n_layers)
        ids = torch.from_numpy(ob.local_cat(0)).long().to(dev)
        assert torch.equal(x0[:ids.numel()], w.feat[ids])
        of = R.sp_forward(ob, w.feat[ids].float().cpu().numpy(), op)
        y = w.labels[torch.from_numpy(tg.cpu().numpy()[ob.target_perm]).to(dev).long()].cpu().numpy()
        _, g = R.softmax_xent(of.logits, y)
        obw, report = SC.conditioned_backward(ob, of, op, g, SC.device_activations(ctx, w.dims, False), SC.TAU_F32,
                                              who=f"{w.name} it {it}")
        e_f = R.max_rel_err(logits.cpu().numpy(), of.logits)
        say(f"ReLU band per layer (entries with |z| <= {SC.TAU_F32:g} max|z|, decided otherwise by the device, "
            f"disagreements outside): {report}")
        errs = SC.grad_errors(gws, gwn, gb, obw)
        say("per layer (w_self, w_neigh, bias) elementwise errors, no allowance: " + SC.fmt(errs))
        e_b = max(max(e) for e in errs)
        say(f"max rel err: logits {e_f:.2e}, gradients {e_b:.2e}")
        assert e_f < TOL_F32 and e_b < TOL_F32
        for l in range(w.n_layers):
            SC.assert_shuffle_index_equal(ctx, ob, l, has_rev=l >= 1)
        say("both sides of the shuffle index equal the oracle's")
    ctx.close()


def test_large_fp32_full_size():
    dev = torch.device("cuda:0")
    w = workloads.large(device=dev, progress=say)
    say(str(w.describe()))
    _run(w, dev)


def test_skewed_fp32_full_size():
    dev = torch.device("cuda:0")
    w = workloads.skewed(device=dev, progress=say)
    say(str(w.describe()))
    _run(w, dev, iters=(0,))


def test_large_gat_statistics_and_counts_full_size():
    """The GAT model (paper section 7.1), the split statistics (section 7.2) and the pre-sampling
    counts (section 5) on the large graph: every logit, every parameter gradient and every counter
    against the oracle on one full-size batch."""
    from paper_2303_13775_amd import Context, GatParams
    from oracle import gat as G
    from test_gpu_gat import attention_grad_err, conditioned_gat_backward
    dev = torch.device("cuda:0")
    w = workloads.large(device=dev, progress=say)
    say(str(w.describe()))
    heads = [4, 4, 1]
    ctx = Context(w.indptr, w.indices, w.pmap, w.n_splits, w.fanouts, w.batch, gat_index=True)
    host = dict(indptr=w.indptr.cpu().numpy(), indices=w.indices.cpu().numpy(), pmap=w.pmap.cpu().numpy())
    tg = w.targets(0)
    ctx.gsplit_sample_split(tg, 4242, 0)
    x0 = torch.empty((ctx.gsplit_max_rows(0), w.dims[0]), dtype=torch.float32, device=dev)
    ctx.gsplit_gather_features(w.feat, x0)
    wt, a_s, a_d, b = workloads.gat_weights(w.dims, heads, seed=w.seed)
    params = GatParams(w.dims, heads, [t.to(dev) for t in wt], [t.to(dev) for t in a_s],
                       [t.to(dev) for t in a_d], [t.to(dev) for t in b])
    logits = torch.empty((w.batch, w.dims[-1]), device=dev)
    ctx.gsplit_gat_fwd(params, x0, logits)
    L, S = w.n_layers, w.n_splits
    edges = torch.zeros(L * S, dtype=torch.int64, device=dev)
    cross = torch.zeros(L * S, dtype=torch.int64, device=dev)
    ctx.gsplit_batch_stats(edges, cross)
    count = torch.zeros(w.n_vertices, dtype=torch.int32, device=dev)
    ctx.gsplit_input_counts_accumulate(count)
    torch.cuda.synchronize()
    say("GPU side done; the oracle samples the batch")
    ob = R.sp_sample(host["indptr"], host["indices"], host["pmap"], w.n_splits, w.fanouts,
                     tg.cpu().numpy(), 4242, 0)
    e, c = R.batch_stats(ob, host["pmap"])
    assert np.array_equal(edges.cpu().numpy().reshape(L, S), e)
    assert np.array_equal(cross.cpu().numpy().reshape(L, S), c)
    say(f"edges {int(e.sum())}, crossing {int(c.sum())} ({100.0 * c.sum() / e.sum():.1f} %)")
    ids = ob.local_cat(0)
    nz = torch.nonzero(count).flatten().cpu().numpy()
    assert np.array_equal(nz, np.sort(ids)) and int(count.sum().item()) == ids.size
    op = G.GatParams(list(heads), [t.numpy() for t in wt], [t.numpy() for t in a_s], [t.numpy() for t in a_d],
                     [t.numpy() for t in b])
    t0 = time.time()
    of = G.gat_forward(ob, w.feat[torch.from_numpy(ids).long().to(dev)].double().cpu().numpy(), op)
    say(f"oracle forward in {time.time() - t0:.1f} s")
    e_f = R.max_rel_err(logits.cpu().numpy(), of.logits)
    say(f"logits max rel err {e_f:.2e}")
    assert e_f < TOL_F32
    lab = w.labels.cpu().numpy()[tg.cpu().numpy()[ob.target_perm]]
    _, g = R.softmax_xent(of.logits, lab)
    gw = [torch.empty_like(t, device=dev) for t in wt]
    gas = [torch.empty_like(t, device=dev) for t in a_s]
    gad = [torch.empty_like(t, device=dev) for t in a_d]
    gb = [torch.empty_like(t, device=dev) for t in b]
    ctx.gsplit_gat_bwd(params, x0, torch.from_numpy(g.astype(np.float32)).to(dev), gw, gas, gad, gb)
    torch.cuda.synchronize()
    t0 = time.time()
    obw, _ = conditioned_gat_backward(ctx, ob, of, op, g, heads, who="gat")
    say(f"oracle backward in {time.time() - t0:.1f} s")
    for l in range(w.n_layers):
        o_src, o_dst = obw.ga_src[l], obw.ga_dst[l]
        errs = (R.max_rel_err(gw[l].cpu().numpy(), obw.gw[l]),
                attention_grad_err(gas[l].cpu().numpy(), o_src, o_src, o_dst, obw.ga_terms[l]),
                attention_grad_err(gad[l].cpu().numpy(), o_dst, o_src, o_dst, obw.ga_terms[l]),
                R.max_rel_err(gb[l].cpu().numpy().reshape(-1), obw.gbias[l].reshape(-1)))
        say(f"layer {l} (w, a_src, a_dst, bias) errors: " + ", ".join(f"{x:.1e}" for x in errs))
        assert max(errs) < TOL_F32, l
    ctx.close()


@pytest.mark.parametrize("n_splits", [1, 2, 4, 8])
def test_sweep_bf16_full_size(n_splits):
    """The split sweep of `bench.py --workload sweep`: the large graph, 8192 targets, four layers of
    fanout 10, bf16 storage, with one split (both keys of a vertex are the same key and one table
    serves) and with eight (every class of the partition in use).  Every integer output of the
    sampled batch is compared, and the bf16 forward pass with the loss gradient's backward pass
    against the oracle that rounds the same stored values."""
    from paper_2303_13775_amd import Context, SageParams, GSPLIT_BF16
    dev = torch.device("cuda:0")
    w = workloads.large(device=dev, n_splits=n_splits, feat_dtype=torch.bfloat16, batch=8192,
                        fanouts=(10, 10, 10, 10), dims=(128, 256, 256, 256, 172), progress=say)
    say(str(w.describe()))
    ctx = Context(w.indptr, w.indices, w.pmap, w.n_splits, w.fanouts, w.batch)
    host = dict(indptr=w.indptr.cpu().numpy(), indices=w.indices.cpu().numpy(), pmap=w.pmap.cpu().numpy())
    params = SageParams(w.dims, w.w_self, w.w_neigh, w.bias, dtype=GSPLIT_BF16)
    op = R.SageParams([t.cpu().numpy() for t in w.w_self], [t.cpu().numpy() for t in w.w_neigh],
                      [t.cpu().numpy() for t in w.bias])
    x0 = torch.empty((ctx.gsplit_max_rows(0), w.dims[0]), dtype=torch.bfloat16, device=dev)
    logits = torch.empty((w.batch, w.dims[-1]), device=dev)
    gws = [torch.empty_like(t) for t in w.w_self]
    gwn = [torch.empty_like(t) for t in w.w_neigh]
    gb = [torch.empty_like(t) for t in w.bias]
    it = 1
    tg = w.targets(it)
    ctx.gsplit_sample_split(tg, 777, it)
    ctx.gsplit_gather_features(w.feat, x0)
    ctx.gsplit_sage_fwd(params, x0, logits)
    torch.cuda.synchronize()
    t0 = time.time()
    ob = R.sp_sample(host["indptr"], host["indices"], host["pmap"], w.n_splits, w.fanouts, tg.cpu().numpy(), 777, it)
    say(f"oracle sampled the batch in {time.time() - t0:.1f} s; rows/level {[len(ob.local_cat(l)) for l in range(w.n_layers + 1)]}")
    assert_batch_equal(ctx.fetch_batch(), ob, w.n_splits, w.n_layers)
    ids = torch.from_numpy(ob.local_cat(0)).long().to(dev)
    assert torch.equal(x0[:ids.numel()].view(torch.int16), w.feat[ids].view(torch.int16))
    t0 = time.time()
    of = R.sp_forward(ob, w.feat[ids].float().cpu().numpy(), op, store_bf16=True)
    y = w.labels[torch.from_numpy(tg.cpu().numpy()[ob.target_perm]).to(dev).long()].cpu().numpy()
    _, g = R.softmax_xent(of.logits, y)
    ctx.gsplit_sage_bwd(params, torch.from_numpy(g.astype(np.float32)).to(dev), gws, gwn, gb)
    torch.cuda.synchronize()
    rows = w.feat[ids].float().cpu().numpy()
    r = dict(logits=logits.cpu().numpy(), gws=[t.cpu().numpy() for t in gws], gwn=[t.cpu().numpy() for t in gwn],
             gb=[t.cpu().numpy() for t in gb], of=of, batch=ob, op=op, rows=rows, g=g,
             act=SC.device_activations(ctx, w.dims, True))
    r["ob"], r["report"] = SC.conditioned_backward(ob, of, op, g, r["act"], SC.TAU_BF16_ROUNDED, store_bf16=True,
                                                   who=w.name)
    say(f"oracle forward/backward in {time.time() - t0:.1f} s")
    check_sage(r, w.n_layers, bf16=True, tag=f"sweep-S{n_splits}")
    for l in range(w.n_layers):
        SC.assert_shuffle_index_equal(ctx, ob, l, has_rev=l >= 1)
    ctx.close()
