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
from test_gpu_parity import assert_batch_equal, TOL_F32

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
        obw = R.sp_backward(ob, of, op, g)
        e_f = R.max_rel_err(logits.cpu().numpy(), of.logits)
        sws, swn, sb, n_und = R.relu_decision_slack(ob, of, op, obw)
        say(f"{n_und} pre-activations are too close to zero for float32 to decide their ReLU")
        errs = [(R.grad_err(gws[l].cpu().numpy(), obw.gw_self[l], sws[l]),
                 R.grad_err(gwn[l].cpu().numpy(), obw.gw_neigh[l], swn[l]),
                 R.grad_err(gb[l].cpu().numpy(), obw.gbias[l], sb[l])) for l in range(w.n_layers)]
        say("per layer (w_self, w_neigh, bias) errors: " + str([tuple(f"{x:.1e}" for x in e) for e in errs]))
        e_b = max(max(e) for e in errs)
        say(f"max rel err: logits {e_f:.2e}, gradients {e_b:.2e}")
        assert e_f < TOL_F32 and e_b < TOL_F32
        # the same gradients as whole matrices, without the allowance for undecidable ReLU decisions
        # (a few flipped decisions among millions of rows do not move a norm)
        fro = lambda x, o: float(np.linalg.norm(x.cpu().numpy().astype(np.float64) - o) / max(np.linalg.norm(o), 1e-300))
        norms = [(fro(gws[l], obw.gw_self[l]), fro(gwn[l], obw.gw_neigh[l]), fro(gb[l], obw.gbias[l]))
                 for l in range(w.n_layers)]
        say("relative Frobenius errors per layer: " + str([tuple(f"{x:.1e}" for x in e) for e in norms]))
        assert max(max(e) for e in norms) < TOL_F32
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
    from test_gpu_gat import attention_grad_err
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
    obw = G.gat_backward(ob, of, op, g)
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


@pytest.mark.parametrize("n_splits", [1, 8])
def test_sweep_bf16_full_size(n_splits):
    """The split sweep of `bench.py --workload sweep`: the large graph, 8192 targets, four layers of
    fanout 10, bf16 storage, with one split (both keys of a vertex are the same key and one table
    serves) and with eight (every class of the partition in use).  Every integer output of the
    sampled batch is compared, and the bf16 forward pass with the loss gradient's backward pass
    against the oracle that rounds the same stored values."""
    from paper_2303_13775_amd import Context, SageParams, GSPLIT_BF16
    from test_gpu_parity import FLOOR_BF16, TOL_BF16
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
    obw = R.sp_backward(ob, of, op, g, store_bf16=True)
    sws, swn, sb, _ = R.relu_decision_slack(ob, of, op, obw, rel_tau=1e-3, store_bf16=True)
    say(f"oracle forward/backward in {time.time() - t0:.1f} s")
    e_f = R.max_rel_err(logits.cpu().numpy(), of.logits, floor=FLOOR_BF16)
    errs = [(R.grad_err(gws[l].cpu().numpy(), obw.gw_self[l], sws[l], floor=FLOOR_BF16),
             R.grad_err(gwn[l].cpu().numpy(), obw.gw_neigh[l], swn[l], floor=FLOOR_BF16),
             R.grad_err(gb[l].cpu().numpy(), obw.gbias[l], sb[l], floor=FLOOR_BF16)) for l in range(w.n_layers)]
    say(f"max rel err: logits {e_f:.2e}; per layer " + str([tuple(f"{x:.1e}" for x in e) for e in errs]))
    assert e_f < TOL_BF16 and max(max(e) for e in errs) < TOL_BF16
    # With millions of rows the undecidable ReLU decisions explain most elementwise differences of
    # the lower layers' gradients, so those are also compared as whole matrices, without that
    # allowance: a handful of flipped decisions does not move a norm over millions of rows.
    fro = lambda a, o: float(np.linalg.norm(a.cpu().numpy().astype(np.float64) - o) / max(np.linalg.norm(o), 1e-300))
    norms = [(fro(gws[l], obw.gw_self[l]), fro(gwn[l], obw.gw_neigh[l]), fro(gb[l], obw.gbias[l]))
             for l in range(w.n_layers)]
    say("relative Frobenius errors per layer: " + str([tuple(f"{x:.1e}" for x in e) for e in norms]))
    assert max(max(e) for e in norms) < TOL_BF16
    ctx.close()
