"""Parity at the sizes of the large configurations (111M-vertex / 1.6B-edge graph, int64 indptr,
57 GB feature table resident in HBM).  Generating these graphs takes a minute or two of GPU time,
so the tests only run when GSPLIT_BIG=1 is set; they print their progress."""
import os
import time

import numpy as np
import pytest
import torch

import workloads
from oracle import reference as R
from test_gpu_parity import assert_batch_equal, TOL_F32

pytestmark = [pytest.mark.gpu,
              pytest.mark.skipif(os.environ.get("GSPLIT_BIG") != "1", reason="set GSPLIT_BIG=1 (minutes of GPU time)")]


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
