"""A whole step (sample + split, gather, forward, loss, backward) captured into a HIP graph and
replayed for several iterations, with eager work and synchronisations between the replays: every
replay must give what the eager path gives for the same targets, seed and iteration (integer
outputs and logits bit for bit; gradients up to the summation order of the reverse shuffle)."""
import numpy as np
import pytest
import torch

import workloads
from test_gpu_parity import TOL_F32

pytestmark = pytest.mark.gpu


def _dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


class _Step:
    def __init__(self, w, dev, model):
        from paper_2303_13775_amd import Context, SageParams, GatParams
        self.w, self.model = w, model
        self.ctx = Context(w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev), w.n_splits, w.fanouts, w.batch,
                           gat_index=model == "gat")
        self.feat, self.labels = w.feat.to(dev), w.labels.to(dev)
        if model == "gat":
            heads = [2] * (w.n_layers - 1) + [1]
            wt = workloads.gat_weights(w.dims, heads, seed=w.seed, device=dev)
            self.params = GatParams(w.dims, heads, *wt)
            self.grads = [[torch.zeros_like(t) for t in lst] for lst in wt]
        else:
            ws = [[t.to(dev) for t in lst] for lst in (w.w_self, w.w_neigh, w.bias)]
            self.params = SageParams(w.dims, *ws)
            self.grads = [[torch.zeros_like(t) for t in lst] for lst in ws]
        self.x0 = torch.zeros((self.ctx.gsplit_max_rows(0), w.dims[0]), device=dev)
        self.logits = torch.zeros((w.batch, w.dims[-1]), device=dev)
        self.glog = torch.zeros_like(self.logits)
        self.tg = torch.zeros(w.batch, dtype=torch.int32, device=dev)
        self.seed_iter = torch.zeros(2, dtype=torch.int64, device=dev)

    def rest(self):
        c = self.ctx
        c.gsplit_gather_features(self.feat, self.x0)
        if self.model == "gat":
            c.gsplit_gat_fwd(self.params, self.x0, self.logits)
            c.gsplit_softmax_xent(self.logits, self.labels, self.glog)
            c.gsplit_gat_bwd(self.params, self.x0, self.glog, *self.grads)
        else:
            c.gsplit_sage_fwd(self.params, self.x0, self.logits)
            c.gsplit_softmax_xent(self.logits, self.labels, self.glog)
            c.gsplit_sage_bwd(self.params, self.glog, *self.grads)

    def eager(self, targets, seed, it):
        self.ctx.gsplit_sample_split(targets, seed, it)
        self.rest()

    def from_device_state(self):
        self.ctx.gsplit_sample_split_dev(self.tg, self.seed_iter)
        self.rest()


@pytest.mark.parametrize("model", ["sage", "gat"])
def test_captured_step_replays_match_eager(model):
    dev = _dev()
    w = workloads.tiny()
    seed = 0xABCDEF
    ref, cap = _Step(w, dev, model), _Step(w, dev, model)
    # one eager step sizes the internal buffers; then the capture
    cap.tg.copy_(w.targets(9).to(dev)); cap.seed_iter.copy_(torch.tensor([seed, 9]))
    cap.from_device_state()
    torch.cuda.synchronize()
    side = torch.cuda.Stream(device=dev)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        cap.from_device_state()
    torch.cuda.synchronize()
    for it in (3, 1, 4, 1, 2):
        tg = w.targets(it).to(dev)
        # eager work and synchronisations between the replays
        cap.tg.copy_(tg)
        cap.seed_iter.copy_(torch.tensor([seed, it]))
        for lst in cap.grads:
            for t in lst:
                t.fill_(7.0)
        cap.logits.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref.eager(tg, seed, it)
        torch.cuda.synchronize()
        a, b = cap.ctx.fetch_batch(), ref.ctx.fetch_batch()
        assert a["n_local"] == b["n_local"] and a["n_edges"] == b["n_edges"] and a["bucket"] == b["bucket"], it
        for l in range(w.n_layers + 1):
            for s in range(w.n_splits):
                assert torch.equal(a["local_front"][l][s], b["local_front"][l][s]), (it, l, s)
        for l in range(w.n_layers):
            for key in ("nbr", "cnt", "blk_indptr", "blk_src", "recv"):
                assert torch.equal(a["layers"][l][key], b["layers"][l][key]), (it, l, key)
        assert torch.equal(cap.logits, ref.logits), it
        for la, lb in zip(cap.grads, ref.grads):
            for ta, tb in zip(la, lb):
                scale = float(tb.abs().max()) + 1e-30
                assert float((ta - tb).abs().max()) / scale < TOL_F32, it
    cap.ctx.close(); ref.ctx.close()
