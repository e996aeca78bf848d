"""The schedules bench.py times, checked as they are timed, on the benchmark workload at its full
size: (groups, the default) two groups of eight batch slots, the mini-batches of a group sampled by
one gsplit_sample_split_multi call on a sampling stream while the training stream works through
the group before; (streams, `--multi 1`) three batch slots, two sampling streams and a training
stream.  Contexts whose sampling kernels may occupy two workgroups per compute unit, two host
threads, events handing the slots over in both directions.  After a run every slot still holds its last step: the integer outputs, the
gathered rows, the logits and every gradient of those steps against the oracle (GraphSAGE), and
for both models the logits against a strictly serial run of the same steps on one stream
(bit-equal: same kernels, same inputs)."""
import numpy as np
import pytest
import torch

import bench
import workloads
from oracle import reference as R
from test_gpu_parity import TOL_F32, assert_batch_equal
import sage_check as SC

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("model,schedule", [("sage", "groups"), ("sage", "streams"), ("gat", "groups"), ("gat", "streams")])
def test_pipelined_schedule_leaves_the_oracles_results_in_every_slot(model, schedule):
    assert torch.cuda.is_available(), "needs the MI355X"
    dev = torch.device("cuda:0")
    w = workloads.medium(device=dev)
    n_steps = 27 if schedule == "groups" else 11     # groups of 2, 4, 8, 8 and a partial last one of 5
    targets = [w.targets(i) for i in range(n_steps)]
    torch.cuda.synchronize()
    if schedule == "groups":
        pipe = bench.PipelinedGroups(w, dev, 8, model, 4, 2)
        slot_of = lambda i: pipe.slot_of_step(i, 0, n_steps)
    else:
        pipe = bench.Pipelined(w, dev, 2, model, 4, 2)
        slot_of = lambda i: pipe.slots[i % pipe.n]
    pipe.run(targets, 0, n_steps)
    torch.cuda.synchronize()
    last = {}                                       # the last step every slot worked on
    for i in range(n_steps):
        last[id(slot_of(i))] = i
    host = dict(indptr=w.indptr.cpu().numpy(), indices=w.indices.cpu().numpy(), pmap=w.pmap.cpu().numpy())
    op = R.SageParams([t.cpu().numpy() for t in w.w_self], [t.cpu().numpy() for t in w.w_neigh],
                      [t.cpu().numpy() for t in w.bias])
    serial = bench.Runner(w, dev, model, 4)
    assert len(last) >= 3
    for i in sorted(last.values()):
        r = slot_of(i)
        tg = targets[i]
        ob = R.sp_sample(host["indptr"], host["indices"], host["pmap"], w.n_splits, w.fanouts,
                         tg.cpu().numpy(), r.seed, i)
        assert_batch_equal(r.ctx.fetch_batch(), ob, w.n_splits, w.n_layers)
        ids = torch.from_numpy(ob.local_cat(0)).long().to(dev)
        assert torch.equal(r.x0[:ids.numel()], w.feat[ids]), ("gathered rows", i)
        serial.step(tg, i)
        torch.cuda.synchronize()
        assert torch.equal(serial.logits, r.logits), ("serial and pipelined logits differ", i)
        if model != "sage":         # the GAT kernels' own parity at this size is test_gpu_medium_rows'
            continue
        of = R.sp_forward(ob, w.feat[ids].cpu().numpy(), op)
        y = w.labels[torch.from_numpy(tg.cpu().numpy()[ob.target_perm]).to(dev).long()].cpu().numpy()
        _, g = R.softmax_xent(of.logits, y)
        obw, report = SC.conditioned_backward(ob, of, op, g, SC.device_activations(r.ctx, w.dims, False), SC.TAU_F32,
                                              who=f"slot of step {i}")
        assert R.max_rel_err(r.logits.cpu().numpy(), of.logits) < TOL_F32, ("logits", i)
        gws, gwn, gb = r.grads
        errs = SC.grad_errors(gws, gwn, gb, obw)
        print(f"\n[pipelined step {i}] per layer (gw_self, gw_neigh, gbias) {SC.fmt(errs)}; ReLU band {report}", flush=True)
        for l in range(w.n_layers):
            assert max(errs[l]) < TOL_F32, ("gradients of layer", i, l, errs[l])
    for r in pipe.slots + [serial]:
        r.ctx.close()
