#!/usr/bin/env python3
"""Benchmark of the split-parallel hot path on one MI355X.

One step = one whole iteration over a fresh synthetic mini-batch, all inputs resident in HBM:
gsplit_sample_split -> gsplit_gather_features -> gsplit_sage_fwd -> gsplit_softmax_xent (loss
gradient of the logits) -> gsplit_sage_bwd.  Prints ONE JSON line.  `--model gat` runs the paper's
second model (gsplit_gat_fwd / gsplit_gat_bwd) through the same steps.

The workload is the "medium" configuration (2.4M-vertex / ~124M-edge R-MAT graph, 100-d fp32
features, 47 classes, range partition map, 4 logical splits, batch 1024, fanouts [15,10,5],
hidden 256); `--workload tiny` selects the small case.  All data is synthetic and seeded.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
FP32_MFMA_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix
BF16_MFMA_PEAK_TFLOPS = 2500.0 # MI355X dense bf16 matrix


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="medium", choices=["medium", "tiny", "large", "skewed", "sweep"])
    ap.add_argument("--dtype", default=None, choices=["f32", "bf16"],
                    help="storage/compute type of the GraphSAGE layers (default f32; sweep: bf16)")
    ap.add_argument("--splits", type=int, default=4, help="number of logical splits")
    ap.add_argument("--model", default="sage", choices=["sage", "gat"])
    ap.add_argument("--heads", type=int, default=4, help="GAT: attention heads of the hidden layers (the last has one)")
    ap.add_argument("--separate-calls", action="store_true",
                    help="GraphSAGE: forward, loss and backward as three calls (gsplit_sage_fwd, gsplit_softmax_xent, "
                         "gsplit_sage_bwd) instead of gsplit_sage_step, which runs the top layer as one kernel")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-iters", type=int, default=120)
    ap.add_argument("--no-pipeline", action="store_true",
                    help="time strictly serial steps on one stream (default: sampling+gather of step i+1 "
                         "overlaps forward/backward of step i on a second stream)")
    ap.add_argument("--ahead", type=int, default=2, help="sampling streams (steps sampled ahead); used with --multi 1")
    ap.add_argument("--multi", type=int, default=8,
                    help="mini-batches sampled per gsplit_sample_split_multi call (sampling does not depend on the "
                         "weights: the batches of the next K steps go through one set of launches); 1 = one call per step")
    ap.add_argument("--sampler-blocks", type=int, default=2,
                    help="pipelined schedule: workgroups per compute unit the sampling kernels may occupy")
    ap.add_argument("--graph", action="store_true",
                    help="replay the timed steps as captured HIP graphs instead of enqueueing every kernel from the "
                         "host (measured: no faster here, the steps are bound by the device-side kernel boundaries, "
                         "not by the host's launch rate)")
    ap.add_argument("--presample", action="store_true",
                    help="measure the offline pre-sampling stage instead (sampling + counting of k_v, k_e)")
    ap.add_argument("--redundancy", action="store_true",
                    help="data-parallel micro-batch mode against split mode: one mini-batch of splits x batch "
                         "targets, once split and once as `splits` independent micro-batches (Table 1 counters, "
                         "workload imbalance, cross-edge share, time per iteration)")
    ap.add_argument("--cache-frac", type=float, default=None,
                    help="keep the feature table in pinned host memory and cache this fraction of every split's "
                         "vertices in HBM, ranked by pre-sampled input-layer frequency; the loading step then is "
                         "gsplit_gather_features_cached (0 = everything over the host link)")
    ap.add_argument("--cache-presample", type=int, default=200, help="sampling iterations that rank the cache")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference point for HBM byte counters)")
    ap.add_argument("--stage-iters", type=int, default=50)
    ap.add_argument("--extra-configs", dest="extra_configs", action="store_true", default=None,
                    help="after the benchmark workload also time large (f32, bf16), skewed and the split sweep "
                         "(S = 1, 2, 4, 8), serially, and report them under extra_configs (default: on for the "
                         "default medium / sage / f32 run)")
    ap.add_argument("--no-extra-configs", dest="extra_configs", action="store_false")
    return ap.parse_args()


class Runner:
    """Holds the device-resident inputs, the context and the preallocated outputs of a step."""

    separate_calls = False      # set from --separate-calls

    def __init__(self, w, dev, model="sage", heads=4, sampler_blocks_per_cu=0):
        import torch
        import workloads
        from paper_2303_13775_amd import Context, SageParams, GatParams
        self.torch = torch
        self.w, self.dev, self.model = w, dev, model
        from paper_2303_13775_amd import GSPLIT_BF16, GSPLIT_F32
        self.ctx = Context(w.indptr, w.indices, w.pmap, w.n_splits, w.fanouts, w.batch, gat_index=model == "gat",
                           sampler_blocks_per_cu=sampler_blocks_per_cu)
        if model == "gat":
            self.heads = [heads] * (w.n_layers - 1) + [1]
            self.gat_w = workloads.gat_weights(w.dims, self.heads, seed=w.seed, device=dev)
            self.params = GatParams(w.dims, self.heads, *self.gat_w)
            self.grads = [[torch.empty_like(t) for t in lst] for lst in self.gat_w]
        else:
            self.params = SageParams(w.dims, w.w_self, w.w_neigh, w.bias,
                                     dtype=GSPLIT_BF16 if w.feat.dtype == torch.bfloat16 else GSPLIT_F32)
            self.grads = [[torch.empty_like(t) for t in lst] for lst in (w.w_self, w.w_neigh, w.bias)]
        self.x0 = torch.empty((self.ctx.gsplit_max_rows(0), w.dims[0]), dtype=w.feat.dtype, device=dev)
        self.logits = torch.empty((w.batch, w.dims[-1]), device=dev)
        self.glogits = torch.empty_like(self.logits)
        self.seed = 0xC0FFEE

    def enable_cache(self, host_table, cache_ids, n_cache):
        self.ctx.gsplit_cache_build(host_table, cache_ids, n_cache)
        self.cached = True
        S = self.w.n_splits
        self.hits = self.torch.zeros(S, dtype=self.torch.int64, device=self.dev)
        self.misses = self.torch.zeros(S, dtype=self.torch.int64, device=self.dev)

    def load(self, count=False):
        if getattr(self, "cached", False):
            # the hit / miss counters are an extra pass over the rows: only when asked for
            self.ctx.gsplit_gather_features_cached(self.x0, self.hits if count else None, self.misses if count else None)
        else:
            self.ctx.gsplit_gather_features(self.w.feat, self.x0)

    # -- captured steps: the targets of step i are row i of one device table, the step counter lives
    # in device memory and advances with every replay, so a replay needs nothing from the host
    def prepare_graphs(self, targets_all, stride):
        torch = self.torch
        self.targets_all = targets_all
        self.tg_buf = torch.zeros(self.w.batch, dtype=torch.int32, device=self.dev)
        self.seed_iter = torch.tensor([self.seed, 0], dtype=torch.int64, device=self.dev)
        self.step_idx = torch.zeros(1, dtype=torch.int64, device=self.dev)
        self.stride = stride

    def _next_targets(self):
        self.tg_buf.view(1, -1).copy_(self.targets_all.index_select(0, self.step_idx))
        self.seed_iter[1:2].copy_(self.step_idx)
        self.step_idx.add_(self.stride)

    def _sample_from_device_state(self):
        self._next_targets()
        self.ctx.gsplit_sample_split_dev(self.tg_buf, self.seed_iter)
        self.load()

    def _train(self):
        self.train()

    def train(self):
        """Forward, loss and backward of the current batch: one call for GraphSAGE unless told otherwise."""
        if self.model == "sage" and not Runner.separate_calls:
            self.ctx.gsplit_sage_step(self.params, self.x0, self.w.labels, self.logits, *self.grads)
        else:
            self.forward()
            self.loss()
            self.backward()

    def capture(self, stream, parts):
        """One graph per element of parts ('sample', 'train', or 'step' for both)."""
        torch = self.torch
        out = {}
        for part in parts:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                if part in ("sample", "step"):
                    self._sample_from_device_state()
                if part in ("train", "step"):
                    self._train()
            out[part] = g
        return out

    def forward(self):
        if self.model == "gat":
            self.ctx.gsplit_gat_fwd(self.params, self.x0, self.logits)
        else:
            self.ctx.gsplit_sage_fwd(self.params, self.x0, self.logits)

    def loss(self):
        self.ctx.gsplit_softmax_xent(self.logits, self.w.labels, self.glogits)

    def backward(self):
        if self.model == "gat":
            self.ctx.gsplit_gat_bwd(self.params, self.x0, self.glogits, *self.grads)
        else:
            self.ctx.gsplit_sage_bwd(self.params, self.glogits, *self.grads)

    def step(self, targets, it, events=None):
        c = self.ctx
        rec = (lambda k: events[k].record()) if events is not None else (lambda k: None)
        rec(0)
        c.gsplit_sample_split(targets, self.seed, it)
        rec(1)
        self.load()
        rec(2)
        if self.model == "sage" and not Runner.separate_calls:
            self.train()
            rec(3)
            return
        self.forward()
        rec(3)
        self.loss()
        rec(4)
        self.backward()
        rec(5)


class Pipelined:
    """Batch slots on several streams: while the forward/backward pass of step i runs on the
    training stream, sampling, splitting and the feature gather of the next steps run on
    sampling streams (they do not depend on the weights; forward/backward of consecutive steps
    stay strictly ordered, as synchronous training requires).  Every step still does all of its
    work; nothing is cached or skipped.  Events order the hand-over of a slot in both directions."""

    def __init__(self, w, dev, n_ahead=2, model="sage", heads=4, sampler_blocks=2):
        import torch
        self.torch = torch
        self.n = n_ahead + 1
        # sampling kernels are latency-bound: two workgroups per compute unit instead of eight cost them
        # about 1 % and leave wave slots for the training stream's workgroups (medium: +5 % throughput)
        self.slots = [Runner(w, dev, model, heads, sampler_blocks_per_cu=sampler_blocks) for _ in range(self.n)]
        self.s_sample = [torch.cuda.Stream(device=dev) for _ in range(n_ahead)]
        self.s_train = torch.cuda.Stream(device=dev)
        self.ready = [torch.cuda.Event() for _ in range(self.n)]
        self.free = [torch.cuda.Event() for _ in range(self.n)]
        for e in self.free:
            e.record()
        # HIP binds a stream to one of its four hardware queues at first use, in order of first use,
        # and which streams end up sharing a queue changes the throughput of this schedule by up to
        # 20 % (measured: 2410 .. 3045 mini-batches/s over first-use orders).  Fix the order here
        # instead of leaving it to the race between the two enqueueing threads.
        for s in [self.s_train] + self.s_sample:
            with torch.cuda.stream(s):
                torch.zeros(1, device=dev)
        torch.cuda.synchronize()

    def enable_graphs(self, targets_all):
        """Captures, per slot, a sampling graph and a training graph (after every slot has run eagerly
        once, which sizes the library's buffers)."""
        torch = self.torch
        self.graphs = []
        for k, r in enumerate(self.slots):
            r.prepare_graphs(targets_all, self.n)
            self.graphs.append(r.capture(self.s_train, ("sample", "train")))
        torch.cuda.synchronize()

    def run(self, targets, first, count):
        """Two host threads enqueue (a launch costs the host a few microseconds and a step has
        about sixty): one feeds the sampling streams, this one the training stream.  The queues only
        order the host-side event calls: a stream may wait on an event only after the other thread
        has recorded it for that step."""
        import queue
        import threading
        torch = self.torch
        sampled, freed = queue.Queue(), queue.Queue()
        for _ in range(self.n):
            freed.put(None)
        failure = []
        graphs = getattr(self, "graphs", None)
        if graphs:      # slot k replays steps k, k + n, ...: point its device-side counter at its first one
            for k, r in enumerate(self.slots):
                r.step_idx.fill_(first + ((k - first) % self.n))
            torch.cuda.synchronize()

        def sampler():
            try:
                torch.cuda.set_device(self.slots[0].dev)
                for i in range(first, first + count):
                    freed.get()
                    k = i % self.n
                    r = self.slots[k]
                    ss = self.s_sample[i % len(self.s_sample)]
                    with torch.cuda.stream(ss):
                        ss.wait_event(self.free[k])
                        if graphs:
                            graphs[k]["sample"].replay()
                        else:
                            r.ctx.gsplit_sample_split(targets[i], r.seed, i)
                            r.load()
                        self.ready[k].record(ss)
                    sampled.put(i)
            except BaseException as e:      # hand the failure to the training thread
                failure.append(e)
                sampled.put(-1)

        th = threading.Thread(target=sampler, name="gsplit-sampler")
        th.start()
        try:
            for i in range(first, first + count):
                got = sampled.get()
                if got != i:
                    raise RuntimeError(f"sampling thread failed: {failure}")
                k = i % self.n
                r = self.slots[k]
                with torch.cuda.stream(self.s_train):
                    self.s_train.wait_event(self.ready[k])
                    if graphs:
                        graphs[k]["train"].replay()
                    else:
                        r.train()
                    self.free[k].record(self.s_train)
                freed.put(None)
        finally:
            for _ in range(count):      # a sampler left waiting for a slot can always finish
                freed.put(None)
            th.join()


def load_group(rs):
    """Loading step of a group of runners: one launch for all of them (the cached loading step, which
    reads host memory, stays one call per batch)."""
    if len(rs) == 1 or getattr(rs[0], "cached", False):
        for r in rs:
            r.load()
        return
    from paper_2303_13775_amd import gsplit_gather_features_multi
    gsplit_gather_features_multi([r.ctx for r in rs], rs[0].w.feat, [r.x0 for r in rs])


class PipelinedGroups:
    """The overlap schedule with sampling in groups: the mini-batches of the next K steps are sampled
    and split by one gsplit_sample_split_multi call (one set of launches for all K) and loaded on a
    sampling stream, while the training stream runs forward / loss / backward of the K steps of the
    group before, one after the other (synchronous training: consecutive steps stay ordered).  Two
    groups of K batch slots alternate; events hand a group over in both directions.  Every step
    does all of its work."""

    def __init__(self, w, dev, k, model="sage", heads=4, sampler_blocks=2):
        import torch
        self.torch = torch
        self.k = k
        self.groups = [[Runner(w, dev, model, heads, sampler_blocks_per_cu=sampler_blocks) for _ in range(k)]
                       for _ in range(2)]
        self.slots = [r for g in self.groups for r in g]
        self.s_sample = torch.cuda.Stream(device=dev)
        self.s_train = torch.cuda.Stream(device=dev)
        self.ready = [torch.cuda.Event() for _ in range(2)]
        self.free = [torch.cuda.Event() for _ in range(2)]
        for e in self.free:
            e.record()
        # a fixed order of first use fixes which hardware queue each stream gets
        for s in (self.s_train, self.s_sample):
            with torch.cuda.stream(s):
                torch.zeros(1, device=dev)
        torch.cuda.synchronize()

    def plan(self, first, count):
        """(first step, size) of every group of a run: sizes 2, 4, ... up to K, then K.  The first
        group is sampled before any training can start, so it is the shortest; each later group is sampled
        while the one before it, half its size or as large, trains."""
        out, lo, n = [], first, 2
        while lo < first + count:
            m = min(n, self.k, first + count - lo)
            out.append((lo, m))
            lo += m
            n *= 2
        return out

    def slot_of_step(self, i, first, count):
        for j, (lo, n) in enumerate(self.plan(first, count)):
            if lo <= i < lo + n:
                return self.groups[j % 2][i - lo]
        raise IndexError(i)

    def run(self, targets, first, count):
        import queue
        import threading
        from paper_2303_13775_amd import gsplit_sample_split_multi
        torch = self.torch
        plan = self.plan(first, count)
        n_groups = len(plan)
        sampled, freed = queue.Queue(), queue.Queue()
        for _ in range(2):
            freed.put(None)
        failure = []

        def sampler():
            try:
                torch.cuda.set_device(self.slots[0].dev)
                for j in range(n_groups):
                    freed.get()
                    g = j % 2
                    lo, n = plan[j]
                    rs = self.groups[g][:n]
                    with torch.cuda.stream(self.s_sample):
                        self.s_sample.wait_event(self.free[g])
                        gsplit_sample_split_multi([r.ctx for r in rs], [targets[lo + b] for b in range(n)], rs[0].seed,
                                                  [lo + b for b in range(n)])
                        load_group(rs)
                        self.ready[g].record(self.s_sample)
                    sampled.put(j)
            except BaseException as e:      # hand the failure to the training thread
                failure.append(e)
                sampled.put(-1)

        th = threading.Thread(target=sampler, name="gsplit-sampler")
        th.start()
        try:
            for j in range(n_groups):
                got = sampled.get()
                if got != j:
                    raise RuntimeError(f"sampling thread failed: {failure}")
                g = j % 2
                lo, n = plan[j]
                with torch.cuda.stream(self.s_train):
                    self.s_train.wait_event(self.ready[g])
                    for r in self.groups[g][:n]:
                        r.train()
                    self.free[g].record(self.s_train)
                freed.put(None)
        finally:
            for _ in range(n_groups):
                freed.put(None)
            th.join()


def cpu_baseline(w_host, iters, budget_s=14.0):
    """The oracle as it stands, timed on the host cores on whole iterations of the same workload:
    once as it runs by default (C steps on one thread, numpy float64 products on all BLAS threads)
    and once held to a single thread throughout."""
    from oracle import reference as R
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threadpool_limits = None
        threads = 1
    ip, ix, pm = w_host["indptr"], w_host["indices"], w_host["pmap"]
    params = R.SageParams(w_host["w_self"], w_host["w_neigh"], w_host["bias"])

    def run(limit_s):
        t0 = time.perf_counter()
        done = 0
        for it in range(iters):
            tg = w_host["targets"][it]
            b = R.sp_sample(ip, ix, pm, w_host["S"], w_host["fanouts"], tg, 0xC0FFEE, it)
            x0 = R.gather_rows(w_host["feat"], b.local_cat(0))
            f = R.sp_forward(b, x0, params)
            _, g = R.softmax_xent(f.logits, w_host["labels"][tg[b.target_perm]])
            R.sp_backward(b, f, params, g)
            done += 1
            if time.perf_counter() - t0 > limit_s:      # the sample stays bounded
                break
        return done, time.perf_counter() - t0

    n_all, dt_all = run(budget_s)
    out = {"value": n_all / dt_all, "unit": "mini-batches/s", "cores": int(threads), "kind": "oracle",
           "sample": f"{n_all} whole iterations of the same workload (C steps single-threaded, "
                     f"numpy float64 matmuls on {threads} BLAS threads), {dt_all:.1f} s"}
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            n_one, dt_one = run(budget_s * 0.6)
        out["one_thread"] = {"value": n_one / dt_one, "unit": "mini-batches/s", "cores": 1,
                             "sample": f"{n_one} whole iterations, every step on one thread, {dt_one:.1f} s"}
    return out


def cpu_baseline_gat(w_host, iters):
    """The GAT oracle as it stands (numpy float64, a Python loop over destinations), whole iterations."""
    from oracle import reference as R
    from oracle import gat as G
    ip, ix, pm = w_host["indptr"], w_host["indices"], w_host["pmap"]
    params = G.GatParams(w_host["heads"], *w_host["gat"])
    t0 = time.perf_counter()
    for it in range(iters):
        tg = w_host["targets"][it]
        b = R.sp_sample(ip, ix, pm, w_host["S"], w_host["fanouts"], tg, 0xC0FFEE, it)
        x0 = R.gather_rows(w_host["feat"], b.local_cat(0))
        f = G.gat_forward(b, x0, params)
        _, g = R.softmax_xent(f.logits, w_host["labels"][tg[b.target_perm]])
        G.gat_backward(b, f, params, g)
    dt = time.perf_counter() - t0
    return {"value": iters / dt, "unit": "mini-batches/s", "cores": 1, "kind": "oracle",
            "sample": f"{iters} whole iteration(s) of the same workload (C sampling steps, numpy float64 GAT with a "
                      f"Python loop over destinations), {dt:.1f} s"}


def presample_bench(a, w, dev, t_gen):
    """Offline pre-sampling (paper section 4): the training sampler plus the counting of k_v and
    k_e, one sample (mini-batch) per step, serial on one stream."""
    import torch
    from paper_2303_13775_amd import Context
    ctx = Context(w.indptr, w.indices, w.pmap, w.n_splits, w.fanouts, w.batch, keep_edge_ids=True)
    k_v = torch.zeros(w.n_vertices, dtype=torch.int32, device=dev)
    k_e = torch.zeros(w.indices.numel(), dtype=torch.int32, device=dev)
    n_total = a.warmup + a.steps
    targets = [w.targets(i) for i in range(n_total)]

    def step(i):
        ctx.gsplit_sample_split(targets[i], 0xC0FFEE, i)
        ctx.gsplit_presample_accumulate(k_v, k_e)

    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.warmup, n_total):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # kernel time of the counting launch and its algorithmic bytes (4-byte id or 8-byte edge
    # position read, one 4-byte counter touched)
    ctx.gsplit_timing_enable(True)
    n_k = min(a.steps, 30)
    work = 0.0
    for i in range(a.warmup, a.warmup + n_k):
        step(i)
        n_local, _, n_edges, _ = ctx.gsplit_batch_sizes()
        rows = [sum(x) for x in n_local]
        slots = sum(rows[l + 1] * w.fanouts[l] for l in range(len(w.fanouts)))
        work += sum(rows[1:]) * 8 + slots * 8 + sum(sum(x) for x in n_edges) * 4
    torch.cuda.synchronize()
    kt = ctx.gsplit_timing_read()
    cnt, ms = kt["presample_accumulate"]
    sec = ms / max(cnt, 1) * 1e-3
    ach = work / n_k / sec / 1e9
    cpu = None
    if not a.no_cpu_baseline:
        from oracle import reference as R
        R.build_oracle()
        ip, ix = w.indptr.cpu().numpy(), w.indices.cpu().numpy()
        n_cpu = max(1, min(a.cpu_iters, 60))
        tc = time.perf_counter()
        R.presample_counts(ip, ix, w.fanouts, [targets[i % len(targets)].cpu().numpy() for i in range(n_cpu)], 0xC0FFEE,
                           list(range(n_cpu)))
        dtc = time.perf_counter() - tc
        cpu = {"value": n_cpu / dtc, "unit": "samples/s", "cores": 1, "kind": "oracle",
               "sample": f"{n_cpu} samples of the same workload, single-threaded C steps, {dtc:.1f} s"}
    out = {
        "metric": "pre-sampling samples/sec (sample + count k_v, k_e) at 1 GPU", "value": a.steps / dt,
        "unit": "samples/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": dt / a.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32", "data": "synthetic",
        "config": dict(w.describe(), graph_gen_s=round(t_gen, 1), schedule="serial, one stream"),
        "kernel_us_per_step": {k: round(v[1] / n_k * 1e3, 2) for k, v in sorted(kt.items(), key=lambda kv: -kv[1][1])},
        "roofline": {"kernel": "presample_accumulate", "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": None,
                     "bytes_per_launch": work / n_k, "launch_ms": ms / max(cnt, 1)},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def redundancy_bench(a, w, dev, t_gen):
    """Paper section 2 (Table 1) and section 7.3 on one GPU: every iteration takes one mini-batch of
    S x batch targets and runs a whole training step on it twice, split S ways (one context with S
    splits) and as S data-parallel micro-batches of `batch` targets (a context with one split,
    called S times with its own random stream each).  Same kernels, all work done, serial on one
    stream."""
    import copy
    import numpy as np
    import torch
    import workloads
    S, L = a.splits, w.n_layers
    w_mini = copy.copy(w)
    w_mini.batch = w.batch * S
    w_micro = copy.copy(w)
    w_micro.n_splits = 1
    w_micro.pmap = torch.zeros_like(w.pmap)
    mini, micro = Runner(w_mini, dev, a.model, a.heads), Runner(w_micro, dev, a.model, a.heads)
    n_total = a.warmup + a.steps
    targets = [w_mini.targets(i) for i in range(n_total)]
    parts = [workloads.micro_batch_parts(t, S) for t in targets]
    torch.cuda.synchronize()

    def run(which, lo, hi):
        t0 = time.perf_counter()
        for i in range(lo, hi):
            if which == "mini":
                mini.step(targets[i], i)
            else:
                for m in range(S):
                    micro.step(parts[i][m], i * S + m)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    run("mini", 0, a.warmup); run("micro", 0, a.warmup)
    dt_mini = run("mini", a.warmup, n_total)
    dt_micro = run("micro", a.warmup, n_total)

    # counters over the same iterations (untimed pass: reading sizes waits for the sampler)
    edges = torch.zeros(L * S, dtype=torch.int64, device=dev)
    cross = torch.zeros(L * S, dtype=torch.int64, device=dev)
    tot = {"edges_micro": 0, "edges_mini": 0, "features_micro": 0, "features_mini": 0}
    imb = []
    mini.ctx.gsplit_timing_enable(True)
    slots = 0
    for i in range(a.warmup, n_total):
        mini.ctx.gsplit_sample_split(targets[i], mini.seed, i)
        before = edges.clone()
        mini.ctx.gsplit_batch_stats(edges, cross)
        n_local, _, n_edges, _ = mini.ctx.gsplit_batch_sizes()
        tot["edges_mini"] += int(np.sum(n_edges)); tot["features_mini"] += int(np.sum(n_local[0]))
        slots += sum(int(np.sum(n_local[l + 1])) * w.fanouts[l] for l in range(L))
        per_split = (edges - before).view(L, S)[1:].sum(0).double()
        imb.append(float(per_split.max() / per_split.mean()) if float(per_split.sum()) > 0 else 1.0)
        for m in range(S):
            micro.ctx.gsplit_sample_split(parts[i][m], micro.seed, i * S + m)
            nl, _, ne, _ = micro.ctx.gsplit_batch_sizes()
            tot["edges_micro"] += int(np.sum(ne)); tot["features_micro"] += int(np.sum(nl[0]))
    torch.cuda.synchronize()
    kt = mini.ctx.gsplit_timing_read()
    cnt, ms = kt["batch_stats"]
    # per slot: the neighbour id (4 bytes) and, for a sampled one, its owner byte
    work = slots * 4 + tot["edges_mini"]
    sec = ms / max(cnt, 1) * 1e-3
    ach = work / max(cnt, 1) / sec / 1e9
    cpu = None
    if not a.no_cpu_baseline:
        from oracle import reference as R
        R.build_oracle()
        ip, ix, pm = w.indptr.cpu().numpy(), w.indices.cpu().numpy(), w.pmap.cpu().numpy()
        n_cpu = max(1, min(a.cpu_iters, 8))
        tc = time.perf_counter()
        for i in range(a.warmup, a.warmup + n_cpu):
            tg = targets[i % len(targets)].cpu().numpy()
            mb = R.sp_sample(ip, ix, pm, S, w.fanouts, tg, mini.seed, i)
            R.redundancy_counts(mb, R.micro_batches(ip, ix, w.fanouts, tg, S, micro.seed, i))
        dtc = time.perf_counter() - tc
        cpu = {"value": n_cpu / dtc, "unit": "iterations/s", "cores": 1, "kind": "oracle",
               "sample": f"{n_cpu} iterations: sampling and counting of the split mini-batch and of its {S} "
                         f"micro-batches (single-threaded C steps, no training step), {dtc:.1f} s"}
    e_all, c_all = int(edges.sum()), int(cross.sum())
    out = {
        "metric": f"mini-batches/sec of {S * w.batch} targets as {S} data-parallel micro-batches "
                  f"(sample+gather+{a.model} fwd/bwd each) at 1 GPU",
        "value": a.steps / dt_micro, "unit": "mini-batches/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": dt_micro / a.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.feat.dtype == torch.float32 else "bf16", "data": "synthetic",
        "config": dict(w_mini.describe(), model=a.model, micro_batches=S, micro_batch=w.batch, graph_gen_s=round(t_gen, 1),
                       schedule="serial, one stream"),
        "split_mode": {"value": a.steps / dt_mini, "ms_per_step": dt_mini / a.steps * 1e3},
        "time_ratio_micro_over_split": dt_micro / dt_mini,
        "table1": dict(tot, edges_ratio=tot["edges_micro"] / max(tot["edges_mini"], 1),
                       features_ratio=tot["features_micro"] / max(tot["features_mini"], 1), iterations=a.steps),
        "split_quality": {"workload_imbalance_mean": sum(imb) / len(imb), "workload_imbalance_max": max(imb),
                          "cross_edge_fraction": c_all / max(e_all, 1)},
        "roofline": {"kernel": "batch_stats", "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": ach / HBM_PEAK_GBS, "traffic": None, "bytes_per_launch": work / max(cnt, 1),
                     "launch_ms": ms / max(cnt, 1)},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def algorithmic_work(w, model, heads, rows, edges, mixed, row_bytes, ip_bytes, S):
    """Algorithmic bytes / flops of one launch of every kernel of a step, from the live sizes of a batch.

    HBM-bound rows follow the per-unit figures of the scope table: sampling = per destination vertex
    its id and two row pointers read and the count written, per sampled edge 4 bytes read and 4
    written; the kernel also makes the hash-table entries of the dedup step (one 8-byte entry per
    element in each table it enters), which are counted with it.  What a kernel moves beyond that
    for its own bookkeeping (the entry indices every element remembers) is returned separately."""
    L = w.n_layers
    work, extra = {}, {}

    def add(label, kind, amount, own=0.0, io=0.0):
        work[label] = (kind, amount)
        if own:
            extra[label] = own
        if io:      # a matrix product's operand and result bytes (its memory-side ceiling)
            extra["io:" + label] = io

    add("gather_rows", "bytes", rows[0] * (2 * row_bytes + 4))
    add("gather_cached", "bytes", rows[0] * (2 * row_bytes + 8))
    es = w.feat.element_size()
    for l in range(L if model == "gat" else 0):
        D, nd, n_lo = w.dims[l], rows[l + 1], rows[l]
        K = heads[l]
        HF = K * w.dims[l + 1] if l == L - 1 else w.dims[l + 1]
        ent = edges[l] + nd
        if l == 0:
            add("gat0_transform.l0", "flops", 2.0 * nd * D * HF)
            add("gat0_grad_p.l0", "flops", 2.0 * nd * D * HF)
            add("gat0_grad_w.l0", "flops", 2.0 * nd * D * HF)
            add("gat0_scores.l0", "bytes", n_lo * 4 * (D + 2 * K))
            add("gat0_aggregate.l0", "bytes", ent * (4 + 4 * D + 8 * K) + nd * 4 * K * D)
            add("gat0_bwd.l0", "bytes", ent * (4 + 4 * D + 8 * K) + nd * 4 * K * D)
        add(f"gat_transform.l{l}", "flops", 2.0 * n_lo * D * (HF + 2 * K))
        add(f"gat_grad_w.l{l}", "flops", 2.0 * n_lo * D * (HF + 2 * K))
        if l > 0:
            add(f"gat_grad_in.l{l}", "flops", 2.0 * n_lo * D * (HF + 2 * K))
        add(f"gat_aggregate.l{l}", "bytes", ent * (4 + 4 * HF + 8 * K) + nd * 4 * w.dims[l + 1])
        add(f"gat_bwd_dst.l{l}", "bytes", ent * (4 + 4 * HF + 8 * K) + nd * (8 * w.dims[l + 1] + 4 * HF + 4 * K))
        add(f"gat_bwd_src.l{l}", "bytes", ent * (8 + 4 * HF + 8 * K) + n_lo * (8 + 4 * (HF + 2 * K)))
    n_tab = 2 if S > 1 else 1
    for l in range(L):
        D, N, nd = w.dims[l], w.dims[l + 1], rows[l + 1]
        # operand bytes: activations and dZ below the top level in the storage type (dZ in bf16 only where
        # its rows are whole 16-byte pieces), logits and input-gradient rows in float, the weights once
        top = l == L - 1
        e_out = 4 if top else es
        e_dz = 4 if (top or es == 4 or N % 8) else 2
        wbytes = 2 * D * N * es
        add(f"linear_fwd.l{l}", "flops", 2.0 * nd * (2 * D) * N, io=nd * (2 * D * es + N * e_out) + wbytes)
        if top:      # the fused top layer: forward, weight-gradient and input-gradient products (plain FMAs)
            add(f"top_fused.l{l}", "flops", 2.0 * nd * (2 * D) * N * 2 + 2.0 * nd * (2 * D + 1) * N)
        add(f"grad_w.l{l}", "flops", 2.0 * nd * (2 * D + 1) * N, io=nd * (2 * D * es + N * e_dz))
        if l > 0:
            add(f"grad_in.l{l}", "flops", 2.0 * nd * N * (2 * D), io=nd * (N * e_dz + 2 * D * 4) + wbytes)
            # float input-gradient rows per entry; per row of the level the stored activation (ReLU mask) read and
            # dZ written, both in the storage type (dZ in bf16 only where its rows are whole 16-byte pieces)
            e_dzl = 2 if (es == 2 and D % 8 == 0) else 4
            add(f"pull_input_grad.l{l}", "bytes", (nd + edges[l]) * (4 + 4 * D) + rows[l] * (8 + (es + e_dzl) * D))
        # no-reuse model: one source row per edge, one self row and one [self | mean] row per destination
        add(f"assemble_input.l{l}", "bytes", edges[l] * (4 + es * D) + nd * (4 + es * D) + nd * 2 * es * D)
        items = nd + edges[l]
        add(f"sample_layer.l{l}", "bytes", nd * (8 + 2 * ip_bytes) + edges[l] * 8 + items * 8 * n_tab, own=items * 8)
        slots = nd * w.fanouts[l]
        # split assignment and buckets: per sampled id 1 (owner byte) + 4 read + 4 written; the dedup's table
        # look-ups of the same pass 8 bytes per table; own: the entry indices and class masks
        add(f"mixed_buckets_count.l{l}", "bytes", edges[l] * (1 + 4 + 8 * n_tab), own=slots * 12)
        add(f"mixed_buckets_scatter.l{l}", "bytes", edges[l] * 4 + mixed[l] * (4 + 4 + 4 * n_tab) + rows[l] * 4,
            own=slots * 4 + mixed[l] * 4)
        add(f"shuffle_index.l{l}", "bytes", (mixed[l] + nd) * 8 + edges[l] * (4 * n_tab + 8), own=slots * 8 + mixed[l] * 4)
        # a wide layer relabels its edges in a launch of its own: that launch's share of the line above
        # (the caller takes it off the line above when the launch was there)
        add(f"shuffle_edges.l{l}", "bytes", edges[l] * (4 * n_tab + 8), own=slots * 4)
    return work, extra


def percentile(xs, q):
    xs = sorted(xs)
    if not xs:
        return None
    k = (len(xs) - 1) * q
    lo, hi = int(k), min(int(k) + 1, len(xs) - 1)
    return xs[lo] + (xs[hi] - xs[lo]) * (k - lo)


def profile_traffic(workload, dtype, model, label):
    """HBM bytes per launch of a kernel from the committed rocprofv3 counter summary of this workload
    (FETCH_SIZE + WRITE_SIZE scaled by the copy calibration stated in that file), with the file it
    came from; (None, None) when there is no summary for this workload and type."""
    here = os.path.dirname(os.path.abspath(__file__))
    tag = workload if dtype == "f32" else f"{workload}_{dtype}"
    name = f"{tag}_{'gat_' if model == 'gat' else ''}bench_hbm_traffic.txt"
    path = os.path.join(here, "profiles", name)
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        f = line.split()
        if len(f) >= 5 and f[0] == label:
            try:
                return (float(f[-2]) + float(f[-1])) * 1024.0, "profiles/" + name
            except ValueError:
                return None, None
    return None, None


def measure(a, w, dev, *, workload, dtype, model="sage", heads=4, steps, warmup, pipeline, stage_iters,
            cache=None, use_graph=False, multi=None):
    """All timings of one configuration: K steps pipelined (if asked) and K steps serial between two
    device synchronisations, K steps with one synchronisation per step (mean / p50 / p95), per-stage
    and per-kernel device times, and the rooflines that follow from them."""
    import torch
    r = Runner(w, dev, model, heads)
    if cache:
        r.enable_cache(cache["host_table"], cache["ids"], cache["n_cache"])
    n_total = warmup + steps
    targets = [w.targets(i) for i in range(n_total)]
    torch.cuda.synchronize()
    targets_all = torch.stack(targets).contiguous() if use_graph else None
    for i in range(warmup):
        r.step(targets[i], i)
    torch.cuda.synchronize()
    graph_check = None
    if use_graph:
        # the same step as one captured HIP graph; its first replay is checked against the eager step
        s_cap = torch.cuda.Stream(device=dev)
        r.prepare_graphs(targets_all, 1)
        g_step = r.capture(s_cap, ("step",))["step"]
        torch.cuda.synchronize()
        r.step(targets[0], 0)
        torch.cuda.synchronize()
        want = r.logits.clone()
        r.step_idx.fill_(0)
        r.logits.fill_(0.0)
        g_step.replay()
        torch.cuda.synchronize()
        graph_check = bool(torch.equal(want, r.logits))
        assert graph_check, "a replayed step differs from the eager step"
        r.step_idx.fill_(warmup)
        torch.cuda.synchronize()
    # (1) K steps back to back on one stream, one synchronisation on each side
    t0 = time.perf_counter()
    for i in range(warmup, n_total):
        if use_graph:
            g_step.replay()
        else:
            r.step(targets[i], i)
    torch.cuda.synchronize()
    dt_serial = time.perf_counter() - t0
    # (2) the same steps with one synchronisation at the end of every step: wall time per step
    per_step = []
    if not use_graph:
        for i in range(warmup, n_total):
            t1 = time.perf_counter()
            r.step(targets[i], i)
            torch.cuda.synchronize()
            per_step.append((time.perf_counter() - t1) * 1e3)
    # (2b) one stream, sampling in groups: the next K mini-batches through one set of launches, then
    # the K training steps one after the other
    K = max(1, min(a.multi if multi is None else multi, steps))
    serial_multi = None
    if K > 1 and not use_graph:
        from paper_2303_13775_amd import gsplit_sample_split_multi
        rs = [r] + [Runner(w, dev, model, heads) for _ in range(K - 1)]
        if cache:
            for x in rs[1:]:
                x.enable_cache(cache["host_table"], cache["ids"], cache["n_cache"])

        def run_groups(lo, hi):
            for g0 in range(lo, hi, K):
                n = min(K, hi - g0)
                gsplit_sample_split_multi([x.ctx for x in rs[:n]], [targets[g0 + b] for b in range(n)], r.seed,
                                          [g0 + b for b in range(n)])
                load_group(rs[:n])
                for x in rs[:n]:
                    x.train()

        run_groups(0, warmup)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_groups(warmup, n_total)
        torch.cuda.synchronize()
        dt_multi = time.perf_counter() - t0
        serial_multi = {"value": steps / dt_multi, "ms_per_step": dt_multi / steps * 1e3, "batches_per_sampling_call": K,
                        "schedule": f"one stream; the mini-batches of the next {K} steps are sampled and split by one "
                                    f"gsplit_sample_split_multi call and loaded by one gsplit_gather_features_multi call, "
                                    f"then trained one after the other"}
        # the sampling kernels of a grouped call, timed by the library on the first context of the group:
        # one launch then carries the K mini-batches' work
        n_g = max(1, min(stage_iters, steps) // K)
        rs[0].ctx.gsplit_timing_enable(True)
        rs[0].ctx.gsplit_timing_read()
        grouped_work = {}
        for gi in range(n_g):
            g0 = warmup + gi * K
            n = min(K, n_total - g0)
            gsplit_sample_split_multi([x.ctx for x in rs[:n]], [targets[g0 + b] for b in range(n)], r.seed,
                                      [g0 + b for b in range(n)])
            load_group(rs[:n])
            for x in rs[:n]:
                nl, nm, ne, _ = x.ctx.gsplit_batch_sizes()
                wk, _own = algorithmic_work(w, model, getattr(r, "heads", None), [sum(v) for v in nl], [sum(v) for v in ne],
                                            [sum(v) for v in nm], w.feat.shape[1] * w.feat.element_size(),
                                            w.indptr.element_size(), w.n_splits)
                for kk, (kind, amount) in wk.items():
                    if kk.startswith(("sample_layer", "mixed_buckets", "shuffle_index", "shuffle_edges")) or kk == "gather_rows":
                        grouped_work[kk] = grouped_work.get(kk, 0.0) + amount
        torch.cuda.synchronize()
        gt = rs[0].ctx.gsplit_timing_read()
        rs[0].ctx.gsplit_timing_enable(False)
        if "gather_rows" in gt and gt["gather_rows"][0] > 0 and not cache:
            cnt, ms = gt.pop("gather_rows")
            ach = grouped_work.pop("gather_rows") / (ms * 1e-3) / 1e9
            serial_multi["roofline_gather_grouped"] = {
                "kernel": "gather_rows", "batches_per_launch": K, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "launch_ms": ms / cnt}
        grouped_work.pop("gather_rows", None)
        for l in range(w.n_layers):
            if f"shuffle_edges.l{l}" in gt and gt[f"shuffle_edges.l{l}"][0] > 0 and f"shuffle_index.l{l}" in grouped_work:
                grouped_work[f"shuffle_index.l{l}"] -= grouped_work[f"shuffle_edges.l{l}"]
        cand = {kk: v for kk, v in gt.items() if kk in grouped_work and v[0] > 0}
        if cand:
            big = max(cand, key=lambda kk: cand[kk][1])
            cnt, ms = cand[big]
            ach = grouped_work[big] / (ms * 1e-3) / 1e9
            serial_multi["roofline_sampling_grouped"] = {
                "kernel": big, "batches_per_launch": K, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "bytes_per_launch": grouped_work[big] / cnt, "launch_ms": ms / cnt}
            serial_multi["sampling_kernel_us_per_batch"] = {kk: round(v[1] / v[0] / K * 1e3, 2) for kk, v in
                                                            sorted(cand.items(), key=lambda kv: -kv[1][1])}
        for x in rs[1:]:
            x.ctx.close()
        del rs
    # (3) sampling + splitting + loading of the next steps on a sampling stream beside the training stream
    dt = dt_serial
    if pipeline:
        if K > 1 and not use_graph:
            pipe = PipelinedGroups(w, dev, K, model, heads, a.sampler_blocks)
        else:
            pipe = Pipelined(w, dev, a.ahead, model, heads, a.sampler_blocks)
        if cache:
            for slot in pipe.slots:
                slot.enable_cache(cache["host_table"], cache["ids"], cache["n_cache"])
        pipe.run(targets, 0, warmup)
        torch.cuda.synchronize()
        if use_graph:
            pipe.enable_graphs(targets_all)
            pipe.run(targets, 0, warmup)
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        pipe.run(targets, warmup, steps)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        for slot in pipe.slots:
            slot.ctx.close()
        del pipe

    # per-stage device times (separate instrumented pass; events on the stream the kernels run on)
    n_st = max(1, min(stage_iters, steps))
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(n_st)]
    for i in range(n_st):
        r.step(targets[warmup + i], warmup + i, ev[i])
    torch.cuda.synchronize()
    names = ["sample_split", "gather", f"{model}_fwd", "loss_grad", f"{model}_bwd"]
    if model == "sage" and not Runner.separate_calls:
        names = ["sample_split", "gather", "sage_step"]
    stage_ms = {nm: sum(ev[i][k].elapsed_time(ev[i][k + 1]) for i in range(n_st)) / n_st for k, nm in enumerate(names)}

    # per-kernel device times: the library brackets each of its launches with HIP events on the
    # launch stream; algorithmic bytes / flops are summed over the very same iterations
    L, S = w.n_layers, w.n_splits
    row_bytes = w.dims[0] * w.feat.element_size()
    ip_bytes = w.indptr.element_size()
    totals, own_totals = {}, {}
    r.ctx.gsplit_timing_enable(True)
    n_k = n_st
    shape = None
    for i in range(n_k):
        r.step(targets[warmup + i], warmup + i)
        n_local, n_mixed, n_edges, bucket = r.ctx.gsplit_batch_sizes()     # waits for sampling only
        rows = [sum(x) for x in n_local]
        edges = [sum(x) for x in n_edges]
        mixed = [sum(x) for x in n_mixed]
        shape = (rows, edges, mixed, bucket)
        work, own = algorithmic_work(w, model, getattr(r, "heads", None), rows, edges, mixed, row_bytes, ip_bytes, S)
        for k, (kind, amount) in work.items():
            t = totals.setdefault(k, [kind, 0.0])
            t[1] += amount
        for k, amount in own.items():
            own_totals[k] = own_totals.get(k, 0.0) + amount
    torch.cuda.synchronize()
    ktimes = r.ctx.gsplit_timing_read()
    r.ctx.gsplit_timing_enable(False)
    per_step_us = {k: v[1] / n_k * 1e3 for k, v in ktimes.items()}
    for l in range(L):      # wide layers: the edges' share of the relabelling belongs to the second launch
        if f"shuffle_edges.l{l}" in ktimes and f"shuffle_index.l{l}" in totals:
            totals[f"shuffle_index.l{l}"][1] -= totals[f"shuffle_edges.l{l}"][1]
            own_totals[f"shuffle_index.l{l}"] -= own_totals[f"shuffle_edges.l{l}"]

    def roofline_of(label):
        cnt, ms = ktimes[label]
        kind, amount = totals.get(label, ("bytes", 0.0))
        per_launch = amount / max(cnt, 1)
        sec = ms / max(cnt, 1) * 1e-3
        traffic, src = profile_traffic(workload, dtype, model, label)
        if kind == "flops":
            ach = per_launch / sec / 1e12
            peak = BF16_MFMA_PEAK_TFLOPS if dtype == "bf16" else FP32_MFMA_PEAK_TFLOPS
            alu = label.startswith("top_fused")      # plain float32 FMAs (vector peak 157.3 TFLOP/s), not the matrix cores
            if alu:
                peak = FP32_MFMA_PEAK_TFLOPS
            out = {"kernel": label, "bound": "alu" if alu else "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak,
                   "traffic": traffic, "flops_per_launch": per_launch, "launch_ms": ms / max(cnt, 1)}
            if "io:" + label in own_totals:
                # the same launch against the memory side: operands read once, results written once
                io = own_totals["io:" + label] / max(cnt, 1)
                t_mem, t_mfma = io / (HBM_PEAK_GBS * 1e9), per_launch / (peak * 1e12)
                out["memory_side"] = {"bytes_per_launch": io, "achieved": io / sec / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                      "frac": io / sec / 1e9 / HBM_PEAK_GBS,
                                      "binding_ceiling": "hbm" if t_mem > t_mfma else "mfma",
                                      "frac_of_binding_ceiling": max(t_mem, t_mfma) / sec}
        else:
            ach = per_launch / sec / 1e9
            out = {"kernel": label, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                   "frac": ach / HBM_PEAK_GBS, "traffic": traffic, "bytes_per_launch": per_launch,
                   "launch_ms": ms / max(cnt, 1)}
            if label in own_totals:     # what the kernel moves for its own bookkeeping, not counted above
                out["bookkeeping_bytes_per_launch"] = own_totals[label] / max(cnt, 1)
        if traffic is not None:
            out["traffic_source"] = src + " (a committed rocprofv3 --pmc summary, not measured in this run)"
            out["traffic_GBps"] = traffic / sec / 1e9
        return out

    rows, edges, mixed, bucket = shape
    dominant = max(per_step_us, key=per_step_us.get)
    gather = roofline_of("gather_cached" if cache else "gather_rows")
    sampling = [k for k in per_step_us if k.startswith(("sample_layer", "mixed_buckets", "shuffle_index", "shuffle_edges"))]
    out = {
        "value": steps / dt, "ms_per_step": dt / steps * 1e3,
        "schedule": ("serial, one stream" if not pipeline else
                     (f"1 sampling stream + 1 training stream: sample+split (one gsplit_sample_split_multi call for "
                      f"a group of mini-batches) and gather (one gsplit_gather_features_multi call) of the next group "
                      f"overlap fwd/loss/bwd of the current one; groups of 2, 4, ... up to {K} steps, then {K} (the first "
                      f"group of a run has nothing to overlap with, so it is the shortest); "
                      f"every step does all of its work inside the timed region") if K > 1 and not use_graph else
                     f"{a.ahead} sampling stream(s) + 1 training stream: sample+split+gather of the next {a.ahead} "
                     f"step(s) overlap fwd/loss/bwd of step i; every step does all of its work"),
        "serial": {"value": steps / dt_serial, "ms_per_step": dt_serial / steps * 1e3,
                   "schedule": "one stream, steps enqueued back to back, one device synchronisation after the last"},
        "serial_ms_per_step": dt_serial / steps * 1e3,
        "gather_GBps": gather["achieved"], "stage_ms": stage_ms,
        "kernel_us_per_step": {k: round(v, 2) for k, v in sorted(per_step_us.items(), key=lambda kv: -kv[1])},
        "kernels_per_step": sum(v[0] for v in ktimes.values()) / n_k,
        "kernel_launch_order": list(ktimes.keys()),
        "batch_shape": {"rows_per_level": rows, "edges_per_layer": edges, "mixed_rows_per_layer": mixed,
                        "ids_shuffled_per_layer": [sum(b[s][t] for s in range(S) for t in range(S) if s != t)
                                                   for b in bucket]},
        "roofline": roofline_of(dominant), "roofline_gather": gather,
        "launch": ("every stream replays captured HIP graphs (the step counter and the targets table stay in device "
                   "memory)" if use_graph else "kernels enqueued from the host"),
    }
    if serial_multi:
        out["serial_multi"] = serial_multi
    if per_step:
        mean = sum(per_step) / len(per_step)
        out["serial_sync"] = {"value": 1e3 / mean, "mean_ms": mean, "p50_ms": percentile(per_step, 0.5),
                              "p95_ms": percentile(per_step, 0.95), "steps": len(per_step),
                              "schedule": "one stream, one device synchronisation at the end of every step (host wall time per step)"}
    if sampling:
        big = max(sampling, key=per_step_us.get)
        out["roofline_sampling"] = roofline_of(big)
        out["sampling_target"] = {"target_frac_of_hbm_peak": 0.6, "achieved_frac": out["roofline_sampling"]["frac"],
                                  "note": "algorithmic bytes of a word-granular random-access kernel; every such access "
                                          "moves a whole 128-byte line (traffic, where a profile exists, is the hardware view)"}
        if out["roofline_sampling"].get("traffic_GBps") is not None:
            # the same launch by the lines it moves: measured traffic over the HBM peak (random 4-byte reads by
            # themselves reach 50 G lines/s on this chip, i.e. 0.8 of the peak)
            out["sampling_target"]["achieved_frac_by_measured_traffic"] = out["roofline_sampling"]["traffic_GBps"] / HBM_PEAK_GBS
    if model == "sage":
        out["roofline_linear"] = [roofline_of(k) for k in sorted(per_step_us)
                                  if k.startswith(("linear_fwd", "grad_w", "grad_in"))]
        # mean aggregation (the input assembly of every layer) and its mirror in the backward pass (the pull):
        # against the no-reuse model (one source row per edge), with the perfect-reuse floor beside it
        # (every row of the level below read once)
        agg = []
        for k in sorted(per_step_us):
            if not k.startswith(("assemble_input", "pull_input_grad")):
                continue
            ro = roofline_of(k)
            l = int(k.rsplit(".l", 1)[1])
            D, es = w.dims[l], w.feat.element_size()
            nd, n_lo = rows[l + 1], rows[l]
            if k.startswith("assemble_input"):
                floor_bytes = n_lo * es * D + nd * (4 + 2 * es * D) + edges[l] * 4
            else:
                floor_bytes = nd * 2 * D * 4 + (nd + edges[l]) * 4 + n_lo * (8 + 2 * es * D)
            ro["perfect_reuse_floor_bytes"] = floor_bytes
            ro["perfect_reuse_floor_us"] = floor_bytes / (HBM_PEAK_GBS * 1e9) * 1e6
            agg.append(ro)
        out["roofline_aggregation"] = agg
    if graph_check is not None:
        out["graph_replay_equals_eager"] = graph_check
    if cache:
        # hits and misses of the kernel-timing iterations alone (the counters ran since the cache was built)
        r.hits.zero_(); r.misses.zero_()
        for i in range(n_k):
            r.ctx.gsplit_sample_split(targets[warmup + i], r.seed, warmup + i)
            r.load(count=True)
        torch.cuda.synchronize()
        h, m = int(r.hits.sum()), int(r.misses.sum())
        PCIE_PEAK_GBS = 64.0       # PCIe 5.0 x16, one direction
        link = m / n_k * row_bytes / (gather["launch_ms"] * 1e-3) / 1e9
        gather["cache"] = {"fraction_cached": a.cache_frac, "rows_cached": int(sum(cache["n_cache"])),
                           "hit_rate": h / max(h + m, 1), "miss_bytes_per_launch": m / n_k * row_bytes,
                           "host_link": {"achieved": link, "peak": PCIE_PEAK_GBS, "unit": "GB/s", "frac": link / PCIE_PEAK_GBS}}
    out["_runner"] = r
    return out


def extra_configs(a, dev, say):
    """The other configurations, each timed serially on one stream with its own rooflines: medium in
    bf16, large in float32 and in bf16, skewed, and the split sweep on the large graph (1, 2, 4, 8 logical splits;
    every stage also as a ratio to one split).  A configuration that fails reports its error and the
    others still run."""
    import torch
    import workloads
    out = {}

    def run(tag, w, workload, dtype, steps=20, warmup=3, multi=1):
        # (a context of the sweep or the skewed configuration holds tens of GB of buffers sized from the
        # no-dedup bounds: those run with one context, i.e. without the grouped-sampling figure)
        t0 = time.time()
        try:
            torch.cuda.empty_cache()
            m = measure(a, w, dev, workload=workload, dtype=dtype, steps=steps, warmup=warmup, pipeline=False,
                        stage_iters=min(steps, 10), multi=multi)
            m.pop("_runner").ctx.close()
            m["config"] = w.describe()
            m["dtype"] = dtype
            m["wall_s"] = round(time.time() - t0, 1)
            out[tag] = m
            say(f"extra config {tag}: {m['serial_sync']['mean_ms']:.3f} ms per step, {m['wall_s']} s in all")
        except Exception as e:                     # noqa: BLE001 - reported in the JSON line
            out[tag] = {"error": f"{type(e).__name__}: {e}"}
            say(f"extra config {tag} failed: {out[tag]['error']}")
        torch.cuda.synchronize()
        torch.cuda.empty_cache()

    try:
        w = workloads.medium(device=dev, n_splits=4)
        w.feat = w.feat.to(torch.bfloat16)
        run("medium_bf16", w, "medium", "bf16", steps=100, warmup=10, multi=a.multi)
        del w
    except Exception as e:                         # noqa: BLE001
        out["medium_bf16_error"] = f"{type(e).__name__}: {e}"
    torch.cuda.empty_cache()
    try:
        w = workloads.large(device=dev, n_splits=4, feat_dtype=torch.float32, progress=say)
        run("large_f32", w, "large", "f32", multi=a.multi)
        w.feat = w.feat.to(torch.bfloat16)
        torch.cuda.empty_cache()
        run("large_bf16", w, "large", "bf16", multi=a.multi)
        rank = workloads.bfs_rank(w.indptr, w.indices)
        sweep = {}
        for S in (1, 2, 4, 8):
            v = workloads.variant(w, n_splits=S, pmap_kind="bfs", rank=rank, batch=8192, fanouts=(10, 10, 10, 10),
                                  dims=(128, 256, 256, 256, 172), name=f"sweep-S{S}")
            run(f"sweep_S{S}", v, "sweep", "bf16")
            sweep[S] = out[f"sweep_S{S}"]
            del v
        if all("error" not in sweep[S] for S in sweep):
            base = sweep[1]
            out["sweep_relative_to_one_split"] = {
                f"S{S}": dict({k: sweep[S]["stage_ms"][k] / base["stage_ms"][k] for k in base["stage_ms"]},
                              step=sweep[S]["serial_sync"]["mean_ms"] / base["serial_sync"]["mean_ms"])
                for S in sweep}
        del w, rank, sweep
    except Exception as e:                         # noqa: BLE001
        out["large_graph_error"] = f"{type(e).__name__}: {e}"
    torch.cuda.empty_cache()
    try:
        w = workloads.skewed(device=dev, n_splits=4, progress=say)
        run("skewed_f32", w, "skewed", "f32")
        del w
    except Exception as e:                         # noqa: BLE001
        out["skewed_graph_error"] = f"{type(e).__name__}: {e}"
    torch.cuda.empty_cache()
    return out


def main():
    a = parse()
    Runner.separate_calls = a.separate_calls
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (logical splits share it); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import workloads
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    t0 = time.time()
    dtype = a.dtype or ("bf16" if a.workload == "sweep" else "f32")
    fdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    say = lambda m: print(f"[bench] {m}", file=sys.stderr, flush=True)
    if a.workload == "medium":
        w = workloads.medium(device=dev, n_splits=a.splits)
    elif a.workload == "tiny":
        w = workloads.tiny(device=dev, n_splits=a.splits)
    elif a.workload == "large":
        w = workloads.large(device=dev, n_splits=a.splits, feat_dtype=fdt, progress=say)
    elif a.workload == "skewed":
        w = workloads.skewed(device=dev, n_splits=a.splits, progress=say)
    else:   # split sweep on the large graph: 4 layers, fanout 10, batch 8192
        base = workloads.large(device=dev, n_splits=4, feat_dtype=fdt, progress=say)
        w = workloads.variant(base, n_splits=a.splits, pmap_kind="bfs", rank=workloads.bfs_rank(base.indptr, base.indices),
                              batch=8192, fanouts=(10, 10, 10, 10), dims=(128, 256, 256, 256, 172),
                              name=f"sweep-S{a.splits}")
        del base
    if w.feat.dtype != fdt:
        w.feat = w.feat.to(fdt)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()        # hand the generator's scratch back: the library allocates with hipMalloc
    if a.workload == "sweep":       # tens of GB of buffers per context, kernels that fill the chip: one stream
        a.no_pipeline = True
    t_gen = time.time() - t0
    if a.presample:
        return presample_bench(a, w, dev, t_gen)
    if a.redundancy:
        return redundancy_bench(a, w, dev, t_gen)
    if a.model == "gat" and dtype != "f32":
        print("bench.py: --model gat runs in f32", file=sys.stderr)
        sys.exit(2)
    cache_info = None
    if a.cache_frac is not None:
        # offline: rank every split's vertices by how often the sampler puts them into the input layer
        # (library kernel), keep the hottest fraction (a sort: the caller's policy step), build the cache
        from paper_2303_13775_amd import Context
        pre = Context(w.indptr, w.indices, w.pmap, w.n_splits, w.fanouts, w.batch)
        host_table = torch.empty(w.feat.shape, dtype=w.feat.dtype, pin_memory=True)
        host_table.copy_(w.feat)
        k_in = torch.zeros(w.n_vertices, dtype=torch.int32, device=dev)
        for i in range(a.cache_presample):
            pre.gsplit_sample_split(w.targets(10_000_000 + i), 0xC0FFEE, 10_000_000 + i)
            pre.gsplit_input_counts_accumulate(k_in)
        ids, n_cache = [], []
        for s_ in range(w.n_splits):
            own = torch.nonzero((w.pmap == s_) & (k_in > 0)).flatten()
            order = torch.sort(-k_in[own].long(), stable=True).indices
            keep = int(a.cache_frac * int((w.pmap == s_).sum()))
            ids.append(own[order][:keep].int())
            n_cache.append(int(ids[-1].numel()))
        cache_ids = torch.cat(ids).contiguous()
        cache_info = {"host_table": host_table, "ids": cache_ids, "n_cache": n_cache}
        pre.close()
        del k_in

    m = measure(a, w, dev, workload=a.workload, dtype=dtype, model=a.model, heads=a.heads, steps=a.steps,
                warmup=a.warmup, pipeline=not a.no_pipeline, stage_iters=a.stage_iters, cache=cache_info,
                use_graph=a.graph)
    r = m.pop("_runner")
    out = {
        "metric": f"mini-batches/sec (sample+split+gather+{'GAT' if a.model == 'gat' else 'SAGE'} fwd/bwd) at 1 GPU",
        "value": m.pop("value"), "unit": "mini-batches/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": m.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "value_schedule": m["schedule"],
        "config": dict(w.describe(), model=a.model, **({"heads": r.heads} if a.model == "gat" else {}),
                       fanout_order="fanouts[l] expands layer l+1 into layer l",
                       graph_gen_s=round(t_gen, 1),
                       **({"features": "pinned host memory", "cache_frac": a.cache_frac} if cache_info else {}),
                       launch=m.pop("launch"), schedule=m.pop("schedule")),
    }
    out.update(m)

    if a.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = {"read": src.numel() * 4, "written": dst.numel() * 4}
        del src, dst

    if not a.no_cpu_baseline and a.model == "gat":
        n_cpu = max(1, min(a.cpu_iters, 2 if a.workload == "medium" else 1))
        host = {"indptr": w.indptr.cpu().numpy(), "indices": w.indices.cpu().numpy(),
                "pmap": w.pmap.cpu().numpy(), "feat": w.feat.cpu().numpy(),
                "labels": w.labels.cpu().numpy(), "S": w.n_splits, "fanouts": w.fanouts,
                "heads": r.heads, "gat": [[t.cpu().numpy() for t in lst] for lst in r.gat_w],
                "targets": [w.targets(a.warmup + i).cpu().numpy() for i in range(n_cpu)]}
        out["cpu_baseline"] = cpu_baseline_gat(host, n_cpu)
    elif not a.no_cpu_baseline:
        host = {"indptr": w.indptr.cpu().numpy(), "indices": w.indices.cpu().numpy(),
                "pmap": w.pmap.cpu().numpy(), "feat": w.feat.float().cpu().numpy(),
                "labels": w.labels.cpu().numpy(), "S": w.n_splits, "fanouts": w.fanouts,
                "w_self": [t.cpu().numpy() for t in w.w_self],
                "w_neigh": [t.cpu().numpy() for t in w.w_neigh],
                "bias": [t.cpu().numpy() for t in w.bias],
                "targets": [w.targets(a.warmup + i).cpu().numpy() for i in range(a.cpu_iters)]}
        out["cpu_baseline"] = cpu_baseline(host, a.cpu_iters)
        del host
    r.ctx.close()
    if a.extra_configs is None:
        a.extra_configs = (a.workload == "medium" and a.model == "sage" and dtype == "f32" and cache_info is None
                           and not a.graph and not a.no_pipeline)
    if a.extra_configs:
        del w, r
        torch.cuda.empty_cache()
        out["extra_configs"] = extra_configs(a, dev, say)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
