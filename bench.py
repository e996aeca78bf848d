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
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-iters", type=int, default=120)
    ap.add_argument("--no-pipeline", action="store_true",
                    help="time strictly serial steps on one stream (default: sampling+gather of step i+1 "
                         "overlaps forward/backward of step i on a second stream)")
    ap.add_argument("--ahead", type=int, default=2, help="sampling streams (steps sampled ahead)")
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
    return ap.parse_args()


class Runner:
    """Holds the device-resident inputs, the context and the preallocated outputs of a step."""

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
                        r.forward()
                        r.loss()
                        r.backward()
                    self.free[k].record(self.s_train)
                freed.put(None)
        finally:
            for _ in range(count):      # a sampler left waiting for a slot can always finish
                freed.put(None)
            th.join()


def cpu_baseline(w_host, iters):
    """The oracle as it stands, timed on the host cores on `iters` whole iterations."""
    import numpy as np
    from oracle import reference as R
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = 1
    ip, ix, pm = w_host["indptr"], w_host["indices"], w_host["pmap"]
    params = R.SageParams(w_host["w_self"], w_host["w_neigh"], w_host["bias"])
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
        if time.perf_counter() - t0 > 30.0:      # the sample stays bounded on the larger workloads
            break
    iters = done
    dt = time.perf_counter() - t0
    return {"value": iters / dt, "unit": "mini-batches/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{iters} whole iterations of the same workload (C steps single-threaded, "
                      f"numpy float64 matmuls on {threads} BLAS threads), {dt:.1f} s"}


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


def main():
    a = parse()
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
        w = workloads.large(device=dev, n_splits=a.splits, feat_dtype=fdt, batch=8192, fanouts=(10, 10, 10, 10),
                            dims=(128, 256, 256, 256, 172), progress=say)
        w.name = f"sweep-S{a.splits}"
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
    r = Runner(w, dev, a.model, a.heads)
    cache_info = None
    if a.cache_frac is not None:
        # offline: rank every split's vertices by how often the sampler puts them into the input layer
        # (library kernel), keep the hottest fraction (a sort: the caller's policy step), build the cache
        host_table = torch.empty(w.feat.shape, dtype=w.feat.dtype, pin_memory=True)
        host_table.copy_(w.feat)
        k_in = torch.zeros(w.n_vertices, dtype=torch.int32, device=dev)
        for i in range(a.cache_presample):
            r.ctx.gsplit_sample_split(w.targets(10_000_000 + i), r.seed, 10_000_000 + i)
            r.ctx.gsplit_input_counts_accumulate(k_in)
        ids, n_cache = [], []
        for s_ in range(w.n_splits):
            own = torch.nonzero((w.pmap == s_) & (k_in > 0)).flatten()
            order = torch.sort(-k_in[own].long(), stable=True).indices
            keep = int(a.cache_frac * int((w.pmap == s_).sum()))
            ids.append(own[order][:keep].int())
            n_cache.append(int(ids[-1].numel()))
        cache_ids = torch.cat(ids).contiguous()
        cache_info = {"host_table": host_table, "ids": cache_ids, "n_cache": n_cache}
        r.enable_cache(host_table, cache_ids, n_cache)
        del k_in
    n_total = a.warmup + a.steps
    targets = [w.targets(i) for i in range(n_total)]
    torch.cuda.synchronize()

    # strictly serial steps on one stream
    use_graph = a.graph
    targets_all = torch.stack(targets).contiguous() if use_graph else None
    for i in range(a.warmup):
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
        r.step_idx.fill_(a.warmup)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.warmup, n_total):
        if use_graph:
            g_step.replay()
        else:
            r.step(targets[i], i)
    torch.cuda.synchronize()
    dt_serial = time.perf_counter() - t0
    dt = dt_serial
    if not a.no_pipeline:
        pipe = Pipelined(w, dev, a.ahead, a.model, a.heads, a.sampler_blocks)
        if cache_info:
            for slot in pipe.slots:
                slot.enable_cache(cache_info["host_table"], cache_info["ids"], cache_info["n_cache"])
        pipe.run(targets, 0, a.warmup)
        torch.cuda.synchronize()
        if use_graph:
            pipe.enable_graphs(targets_all)
            pipe.run(targets, 0, a.warmup)
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        pipe.run(targets, a.warmup, a.steps)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    ms_per_step = dt / a.steps * 1e3

    # per-stage device times (separate instrumented pass; events on the stream the kernels run on)
    n_st = min(a.stage_iters, a.steps)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(n_st)]
    for i in range(n_st):
        r.step(targets[a.warmup + i], a.warmup + i, ev[i])
    torch.cuda.synchronize()
    names = ["sample_split", "gather", f"{a.model}_fwd", "loss_grad", f"{a.model}_bwd"]
    stage_ms = {nm: sum(ev[i][k].elapsed_time(ev[i][k + 1]) for i in range(n_st)) / max(n_st, 1)
                for k, nm in enumerate(names)}

    # per-kernel device times: the library brackets each of its launches with HIP events on the
    # launch stream; algorithmic bytes / flops are summed over the very same iterations
    L, S = w.n_layers, w.n_splits
    row_bytes = w.dims[0] * w.feat.element_size()
    ip_bytes = w.indptr.element_size()
    work = {}      # label -> [kind, amount]

    def add(label, kind, amount):
        work.setdefault(label, [kind, 0.0])[1] += amount

    r.ctx.gsplit_timing_enable(True)
    n_k = max(1, min(a.stage_iters, a.steps))
    shape = None
    for i in range(n_k):
        r.step(targets[a.warmup + i], a.warmup + i)
        n_local, n_mixed, n_edges, bucket = r.ctx.gsplit_batch_sizes()     # waits for sampling only
        rows = [sum(x) for x in n_local]
        edges = [sum(x) for x in n_edges]
        mixed = [sum(x) for x in n_mixed]
        shape = (rows, edges, mixed, bucket)
        add("gather_rows", "bytes", rows[0] * (2 * row_bytes + 4))
        add("gather_cached", "bytes", rows[0] * (2 * row_bytes + 8))
        for l in range(L if a.model == "gat" else 0):
            # the transform and both backward products run over the rows of level l; the row kernels
            # move one transformed (or gradient) row per entry (edge or self) and its coefficients
            D, nd, n_lo = w.dims[l], rows[l + 1], rows[l]
            K = r.heads[l]
            HF = K * w.dims[l + 1] if l == L - 1 else w.dims[l + 1]
            ent = edges[l] + nd
            if l == 0:
                # bottom layer, aggregate-then-transform: per-head products over the destinations; the row
                # kernels move one input row per entry
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
        for l in range(L):
            D, N, nd = w.dims[l], w.dims[l + 1], rows[l + 1]
            add(f"linear_fwd.l{l}", "flops", 2.0 * nd * (2 * D) * N)
            add(f"grad_w.l{l}", "flops", 2.0 * nd * (2 * D + 1) * N)
            if l > 0:
                add(f"grad_in.l{l}", "flops", 2.0 * nd * N * (2 * D))
                add(f"pull_input_grad.l{l}", "bytes", (nd + edges[l]) * (4 + 4 * D) + rows[l] * (8 + 8 * D))
            # no-reuse model: one source row per edge, one self row and one [self | mean] row per destination
            es = w.feat.element_size()
            add(f"assemble_input.l{l}", "bytes", edges[l] * (4 + es * D) + nd * (4 + es * D) + nd * 2 * es * D)
            # per destination: id + two indptr words read, count written, and like every edge below an
            # 8-byte entry in each of the two tables and the two 4-byte entry indices it remembers;
            # per edge: 4 read, 4 written, 2 x 8 table bytes, 2 x 4 index bytes
            add(f"sample_layer.l{l}", "bytes", nd * (8 + 2 * ip_bytes + 24) + edges[l] * 32)
            slots = nd * w.fanouts[l]
            add(f"mixed_buckets_count.l{l}", "bytes", slots * (4 + 4 + 8 + 4) + edges[l] * 1)
            add(f"mixed_buckets_scatter.l{l}", "bytes", slots * 4 + edges[l] * 4 + mixed[l] * (4 + 4 + 4 + 8 + 4))
    torch.cuda.synchronize()
    ktimes = r.ctx.gsplit_timing_read()
    r.ctx.gsplit_timing_enable(False)
    kernel_us = {k: v[1] / max(v[0], 1) * 1e3 for k, v in ktimes.items()}
    per_step_us = {k: v[1] / n_k * 1e3 for k, v in ktimes.items()}
    dominant = max(per_step_us, key=per_step_us.get)

    def measured_traffic(label):
        """HBM bytes per launch of this kernel from the committed rocprofv3 counter summary
        (FETCH_SIZE + WRITE_SIZE, scaled by the copy calibration stated there), or None."""
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                            f"{a.workload}_bench_hbm_traffic.txt")
        if a.model == "gat":
            path = path.replace("_bench_", "_gat_bench_")
        if dtype != "f32" or not os.path.exists(path):
            return None
        for line in open(path):
            f = line.split()
            if len(f) >= 6 and f[0] == label:
                try:
                    return (float(f[-2]) + float(f[-1])) * 1024.0
                except ValueError:
                    return None
        return None

    def roofline_of(label):
        cnt, ms = ktimes[label]
        kind, amount = work.get(label, ("bytes", 0.0))
        per_launch = amount / max(cnt, 1)
        sec = ms / max(cnt, 1) * 1e-3
        if kind == "flops":
            ach = per_launch / sec / 1e12
            peak = BF16_MFMA_PEAK_TFLOPS if dtype == "bf16" else FP32_MFMA_PEAK_TFLOPS
            return {"kernel": label, "bound": "mfma", "achieved": ach, "peak": peak,
                    "unit": "TFLOP/s", "frac": ach / peak, "traffic": measured_traffic(label),
                    "flops_per_launch": per_launch, "launch_ms": ms / max(cnt, 1)}
        ach = per_launch / sec / 1e9
        return {"kernel": label, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": measured_traffic(label), "bytes_per_launch": per_launch,
                "launch_ms": ms / max(cnt, 1)}

    rows, edges, mixed, bucket = shape
    gather = roofline_of("gather_cached" if cache_info else "gather_rows")
    if cache_info:
        # hits and misses of the kernel-timing iterations alone (the counters ran since the cache was built)
        r.hits.zero_(); r.misses.zero_()
        for i in range(n_k):
            r.ctx.gsplit_sample_split(targets[a.warmup + i], r.seed, a.warmup + i)
            r.load(count=True)
        torch.cuda.synchronize()
        h, m = int(r.hits.sum()), int(r.misses.sum())
        PCIE_PEAK_GBS = 64.0       # PCIe 5.0 x16, one direction
        link = m / n_k * row_bytes / (gather["launch_ms"] * 1e-3) / 1e9
        gather["cache"] = {"fraction_cached": a.cache_frac, "rows_cached": int(sum(cache_info["n_cache"])),
                           "hit_rate": h / max(h + m, 1), "miss_bytes_per_launch": m / n_k * row_bytes,
                           "host_link": {"achieved": link, "peak": PCIE_PEAK_GBS, "unit": "GB/s", "frac": link / PCIE_PEAK_GBS}}
    out = {
        "metric": f"mini-batches/sec (sample+split+gather+{'GAT' if a.model == 'gat' else 'SAGE'} fwd/bwd) at 1 GPU",
        "value": a.steps / dt, "unit": "mini-batches/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": dict(w.describe(), model=a.model, **({"heads": r.heads} if a.model == "gat" else {}),
                       fanout_order="fanouts[l] expands layer l+1 into layer l",
                       graph_gen_s=round(t_gen, 1),
                       **({"features": "pinned host memory", "cache_frac": a.cache_frac} if cache_info else {}),
                       launch=("every stream replays captured HIP graphs (the step counter and the targets table "
                               "stay in device memory)" if use_graph else "kernels enqueued from the host"),
                       **({"graph_replay_equals_eager": graph_check} if use_graph else {}),
                       schedule=("serial, one stream" if a.no_pipeline else
                                 f"{a.ahead} sampling stream(s) + 1 training stream: sample+split+gather of the "
                                 f"next {a.ahead} step(s) overlap fwd/loss/bwd of step i")),
        "serial_ms_per_step": dt_serial / a.steps * 1e3,
        "gather_GBps": gather["achieved"],
        "stage_ms": stage_ms,
        "kernel_us_per_step": {k: round(v, 2) for k, v in sorted(per_step_us.items(), key=lambda kv: -kv[1])},
        "batch_shape": {"rows_per_level": rows, "edges_per_layer": edges, "mixed_rows_per_layer": mixed,
                        "ids_shuffled_per_layer": [sum(b[s][t] for s in range(S) for t in range(S) if s != t)
                                                   for b in bucket]},
        "roofline": roofline_of(dominant),
        "roofline_gather": gather,
    }

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
                "pmap": w.pmap.cpu().numpy(), "feat": w.feat.cpu().numpy(),
                "labels": w.labels.cpu().numpy(), "S": w.n_splits, "fanouts": w.fanouts,
                "w_self": [t.cpu().numpy() for t in w.w_self],
                "w_neigh": [t.cpu().numpy() for t in w.w_neigh],
                "bias": [t.cpu().numpy() for t in w.bias],
                "targets": [w.targets(a.warmup + i).cpu().numpy() for i in range(a.cpu_iters)]}
        out["cpu_baseline"] = cpu_baseline(host, a.cpu_iters)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
