"""The whole path on randomly drawn configurations (seeded, so every run draws the same ones):
graph size and density, int32 / int64 row pointers, number of layers, fanouts, number of splits,
partition-map kind, batch size, and widths that are and are not multiples of 4.  On each:
sampling and splitting bit-exact against the oracle, GraphSAGE (float32 and the bf16 path) and GAT
forward/backward within their tolerances (paper Algorithms 1 and 2, section 7.1 for the models)."""
import numpy as np
import pytest
import torch

import workloads
from oracle import reference as R
from test_gpu_parity import (FLOOR_BF16, TOL_BF16, TOL_F32, _ctx, _dev, _oracle_batch, _run_fwd_bwd,
                             assert_batch_equal)
from test_gpu_gat import _check as check_gat, _run as run_gat

pytestmark = pytest.mark.gpu

N_CONFIGS = 48


def draw(k: int):
    """Configuration k: the workload and the GAT head counts that fit its widths."""
    rng = np.random.default_rng(9000 + k)
    n = int(10 ** rng.uniform(1.7, 3.9))
    n_directed = max(1, int(n * rng.uniform(0.5, 30.0) / 2))
    L = int(rng.integers(1, 5))
    budget = 40000                                   # bound on destinations + slots of the bottom layer
    batch = int(rng.integers(1, min(n, 500) + 1))
    fanouts = []
    grown = batch
    for _ in range(L):
        f = int(rng.integers(1, 41 if rng.random() < 0.15 else 13))
        while f > 1 and grown * (1 + f) > budget:
            f -= 1
        fanouts.append(f)
        grown = min(n, grown * (1 + f))
    fanouts = fanouts[::-1]                           # fanouts[l] expands level l+1: keep the wide ones on top
    S = int(rng.integers(1, 9))
    heads = [int(rng.integers(1, 5)) for _ in range(L - 1)] + [1]
    by4 = rng.random() < 0.5
    width = lambda lo, hi: int(rng.integers(lo, hi + 1)) * 4 if by4 else int(rng.integers(lo, 4 * hi + 1))
    dims = [width(1, 35)] + [heads[l] * width(1, max(1, 32 // heads[l])) for l in range(L - 1)]
    dims.append(int(rng.integers(2, 61)))
    kind = ["random", "range", "bfs"][int(rng.integers(0, 3))]
    w = workloads.custom(n, n_directed, dims=dims, fanouts=fanouts, batch=batch, n_splits=S, pmap_kind=kind,
                         index64=bool(rng.random() < 0.3), seed=4000 + k, name=f"random-{k}")
    return w, heads


@pytest.mark.parametrize("k", range(N_CONFIGS))
def test_random_configuration(k):
    dev = _dev()
    w, heads = draw(k)
    print(f"\n[random {k}] {w.describe()} heads {heads}", flush=True)
    ctx = _ctx(w, dev)
    for it in (0, 1):
        tg = w.targets(it).to(dev)
        ctx.gsplit_sample_split(tg, 500 + k, it)
        assert_batch_equal(ctx.fetch_batch(), _oracle_batch(w, tg, 500 + k, it), w.n_splits, w.n_layers)
    ctx.close()
    r = _run_fwd_bwd(w, dev, seed=500 + k, it=1)
    assert R.max_rel_err(r["logits"], r["of"].logits) < TOL_F32, "sage logits"
    sws, swn, sb, _ = r["slack"]
    for l in range(w.n_layers):
        assert R.grad_err(r["gws"][l], r["ob"].gw_self[l], sws[l]) < TOL_F32, ("sage gw_self", l)
        assert R.grad_err(r["gwn"][l], r["ob"].gw_neigh[l], swn[l]) < TOL_F32, ("sage gw_neigh", l)
        assert R.grad_err(r["gb"][l], r["ob"].gbias[l], sb[l]) < TOL_F32, ("sage gbias", l)
    check_gat(run_gat(w, heads, dev, seed=500 + k, it=1), w.n_layers)
    if any(d % 4 for d in w.dims[:-1]):
        return                     # the bf16 path takes input and hidden widths that are multiples of 4
    r = _run_fwd_bwd(w, dev, seed=500 + k, it=0, bf16=True)
    assert R.max_rel_err(r["logits"], r["of"].logits, floor=FLOOR_BF16) < TOL_BF16, "bf16 logits"
    sws, swn, sb, _ = r["slack"]
    for l in range(w.n_layers):
        assert R.grad_err(r["gws"][l], r["ob"].gw_self[l], sws[l], floor=FLOOR_BF16) < TOL_BF16, ("bf16 gw_self", l)
        assert R.grad_err(r["gwn"][l], r["ob"].gw_neigh[l], swn[l], floor=FLOOR_BF16) < TOL_BF16, ("bf16 gw_neigh", l)
        assert R.grad_err(r["gb"][l], r["ob"].gbias[l], sb[l], floor=FLOOR_BF16) < TOL_BF16, ("bf16 gbias", l)
