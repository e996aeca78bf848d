"""GPU parity of the GAT layer (paper section 7.1, second model): gsplit_gat_fwd / gsplit_gat_bwd,
called through the C ABI, against oracle/gat.py on the same seeded batch, features and parameters.
Logits and every parameter gradient within 1e-4 of the float64 oracle, measured as
|a - o| / max(|o|, 1e-2 * max|o|); for the two attention-vector gradients of a layer max|o| is
taken over both (see attention_grad_err).  Where a LeakyReLU argument is zero to float32 rounding
the oracle's backward pass takes the slope the device took (read from the score terms the device
stored); everywhere else the two must agree."""
import numpy as np
import pytest
import torch

import workloads
from oracle import reference as R
from oracle import gat as G

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4


def _dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


def _run(w, heads, dev, seed, it, n_splits=None, pmap=None, batch_targets=None):
    from paper_2303_13775_amd import Context, GatParams
    S = n_splits or w.n_splits
    pm = w.pmap if pmap is None else pmap
    ctx = Context(w.indptr.to(dev), w.indices.to(dev), pm.to(dev), S, w.fanouts, w.batch, gat_index=True)
    tg = w.targets(it) if batch_targets is None else batch_targets
    ctx.gsplit_sample_split(tg.to(dev), seed, it)
    x0 = torch.empty((ctx.gsplit_max_rows(0), w.dims[0]), dtype=torch.float32, device=dev)
    ctx.gsplit_gather_features(w.feat.to(dev), x0)
    wt, a_s, a_d, b = workloads.gat_weights(w.dims, heads, seed=w.seed)
    params = GatParams(w.dims, heads, [t.to(dev) for t in wt], [t.to(dev) for t in a_s], [t.to(dev) for t in a_d],
                       [t.to(dev) for t in b])
    logits = torch.full((tg.numel(), w.dims[-1]), 7.0, device=dev)
    ctx.gsplit_gat_fwd(params, x0, logits)
    ob = R.sp_sample(w.indptr.numpy(), w.indices.numpy(), pm.numpy(), S, w.fanouts, tg.numpy(), seed, it)
    op = G.GatParams(list(heads), [t.numpy() for t in wt], [t.numpy() for t in a_s], [t.numpy() for t in a_d],
                     [t.numpy() for t in b])
    of = G.gat_forward(ob, R.gather_rows(w.feat.numpy(), ob.local_cat(0)), op)
    lab = w.labels.numpy()[tg.numpy()[ob.target_perm]]
    _, g = R.softmax_xent(of.logits, lab)
    gw = [torch.full_like(t, 7.0, device=dev) for t in wt]           # must be overwritten
    gas = [torch.full_like(t, 7.0, device=dev) for t in a_s]
    gad = [torch.full_like(t, 7.0, device=dev) for t in a_d]
    gb = [torch.full_like(t, 7.0, device=dev) for t in b]
    ctx.gsplit_gat_bwd(params, x0, torch.from_numpy(g.astype(np.float32)).to(dev), gw, gas, gad, gb)
    torch.cuda.synchronize()
    obw, report = conditioned_gat_backward(ctx, ob, of, op, g, heads, who=w.name)
    res = dict(logits=logits.cpu().numpy(), gw=[t.cpu().numpy() for t in gw], gas=[t.cpu().numpy() for t in gas],
               gad=[t.cpu().numpy() for t in gad], gb=[t.cpu().numpy() for t in gb], of=of, ob=obw, report=report)
    ctx.close()
    return res


# a LeakyReLU argument closer to zero than this (relative to the layer's largest) is not decided
# by a float32 evaluation of the scores (the scores are sums of a few hundred float32 products)
TAU_SCORE = 2e-6


def conditioned_gat_backward(ctx, ob, of, op, g, heads, who=""):
    """Oracle backward pass with the device's LeakyReLU slope decisions inside the rounding band
    only; a disagreement outside the band fails the test."""
    terms = [tuple(t.cpu().numpy() for t in ctx.fetch_gat_score_terms(l, heads[l])) for l in range(len(heads))]
    slopes, report = G.conditioned_slopes(ob, of, op, terms, TAU_SCORE)
    for l, (n_band, n_flip, n_bad) in enumerate(report):
        assert n_bad == 0, (f"{who}: layer {l}: {n_bad} LeakyReLU slopes differ from the oracle's although |score| > "
                            f"{TAU_SCORE:g} * max|score|")
    return G.gat_backward(ob, of, op, g, slope_positive=slopes), report


def attention_grad_err(a, o, o_src, o_dst, terms=None) -> float:
    """Error of an attention-vector gradient, judged against the common scale of the layer's two
    attention gradients: d a_dst sums the very terms of d a_src, but over the neighbours of a
    destination first, where they cancel (with every score in the linear part of the LeakyReLU
    the softmax does not depend on the destination term at all and d a_dst is identically zero),
    so its entries are small differences of terms of the size of d a_src."""
    a = np.asarray(a, np.float64).reshape(-1); o = np.asarray(o, np.float64).reshape(-1)
    scale = np.maximum(np.abs(o), 1e-2 * max(np.abs(o_src).max(), np.abs(o_dst).max()))
    # Both gradients are sums of terms that cancel (inside the softmax backward, then over the
    # edges): with few neighbours and near-uniform attention d a_src cancels to 10^-4 of its terms
    # as well.  A float32 sum carries a rounding error proportional to the magnitudes summed
    # (|fl(sum x) - sum x| <= gamma_n sum |x|), which the oracle reports per entry; that much of the
    # difference is rounding, whatever the size of the result (measured: up to 2 units of 2^-24).
    noise = 0.0 if terms is None else 8.0 * 2.0 ** -24 * np.asarray(terms, np.float64).reshape(-1)
    return float((np.maximum(np.abs(a - o) - noise, 0.0) / np.where(scale == 0, 1.0, scale)).max())


def _check(r, L):
    """Logits and every parameter gradient against the oracle, every entry, no allowance."""
    assert R.max_rel_err(r["logits"], r["of"].logits) < TOL_F32, "logits"
    if any(x[1] for x in r["report"]):
        print(f"[gat] LeakyReLU band per layer (scores, decided otherwise by the device, outside): {r['report']}", flush=True)
    for l in range(L):
        o_src, o_dst = r["ob"].ga_src[l], r["ob"].ga_dst[l]
        terms = r["ob"].ga_terms[l]
        errs = {"gw": R.max_rel_err(r["gw"][l], r["ob"].gw[l]),
                "ga_src": attention_grad_err(r["gas"][l], o_src, o_src, o_dst, terms),
                "ga_dst": attention_grad_err(r["gad"][l], o_dst, o_src, o_dst, terms),
                "gbias": R.max_rel_err(r["gb"][l].reshape(-1), r["ob"].gbias[l].reshape(-1))}
        bad = {k: v for k, v in errs.items() if not v < TOL_F32}
        assert not bad, (l, bad)


# name -> (workload, heads): widths that take the 16-byte and the scalar lane layouts, head counts
# that are and are not powers of two, one to sixteen values per lane, S = 1 .. 8; bottom layers
# that run aggregate-then-transform (input width and features per head multiples of 4) and ones
# that run transform-then-aggregate like the layers above
CASES = {
    "tiny-2x1": (lambda: workloads.tiny(), None),
    "heads-4-4-1": (lambda: workloads.custom(6000, 150000, dims=[100, 64, 64, 47], fanouts=[6, 5, 4], batch=300,
                                             n_splits=4, name="gat-a"), [4, 4, 1]),
    "heads-3-odd-widths": (lambda: workloads.custom(3000, 50000, dims=[30, 33, 10], fanouts=[5, 4], batch=129,
                                                    n_splits=3, name="gat-b"), [3, 2]),
    "wide-single-head": (lambda: workloads.custom(8000, 200000, dims=[128, 512, 172], fanouts=[6, 5], batch=256,
                                                  n_splits=4, pmap_kind="range", name="gat-c"), [1, 1]),
    "heads-8-S8-fan20": (lambda: workloads.custom(5000, 200000, dims=[64, 256, 40], fanouts=[20, 15], batch=200,
                                                  n_splits=8, name="gat-d"), [8, 6]),
    # 320 input features: two 16-byte vectors per lane in the bottom-layer kernels
    "input-320": (lambda: workloads.custom(4000, 90000, dims=[320, 64, 10], fanouts=[7, 5], batch=200,
                                           n_splits=4, name="gat-f"), [2, 2]),
    # one layer only: the bottom layer is also the last one
    "single-layer": (lambda: workloads.custom(3000, 60000, dims=[64, 12], fanouts=[9], batch=150,
                                              n_splits=2, name="gat-g"), [3]),
    "S1-scalar-wide": (lambda: workloads.custom(2000, 30000, dims=[18, 250, 7], fanouts=[5, 5], batch=300,
                                                n_splits=1, name="gat-e"), [2, 5]),
}


@pytest.mark.parametrize("name", list(CASES))
def test_gat_forward_backward_within_tolerance(name):
    make, heads = CASES[name]
    w = make()
    if heads is None:
        heads = [2] * (w.n_layers - 1) + [1]
        assert all(w.dims[l + 1] % heads[l] == 0 for l in range(w.n_layers - 1))
    for seed, it in ((55, 1), (333, 3)):
        _check(_run(w, heads, _dev(), seed=seed, it=it), w.n_layers)


def _hub_workloads():
    from test_gpu_parity import _star_workload
    return {
        # a skewed graph without id permutation: the busiest rows feed hundreds of destinations (more than a
        # wave sorts at once: windows of ascending codes)
        "hubs": (lambda: workloads.custom(20000, 1200000, dims=[32, 64, 64, 16], fanouts=[12, 12, 12], batch=2000,
                                          n_splits=4, abc=(0.7, 0.1, 0.1), permute_ids=False, name="gat-hubs"), [2, 2, 1]),
        # every vertex aggregates from vertex 0: one row with thousands of entries
        "huge-hub": (_star_workload, [2, 1]),
    }


@pytest.mark.parametrize("name", ["hubs", "huge-hub"])
def test_gat_gradients_are_bit_reproducible(name):
    """Three backward passes over the same batch give bit-equal gradients (the pull over the scatter
    side of the shuffle index sums a row's entries in ascending code order, whatever order the atomic
    cursor filled them in), and they are within tolerance of the oracle."""
    from paper_2303_13775_amd import Context, GatParams
    dev = _dev()
    make, heads = _hub_workloads()[name]
    w = make()
    _check(_run(w, heads, dev, seed=9, it=2), w.n_layers)
    ctx = Context(w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev), w.n_splits, w.fanouts, w.batch, gat_index=True)
    wt, a_s, a_d, b = workloads.gat_weights(w.dims, heads, seed=w.seed)
    params = GatParams(w.dims, heads, [t.to(dev) for t in wt], [t.to(dev) for t in a_s], [t.to(dev) for t in a_d],
                       [t.to(dev) for t in b])
    x0 = torch.empty((ctx.gsplit_max_rows(0), w.dims[0]), dtype=torch.float32, device=dev)
    logits = torch.empty((w.batch, w.dims[-1]), device=dev)
    glog = torch.randn((w.batch, w.dims[-1]), generator=torch.Generator().manual_seed(5)).to(dev)
    outs = [[torch.empty_like(t, device=dev) for t in lst] for lst in (wt, a_s, a_d, b)]
    runs = []
    for _ in range(3):
        ctx.gsplit_sample_split(w.targets(2).to(dev), 9, 2)
        ctx.gsplit_gather_features(w.feat.to(dev), x0)
        ctx.gsplit_gat_fwd(params, x0, logits)
        ctx.gsplit_gat_bwd(params, x0, glog, *outs)
        torch.cuda.synchronize()
        runs.append([logits.clone()] + [t.clone() for lst in outs for t in lst])
    longest = max(int(ctx.fetch_shuffle(l)["rev_cnt"].max()) for l in range(w.n_layers))
    print(f"\n[gat reproducible {name}] longest reverse-index row {longest} entries", flush=True)
    assert longest > 64
    for other in runs[1:]:
        for x, y in zip(runs[0], other):
            assert torch.equal(x, y), "results of two runs of the same batch differ in some bit"
    ctx.close()


def test_gat_edge_cases_isolated_targets_and_one_owner():
    dev = _dev()
    w = workloads.custom(500, 1500, dims=[8, 8, 4], fanouts=[3, 2], batch=16, n_splits=4, name="edge")
    ip = w.indptr.numpy().astype(np.int64)
    iso = torch.from_numpy(np.nonzero((ip[1:] - ip[:-1]) == 0)[0][:5].astype(np.int32))
    assert iso.numel() > 0
    # isolated targets: every neighbourhood is the vertex itself, alpha = 1
    _check(_run(w, [2, 3], dev, seed=3, it=0, batch_targets=iso), 2)
    # all targets owned by one split
    pm = w.pmap.numpy()
    own = torch.from_numpy(np.nonzero(pm == 2)[0][:16].astype(np.int32))
    _check(_run(w, [2, 3], dev, seed=3, it=0, batch_targets=own), 2)


def test_gat_rejects_bad_arguments():
    from paper_2303_13775_amd import Context, GatParams, GsplitError
    dev = _dev()
    w = workloads.tiny()
    heads = [2] * (w.n_layers - 1) + [1]
    wt, a_s, a_d, b = workloads.gat_weights(w.dims, heads, seed=w.seed)
    params = GatParams(w.dims, heads, [t.to(dev) for t in wt], [t.to(dev) for t in a_s], [t.to(dev) for t in a_d],
                       [t.to(dev) for t in b])
    tg = w.targets(0)
    logits = torch.empty((tg.numel(), w.dims[-1]), device=dev)
    # a context without the bottom-layer reverse index
    ctx = Context(w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev), w.n_splits, w.fanouts, w.batch)
    ctx.gsplit_sample_split(tg.to(dev), 1, 0)
    x0 = torch.zeros((ctx.gsplit_max_rows(0), w.dims[0]), device=dev)
    with pytest.raises(GsplitError):
        ctx.gsplit_gat_fwd(params, x0, logits)
    ctx.close()
    ctx = Context(w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev), w.n_splits, w.fanouts, w.batch, gat_index=True)
    x0 = torch.zeros((ctx.gsplit_max_rows(0), w.dims[0]), device=dev)
    with pytest.raises(GsplitError):          # no batch yet
        ctx.gsplit_gat_fwd(params, x0, logits)
    ctx.gsplit_sample_split(tg.to(dev), 1, 0)
    gw = [torch.empty_like(t, device=dev) for t in wt]
    ga = [torch.empty_like(t, device=dev) for t in a_s]
    gd = [torch.empty_like(t, device=dev) for t in a_d]
    gb = [torch.empty_like(t, device=dev) for t in b]
    with pytest.raises(GsplitError):          # backward before forward
        ctx.gsplit_gat_bwd(params, x0, logits, gw, ga, gd, gb)
    ctx.gsplit_gat_fwd(params, x0, logits)
    ctx.gsplit_sample_split(w.targets(1).to(dev), 1, 1)
    with pytest.raises(GsplitError):          # the forward pass belongs to another batch
        ctx.gsplit_gat_bwd(params, x0, logits, gw, ga, gd, gb)
    torch.cuda.synchronize()
    ctx.close()
