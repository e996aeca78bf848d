"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Integer outputs (sampling, splits, dedup, relabel, buckets, both sides of the shuffle
index) must be bit-exact; fp32 GraphSAGE outputs and gradients within 1e-4 max relative error
(|a - o| / max(|o|, 1e-2 * max|o|)), every entry, with no allowance: where a pre-activation is zero
to the forward pass's rounding the oracle's backward pass takes the device's ReLU decision (read
from the activations the device stored), everywhere else the decisions must agree.  The bf16 path
is held to 1e-2 against two oracles: the one that rounds the values the device stores in bf16
(entry by entry, floor 1e-2 * max|o| like fp32) and the one that rounds nothing but the inputs
and weights it is given (the plain definition of Algorithm 2)."""
import numpy as np
import pytest
import torch

import workloads
from oracle import reference as R
import sage_check as SC
from sage_check import TOL_F32, TOL_BF16

pytestmark = pytest.mark.gpu


def _dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


def _ctx(w, dev, max_targets=None, table_mode=0):
    from paper_2303_13775_amd import Context
    return Context(w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev), w.n_splits, w.fanouts,
                   max_targets or w.batch, table_mode=table_mode)


def _oracle_batch(w, tg, seed, it, n_splits=None, pmap=None):
    pm = w.pmap.cpu().numpy() if pmap is None else pmap
    return R.sp_sample(w.indptr.cpu().numpy(), w.indices.cpu().numpy(), pm,
                       n_splits or w.n_splits, w.fanouts, tg.cpu().numpy(), seed, it)


def assert_batch_equal(got, ob, S, L):
    """Every integer output of sample+split, element by element."""
    for l in range(L + 1):
        for s in range(S):
            assert np.array_equal(got["local_front"][l][s].cpu().numpy(), ob.local_front[l][s]), ("front", l, s)
    for l in range(L):
        lay = got["layers"][l]
        nbr = np.concatenate([b.nbr for b in ob.blocks[l]]) if S else np.zeros((0, 1))
        cnt = np.concatenate([b.cnt for b in ob.blocks[l]])
        assert np.array_equal(lay["nbr"].cpu().numpy(), nbr), ("nbr", l)
        assert np.array_equal(lay["cnt"].cpu().numpy(), cnt), ("cnt", l)
        indptr = lay["blk_indptr"].cpu().numpy()
        src = lay["blk_src"].cpu().numpy()
        row0 = 0
        for s in range(S):
            b = ob.blocks[l][s]
            n_dst = b.dst.shape[0]
            assert np.array_equal(lay["mixed"][s].cpu().numpy(), b.mixed_front), ("mixed", l, s)
            ip = indptr[row0:row0 + n_dst + 1]
            assert np.array_equal(ip - ip[0], b.blk_indptr), ("blk_indptr", l, s)
            assert np.array_equal(src[ip[0]:ip[-1]], b.blk_src), ("blk_src", l, s)
            assert np.array_equal(lay["shuffle_src_row"][s].cpu().numpy(), b.shuffle_src_row), ("shuffle", l, s)
            for t in range(S):
                assert got["bucket"][l][s][t] == b.buckets[t].shape[0], ("bucket size", l, s, t)
            row0 += n_dst
        recv = np.concatenate([ob.blocks[l][s].buckets[t] for t in range(S) for s in range(S)]) \
            if S else np.zeros(0, np.int32)
        assert np.array_equal(lay["recv"].cpu().numpy(), recv), ("recv", l)


CASES = {
    "tiny": lambda: workloads.tiny(),
    "ragged-S3": lambda: workloads.custom(3001, 41000, dims=[20, 12, 6], fanouts=[7, 3], batch=257,
                                          n_splits=3, name="ragged"),
    "fan32-S8-int64": lambda: workloads.custom(5000, 200000, dims=[8, 8, 8, 4], fanouts=[33, 20, 17],
                                               batch=100, n_splits=8, index64=True, name="wide"),
    "S1": lambda: workloads.custom(2000, 30000, dims=[16, 16, 4], fanouts=[5, 5], batch=300, n_splits=1,
                                   name="s1"),
    "range-map-deep": lambda: workloads.custom(20000, 600000, dims=[8, 8, 8, 8, 4], fanouts=[4, 3, 3, 2],
                                               batch=500, n_splits=4, pmap_kind="range", name="deep"),
    "fan64": lambda: workloads.custom(1500, 120000, dims=[8, 8], fanouts=[64], batch=64, n_splits=2,
                                      name="fan64"),
    # many distinct vertices per sampled slot and eight keys per vertex: the hashed table at its highest
    # load, full lines and probes that run over into the next line
    "table-load": lambda: workloads.custom(200000, 1200000, dims=[8, 8, 4], fanouts=[4, 3], batch=20000,
                                           n_splits=8, name="load"),
    # more than 2**20 slots at the upper bound of the bottom layer: the 1024-chunk partition
    "many-chunks": lambda: workloads.custom(60000, 1500000, dims=[8, 8, 8, 4], fanouts=[15, 10, 5], batch=2048,
                                            n_splits=4, pmap_kind="range", name="chunks"),
}


@pytest.mark.parametrize("table_mode", [1, 2], ids=["hashed", "direct"])
@pytest.mark.parametrize("name", list(CASES))
def test_sample_split_bit_exact(name, table_mode):
    """Both forms of the dedup tables (hashed; indexed by the key itself) give the oracle's batch."""
    dev = _dev()
    w = CASES[name]()
    ctx = _ctx(w, dev, table_mode=table_mode)
    for it in (0, 1):
        tg = w.targets(it)
        ctx.gsplit_sample_split(tg.to(dev), seed=1234 + it, it=it)
        got = ctx.fetch_batch()
        ob = _oracle_batch(w, tg, 1234 + it, it)
        assert_batch_equal(got, ob, w.n_splits, w.n_layers)
        for l in range(w.n_layers):
            SC.assert_shuffle_index_equal(ctx, ob, l, has_rev=l >= 1)
    ctx.close()


@pytest.mark.parametrize("name", list(CASES))
def test_wide_layer_relabelling_bit_exact(name, monkeypatch):
    """The relabelling of wide layers (the slots in a launch of their own, one access per slot) on every
    layer of every case: the bar that selects it is lowered to one slot.  A context that keeps the
    scatter side for the bottom layer too, so every layer counts its reverse index on this path."""
    from paper_2303_13775_amd import Context
    monkeypatch.setenv("GSPLIT_WIDE_SLOTS", "1")
    dev = _dev()
    w = CASES[name]()
    ctx = Context(w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev), w.n_splits, w.fanouts, w.batch,
                  gat_index=True, table_mode=1 + len(name) % 2)
    for it in (0, 1):
        tg = w.targets(it)[:w.batch - 11 * it]
        ctx.gsplit_sample_split(tg.to(dev), seed=4321 + it, it=it)
        ob = _oracle_batch(w, tg, 4321 + it, it)
        assert_batch_equal(ctx.fetch_batch(), ob, w.n_splits, w.n_layers)
        for l in range(w.n_layers):
            SC.assert_shuffle_index_equal(ctx, ob, l, has_rev=True, has_eid=True)
    ctx.close()


@pytest.mark.parametrize("name", ["tiny", "ragged-S3", "fan32-S8-int64", "S1"])
def test_shuffle_index_scatter_side_with_edge_ids(name):
    """A context that keeps the scatter side for the bottom layer too (gat_index): every layer's
    transpose of (self_row, edge_row) and the edge number behind every entry."""
    from paper_2303_13775_amd import Context
    dev = _dev()
    w = CASES[name]()
    ctx = Context(w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev), w.n_splits, w.fanouts, w.batch, gat_index=True)
    tg = w.targets(3)
    ctx.gsplit_sample_split(tg.to(dev), 99, 3)
    ob = _oracle_batch(w, tg, 99, 3)
    assert_batch_equal(ctx.fetch_batch(), ob, w.n_splits, w.n_layers)
    for l in range(w.n_layers):
        SC.assert_shuffle_index_equal(ctx, ob, l, has_rev=True, has_eid=True)
    ctx.close()


@pytest.mark.parametrize("name,n_batches", [("tiny", 4), ("ragged-S3", 3), ("fan32-S8-int64", 8), ("S1", 2),
                                            ("many-chunks", 2)])
def test_multi_batch_sampling_bit_exact(name, n_batches):
    """gsplit_sample_split_multi: several mini-batches through one set of launches, every one of them
    bit-equal to the oracle's (and hence to gsplit_sample_split's), batches of different sizes
    (the last one empty when there are more than two), both sides of the shuffle index included;
    then a training step on one of them."""
    from paper_2303_13775_amd import Context, GsplitError, gsplit_sample_split_multi, gsplit_gather_features_multi
    dev = _dev()
    w = CASES[name]()
    gi, gx, gp = w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev)
    ctxs = [Context(gi, gx, gp, w.n_splits, w.fanouts, w.batch, table_mode=1 + n_batches % 2) for _ in range(n_batches)]
    table = w.feat.to(dev)
    for rnd in (0, 1):
        its = [10 * rnd + b for b in range(n_batches)]
        tgs = [w.targets(it)[:max(0, w.batch - 37 * b)] for b, it in enumerate(its)]
        if n_batches > 2:
            tgs[-1] = tgs[-1][:0]
        gsplit_sample_split_multi(ctxs, [t.to(dev) for t in tgs], 777, its)
        # the loading step of all of them in one launch: byte for byte the table's rows
        outs = [torch.full((c.gsplit_max_rows(0), w.dims[0]), 7.0, device=dev) for c in ctxs]
        gsplit_gather_features_multi(ctxs, table, outs)
        for b in range(n_batches):
            ob = _oracle_batch(w, tgs[b], 777, its[b])
            assert_batch_equal(ctxs[b].fetch_batch(), ob, w.n_splits, w.n_layers)
            for l in range(w.n_layers):
                SC.assert_shuffle_index_equal(ctxs[b], ob, l, has_rev=l >= 1)
            ids = torch.from_numpy(ob.local_cat(0)).long().to(dev)
            assert torch.equal(outs[b][:ids.numel()], table[ids]), ("rows loaded by the grouped call", b)
            assert bool((outs[b][ids.numel():] == 7.0).all()), ("rows past the batch written", b)
    with pytest.raises(GsplitError):                       # the same context twice
        gsplit_sample_split_multi([ctxs[0], ctxs[0]], [tgs[0].to(dev)] * 2, 1, [0, 1])
    other = Context(gi, gx, gp, w.n_splits, w.fanouts, max(1, w.batch // 2), table_mode=1 + n_batches % 2)
    with pytest.raises(GsplitError):                       # another configuration
        gsplit_sample_split_multi([ctxs[0], other], [tgs[0].to(dev)[:1]] * 2, 1, [0, 1])
    for c in ctxs + [other]:
        c.close()


def test_edge_cases_empty_isolated_and_unowned_split():
    dev = _dev()
    w = workloads.custom(500, 1500, dims=[8, 8, 4], fanouts=[3, 2], batch=16, n_splits=4, name="edge")
    ip = w.indptr.cpu().numpy().astype(np.int64)
    deg = ip[1:] - ip[:-1]
    iso = np.nonzero(deg == 0)[0][:5].astype(np.int32)
    assert iso.shape[0] > 0
    ctx = _ctx(w, dev)
    # empty mini-batch
    ctx.gsplit_sample_split(torch.empty(0, dtype=torch.int32, device=dev), 1, 0)
    n_local, n_mixed, n_edges, _ = ctx.gsplit_batch_sizes()
    assert all(x == 0 for row in n_local for x in row) and all(x == 0 for row in n_edges for x in row)
    # isolated targets only: nothing is sampled, frontiers are the targets themselves
    tg = torch.from_numpy(iso)
    ctx.gsplit_sample_split(tg.to(dev), 1, 0)
    assert_batch_equal(ctx.fetch_batch(), _oracle_batch(w, tg, 1, 0), 4, 2)
    # targets all owned by one split, so the other splits start with nothing
    own0 = torch.nonzero(w.pmap == 0).flatten()[:16].to(torch.int32)
    ctx.gsplit_sample_split(own0.to(dev), 9, 4)
    assert_batch_equal(ctx.fetch_batch(), _oracle_batch(w, own0, 9, 4), 4, 2)
    # a single target, and the largest batch the context allows
    one = w.targets(3)[:1]
    ctx.gsplit_sample_split(one.to(dev), 2, 2)
    assert_batch_equal(ctx.fetch_batch(), _oracle_batch(w, one, 2, 2), 4, 2)
    ctx.close()


def test_error_paths():
    from paper_2303_13775_amd import Context, GsplitError
    dev = _dev()
    w = workloads.custom(500, 1500, dims=[8, 8, 4], fanouts=[3, 2], batch=16, n_splits=4, name="err")
    ctx = _ctx(w, dev)
    with pytest.raises(GsplitError) as e:
        ctx.gsplit_sample_split(w.targets(0)[:16].repeat(2).contiguous().to(dev), 0, 0)   # 32 > max_targets
    assert e.value.code == -3
    with pytest.raises(GsplitError):
        ctx.gsplit_max_rows(99)
    with pytest.raises(GsplitError) as e:
        Context(w.indptr.to(dev), w.indices.to(dev), w.pmap.to(dev), 4, [3, 200], 16)   # fanout too large
    assert e.value.code == -1
    bad = w.targets(0)[:8].clone(); bad[3] = w.n_vertices + 5            # id outside the graph
    ctx.gsplit_sample_split(bad.to(dev), 0, 0)
    with pytest.raises(GsplitError) as e:
        ctx.gsplit_batch_sizes()
    assert e.value.code == -1
    ctx.gsplit_sample_split(w.targets(0).to(dev), 0, 0)                   # the context stays usable
    ctx.gsplit_batch_sizes()
    ctx2 = _ctx(w, dev)
    with pytest.raises(GsplitError) as e:    # gather before any batch
        ctx2.gsplit_gather_features(w.feat.to(dev), torch.empty((ctx2.gsplit_max_rows(0), 8), device=dev))
    assert e.value.code == -5
    ctx.close(); ctx2.close()


@pytest.mark.parametrize("dim,dtype", [(64, torch.float32), (100, torch.float32), (128, torch.bfloat16),
                                       (7, torch.float32), (5, torch.bfloat16), (128, torch.float32)])
def test_gather_is_exact(dim, dtype):
    dev = _dev()
    w = workloads.custom(4000, 60000, dims=[dim, 8, 4], fanouts=[6, 4], batch=333, n_splits=4, name="gather")
    table = w.feat.to(dtype).to(dev)
    ctx = _ctx(w, dev)
    tg = w.targets(0)
    ctx.gsplit_sample_split(tg.to(dev), 3, 0)
    out = torch.full((ctx.gsplit_max_rows(0), dim), float("nan"), dtype=dtype, device=dev)
    ctx.gsplit_gather_features(table, out)
    ob = _oracle_batch(w, tg, 3, 0)
    ids = ob.local_cat(0)
    as_int = torch.int16 if dtype == torch.bfloat16 else torch.int32
    want = R.gather_rows(table.cpu().view(as_int).numpy(), ids)
    assert np.array_equal(out[:ids.shape[0]].cpu().view(as_int).numpy(), want)
    # an independent library routine agrees as well, and rows past the frontier are untouched
    assert torch.equal(out[:ids.shape[0]], table[torch.from_numpy(ids).long().to(dev)])
    assert torch.isnan(out[ids.shape[0]:].float()).all()
    ctx.close()


def _run_fwd_bwd(w, dev, seed, it, n_splits=None, pmap=None, bf16=False, step=False):
    """One iteration on the device and on the oracle.  The device's backward pass is fed the
    oracle's loss gradient; the oracle's backward pass is conditioned on the device's ReLU
    decisions inside the rounding band (sage_check.conditioned_backward)."""
    from paper_2303_13775_amd import Context, SageParams, GSPLIT_BF16, GSPLIT_F32
    S = n_splits or w.n_splits
    pm = w.pmap if pmap is None else pmap
    ctx = Context(w.indptr.to(dev), w.indices.to(dev), pm.to(dev), S, w.fanouts, w.batch)
    tg = w.targets(it)
    ctx.gsplit_sample_split(tg.to(dev), seed, it)
    table = w.feat.to(torch.bfloat16) if bf16 else w.feat
    x0 = torch.empty((ctx.gsplit_max_rows(0), w.dims[0]), dtype=table.dtype, device=dev)
    ctx.gsplit_gather_features(table.to(dev), x0)
    params = SageParams(w.dims, [t.to(dev) for t in w.w_self], [t.to(dev) for t in w.w_neigh],
                        [t.to(dev) for t in w.bias], dtype=GSPLIT_BF16 if bf16 else GSPLIT_F32)
    logits = torch.empty((tg.numel(), w.dims[-1]), device=dev)
    gws = [torch.full_like(t, 7.0, device=dev) for t in w.w_self]      # must be overwritten
    gwn = [torch.full_like(t, 7.0, device=dev) for t in w.w_neigh]
    gb = [torch.full_like(t, 7.0, device=dev) for t in w.bias]
    row_loss = torch.full((tg.numel(),), 7.0, device=dev)
    if step:        # forward, loss and backward as one call (the device forms the loss gradient itself)
        ctx.gsplit_sage_step(params, x0, w.labels.to(dev), logits, gws, gwn, gb, row_loss)
    else:
        ctx.gsplit_sage_fwd(params, x0, logits)
    ob = _oracle_batch(w, tg, seed, it, n_splits=S, pmap=pm.cpu().numpy())
    op = R.SageParams([t.numpy() for t in w.w_self], [t.numpy() for t in w.w_neigh],
                      [t.numpy() for t in w.bias])
    rows = R.gather_rows(table.float().numpy(), ob.local_cat(0))
    of = R.sp_forward(ob, rows, op, store_bf16=bf16)
    lab = w.labels.numpy()[tg.numpy()[ob.target_perm]]
    loss, g = R.softmax_xent(of.logits, lab)
    if step:
        got_loss = float(row_loss.double().mean()) if tg.numel() else 0.0
        assert abs(got_loss - loss) <= (2e-2 if bf16 else 1e-5) * max(1.0, abs(loss)), ("loss", got_loss, loss)
    else:
        ctx.gsplit_sage_bwd(params, torch.from_numpy(g.astype(np.float32)).to(dev), gws, gwn, gb)
    torch.cuda.synchronize()
    act = SC.device_activations(ctx, w.dims, bf16)
    obw, report = SC.conditioned_backward(ob, of, op, g, act, SC.TAU_BF16_ROUNDED if bf16 else SC.TAU_F32,
                                          store_bf16=bf16, who=w.name)
    res = dict(logits=logits.cpu().numpy(), gws=[t.cpu().numpy() for t in gws],
               gwn=[t.cpu().numpy() for t in gwn], gb=[t.cpu().numpy() for t in gb],
               perm=ob.target_perm, of=of, ob=obw, report=report, batch=ob, act=act, op=op, rows=rows, g=g)
    ctx.close()
    return res


# bf16 path: the tolerance 1e-2 is held against the largest entry of each output (floor 1: max|a - o| /
# max|o|).  Every operand of a bf16 product carries 2^-9 of relative rounding, so an output formed
# from K terms carries an absolute error of the order of 2^-9 * max|o| whatever its own size (and a
# stored activation that sits on a rounding boundary may round the other way on the two sides,
# a whole bf16 step); an entry that cancelled to 1e-2 * max|o| cannot be within 1e-2 of itself.
# The entry-by-entry figure with the fp32 tests' floor (1e-2 * max|o|) is printed beside it.
FLOOR_BF16 = 1.0


def check_sage(r, L, bf16=False, tag=""):
    """Logits and every gradient entry against the oracle, no allowance for ReLU decisions; for bf16
    also against the oracle that rounds only inputs and weights."""
    tol, floor = (TOL_BF16, FLOOR_BF16) if bf16 else (TOL_F32, 1e-2)
    e_log = R.max_rel_err(r["logits"], r["of"].logits, floor)
    errs = SC.grad_errors(r["gws"], r["gwn"], r["gb"], r["ob"], floor)
    print(f"\n[sage {tag}{' bf16, floor 1' if bf16 else ''}] logits {e_log:.1e}; per layer (gw_self, gw_neigh, gbias) "
          f"{SC.fmt(errs)}; ReLU band (entries, decided otherwise by the device, outside) {r['report']}", flush=True)
    # a second floor beside the one the tolerance is stated on: fp32 1e-3 * max|o| (the finer one),
    # bf16 1e-2 * max|o| (the fp32 tests' floor)
    f2 = 1e-2 if bf16 else 1e-3
    e2 = SC.grad_errors(r["gws"], r["gwn"], r["gb"], r["ob"], floor=f2)
    print(f"[sage {tag}] entry by entry with the floor at {f2:g} * max|o|: logits "
          f"{R.max_rel_err(r['logits'], r['of'].logits, f2):.1e}, gradients {SC.fmt(e2)}", flush=True)
    assert e_log < tol, "logits"
    for l in range(L):
        assert max(errs[l]) < tol, ("gradients of layer", l, errs[l])
    if not bf16:
        return
    # the same device results against the plain definition: float64 throughout, only the inputs and
    # the weights are the bfloat16 values the device was given
    ob = r["batch"]
    pq, of = SC.bf16_plain_oracle(ob, r["rows"], r["op"])
    obw, rep = SC.conditioned_backward(ob, of, pq, r["g"], r["act"], SC.TAU_BF16_PLAIN, who=tag + " plain")
    e_log = R.max_rel_err(r["logits"], of.logits, floor)
    errs = SC.grad_errors(r["gws"], r["gwn"], r["gb"], obw, floor)
    e2 = SC.grad_errors(r["gws"], r["gwn"], r["gb"], obw, floor=f2)
    print(f"[sage {tag} bf16 against the oracle that rounds only inputs and weights, floor 1] logits {e_log:.1e}, "
          f"gradients {SC.fmt(errs)}; entry by entry with the floor at {f2:g} * max|o|: logits "
          f"{R.max_rel_err(r['logits'], of.logits, f2):.1e}, gradients {SC.fmt(e2)}; ReLU band {rep}", flush=True)
    assert e_log < tol, "logits against the unrounded oracle"
    for l in range(L):
        assert max(errs[l]) < tol, ("gradients of layer against the unrounded oracle", l, errs[l])


SAGE_CASES = {
    "tiny": lambda: workloads.tiny(),
    "ragged-dims": lambda: workloads.custom(6000, 150000, dims=[100, 72, 47], fanouts=[9, 6], batch=700,
                                            n_splits=4, name="ragged-dims"),
    "odd-width": lambda: workloads.custom(3000, 50000, dims=[30, 33, 10, 3], fanouts=[5, 4, 3], batch=129,
                                          n_splits=3, name="odd"),
    "wide": lambda: workloads.custom(8000, 200000, dims=[128, 256, 256, 172], fanouts=[6, 5, 4], batch=256,
                                     n_splits=4, pmap_kind="range", name="wide"),
}


@pytest.mark.parametrize("name", list(SAGE_CASES))
def test_sage_forward_backward_within_tolerance(name):
    dev = _dev()
    w = SAGE_CASES[name]()
    check_sage(_run_fwd_bwd(w, dev, seed=77, it=2), w.n_layers, tag=name)


# gsplit_sage_step: the top layer as one fused kernel (tiny: 16 classes; ragged-dims: 47 classes, 72 inputs; wide and
# the bf16 run: shapes it does not take, which run the three steps one after the other); several rounds of
# rows per workgroup ("many-targets": 6000 targets over 256 workgroups of 8 rows)
STEP_CASES = dict(SAGE_CASES)
STEP_CASES["many-targets"] = lambda: workloads.custom(20000, 400000, dims=[16, 32, 40], fanouts=[3, 2], batch=6000,
                                                      n_splits=4, name="many-targets")
STEP_CASES["top-width-384"] = lambda: workloads.custom(4000, 80000, dims=[24, 384, 64], fanouts=[4, 3], batch=333,
                                                       n_splits=2, name="top-384")


@pytest.mark.parametrize("name", list(STEP_CASES))
def test_sage_step_within_tolerance(name):
    dev = _dev()
    w = STEP_CASES[name]()
    check_sage(_run_fwd_bwd(w, dev, seed=78, it=3, step=True), w.n_layers, tag=name + " step")
    if name == "tiny":
        check_sage(_run_fwd_bwd(w, dev, seed=78, it=3, step=True, bf16=True), w.n_layers, bf16=True, tag=name + " step")


def test_sage_step_then_backward_needs_a_forward():
    from paper_2303_13775_amd import Context, SageParams, GsplitError
    dev = _dev()
    w = workloads.tiny()
    ctx = _ctx(w, dev)
    ctx.gsplit_sample_split(w.targets(0).to(dev), 1, 0)
    x0 = torch.empty((ctx.gsplit_max_rows(0), w.dims[0]), device=dev)
    ctx.gsplit_gather_features(w.feat.to(dev), x0)
    params = SageParams(w.dims, [t.to(dev) for t in w.w_self], [t.to(dev) for t in w.w_neigh], [t.to(dev) for t in w.bias])
    logits = torch.empty((w.batch, w.dims[-1]), device=dev)
    grads = [[torch.empty_like(t, device=dev) for t in lst] for lst in (w.w_self, w.w_neigh, w.bias)]
    ctx.gsplit_sage_step(params, x0, w.labels.to(dev), logits, *grads)
    with pytest.raises(GsplitError) as e:
        ctx.gsplit_sage_bwd(params, logits, *grads)
    assert e.value.code == -5
    ctx.close()


BF16_CASES = {
    "tiny": lambda: workloads.tiny(),
    "wide": lambda: workloads.custom(8000, 200000, dims=[128, 256, 256, 172], fanouts=[6, 5, 4], batch=256,
                                     n_splits=4, pmap_kind="range", name="wide"),
    "medium-dims": lambda: workloads.custom(30000, 900000, dims=[100, 256, 256, 47], fanouts=[15, 10, 5],
                                            batch=512, n_splits=4, pmap_kind="range", name="mdims"),
    "deep-S8": lambda: workloads.custom(20000, 500000, dims=[128, 256, 256, 256, 172], fanouts=[10, 10, 10, 10],
                                        batch=300, n_splits=8, name="deep"),
    # levels of more than 32768 rows (by their bound) with contractions of 256 and 512: the streaming
    # row-block kernel (weights in registers, rows through LDS) for forward and input-gradient products
    "streamed": lambda: workloads.custom(200000, 3000000, dims=[128, 256, 256, 256, 64], fanouts=[4, 5, 6, 6],
                                         batch=700, n_splits=4, pmap_kind="range", name="streamed"),
    "streamed-512": lambda: workloads.custom(150000, 2500000, dims=[128, 256, 512, 64], fanouts=[5, 10, 10],
                                             batch=3000, n_splits=3, name="streamed512"),
    # output widths that end inside a column block of the streaming kernels (136 = 128 + 8)
    "streamed-ragged-256": lambda: workloads.custom(150000, 2500000, dims=[128, 136, 64], fanouts=[10, 10],
                                                    batch=3000, n_splits=2, name="streamedr256"),
    "streamed-ragged-512": lambda: workloads.custom(150000, 2500000, dims=[128, 256, 136, 64], fanouts=[5, 10, 10],
                                                    batch=3000, n_splits=3, name="streamedr512"),
    # hidden widths that are multiples of 4 but not of 8: dZ stays in float below the top level
    "width-mod-4": lambda: workloads.custom(6000, 150000, dims=[100, 60, 44, 10], fanouts=[8, 6, 4], batch=300,
                                            n_splits=3, name="mod4"),
}


@pytest.mark.parametrize("name", list(BF16_CASES))
def test_sage_bf16_path_within_tolerance(name, monkeypatch):
    """bf16 storage + bf16 MFMA products (float accumulation) against the oracle that rounds the
    same stored values to bf16, and against the one that rounds only inputs and weights."""
    dev = _dev()
    w = BF16_CASES[name]()
    # levels of these sizes stay with the tiled weight-gradient kernel by default (the streaming one takes
    # over from 131072 rows, which the big configurations reach): a lower bar for these cases.  "streamed":
    # level 1 (18017 rows) above the bar, level 2 (7122 rows) below it, so both kernels of the pair of launches
    # work once; "streamed-512": both levels above it (the middle layer has two 256-row blocks of outputs)
    bar = {"streamed": 10000, "streamed-512": 4096, "streamed-ragged-256": 4096, "streamed-ragged-512": 4096}.get(name)
    if bar:
        monkeypatch.setenv("GSPLIT_GRADW_STREAM_ROWS", str(bar))
    r = _run_fwd_bwd(w, dev, seed=31, it=1, bf16=True)
    if bar and w.n_layers >= 3:
        n1, n2 = (r["batch"].local_cat(l).shape[0] for l in (1, 2))
        assert n1 >= bar and (n2 < bar) == (name == "streamed"), (n1, n2, bar)
    check_sage(r, w.n_layers, bf16=True, tag=name)


def test_softmax_xent_matches_oracle():
    dev = _dev()
    w = workloads.custom(6000, 150000, dims=[16, 16, 47], fanouts=[4, 3], batch=333, n_splits=4, name="loss")
    ctx = _ctx(w, dev)
    tg = w.targets(1)
    ctx.gsplit_sample_split(tg.to(dev), 8, 1)
    ob = _oracle_batch(w, tg, 8, 1)
    rng = np.random.default_rng(5)
    logits = (rng.standard_normal((tg.numel(), 47)) * 3).astype(np.float32)
    g = torch.empty((tg.numel(), 47), device=dev)
    rl = torch.empty(tg.numel(), device=dev)
    ctx.gsplit_softmax_xent(torch.from_numpy(logits).to(dev), w.labels.to(dev), g, rl)
    y = w.labels.numpy()[tg.numpy()[ob.target_perm]]
    loss, want = R.softmax_xent(logits.astype(np.float64), y)
    assert R.max_rel_err(g.cpu().numpy(), want) < TOL_F32
    assert abs(float(rl.mean()) - loss) < 1e-5 * max(1.0, abs(loss))
    ctx.close()


def test_split_equals_unsplit_on_gpu():
    dev = _dev()
    w = workloads.tiny()
    a = _run_fwd_bwd(w, dev, seed=5, it=0)
    b = _run_fwd_bwd(w, dev, seed=5, it=0, n_splits=1, pmap=torch.zeros_like(w.pmap))
    la = np.empty_like(a["logits"]); la[a["perm"]] = a["logits"]
    lb = np.empty_like(b["logits"]); lb[b["perm"]] = b["logits"]
    assert R.max_rel_err(la, lb) < TOL_F32
    # each run is within tolerance of its own oracle (conditioned on its own decisions in the band),
    # and the two oracles are one computation when no decision in the band was taken differently
    for r in (a, b):
        check_sage(r, w.n_layers, tag="split-vs-unsplit")
    if all(x[1] == 0 for x in a["report"] + b["report"]):
        for l in range(w.n_layers):
            assert R.max_rel_err(a["gws"][l], b["gws"][l]) < 2 * TOL_F32
            assert R.max_rel_err(a["gwn"][l], b["gwn"][l]) < 2 * TOL_F32


def test_medium_workload_full_size():
    """The benchmark workload at its real size (2.4M vertices, about 131M edges, batch 1024,
    fanouts [15,10,5], 100-256-256-47): every integer output and the fp32 forward/backward
    against the oracle, generated on the GPU and handed to both sides."""
    from paper_2303_13775_amd import Context, SageParams
    dev = _dev()
    w = workloads.medium(device=dev)
    ctx = Context(w.indptr, w.indices, w.pmap, w.n_splits, w.fanouts, w.batch)
    host = dict(indptr=w.indptr.cpu().numpy(), indices=w.indices.cpu().numpy(), pmap=w.pmap.cpu().numpy())
    params = SageParams(w.dims, w.w_self, w.w_neigh, w.bias)
    op = R.SageParams([t.cpu().numpy() for t in w.w_self], [t.cpu().numpy() for t in w.w_neigh],
                      [t.cpu().numpy() for t in w.bias])
    x0 = torch.empty((ctx.gsplit_max_rows(0), w.dims[0]), device=dev)
    logits = torch.empty((w.batch, w.dims[-1]), device=dev)
    glog = torch.empty_like(logits)
    gws = [torch.empty_like(t) for t in w.w_self]
    gwn = [torch.empty_like(t) for t in w.w_neigh]
    gb = [torch.empty_like(t) for t in w.bias]
    for it in (0, 5):
        tg = w.targets(it)
        ctx.gsplit_sample_split(tg, 99, it)
        ob = R.sp_sample(host["indptr"], host["indices"], host["pmap"], w.n_splits, w.fanouts,
                         tg.cpu().numpy(), 99, it)
        assert_batch_equal(ctx.fetch_batch(), ob, w.n_splits, w.n_layers)
        ctx.gsplit_gather_features(w.feat, x0)
        ids = torch.from_numpy(ob.local_cat(0)).long().to(dev)
        assert torch.equal(x0[:ids.numel()], w.feat[ids])
        ctx.gsplit_sage_fwd(params, x0, logits)
        ctx.gsplit_softmax_xent(logits, w.labels, glog)
        ctx.gsplit_sage_bwd(params, glog, gws, gwn, gb)
        of = R.sp_forward(ob, w.feat[ids].cpu().numpy(), op)
        y = w.labels[torch.from_numpy(tg.cpu().numpy()[ob.target_perm]).to(dev).long()].cpu().numpy()
        _, g = R.softmax_xent(of.logits, y)
        act = SC.device_activations(ctx, w.dims, False)
        obw, report = SC.conditioned_backward(ob, of, op, g, act, SC.TAU_F32, who=f"medium it {it}")
        assert R.max_rel_err(logits.cpu().numpy(), of.logits) < TOL_F32
        assert R.max_rel_err(glog.cpu().numpy(), g) < TOL_F32
        errs = SC.grad_errors(gws, gwn, gb, obw)
        print(f"\n[medium it {it}] per layer (gw_self, gw_neigh, gbias) {SC.fmt(errs)}; ReLU band {report}", flush=True)
        for l in range(w.n_layers):
            assert max(errs[l]) < TOL_F32, ("gradients of layer", l, errs[l])
            SC.assert_shuffle_index_equal(ctx, ob, l, has_rev=l >= 1)
        # what the check must catch: 1 % on one entry of the bottom layer's weight gradient, planted
        # in the oracle's result
        bad = obw.gw_self[0].copy()
        idx = np.unravel_index(np.abs(bad).argmax(), bad.shape)
        bad[idx] *= 1.01
        assert R.max_rel_err(gws[0].cpu().numpy(), bad) > 50 * TOL_F32
    ctx.close()


def test_repeatable_across_runs():
    """Race check: integer outputs of three runs of the same batch are identical."""
    dev = _dev()
    w = workloads.tiny()
    ctx = _ctx(w, dev)
    tg = w.targets(7).to(dev)
    ref = None
    for _ in range(3):
        ctx.gsplit_sample_split(tg, 42, 7)
        got = ctx.fetch_batch()
        flat = [t.cpu() for l in got["local_front"] for t in l] + \
               [lay[k].cpu() for lay in got["layers"] for k in ("nbr", "blk_src", "recv")]
        if ref is None:
            ref = flat
        else:
            assert all(torch.equal(x, y) for x, y in zip(ref, flat))
    ctx.close()


HUB_CASES = {
    "tiny": (lambda: workloads.tiny(), False),
    # hubs: a skewed graph without id permutation; the busiest row of a level feeds hundreds of destinations
    # (more than a wave holds: the workgroup path of the backward pull)
    "hubs": (lambda: workloads.custom(20000, 1200000, dims=[32, 64, 64, 16], fanouts=[12, 12, 12], batch=2000, n_splits=4,
                                      abc=(0.7, 0.1, 0.1), permute_ids=False, name="hubs"), False),
    # a row with more entries than the workgroup path sorts at once (two windows): every vertex aggregates from vertex 0
    "huge-hub": (lambda: _star_workload(), True),
}


def _star_workload():
    """20000 vertices; vertex v aggregates from vertex 0 and two more (fewer than any fanout, so every
    destination keeps all three): the row of vertex 0 feeds every destination of a layer."""
    from workloads import synth
    n = 20000
    v = torch.arange(1, n, dtype=torch.int64)
    nb = torch.stack([torch.zeros_like(v), (v * 7 + 1) % n, (v * 13 + 5) % n], 1)
    nb = torch.sort(nb, 1).values
    keep = torch.ones_like(nb, dtype=torch.bool)
    keep[:, 1:] &= nb[:, 1:] != nb[:, :-1]
    keep &= nb != v[:, None]
    rows = [torch.tensor([1, 2, 3])] + [nb[i][keep[i]] for i in range(n - 1)]
    deg = torch.tensor([r.numel() for r in rows])
    indptr = torch.cat([torch.zeros(1, dtype=torch.int64), torch.cumsum(deg, 0)]).to(torch.int32)
    indices = torch.cat(rows).to(torch.int32)
    pmap = synth.pmap_random(n, 2, seed=synth.MASTER_SEED)
    return synth._finish("huge-hub", n, indptr, indices, pmap, 2, [16, 32, 8], [5, 4], 6000, synth.MASTER_SEED, "cpu")


@pytest.mark.parametrize("name", list(HUB_CASES))
@pytest.mark.parametrize("bf16", [False, True])
def test_training_results_are_bit_reproducible(name, bf16):
    """Logits and every gradient of three runs of the same batch are bit-equal (the backward pull
    sums the entries of a reverse-index row in ascending code order, whatever order the atomic
    cursor filled them in), and within tolerance of the oracle; also through gsplit_sage_step."""
    from paper_2303_13775_amd import Context, SageParams, GSPLIT_BF16, GSPLIT_F32
    dev = _dev()
    make, beyond_cap = HUB_CASES[name]
    w = make()
    r = _run_fwd_bwd(w, dev, seed=11, it=4, bf16=bf16)
    check_sage(r, w.n_layers, bf16=bf16, tag=name + " hubs")
    ctx = _ctx(w, dev)
    table = (w.feat.to(torch.bfloat16) if bf16 else w.feat).to(dev)
    params = SageParams(w.dims, [t.to(dev) for t in w.w_self], [t.to(dev) for t in w.w_neigh],
                        [t.to(dev) for t in w.bias], dtype=GSPLIT_BF16 if bf16 else GSPLIT_F32)
    x0 = torch.empty((ctx.gsplit_max_rows(0), w.dims[0]), dtype=table.dtype, device=dev)
    logits = torch.empty((w.batch, w.dims[-1]), device=dev)
    grads = [[torch.empty_like(t, device=dev) for t in lst] for lst in (w.w_self, w.w_neigh, w.bias)]
    labels = w.labels.to(dev)
    runs = []
    for k in range(3):
        ctx.gsplit_sample_split(w.targets(4).to(dev), 11, 4)
        ctx.gsplit_gather_features(table, x0)
        ctx.gsplit_sage_step(params, x0, labels, logits, *grads)
        torch.cuda.synchronize()
        runs.append([logits.clone()] + [t.clone() for lst in grads for t in lst])
    cnt = [ctx.fetch_shuffle(l)["rev_cnt"] for l in range(1, w.n_layers)]
    longest = max(int(c.max()) for c in cnt)
    print(f"\n[reproducible {name}] longest reverse-index row {longest} entries, rows with more than 256 (workgroup path): "
          f"{[int((c > 256).sum()) for c in cnt]}", flush=True)
    if name != "tiny":
        assert longest > 64
    if beyond_cap:      # (taken in windows of ascending values, 4096 codes at a time)
        assert longest > 4096
    for other in runs[1:]:
        for x, y in zip(runs[0], other):
            assert torch.equal(x, y), "results of two runs of the same batch differ in some bit"
    ctx.close()
