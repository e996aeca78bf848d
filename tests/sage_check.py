"""Shared pieces of the GPU parity tests of the GraphSAGE path (not a test module itself).

Gradient checks are elementwise with no allowance: the oracle's backward pass takes the device's
ReLU decisions only where its own float64 pre-activation lies within the forward pass's rounding
band of zero, asserts that the two agree everywhere else, and every gradient entry is then held to
the tolerance (paper Algorithm 2 and the backward description after it)."""
import numpy as np
import torch

from oracle import reference as R

TOL_F32 = 1e-4
TOL_BF16 = 1e-2
# |z| <= tau * max|z| of the layer: where the sign of a pre-activation is not decided by
#   float32 arithmetic against float64 (products of a few hundred terms: 1e-5),
#   bf16 storage against the oracle that rounds the same stored values (an activation on a rounding
#     boundary may round the other way, which moves z by a bf16 step of one term: 1e-3),
#   bf16 storage against the oracle that rounds nothing but inputs and weights (every stored
#     operand carries 2^-9 of relative rounding: 1e-2).
TAU_F32 = 1e-5
TAU_BF16_ROUNDED = 1e-3
TAU_BF16_PLAIN = 1e-2


def device_activations(ctx, dims, bf16):
    """What the forward pass stored for local_cat[1 .. L-1], as float32 numpy arrays (index = level)."""
    L = len(dims) - 1
    dt = torch.bfloat16 if bf16 else torch.float32
    return [None] + [ctx.fetch_sage_activations(l, dims[l], dt).float().cpu().numpy() for l in range(1, L)]


def conditioned_backward(ob, of, op, g, act, rel_tau, store_bf16=False, who=""):
    """Oracle backward pass with the device's ReLU decisions inside the rounding band only.  A
    disagreement outside the band fails the test."""
    masks, report = R.conditioned_relu_masks(ob, of, act, rel_tau)
    for l, (n_band, n_flip, n_bad) in enumerate(report):
        assert n_bad == 0, (f"{who}: layer {l}: {n_bad} ReLU decisions differ from the oracle's although |z| > "
                            f"{rel_tau:g} * max|z|")
    return R.sp_backward(ob, of, op, g, store_bf16=store_bf16, relu_mask=masks), report


def norm_err(a, o):
    """max|a - o| / max|o|"""
    o = np.asarray(o, np.float64)
    return float(np.abs(np.asarray(a, np.float64) - o).max() / max(np.abs(o).max(), 1e-300)) if o.size else 0.0


def grad_errors(gws, gwn, gb, obw, floor=1e-2):
    """Per layer (gw_self, gw_neigh, gbias) elementwise errors max|a - o| / max(|o|, floor * max|o|)."""
    as_np = lambda t: t.cpu().numpy() if hasattr(t, "cpu") else np.asarray(t)
    return [(R.max_rel_err(as_np(gws[l]), obw.gw_self[l], floor), R.max_rel_err(as_np(gwn[l]), obw.gw_neigh[l], floor),
             R.max_rel_err(as_np(gb[l]), obw.gbias[l], floor)) for l in range(len(gws))]


def fmt(errs):
    return "[" + ", ".join("(" + ", ".join(f"{x:.1e}" for x in e) + ")" for e in errs) + "]"


def bf16_plain_oracle(ob, feat_rows_f32, op, labels_or_none=None):
    """The oracle that knows nothing of the device's storage scheme: inputs and weights are the
    bfloat16 values the device is given, everything after that is float64."""
    q = R.to_bf16_rne
    pq = R.SageParams([q(w) for w in op.w_self], [q(w) for w in op.w_neigh], list(op.bias))
    return pq, R.sp_forward(ob, q(np.asarray(feat_rows_f32, np.float32)), pq)


def shuffle_transpose(ob, l):
    """The scatter side of shuffle_idx[l] from the oracle's batch: for every row u of local_cat[l] the
    sorted codes 2 * i (u is destination i's own row) and 2 * i + 1 (u is the source of an edge of
    destination i), destinations numbered over local_cat[l + 1]; plus the composed gather side
    (self_row, edge_row) and the edge number behind every code."""
    self_row, edge_row = [], []
    for b in ob.blocks[l]:
        n_dst = b.dst.shape[0]
        self_row.append(b.shuffle_src_row[:n_dst])
        edge_row.append(b.shuffle_src_row[b.blk_src])
    self_row = np.concatenate(self_row).astype(np.int64)
    edge_row = np.concatenate(edge_row).astype(np.int64)
    cnt = np.concatenate([b.cnt for b in ob.blocks[l]]).astype(np.int64)
    edge_dst = np.repeat(np.arange(cnt.shape[0]), cnt)
    rows = np.concatenate([self_row, edge_row])
    codes = np.concatenate([2 * np.arange(self_row.shape[0]), 2 * edge_dst + 1])
    eids = np.concatenate([np.full(self_row.shape[0], -1, np.int64), np.arange(edge_row.shape[0])])
    order = np.lexsort((codes, rows))
    return self_row, edge_row, rows[order], codes[order], eids[order]


def assert_shuffle_index_equal(ctx, ob, l, has_rev, has_eid=False):
    """Composed gather side and scatter side of shuffle_idx[l], bit for bit (the entries of a row as
    a sorted segment: their order inside a row is not part of the result)."""
    got = ctx.fetch_shuffle(l)
    self_row, edge_row, rows, codes, eids = shuffle_transpose(ob, l)
    assert np.array_equal(got["self_row"].cpu().numpy(), self_row), ("self_row", l)
    assert np.array_equal(got["edge_row"].cpu().numpy(), edge_row), ("edge_row", l)
    if not has_rev:
        assert got["rev_list"] is None, ("unexpected scatter side", l)
        return
    n_lo = ob.local_cat(l).shape[0]
    ptr = got["rev_ptr"].cpu().numpy().astype(np.int64)
    cnt = got["rev_cnt"].cpu().numpy().astype(np.int64)
    lst = got["rev_list"].cpu().numpy().astype(np.int64)
    want_cnt = np.bincount(rows, minlength=n_lo)
    assert np.array_equal(cnt, want_cnt), ("rev_cnt", l)
    # segments tile rev_list without overlap
    order = np.argsort(ptr, kind="stable")
    nz = order[cnt[order] > 0]
    assert np.array_equal(ptr[nz], np.cumsum(cnt[nz]) - cnt[nz]), ("rev_ptr", l)
    # entry e of rev_list belongs to the row whose segment holds it
    seg_row = np.repeat(np.arange(n_lo), cnt)
    start = np.cumsum(cnt) - cnt
    pos = np.repeat(ptr, cnt) + (np.arange(int(cnt.sum())) - np.repeat(start, cnt))
    got_codes = lst[pos]
    o = np.lexsort((got_codes, seg_row))
    assert np.array_equal(seg_row[o], rows) and np.array_equal(got_codes[o], codes), ("rev_list", l)
    if has_eid:
        eid = got["rev_eid"].cpu().numpy().astype(np.int64)[pos]
        assert np.array_equal(eid[o], eids), ("rev_eid", l)
    else:
        assert got["rev_eid"] is None
