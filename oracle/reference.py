"""CPU ORACLE (test infrastructure only) -- Python side.

Drives the plain C steps of `gsplit_oracle.c` in the order of the paper's Algorithm 1
(`sp_sample`) and Algorithm 2 (`sp_forward`) and the backward description that follows it, for
all S splits in lock-step (each split plays the role of one GPU of the paper; the all-to-all
shuffles become list concatenations).  Dense products are numpy float64 matmuls.

Nothing in the product path may import this module.  It shares no code with the HIP library.

Readings of the paper that this file fixes (the paper is silent on them):
  * fanouts[l] is used when layer l+1 is expanded into layer l (l is Algorithm 1's loop variable).
  * neighbours are taken without replacement; a vertex with degree <= fanout keeps all of them.
  * a vertex of local_front[l+1] is also a member of layer l (its own lower-layer row feeds the
    GraphSAGE self term), so both the next local frontier and every mixed frontier start with the
    destination vertices themselves ("the next layer is the union of the new local frontier and
    the previous mixed frontier", section 3).
  * local numbering everywhere = order of first occurrence; what a split hands to owner t is the
    sampled part of its (already duplicate-free) mixed frontier that t owns, in mixed-frontier
    order; received buckets are concatenated by sending split.
  * GraphSAGE layer: relu(H_dst W_self + mean(H_nbr) W_neigh + b), no activation on the last layer,
    mean of an empty neighbourhood = 0.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gsplit_oracle.c")
_LIB = os.path.join(_HERE, "libgsplit_oracle.so")


def build_oracle(force: bool = False) -> str:
    """Compile the C steps with gcc (-O2, no OpenMP, no fast-math)."""
    if force or (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None

_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build_oracle())
        L.gso_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        L.gso_philox4x32_10.restype = None
        L.gso_philox_word.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
        L.gso_philox_word.restype = C.c_uint32
        L.gso_floyd_select.argtypes = [C.c_int64, C.c_int32, _u32p, _i64p]
        L.gso_floyd_select.restype = None
        L.gso_sample_layer.argtypes = [_i64p, _i32p, _i32p, C.c_int64, C.c_int32, C.c_uint32,
                                       C.c_uint64, C.c_uint64, _i32p, _i32p, C.c_void_p]
        L.gso_sample_layer.restype = None
        L.gso_slot_stream.argtypes = [_i32p, _i32p, C.c_int64, C.c_int32, _i32p]
        L.gso_slot_stream.restype = C.c_int64
        L.gso_split_buckets.argtypes = [_i32p, C.c_int64, _u8p, C.c_int32, _i32p, _i64p]
        L.gso_split_buckets.restype = None
        L.gso_unique_first.argtypes = [_i32p, C.c_int64, _i32p, _i32p, C.c_void_p]
        L.gso_unique_first.restype = C.c_int64
        L.gso_positions_in.argtypes = [_i32p, C.c_int64, _i32p, C.c_int64, _i32p, _i32p]
        L.gso_positions_in.restype = None
        L.gso_gather_rows.argtypes = [C.c_void_p, C.c_int64, C.c_int64, _i32p, C.c_int64, C.c_void_p]
        L.gso_gather_rows.restype = None
        L.gso_mean_aggregate.argtypes = [C.c_int64, C.c_int64, _i64p, _i32p, _f64p, _f64p]
        L.gso_mean_aggregate.restype = None
        L.gso_mean_aggregate_adjoint.argtypes = [C.c_int64, C.c_int64, _i64p, _i32p, _f64p, _f64p]
        L.gso_mean_aggregate_adjoint.restype = None
        L.gso_rows_take.argtypes = [_f64p, C.c_int64, _i32p, C.c_int64, _f64p]
        L.gso_rows_take.restype = None
        L.gso_rows_add_into.argtypes = [_f64p, C.c_int64, _i32p, C.c_int64, _f64p]
        L.gso_rows_add_into.restype = None
        _lib = L
    return _lib


# --------------------------------------------------------------------------------------------
# thin wrappers, one per C step
# --------------------------------------------------------------------------------------------
def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> np.ndarray:
    out = np.zeros(4, np.uint32)
    lib().gso_philox4x32_10(np.asarray(ctr, np.uint32), np.asarray(key, np.uint32), out)
    return out


def philox_word(seed: int, it: int, layer: int, v: int, draw: int) -> int:
    return int(lib().gso_philox_word(seed, it, layer, v, draw))


def floyd_select(d: int, k: int, words: np.ndarray) -> np.ndarray:
    assert 0 < k < d
    chosen = np.zeros(k, np.int64)
    lib().gso_floyd_select(d, k, np.ascontiguousarray(words, np.uint32), chosen)
    return chosen


def sample_layer(indptr64, indices, frontier, fan, layer, seed, it, want_edge_pos=False):
    frontier = np.ascontiguousarray(frontier, np.int32)
    n = frontier.shape[0]
    nbr = np.empty(n * fan, np.int32)
    cnt = np.empty(n, np.int32)
    epos = np.empty(n * fan, np.int64) if want_edge_pos else None
    lib().gso_sample_layer(indptr64, indices, frontier, n, fan, layer, seed, it, nbr, cnt,
                           epos.ctypes.data if want_edge_pos else None)
    if want_edge_pos:
        return nbr.reshape(n, fan), cnt, epos.reshape(n, fan)
    return nbr.reshape(n, fan), cnt


def slot_stream(nbr, cnt):
    n, fan = nbr.shape
    sigma = np.empty(n * fan, np.int32)
    m = lib().gso_slot_stream(np.ascontiguousarray(nbr).reshape(-1), cnt, n, fan, sigma)
    return sigma[:m].copy()


def split_buckets(sigma, pmap, n_splits):
    out = np.empty(sigma.shape[0], np.int32)
    off = np.zeros(n_splits + 1, np.int64)
    lib().gso_split_buckets(sigma, sigma.shape[0], pmap, n_splits, out, off)
    return [out[off[t]:off[t + 1]].copy() for t in range(n_splits)]


class _Scratch:
    """The n_vertices-sized 'where' array the dedup steps need, kept at -1 between calls."""

    def __init__(self, n_vertices: int):
        self.where = np.full(n_vertices, -1, np.int32)


def unique_first(seq, scratch: _Scratch, want_local: bool = False):
    seq = np.ascontiguousarray(seq, np.int32)
    uniq = np.empty(seq.shape[0], np.int32)
    local = np.empty(seq.shape[0], np.int32) if want_local else None
    m = lib().gso_unique_first(seq, seq.shape[0], scratch.where, uniq,
                               local.ctypes.data if want_local else None)
    return (uniq[:m].copy(), local) if want_local else uniq[:m].copy()


def positions_in(lst, ids, scratch: _Scratch):
    pos = np.empty(ids.shape[0], np.int32)
    lib().gso_positions_in(np.ascontiguousarray(lst, np.int32), lst.shape[0],
                           np.ascontiguousarray(ids, np.int32), ids.shape[0], scratch.where, pos)
    return pos


def gather_rows(table: np.ndarray, ids: np.ndarray) -> np.ndarray:
    """Loading step: table[ids] as a byte copy (any dtype, row-major, contiguous rows)."""
    assert table.ndim == 2 and table.strides[1] == table.itemsize
    ids = np.ascontiguousarray(ids, np.int32)
    out = np.empty((ids.shape[0], table.shape[1]), table.dtype)
    lib().gso_gather_rows(table.ctypes.data, table.strides[0], table.shape[1] * table.itemsize,
                          ids, ids.shape[0], out.ctypes.data)
    return out


def mean_aggregate(blk_indptr, blk_src, H):
    n_dst = blk_indptr.shape[0] - 1
    M = np.empty((n_dst, H.shape[1]), np.float64)
    lib().gso_mean_aggregate(n_dst, H.shape[1], blk_indptr, blk_src, np.ascontiguousarray(H), M)
    return M


def mean_aggregate_adjoint(blk_indptr, blk_src, dM, n_src):
    dH = np.zeros((n_src, dM.shape[1]), np.float64)
    lib().gso_mean_aggregate_adjoint(blk_indptr.shape[0] - 1, dM.shape[1], blk_indptr, blk_src,
                                     np.ascontiguousarray(dM), dH)
    return dH


def rows_take(src, rows):
    out = np.empty((rows.shape[0], src.shape[1]), np.float64)
    lib().gso_rows_take(np.ascontiguousarray(src), src.shape[1], rows, rows.shape[0], out)
    return out


def rows_add_into(dst, rows, src):
    lib().gso_rows_add_into(dst, dst.shape[1], rows, rows.shape[0], np.ascontiguousarray(src))


# --------------------------------------------------------------------------------------------
# Algorithm 1: split-parallel sampling
# --------------------------------------------------------------------------------------------
@dataclass
class Block:
    """What split s holds for sampling layer l: edges[l] in local ids plus shuffle_idx[l]."""
    dst: np.ndarray               # local_front[l+1]_s, global ids (n_dst)
    nbr: np.ndarray               # [n_dst, fan] sampled global ids, -1 padded
    cnt: np.ndarray               # [n_dst]
    buckets: List[np.ndarray]     # bucket[s->t], t = 0..S-1: sampled part of mixed_front owned by t
    mixed_front: np.ndarray       # global ids; first n_dst entries are dst
    blk_indptr: np.ndarray        # int64 [n_dst+1]
    blk_src: np.ndarray           # int32 [nnz] rows of mixed_front
    shuffle_src_row: np.ndarray   # int32 [n_src] row of local_cat[l] holding each mixed vertex


@dataclass
class Batch:
    n_splits: int
    n_layers: int
    local_front: List[List[np.ndarray]]      # [l][s], l = 0..L
    blocks: List[List[Block]]                # [l][s], l = 0..L-1
    target_perm: np.ndarray                  # row r of local_cat[L] is targets[target_perm[r]]

    def local_cat(self, l: int) -> np.ndarray:
        return np.concatenate(self.local_front[l]) if self.n_splits else np.empty(0, np.int32)

    def local_off(self, l: int) -> np.ndarray:
        return np.concatenate([[0], np.cumsum([f.shape[0] for f in self.local_front[l]])]).astype(np.int64)


def as_int64_indptr(indptr) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(indptr), np.int64)


def sp_sample(indptr, indices, pmap, n_splits: int, fanouts: Sequence[int], targets, seed: int,
              it: int) -> Batch:
    """Algorithm 1 executed by all splits in lock-step.  Targets must be distinct."""
    indptr64 = as_int64_indptr(indptr)
    indices = np.ascontiguousarray(np.asarray(indices), np.int32)
    pmap = np.ascontiguousarray(np.asarray(pmap), np.uint8)
    targets = np.ascontiguousarray(np.asarray(targets), np.int32)
    n_vertices = indptr64.shape[0] - 1
    S, L = n_splits, len(fanouts)
    assert np.unique(targets).shape[0] == targets.shape[0], "targets must be distinct"
    scratch = _Scratch(n_vertices)

    local_front: List[Optional[List[np.ndarray]]] = [None] * (L + 1)
    blocks: List[Optional[List[Block]]] = [None] * L
    owner_of_target = pmap[targets]
    # local_front[L] = local_targets: the targets each split owns, in the caller's order
    local_front[L] = [targets[owner_of_target == s] for s in range(S)]
    target_perm = np.concatenate([np.nonzero(owner_of_target == s)[0] for s in range(S)]).astype(np.int64) \
        if S else np.empty(0, np.int64)

    for l in range(L - 1, -1, -1):
        fan = int(fanouts[l])
        partial = []
        for s in range(S):
            dst = local_front[l + 1][s]
            n_dst = dst.shape[0]
            # mixed_front, edges[l] = sample_layer(local_front[l+1]): the mixed frontier is the
            # SET of vertices the layer needs (destination vertices first, then sampled ones in
            # order of first appearance); edges[l] point at its rows
            nbr, cnt = sample_layer(indptr64, indices, dst, fan, l, seed, it)
            sigma = slot_stream(nbr, cnt)
            mixed, local_ids = unique_first(np.concatenate([dst, sigma]), scratch, want_local=True)
            blk_src = np.ascontiguousarray(local_ids[n_dst:], np.int32)
            blk_indptr = np.concatenate([[0], np.cumsum(cnt, dtype=np.int64)]).astype(np.int64)
            # split(): owner lookup through f_G for the sampled part of the mixed frontier, one
            # stable bucket per owner (bucket[s->s] is the local part, the others are remote)
            buckets = split_buckets(np.ascontiguousarray(mixed[n_dst:]), pmap, S)
            partial.append((dst, nbr, cnt, buckets, mixed, blk_indptr, blk_src))
        # the sampling shuffle: split t receives bucket[s->t] from every s, in order of s
        recv = [np.concatenate([partial[s][3][t] for s in range(S)]) for t in range(S)]
        # new local frontier: own destination vertices first, then what arrived
        local_front[l] = [unique_first(np.concatenate([local_front[l + 1][t], recv[t]]), scratch)
                          for t in range(S)]
        off = np.concatenate([[0], np.cumsum([f.shape[0] for f in local_front[l]])])
        blocks[l] = []
        for s in range(S):
            dst, nbr, cnt, buckets, mixed, blk_indptr, blk_src = partial[s]
            # shuffle index: where each mixed-frontier vertex lives in the owners' local frontiers
            src_row = np.empty(mixed.shape[0], np.int32)
            own = pmap[mixed]
            for t in range(S):
                sel = np.nonzero(own == t)[0]
                if sel.shape[0]:
                    p = positions_in(local_front[l][t], mixed[sel], scratch)
                    assert (p >= 0).all()
                    src_row[sel] = p + off[t]
            blocks[l].append(Block(dst, nbr, cnt, buckets, mixed, blk_indptr, blk_src, src_row))
    return Batch(S, L, local_front, blocks, target_perm)


# --------------------------------------------------------------------------------------------
# split-quality figures defined in the paper's splitting-algorithm evaluation
# --------------------------------------------------------------------------------------------
def split_quality(batch: Batch, pmap) -> dict:
    """workload imbalance = max over splits of #edges at layers l > 0, divided by the average;
    communication cost = cross-split edges / all edges of the mini-batch."""
    pmap = np.asarray(pmap)
    S = batch.n_splits
    per_split = np.zeros(S, np.int64)
    cross = total = sent = 0
    for l in range(batch.n_layers):
        for s in range(S):
            b = batch.blocks[l][s]
            n_e = int(b.blk_indptr[-1])
            total += n_e
            if l > 0:
                per_split[s] += n_e
            cross += int((pmap[b.mixed_front[b.blk_src]] != s).sum())
            sent += int(sum(b.buckets[t].shape[0] for t in range(S) if t != s))
    imb = float(per_split.max() / per_split.mean()) if per_split.sum() else 1.0
    return {"workload_imbalance": imb, "cross_edge_fraction": cross / max(total, 1),
            "edges": total, "ids_shuffled": sent}


def batch_stats(batch: Batch, pmap):
    """Per sampling layer and split: the edges the split computes and how many of them are cross
    edges (source vertex owned by another split).  The two figures of the paper's partitioning
    evaluation (section 7.3) follow from them: workload imbalance = max over splits of the edges
    at layers l > 0 divided by their average; communication cost = cross edges / all edges."""
    pmap = np.asarray(pmap)
    L, S = batch.n_layers, batch.n_splits
    edges = np.zeros((L, S), np.int64)
    cross = np.zeros((L, S), np.int64)
    for l in range(L):
        for s in range(S):
            b = batch.blocks[l][s]
            for i in range(b.dst.shape[0]):
                for q in range(int(b.cnt[i])):
                    edges[l, s] += 1
                    if pmap[b.nbr[i, q]] != s:
                        cross[l, s] += 1
    return edges, cross


def quality_from_stats(edges: np.ndarray, cross: np.ndarray) -> dict:
    upper = edges[1:].sum(0) if edges.shape[0] > 1 else np.zeros(edges.shape[1], np.int64)
    imb = float(upper.max() / upper.mean()) if upper.sum() else 1.0
    return {"workload_imbalance": imb, "cross_edge_fraction": float(cross.sum()) / max(int(edges.sum()), 1)}


# --------------------------------------------------------------------------------------------
# data-parallel micro-batches (paper section 2, "Redundant loading and computation", Table 1)
# --------------------------------------------------------------------------------------------
def micro_batches(indptr, indices, fanouts: Sequence[int], targets, n_micro: int, seed: int, it: int):
    """The mini-batch's targets dealt to n_micro micro-batches by position (equal contiguous parts,
    the remainder to the first ones), each sampled on its own as data-parallel training does:
    one split, no partition map, and its own random stream (iteration counter it * n_micro + m)."""
    targets = np.asarray(targets, np.int32)
    n_vertices = len(indptr) - 1
    pm = np.zeros(n_vertices, np.uint8)
    base, rem = divmod(targets.shape[0], n_micro)
    out, pos = [], 0
    for m in range(n_micro):
        n = base + (1 if m < rem else 0)
        out.append(sp_sample(indptr, indices, pm, 1, fanouts, targets[pos:pos + n], seed, it * n_micro + m))
        pos += n
    return out


def redundancy_counts(mini: Batch, micro: Sequence[Batch]) -> dict:
    """Table 1's two columns for one iteration: edges computed (all sampling layers) and feature
    rows loaded (input layer), for the micro-batches together and for the one mini-batch."""
    def edges_of(b):
        return sum(int(blk.blk_indptr[-1]) for layer in b.blocks for blk in layer)
    def feats_of(b):
        return int(b.local_cat(0).shape[0])
    return {"edges_micro": sum(edges_of(b) for b in micro), "edges_mini": edges_of(mini),
            "features_micro": sum(feats_of(b) for b in micro), "features_mini": feats_of(mini)}


# --------------------------------------------------------------------------------------------
# Algorithm 2 (forward) and the backward pass
# --------------------------------------------------------------------------------------------
def to_bf16_rne(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (round to nearest, ties to even); result kept as float32."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(np.shape(x))


@dataclass
class SageParams:
    w_self: List[np.ndarray]     # [D_l, D_{l+1}]
    w_neigh: List[np.ndarray]
    bias: List[np.ndarray]


@dataclass
class Forward:
    logits: np.ndarray                         # [n_targets, D_L], rows in local_cat[L] order
    hidden: List[np.ndarray]                   # local_cat activations per layer 0..L
    mixed: List[List[np.ndarray]] = field(default_factory=list)   # [l][s]
    mean: List[List[np.ndarray]] = field(default_factory=list)    # [l][s]
    z: List[List[np.ndarray]] = field(default_factory=list)       # [l][s] pre-activation


def sp_forward(batch: Batch, feat_local_cat: np.ndarray, params: SageParams,
               store_bf16: bool = False) -> Forward:
    """Algorithm 2, bottom-up.  feat_local_cat = input features of local_cat[0] rows.

    With store_bf16 every value the device holds in bfloat16 (features, weights, activations
    between layers, and the neighbourhood mean that enters the matrix product) is first rounded to
    bfloat16; the arithmetic itself stays in float64."""
    S, L = batch.n_splits, batch.n_layers
    q = (lambda a: to_bf16_rne(np.asarray(a, np.float32)).astype(np.float64)) if store_bf16 \
        else (lambda a: np.asarray(a, np.float64))
    hidden = [q(feat_local_cat)]
    out = Forward(None, hidden)
    for l in range(L):
        Ws, Wn, b = q(params.w_self[l]), q(params.w_neigh[l]), np.asarray(params.bias[l], np.float64)
        parts, mixed_l, mean_l, z_l = [], [], [], []
        for s in range(S):
            blk = batch.blocks[l][s]
            n_dst = blk.dst.shape[0]
            # mixed_hidden = shuffle(shuffle_idx[l], local_hidden)
            mixed = rows_take(hidden[l], blk.shuffle_src_row)
            # local_hidden = gnn_layer(edges[l], mixed_hidden)
            M = mean_aggregate(blk.blk_indptr, blk.blk_src, mixed)
            if store_bf16:          # the mean is an operand of the bf16 matrix product: stored rounded
                M = q(M)
            Z = mixed[:n_dst] @ Ws + M @ Wn + b
            H = Z if l == L - 1 else np.maximum(Z, 0.0)
            parts.append(H)
            mixed_l.append(mixed); mean_l.append(M); z_l.append(Z)
        nxt = np.concatenate(parts, 0) if parts else np.zeros((0, params.w_self[l].shape[1]))
        if store_bf16 and l < L - 1:
            nxt = q(nxt)
        hidden.append(nxt)
        out.mixed.append(mixed_l); out.mean.append(mean_l); out.z.append(z_l)
    out.logits = hidden[L]
    return out


@dataclass
class Backward:
    gw_self: List[np.ndarray]
    gw_neigh: List[np.ndarray]
    gbias: List[np.ndarray]
    ghidden: List[Optional[np.ndarray]]   # d loss / d local_cat[l] for l >= 1 (None for l = 0)


def sp_backward(batch: Batch, fwd: Forward, params: SageParams, grad_logits: np.ndarray,
                store_bf16: bool = False, relu_mask=None) -> Backward:
    """Top layer down.  Gradients of remote rows travel back through the same shuffle index,
    reversed; weight gradients are summed over splits (the gradient aggregation step).  No
    gradient is formed for the input features.

    relu_mask (optional): relu_mask[l][s], a boolean array like fwd.z[l][s], replaces [z > 0] of
    layer l (see conditioned_relu_masks); None keeps this pass's own decisions."""
    S, L = batch.n_splits, batch.n_layers
    q = (lambda a: to_bf16_rne(np.asarray(a, np.float32)).astype(np.float64)) if store_bf16 \
        else (lambda a: np.asarray(a, np.float64))
    gws = [np.zeros(w.shape, np.float64) for w in params.w_self]
    gwn = [np.zeros(w.shape, np.float64) for w in params.w_neigh]
    gb = [np.zeros(b.shape, np.float64) for b in params.bias]
    ghid: List[Optional[np.ndarray]] = [None] * (L + 1)
    ghid[L] = np.asarray(grad_logits, np.float64)
    for l in range(L - 1, -1, -1):
        Ws, Wn = q(params.w_self[l]), q(params.w_neigh[l])
        off = batch.local_off(l + 1)
        if l > 0:
            ghid[l] = np.zeros(fwd.hidden[l].shape, np.float64)
        for s in range(S):
            blk = batch.blocks[l][s]
            n_dst = blk.dst.shape[0]
            dH = ghid[l + 1][off[s]:off[s + 1]]
            if l == L - 1:
                dZ = dH
            else:
                dZ = dH * (fwd.z[l][s] > 0.0 if relu_mask is None else relu_mask[l][s])
            mixed, M = fwd.mixed[l][s], fwd.mean[l][s]
            # with bf16 storage every matrix product takes bf16 operands, so dZ enters the
            # weight-gradient and the input-gradient products rounded like the other operands
            # (the bias gradient is the product of dZ with a column of ones)
            dZq = q(dZ) if store_bf16 else dZ
            gws[l] += mixed[:n_dst].T @ dZq
            gwn[l] += M.T @ dZq
            gb[l] += dZq.sum(0)
            if l > 0:
                dmixed = mean_aggregate_adjoint(blk.blk_indptr, blk.blk_src, dZq @ Wn.T,
                                                mixed.shape[0])
                dmixed[:n_dst] += dZq @ Ws.T
                rows_add_into(ghid[l], blk.shuffle_src_row, dmixed)
    return Backward(gws, gwn, gb, ghid)


def conditioned_relu_masks(batch: Batch, fwd: Forward, device_act: Sequence[Optional[np.ndarray]],
                           rel_tau: float):
    """ReLU decisions for a backward pass that is compared with a device's, conditioned on the
    decisions the device took where the sign of a pre-activation is below the forward pass's
    rounding noise.

    The backward pass multiplies by [z > 0].  This oracle forms z in float64, a device in float32
    (or from bfloat16 operands): where |z| <= rel_tau * max|z| of the layer the two may legitimately
    land on different sides of zero, and one flipped decision moves a whole gradient row.  There
    the device's own decision is taken (device_act[l + 1] > 0: the activations it stored for
    local_cat[l + 1], rows in the order of that level); everywhere else the oracle's.  A
    disagreement outside the band is a wrong result on the device and is counted, not excused.

    Returns (masks, report): masks[l][s] a boolean array like fwd.z[l][s] for l < L - 1 (None for the
    last layer, which has no activation); report = per layer (entries in the band, of which the
    device decided the other way, disagreements outside the band)."""
    S, L = batch.n_splits, batch.n_layers
    masks: List[Optional[List[np.ndarray]]] = [None] * L
    report = []
    for l in range(L - 1):
        off = batch.local_off(l + 1)
        zmax = max([float(np.abs(z).max()) if z.size else 0.0 for z in fwd.z[l]] + [0.0])
        act = np.asarray(device_act[l + 1])
        assert act.shape[0] == off[-1], "device activations do not match the level's row count"
        masks[l] = []
        n_band = n_flip = n_bad = 0
        for s in range(S):
            z = fwd.z[l][s]
            own = z > 0.0
            dev = act[off[s]:off[s + 1]] > 0
            band = np.abs(z) <= rel_tau * zmax
            n_band += int(band.sum())
            n_flip += int((band & (own != dev)).sum())
            n_bad += int((~band & (own != dev)).sum())
            masks[l].append(np.where(band, dev, own))
        report.append((n_band, n_flip, n_bad))
    return masks, report


def softmax_xent(logits: np.ndarray, labels: np.ndarray):
    """Mean softmax cross-entropy and its gradient w.r.t. the logits (the harness-side loss)."""
    z = logits - logits.max(1, keepdims=True)
    p = np.exp(z)
    p /= p.sum(1, keepdims=True)
    n = logits.shape[0]
    loss = -np.log(p[np.arange(n), labels]).mean() if n else 0.0
    g = p.copy()
    g[np.arange(n), labels] -= 1.0
    return float(loss), g / max(n, 1)


def max_rel_err(a: np.ndarray, o: np.ndarray, floor: float = 1e-2) -> float:
    """max_i |a_i - o_i| / max(|o_i|, floor * max|o|): the tolerance measure used by the tests.

    The floor keeps entries that are small only because large terms cancelled (every output is a
    sum of hundreds of products of size about max|o|) from being judged against their own size,
    which no fixed-precision arithmetic can meet: an fp32 dot product of length K carries an
    absolute error of roughly sqrt(K) * 2^-24 * (size of its terms), whatever the size of the sum."""
    a = np.asarray(a, np.float64); o = np.asarray(o, np.float64)
    if o.size == 0:
        return 0.0
    scale = np.maximum(np.abs(o), floor * np.abs(o).max())
    scale = np.where(scale == 0, 1.0, scale)
    return float((np.abs(a - o) / scale).max())


# ---------------------------------------------------------------------------------------------
# Offline pre-sampling (section 4, "pre-sampling stage" and the analysis after Eq. 2)
# ---------------------------------------------------------------------------------------------
def presample_counts(indptr, indices, fanouts, batches, seed, iters):
    """Runs the training sampler (the whole mini-batch, no splitting) on every batch and counts
    k_v = number of (sample, layer l > 0) pairs in which vertex v appears (layers are the levels of
    Algorithm 1: level L holds the targets, level 0 the input layer, which does not count) and
    k_e = number of times CSR edge e is sampled, over all samples and layers.  The weights of the
    weighted graph G_w are w_V = k_v / N and w_E = k_e / N with N = len(batches)."""
    indptr64 = np.ascontiguousarray(indptr, np.int64)
    indices = np.ascontiguousarray(indices, np.int32)
    n_vertices, L = indptr64.shape[0] - 1, len(fanouts)
    k_v = np.zeros(n_vertices, np.int64)
    k_e = np.zeros(indices.shape[0], np.int64)
    scratch = _Scratch(n_vertices)
    for targets, it in zip(batches, iters):
        front = np.ascontiguousarray(targets, np.int32)          # level L (distinct ids)
        k_v[front] += 1
        for l in range(L - 1, -1, -1):
            nbr, cnt, epos = sample_layer(indptr64, indices, front, fanouts[l], l, seed, it, want_edge_pos=True)
            np.add.at(k_e, epos[epos >= 0], 1)
            front = unique_first(np.concatenate([front, slot_stream(nbr, cnt)]), scratch)   # level l
            if l > 0:
                k_v[front] += 1
    return k_v, k_e


def presample_weights(k_v, k_e, n_samples):
    """w_V(v) = k_v / N, w_E(e) = k_e / N."""
    return k_v.astype(np.float64) / n_samples, k_e.astype(np.float64) / n_samples


# --------------------------------------------------------------------------------------------
# partial feature cache aligned with f_G and the host-memory miss path (sections 3, 4 and 7.1)
# --------------------------------------------------------------------------------------------
def input_counts(indptr, indices, fanouts, batches, seed, iters):
    """k_in[v] = number of samples whose input layer (level 0) holds v: the sampling-frequency
    criterion by which input features are ranked for caching (section 7.1).  Same unsplit sampler as
    presample_counts."""
    indptr64 = np.ascontiguousarray(indptr, np.int64)
    indices = np.ascontiguousarray(indices, np.int32)
    n_vertices, L = indptr64.shape[0] - 1, len(fanouts)
    k_in = np.zeros(n_vertices, np.int64)
    scratch = _Scratch(n_vertices)
    for targets, it in zip(batches, iters):
        front = np.ascontiguousarray(targets, np.int32)
        for l in range(L - 1, -1, -1):
            nbr, cnt = sample_layer(indptr64, indices, front, fanouts[l], l, seed, it)[:2]
            front = unique_first(np.concatenate([front, slot_stream(nbr, cnt)]), scratch)
        k_in[front] += 1
    return k_in


def cache_select(k_in, pmap, n_splits: int, capacity: Sequence[int]):
    """Static cache content: split s caches the capacity[s] most frequently sampled vertices among
    those f_G assigns to it (f_G also decides where a vertex's input features are cached, section
    4, so that caches are consistent with the splits); ties go to the smaller id; a vertex that
    was never sampled is not cached.  Returns one id array per split, hottest first."""
    k_in = np.asarray(k_in, np.int64)
    pmap = np.asarray(pmap)
    out = []
    for s in range(n_splits):
        own = np.nonzero((pmap == s) & (k_in > 0))[0]
        order = sorted(own.tolist(), key=lambda v: (-int(k_in[v]), v))
        out.append(np.asarray(order[:int(capacity[s])], np.int32))
    return out


def cached_gather(host_table: np.ndarray, cache_ids, cache_rows, batch: Batch):
    """Loading step with a cache: a row of split s's input layer comes from s's cache if s cached
    that vertex, otherwise from the host table.  Returns the gathered rows (splits concatenated)
    and the hits and misses per split."""
    S = batch.n_splits
    hits, misses = np.zeros(S, np.int64), np.zeros(S, np.int64)
    parts = []
    for s in range(S):
        where = {int(v): j for j, v in enumerate(cache_ids[s])}
        ids = batch.local_front[0][s]
        rows = np.empty((ids.shape[0], host_table.shape[1]), host_table.dtype)
        for r, v in enumerate(ids):
            j = where.get(int(v))
            if j is None:
                rows[r] = host_table[v]
                misses[s] += 1
            else:
                rows[r] = cache_rows[s][j]
                hits[s] += 1
        parts.append(rows)
    out = np.concatenate(parts, 0) if parts else np.zeros((0, host_table.shape[1]), host_table.dtype)
    return out, hits, misses
