"""Plain CPU reference of the GAT layer on the split mini-batch (test infrastructure only: used by
tests/, __graft_entry__.smoke() and bench.py's cpu_baseline; the product never imports it).

The paper evaluates GAT as its second model (section 7.1) and cites Velickovic et al. (ICLR 2018)
for it without restating the formula; Algorithm 2 fixes how a layer runs on a split:
`mixed_hidden = shuffle(shuffle_idx[l], local_hidden)`, then `gnn_layer(edges[l], mixed_hidden)`.
The layer taken here is the cited one:

    z_j      = h_j W                                   (per head k: z_j^k, F features)
    e_ij^k   = LeakyReLU_0.2( a_dst^k . z_i^k + a_src^k . z_j^k )
    alpha_ij = softmax over j in N(i) of e_ij,          N(i) = {i} + the sampled neighbours of i
    out_i^k  = sum_j alpha_ij^k z_j^k
    hidden layers : h'_i = ELU( concat_k out_i^k + b )
    last layer    : logits_i = mean_k out_i^k + b

All arithmetic in float64, one split after the other, every step a loop or a numpy primitive."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from .reference import Batch, rows_take, rows_add_into

NEG_SLOPE = 0.2


@dataclass
class GatParams:
    heads: List[int]             # heads of layer l
    w: List[np.ndarray]          # [D_l, heads_l * F_l]
    a_src: List[np.ndarray]      # [heads_l * F_l]
    a_dst: List[np.ndarray]      # [heads_l * F_l]
    bias: List[np.ndarray]       # [heads_l * F_l] (hidden layers, concatenated heads) or [F_L] (last layer)


@dataclass
class GatForward:
    logits: np.ndarray
    hidden: List[np.ndarray]                                   # local_cat activations per level
    mixed: List[List[np.ndarray]] = field(default_factory=list)    # [l][s] shuffled inputs
    z: List[List[np.ndarray]] = field(default_factory=list)        # [l][s] transformed mixed rows [n, K, F]
    alpha: List[List[list]] = field(default_factory=list)          # [l][s][i] -> [1 + cnt_i, K]
    pre: List[List[np.ndarray]] = field(default_factory=list)      # [l][s] value before the activation


def _leaky(x):
    return np.where(x > 0.0, x, NEG_SLOPE * x)


def _elu(x):
    return np.where(x > 0.0, x, np.expm1(np.minimum(x, 0.0)))


def gat_forward(batch: Batch, feat_local_cat: np.ndarray, params: GatParams) -> GatForward:
    S, L = batch.n_splits, batch.n_layers
    hidden = [np.asarray(feat_local_cat, np.float64)]
    out = GatForward(None, hidden)
    for l in range(L):
        K = params.heads[l]
        W = np.asarray(params.w[l], np.float64)
        F = W.shape[1] // K
        a_s = np.asarray(params.a_src[l], np.float64).reshape(K, F)
        a_d = np.asarray(params.a_dst[l], np.float64).reshape(K, F)
        b = np.asarray(params.bias[l], np.float64)
        last = l == L - 1
        parts, mixed_l, z_l, alpha_l, pre_l = [], [], [], [], []
        for s in range(S):
            blk = batch.blocks[l][s]
            n_dst = blk.dst.shape[0]
            mixed = rows_take(hidden[l], blk.shuffle_src_row)             # shuffle
            z = (mixed @ W).reshape(-1, K, F)                              # gnn_layer from here on
            e_src = (z * a_s).sum(2)                                       # [n_mixed, K]
            e_dst = (z * a_d).sum(2)
            agg = np.zeros((n_dst, K, F))
            alphas = []
            for i in range(n_dst):
                nbrs = np.concatenate([[i], blk.blk_src[blk.blk_indptr[i]:blk.blk_indptr[i + 1]]]).astype(np.int64)
                e = _leaky(e_dst[i][None, :] + e_src[nbrs])                # [1 + cnt, K]
                e = e - e.max(0, keepdims=True)
                a = np.exp(e)
                a = a / a.sum(0, keepdims=True)
                agg[i] = (a[:, :, None] * z[nbrs]).sum(0)
                alphas.append(a)
            pre = (agg.mean(1) if last else agg.reshape(n_dst, K * F)) + b
            parts.append(pre if last else _elu(pre))
            mixed_l.append(mixed); z_l.append(z); alpha_l.append(alphas); pre_l.append(pre)
        width = F if last else K * F
        hidden.append(np.concatenate(parts, 0) if parts else np.zeros((0, width)))
        out.mixed.append(mixed_l); out.z.append(z_l); out.alpha.append(alpha_l); out.pre.append(pre_l)
    out.logits = hidden[L]
    return out


@dataclass
class GatBackward:
    gw: List[np.ndarray]
    ga_src: List[np.ndarray]
    ga_dst: List[np.ndarray]
    gbias: List[np.ndarray]
    ghidden: List[Optional[np.ndarray]]
    # per entry of ga_src / ga_dst: the sum of the magnitudes of the terms that the entry adds up
    # (the softmax backward subtracts terms of the same size, the sum over edges mixes signs), i.e.
    # the quantity a floating-point evaluation's rounding error is proportional to.  Not a result
    # of the method: tests use it to tell rounding noise in an entry that cancels to almost
    # nothing from a wrong entry.
    ga_terms: List[np.ndarray]


def gat_backward(batch: Batch, fwd: GatForward, params: GatParams, grad_logits: np.ndarray,
                 slope_positive=None) -> GatBackward:
    """Top layer down; gradients of remote rows go back through the reversed shuffle index; weight
    gradients are summed over the splits.  No gradient for the input features.

    slope_positive (optional): slope_positive[l][s][i], a boolean array [1 + cnt_i, K], replaces
    [score > 0] in the LeakyReLU derivative of destination i (see conditioned_slopes); None keeps
    this pass's own decisions."""
    S, L = batch.n_splits, batch.n_layers
    gw = [np.zeros(np.shape(w), np.float64) for w in params.w]
    gas = [np.zeros(np.shape(a), np.float64) for a in params.a_src]
    gad = [np.zeros(np.shape(a), np.float64) for a in params.a_dst]
    gb = [np.zeros(np.shape(b), np.float64) for b in params.bias]
    terms = [np.zeros(np.shape(a), np.float64) for a in params.a_src]
    ghid: List[Optional[np.ndarray]] = [None] * (L + 1)
    ghid[L] = np.asarray(grad_logits, np.float64)
    for l in range(L - 1, -1, -1):
        K = params.heads[l]
        W = np.asarray(params.w[l], np.float64)
        F = W.shape[1] // K
        a_s = np.asarray(params.a_src[l], np.float64).reshape(K, F)
        a_d = np.asarray(params.a_dst[l], np.float64).reshape(K, F)
        last = l == L - 1
        off = batch.local_off(l + 1)
        if l > 0:
            ghid[l] = np.zeros(fwd.hidden[l].shape, np.float64)
        for s in range(S):
            blk = batch.blocks[l][s]
            n_dst = blk.dst.shape[0]
            dH = ghid[l + 1][off[s]:off[s + 1]]
            pre, z, mixed = fwd.pre[l][s], fwd.z[l][s], fwd.mixed[l][s]
            if last:
                dpre = dH
                dagg = np.repeat(dpre[:, None, :], K, 1) / K              # mean over heads
            else:
                dpre = dH * np.where(pre > 0.0, 1.0, np.exp(np.minimum(pre, 0.0)))   # ELU'
                dagg = dpre.reshape(n_dst, K, F)
            gb[l] += dpre.sum(0)
            dz = np.zeros(z.shape)
            de_src = np.zeros(z.shape[:2])
            de_dst = np.zeros(z.shape[:2])
            mag = np.zeros(z.shape[:2])
            e_src = (z * a_s).sum(2)
            e_dst = (z * a_d).sum(2)
            for i in range(n_dst):
                nbrs = np.concatenate([[i], blk.blk_src[blk.blk_indptr[i]:blk.blk_indptr[i + 1]]]).astype(np.int64)
                a = fwd.alpha[l][s][i]                                     # [n, K]
                np.add.at(dz, nbrs, a[:, :, None] * dagg[i][None, :, :])
                da = (z[nbrs] * dagg[i][None, :, :]).sum(2)                # [n, K]
                de = a * (da - (a * da).sum(0, keepdims=True))             # softmax backward
                raw = e_dst[i][None, :] + e_src[nbrs]
                pos = raw > 0.0 if slope_positive is None else slope_positive[l][s][i]
                de = de * np.where(pos, 1.0, NEG_SLOPE)                    # LeakyReLU backward
                np.add.at(de_src, nbrs, de)
                de_dst[i] += de.sum(0)
                np.add.at(mag, nbrs, a * (np.abs(da) + (a * np.abs(da)).sum(0, keepdims=True)))
            gas[l] += (de_src[:, :, None] * z).sum(0).reshape(-1)
            gad[l] += (de_dst[:, :, None] * z).sum(0).reshape(-1)
            terms[l] += (mag[:, :, None] * np.abs(z)).sum(0).reshape(-1)
            dz += de_src[:, :, None] * a_s[None] + de_dst[:, :, None] * a_d[None]
            dz2 = dz.reshape(z.shape[0], K * F)
            gw[l] += mixed.T @ dz2
            if l > 0:
                rows_add_into(ghid[l], blk.shuffle_src_row, dz2 @ W.T)
    return GatBackward(gw, gas, gad, gb, ghid, terms)


def conditioned_slopes(batch: Batch, fwd: GatForward, params: GatParams, device_terms, rel_tau: float):
    """LeakyReLU slope decisions for a backward pass that is compared with a device's, conditioned
    on the decisions the device took where a score is zero to the rounding of its forward pass.

    The derivative of the LeakyReLU is 1 or NEG_SLOPE according to the sign of the score
    a_dst . z_i + a_src . z_j.  This oracle forms it in float64; a device that forms it in float32
    may land on the other side of zero when |score| <= rel_tau * (largest |score| of the layer), and
    the gradients of that layer and of everything below it then differ by a whole term without
    either being wrong.  There the device's decision is taken: device_terms[l] = (src, dst), the two
    float32 terms it stored per row of local_cat[l] and head ([rows, K] each), whose float32 sum is
    the score it used.  Everywhere else the oracle's own sign stands; a disagreement outside the
    band is a wrong result on the device and is counted, not excused.

    Returns (slope_positive, report): slope_positive[l][s][i] boolean [1 + cnt_i, K]; report = per
    layer (scores in the band, of which the device decided the other way, disagreements outside)."""
    out, report = [], []
    for l in range(batch.n_layers):
        K = params.heads[l]
        F = np.shape(params.w[l])[1] // K
        a_s = np.asarray(params.a_src[l], np.float64).reshape(K, F)
        a_d = np.asarray(params.a_dst[l], np.float64).reshape(K, F)
        d_src = np.asarray(device_terms[l][0], np.float32)
        d_dst = np.asarray(device_terms[l][1], np.float32)
        raws, devs = [], []
        hi = 0.0
        for s in range(batch.n_splits):
            blk, z = batch.blocks[l][s], fwd.z[l][s]
            e_src, e_dst = (z * a_s).sum(2), (z * a_d).sum(2)
            rows = blk.shuffle_src_row            # row of local_cat[l] behind every mixed row
            r_s, d_s = [], []
            for i in range(blk.dst.shape[0]):
                nbrs = np.concatenate([[i], blk.blk_src[blk.blk_indptr[i]:blk.blk_indptr[i + 1]]]).astype(np.int64)
                raw = e_dst[i][None, :] + e_src[nbrs]
                dev = d_dst[rows[i]][None, :] + d_src[rows[nbrs]]          # float32 sum, as on the device
                hi = max(hi, float(np.abs(raw).max()))
                r_s.append(raw); d_s.append(dev)
            raws.append(r_s); devs.append(d_s)
        n_band = n_flip = n_bad = 0
        layer = []
        for r_s, d_s in zip(raws, devs):
            per = []
            for raw, dev in zip(r_s, d_s):
                own, theirs = raw > 0.0, dev > np.float32(0.0)
                band = np.abs(raw) <= rel_tau * hi
                n_band += int(band.sum())
                n_flip += int((band & (own != theirs)).sum())
                n_bad += int((~band & (own != theirs)).sum())
                per.append(np.where(band, theirs, own))
            layer.append(per)
        out.append(layer)
        report.append((n_band, n_flip, n_bad))
    return out, report
