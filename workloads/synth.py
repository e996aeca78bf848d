"""Seeded synthetic inputs shaped like the paper's workloads (Table 2 and the experiment settings).

This module only *draws inputs*: graphs, partition maps, features, labels, weights and target
batches.  It contains none of the method's arithmetic (no sampling, splitting, dedup or GNN
maths) and is the one piece of code that the CPU oracle's tests and the HIP path's tests both
use, so that the two sides see the very same arrays.

Everything is written with torch tensor ops so that the large graphs can be generated on the GPU
in seconds; the arrays are then handed (or copied to the host) unchanged to whichever side needs
them.  A torch.Generator seeded from one master seed plus a fixed per-purpose offset drives every
draw.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import torch

MASTER_SEED = 0x5EED

_OFF_GRAPH = 1
_OFF_PERM = 2
_OFF_FEAT = 3
_OFF_LABEL = 4
_OFF_WEIGHT = 5
_OFF_PMAP = 6
_OFF_TARGET = 7


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    return g


def rmat_edge_chunks(scale: int, n_draws: int, a: float, b: float, c: float, *, seed: int,
                     device="cpu", chunk: int = 1 << 26):
    """Yield `n_draws` directed (src, dst) pairs from the recursive-matrix model on 2**scale ids,
    `chunk` pairs at a time.

    Each of the `scale` bit levels picks one of four quadrants with probabilities (a, b, c, 1-a-b-c):
    a = (0,0), b = (0,1), c = (1,0), d = (1,1) for the (src bit, dst bit) pair.
    """
    g = _gen(device, seed)
    done = 0
    while done < n_draws:
        m = min(chunk, n_draws - done)
        src = torch.zeros(m, dtype=torch.int64, device=device)
        dst = torch.zeros(m, dtype=torch.int64, device=device)
        for _ in range(scale):
            u = torch.rand(m, generator=g, device=device)
            sbit = (u >= a + b).to(torch.int64)
            dbit = (((u >= a) & (u < a + b)) | (u >= a + b + c)).to(torch.int64)
            src = (src << 1) | sbit
            dst = (dst << 1) | dbit
        yield src, dst
        done += m


def rmat_edges(scale: int, n_draws: int, a: float, b: float, c: float, *, seed: int, device="cpu",
               chunk: int = 1 << 26):
    parts = list(rmat_edge_chunks(scale, n_draws, a, b, c, seed=seed, device=device, chunk=chunk))
    return torch.cat([p[0] for p in parts]), torch.cat([p[1] for p in parts])


def _unique_sorted(keys: torch.Tensor, limit: int = (1 << 31) - (1 << 24)) -> torch.Tensor:
    """torch.unique (sorted) for inputs of any length: the device sort handles fewer than 2**31
    elements, so longer inputs are cut at splitters taken from a sorted random sample and every
    part is deduplicated on its own (parts are disjoint value ranges, so concatenation is sorted)."""
    n = keys.numel()
    if n <= limit:
        return torch.unique(keys)
    parts = 2 * ((n + limit - 1) // limit)
    g = _gen(keys.device, 12345)
    sample = keys[torch.randint(0, n, (1 << 20,), generator=g, device=keys.device)]
    sample = torch.sort(sample).values
    cuts = sample[torch.arange(1, parts, device=keys.device) * (sample.numel() // parts)]
    cuts = torch.unique(cuts)
    out = []
    lo = None
    step = 1 << 29
    for i in range(cuts.numel() + 1):
        hi = cuts[i] if i < cuts.numel() else None
        piece = []
        for s0 in range(0, n, step):                      # select in slices: no op sees 2**31 elements
            kk = keys[s0:s0 + step]
            sel = torch.ones(kk.numel(), dtype=torch.bool, device=keys.device) if lo is None else kk >= lo
            if hi is not None:
                sel &= kk < hi
            piece.append(kk[sel])
        part = torch.cat(piece)
        del piece
        assert part.numel() <= limit, "splitters too coarse"
        out.append(torch.unique(part))
        del part
        lo = hi
    return torch.cat(out)


def csr_from_keys(keys: torch.Tensor, n_vertices: int, *, index64: bool):
    """CSR from sorted, duplicate-free keys src * n_vertices + dst."""
    bounds = torch.arange(n_vertices + 1, dtype=torch.int64, device=keys.device) * n_vertices
    indptr = torch.searchsorted(keys, bounds)
    cols = torch.empty(keys.numel(), dtype=torch.int32, device=keys.device)
    step = 1 << 29
    for s0 in range(0, keys.numel(), step):
        kk = keys[s0:s0 + step]
        cols[s0:s0 + step] = (kk - torch.div(kk, n_vertices, rounding_mode="floor") * n_vertices).to(torch.int32)
    if not index64:
        assert int(indptr[-1]) < 2 ** 31
        indptr = indptr.to(torch.int32)
    return indptr.contiguous(), cols


def build_csr(src: torch.Tensor, dst: torch.Tensor, n_vertices: int, *, symmetrise: bool,
              index64: bool):
    """Sorted, duplicate-free, self-loop-free CSR.  Row v lists the vertices v aggregates from."""
    keep = (src != dst) & (src < n_vertices) & (dst < n_vertices)
    src, dst = src[keep], dst[keep]
    if symmetrise:
        src, dst = torch.cat([src, dst]), torch.cat([dst, src])
    keys = _unique_sorted(src * n_vertices + dst)  # sorted ascending => rows sorted, no dups
    return csr_from_keys(keys, n_vertices, index64=index64)


def rmat_graph(n_vertices: int, n_directed_target: int, abc: Sequence[float], *, seed: int,
               symmetrise: bool = True, permute_ids: bool = True, index64: bool = False,
               device="cpu", exact_draws: Optional[int] = None):
    """R-MAT graph with about `n_directed_target` directed edges after clean-up.

    ids >= n_vertices are rejected (scale is the next power of two); a seeded random relabelling
    spreads the hubs over the id range unless permute_ids is False; self loops and duplicates are
    removed; with `symmetrise` every edge is stored in both directions.  If `exact_draws` is given
    that many pairs are drawn once (the Tiny workload fixes the number of draws, not of edges);
    otherwise batches are drawn until the cleaned edge count reaches the target.  Everything runs
    chunk by chunk, so no single tensor op sees more than 2**30 elements.
    """
    scale = max(1, math.ceil(math.log2(n_vertices)))
    a, b, c = abc
    perm = torch.randperm(n_vertices, generator=_gen(device, seed + _OFF_PERM), device=device) \
        if permute_ids else None
    both = 2 if symmetrise else 1

    def clean_keys(n_draws, sd):
        out = []
        for s2, d2 in rmat_edge_chunks(scale, n_draws, a, b, c, seed=sd, device=device):
            ok = (s2 != d2) & (s2 < n_vertices) & (d2 < n_vertices)
            s2, d2 = s2[ok], d2[ok]
            if perm is not None:
                s2, d2 = perm[s2], perm[d2]
            if symmetrise:  # canonical orientation: (u,v) and (v,u) are one undirected edge
                s2, d2 = torch.minimum(s2, d2), torch.maximum(s2, d2)
            out.append(s2 * n_vertices + d2)
        return out

    if exact_draws is not None:
        keys = _unique_sorted(torch.cat(clean_keys(exact_draws, seed + _OFF_GRAPH)))
    else:
        keys = torch.empty(0, dtype=torch.int64, device=device)
        rnd = 0
        while keys.numel() * both < n_directed_target:
            need = max(1, n_directed_target // both // 8,
                       int((n_directed_target - keys.numel() * both) / both * 1.15))
            keys = _unique_sorted(torch.cat([keys] + clean_keys(need, seed + _OFF_GRAPH + 1000 * rnd)))
            rnd += 1
    if symmetrise:
        src = torch.div(keys, n_vertices, rounding_mode="floor")
        swapped = (keys - src * n_vertices) * n_vertices + src
        del src
        keys = _unique_sorted(torch.cat([keys, swapped]))
        del swapped
    return csr_from_keys(keys, n_vertices, index64=index64)


def pmap_random(n_vertices: int, n_splits: int, *, seed: int, device="cpu") -> torch.Tensor:
    """The 'Rand' partitioner of the paper's splitting-algorithm evaluation: uniform owner."""
    g = _gen(device, seed + _OFF_PMAP)
    return torch.randint(0, n_splits, (n_vertices,), generator=g, device=device).to(torch.uint8)


def pmap_range(n_vertices: int, n_splits: int, *, device="cpu") -> torch.Tensor:
    """Contiguous id ranges: owner(v) = floor(v * S / |V|)."""
    v = torch.arange(n_vertices, dtype=torch.int64, device=device)
    return torch.div(v * n_splits, n_vertices, rounding_mode="floor").to(torch.uint8)


def bfs_rank(indptr: torch.Tensor, indices: torch.Tensor) -> torch.Tensor:
    """Rank of every vertex in BFS visit order from the max-degree vertex (ties inside a level by
    id); vertices the search does not reach follow in id order."""
    dev = indptr.device
    n = indptr.numel() - 1
    ip = indptr.to(torch.int64)
    deg = ip[1:] - ip[:-1]
    rank = torch.full((n,), -1, dtype=torch.int64, device=dev)
    next_rank = 0
    frontier = torch.argmax(deg).reshape(1)
    while frontier.numel() > 0:
        rank[frontier] = next_rank + torch.arange(frontier.numel(), device=dev)
        next_rank += frontier.numel()
        # expand the level in slices so that no temporary exceeds about 2**28 entries
        nxt = []
        lens_all = deg[frontier]
        csum = torch.cumsum(lens_all, 0)
        start = 0
        while start < frontier.numel():
            base = int(csum[start - 1]) if start > 0 else 0
            stop = int(torch.searchsorted(csum, torch.tensor(base + (1 << 28), device=dev), right=True))
            stop = max(stop, start + 1)
            f = frontier[start:stop]
            lens = lens_all[start:stop]
            tot = int(lens.sum())
            if tot > 0:
                seg = torch.repeat_interleave(torch.arange(f.numel(), device=dev), lens)
                offs = torch.arange(tot, device=dev) - torch.repeat_interleave(torch.cumsum(lens, 0) - lens, lens)
                nb = indices[ip[f][seg] + offs].to(torch.int64)
                nb = nb[rank[nb] < 0]
                if nb.numel():
                    nxt.append(torch.unique(nb))
                del seg, offs, nb
            start = stop
        frontier = torch.unique(torch.cat(nxt)) if nxt else frontier[:0]
        if frontier.numel():
            frontier = frontier[rank[frontier] < 0]
    rest = torch.nonzero(rank < 0).flatten()
    rank[rest] = next_rank + torch.arange(rest.numel(), device=dev)
    return rank


def pmap_from_rank(rank: torch.Tensor, n_splits: int) -> torch.Tensor:
    """A ranking of the vertices cut into n_splits equal blocks."""
    n = rank.numel()
    return torch.div(rank * n_splits, n, rounding_mode="floor").clamp(0, n_splits - 1).to(torch.uint8)


def pmap_bfs_blocks(indptr: torch.Tensor, indices: torch.Tensor, n_splits: int) -> torch.Tensor:
    """Locality map: the BFS ranking (bfs_rank) cut into n_splits equal blocks."""
    return pmap_from_rank(bfs_rank(indptr, indices), n_splits)


def features(n_vertices: int, dim: int, *, seed: int, device="cpu", dtype=torch.float32,
             chunk_rows: int = 1 << 22) -> torch.Tensor:
    """N(0,1) rows, generated in chunks so that the big tables never need a second copy."""
    g = _gen(device, seed + _OFF_FEAT)
    out = torch.empty((n_vertices, dim), dtype=dtype, device=device)
    for r0 in range(0, n_vertices, chunk_rows):
        r1 = min(n_vertices, r0 + chunk_rows)
        out[r0:r1] = torch.randn((r1 - r0, dim), generator=g, device=device).to(dtype)
    return out


def labels(n_vertices: int, n_classes: int, *, seed: int, device="cpu") -> torch.Tensor:
    g = _gen(device, seed + _OFF_LABEL)
    return torch.randint(0, n_classes, (n_vertices,), generator=g, device=device, dtype=torch.int64)


def sage_weights(dims: Sequence[int], *, seed: int, device="cpu"):
    """Glorot-uniform W_self[l], W_neigh[l] of shape [D_l, D_{l+1}] and a small non-zero bias."""
    g = _gen(device, seed + _OFF_WEIGHT)
    w_self, w_neigh, bias = [], [], []
    for l in range(len(dims) - 1):
        lim = math.sqrt(6.0 / (dims[l] + dims[l + 1]))
        for dstl in (w_self, w_neigh):
            dstl.append(((torch.rand((dims[l], dims[l + 1]), generator=g, device=device) * 2 - 1) * lim)
                        .contiguous())
        bias.append(((torch.rand((dims[l + 1],), generator=g, device=device) * 2 - 1) * 0.1).contiguous())
    return w_self, w_neigh, bias


def micro_batch_parts(targets: torch.Tensor, n_micro: int):
    """The targets of one mini-batch dealt to n_micro data-parallel micro-batches by position: equal
    contiguous parts, the remainder to the first ones."""
    base, rem = divmod(targets.numel(), n_micro)
    out, pos = [], 0
    for m in range(n_micro):
        n = base + (1 if m < rem else 0)
        out.append(targets[pos:pos + n])
        pos += n
    return out


def gat_weights(dims: Sequence[int], heads: Sequence[int], *, seed: int, device="cpu"):
    """Glorot-uniform W[l] of shape [D_l, heads_l * F_l] (F_l = dims[l+1] / heads_l on hidden layers,
    dims[L] on the last, whose heads are averaged), attention vectors a_src[l], a_dst[l] of
    heads_l * F_l entries, and a small non-zero bias of dims[l+1] entries."""
    g = _gen(device, seed + _OFF_WEIGHT + 7)
    L = len(dims) - 1
    w, a_src, a_dst, bias = [], [], [], []
    for l in range(L):
        width = heads[l] * dims[l + 1] if l == L - 1 else dims[l + 1]
        feat = width // heads[l]
        lim = math.sqrt(6.0 / (dims[l] + width))
        w.append(((torch.rand((dims[l], width), generator=g, device=device) * 2 - 1) * lim).contiguous())
        lim_a = math.sqrt(6.0 / (feat + 1))
        a_src.append(((torch.rand((width,), generator=g, device=device) * 2 - 1) * lim_a).contiguous())
        a_dst.append(((torch.rand((width,), generator=g, device=device) * 2 - 1) * lim_a).contiguous())
        bias.append(((torch.rand((dims[l + 1],), generator=g, device=device) * 2 - 1) * 0.1).contiguous())
    return w, a_src, a_dst, bias


def draw_targets(n_vertices: int, batch: int, *, seed: int, it: int, device="cpu") -> torch.Tensor:
    """`batch` distinct vertex ids, uniformly, fresh for every iteration number `it`."""
    g = _gen(device, seed + _OFF_TARGET + 7919 * (it + 1))
    if n_vertices <= (1 << 24):
        return torch.randperm(n_vertices, generator=g, device=device)[:batch].to(torch.int32).contiguous()
    # large id ranges: oversample, dedup keeping first occurrences
    cand = torch.randint(0, n_vertices, (batch * 2 + 64,), generator=g, device=device)
    uniq, inv = torch.unique(cand, return_inverse=True)
    first = torch.full((uniq.numel(),), cand.numel(), dtype=torch.int64, device=device)
    first.scatter_reduce_(0, inv, torch.arange(cand.numel(), device=device), reduce="amin")
    order = torch.sort(first).values[:batch]
    return cand[order].to(torch.int32).contiguous()


@dataclass
class Workload:
    name: str
    n_vertices: int
    indptr: torch.Tensor          # int32 or int64 [n_vertices+1]
    indices: torch.Tensor         # int32 [n_edges]
    pmap: torch.Tensor            # uint8 [n_vertices]
    n_splits: int
    feat: torch.Tensor            # [n_vertices, dims[0]]
    labels: torch.Tensor          # int64 [n_vertices]
    fanouts: List[int]            # fanouts[l] expands layer l+1 into layer l (l = L-1 .. 0)
    dims: List[int]               # dims[0] = input width ... dims[L] = classes
    batch: int
    seed: int = MASTER_SEED
    w_self: list = field(default_factory=list)
    w_neigh: list = field(default_factory=list)
    bias: list = field(default_factory=list)

    @property
    def n_edges(self) -> int:
        return int(self.indices.numel())

    @property
    def n_layers(self) -> int:
        return len(self.fanouts)

    def targets(self, it: int) -> torch.Tensor:
        return draw_targets(self.n_vertices, self.batch, seed=self.seed, it=it,
                            device=self.indptr.device)

    def describe(self) -> dict:
        return {"workload": self.name, "n_vertices": self.n_vertices, "n_edges": self.n_edges,
                "n_splits": self.n_splits, "batch": self.batch, "fanouts": list(self.fanouts),
                "dims": list(self.dims), "feat_dtype": str(self.feat.dtype).replace("torch.", ""),
                "indptr": str(self.indptr.dtype).replace("torch.", "")}


def _finish(name, n, indptr, indices, pmap, n_splits, dims, fanouts, batch, seed, device,
            feat_dtype=torch.float32) -> Workload:
    feat = features(n, dims[0], seed=seed, device=device, dtype=feat_dtype)
    lab = labels(n, dims[-1], seed=seed, device=device)
    ws, wn, b = sage_weights(dims, seed=seed, device=device)
    return Workload(name, n, indptr, indices, pmap, n_splits, feat, lab, list(fanouts), list(dims),
                    batch, seed, ws, wn, b)


def tiny(device="cpu", seed: int = MASTER_SEED, n_splits: int = 4) -> Workload:
    """2**14 vertices, 2**18 R-MAT(.57,.19,.19) draws symmetrised; 64-d features; 16 classes;
    uniform-random partition map; 1024 targets; fanouts [10, 5]; hidden 64."""
    n = 1 << 14
    indptr, indices = rmat_graph(n, 0, (0.57, 0.19, 0.19), seed=seed, symmetrise=True,
                                 permute_ids=False, index64=False, device=device,
                                 exact_draws=1 << 18)
    pmap = pmap_random(n, n_splits, seed=seed, device=device)
    return _finish("tiny", n, indptr, indices, pmap, n_splits, [64, 64, 16], [10, 5], 1024, seed, device)


def medium(device="cpu", seed: int = MASTER_SEED, n_splits: int = 4, scale_down: int = 1) -> Workload:
    """2.4M vertices, about 124M directed edges (symmetric, average degree about 50); 100-d
    features; 47 classes; contiguous-range partition map; batch 1024; fanouts [15,10,5];
    hidden 256.  `scale_down` divides vertex and edge counts (CPU-sized rehearsals only)."""
    n = 2_400_000 // scale_down
    m = 124_000_000 // scale_down
    indptr, indices = rmat_graph(n, m, (0.57, 0.19, 0.19), seed=seed, symmetrise=True,
                                 permute_ids=True, index64=False, device=device)
    pmap = pmap_range(n, n_splits, device=device)
    name = "medium" if scale_down == 1 else f"medium/{scale_down}"
    return _finish(name, n, indptr, indices, pmap, n_splits, [100, 256, 256, 47], [15, 10, 5], 1024,
                   seed, device)


def large(device="cuda", seed: int = MASTER_SEED, n_splits: int = 4, feat_dtype=torch.float32,
          scale_down: int = 1, batch: int = 4096, fanouts=(15, 10, 5), dims=(128, 256, 256, 172),
          progress=None) -> Workload:
    """111M vertices, 1.6B directed edges (not symmetrised: row v lists what v aggregates from),
    int64 indptr; 128-d features (fp32 or bf16), 172 classes; BFS-block partition map; batch 4096;
    fanouts [15,10,5]; hidden 256.  `scale_down` divides vertex and edge counts."""
    say = progress or (lambda m: None)
    n = 111_000_000 // scale_down
    m = 1_600_000_000 // scale_down
    say(f"large: drawing about {m} directed edges on {n} vertices")
    indptr, indices = rmat_graph(n, m, (0.57, 0.19, 0.19), seed=seed, symmetrise=False,
                                 permute_ids=True, index64=True, device=device)
    say(f"large: CSR built, {indices.numel()} edges; partition map")
    pmap = pmap_bfs_blocks(indptr, indices, n_splits)
    say("large: features")
    name = "large" if scale_down == 1 else f"large/{scale_down}"
    return _finish(name, n, indptr, indices, pmap, n_splits, list(dims), list(fanouts), batch, seed,
                   device, feat_dtype=feat_dtype)


def skewed(device="cuda", seed: int = MASTER_SEED, n_splits: int = 4, scale_down: int = 1,
           progress=None) -> Workload:
    """65M vertices, 3.6B directed edges (symmetric), R-MAT(.6,.15,.15,.1) without id permutation
    (hubs stay clustered), int64 indptr; 128-d fp32 features; 64 classes; contiguous-range map;
    batch 4096; fanouts [20,20,20]; hidden 256."""
    say = progress or (lambda m: None)
    n = 65_000_000 // scale_down
    m = 3_600_000_000 // scale_down
    say(f"skewed: drawing about {m} directed edges on {n} vertices")
    indptr, indices = rmat_graph(n, m, (0.6, 0.15, 0.15), seed=seed, symmetrise=True,
                                 permute_ids=False, index64=True, device=device)
    say(f"skewed: CSR built, {indices.numel()} edges")
    pmap = pmap_range(n, n_splits, device=device)
    name = "skewed" if scale_down == 1 else f"skewed/{scale_down}"
    return _finish(name, n, indptr, indices, pmap, n_splits, [128, 256, 256, 64], [20, 20, 20], 4096,
                   seed, device)


def custom(n_vertices: int, n_directed: int, *, dims, fanouts, batch, n_splits=4, pmap_kind="random",
           abc=(0.57, 0.19, 0.19), index64=False, device="cpu", seed: int = MASTER_SEED,
           permute_ids=True, name="custom") -> Workload:
    """Free-form workload for parity cases (ragged sizes, int64 indptr, other split counts)."""
    indptr, indices = rmat_graph(n_vertices, n_directed, abc, seed=seed, symmetrise=True,
                                 permute_ids=permute_ids, index64=index64, device=device)
    if pmap_kind == "random":
        pmap = pmap_random(n_vertices, n_splits, seed=seed, device=device)
    elif pmap_kind == "range":
        pmap = pmap_range(n_vertices, n_splits, device=device)
    elif pmap_kind == "bfs":
        pmap = pmap_bfs_blocks(indptr, indices, n_splits)
    else:
        raise ValueError(pmap_kind)
    return _finish(name, n_vertices, indptr, indices, pmap, n_splits, dims, fanouts, batch, seed, device)


def variant(w: Workload, *, n_splits: Optional[int] = None, batch: Optional[int] = None, fanouts=None, dims=None,
            feat_dtype=None, pmap_kind: Optional[str] = None, name: Optional[str] = None, rank=None) -> Workload:
    """The same graph, features and labels under another model / batch / split configuration (the
    split sweep runs on the large graph): new weights for new dims, a new partition map for a new
    number of splits (pmap_kind 'bfs' cuts `rank`, or a fresh BFS ranking, into blocks; 'range' cuts
    the id range).  Input width and class count must stay what they are.  The tensors that do not
    change are shared, not copied."""
    import copy
    v = copy.copy(w)
    dev = w.indptr.device
    if dims is not None:
        assert dims[0] == w.dims[0] and dims[-1] == w.dims[-1], "features and labels are kept"
        v.dims = list(dims)
        v.w_self, v.w_neigh, v.bias = sage_weights(v.dims, seed=w.seed, device=dev)
    if fanouts is not None:
        v.fanouts = list(fanouts)
    if batch is not None:
        v.batch = int(batch)
    if n_splits is not None and (n_splits != w.n_splits or pmap_kind is not None):
        v.n_splits = int(n_splits)
        kind = pmap_kind or "bfs"
        if kind == "bfs":
            v.pmap = pmap_from_rank(rank if rank is not None else bfs_rank(w.indptr, w.indices), v.n_splits)
        elif kind == "range":
            v.pmap = pmap_range(w.n_vertices, v.n_splits, device=dev)
        else:
            v.pmap = pmap_random(w.n_vertices, v.n_splits, seed=w.seed, device=dev)
    if feat_dtype is not None and feat_dtype != w.feat.dtype:
        v.feat = w.feat.to(feat_dtype)
    if name:
        v.name = name
    return v
