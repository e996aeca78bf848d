"""ctypes binding of libgsplit.so: argument marshalling only.

Every function has the name and the argument order of its C entry point in include/gsplit.h;
tensors are passed as raw device pointers and the current torch stream as a hipStream_t.  There is
no computation here and no fallback: if the HIP library is missing or a call fails, an exception
is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgsplit.so")

GSPLIT_F32, GSPLIT_BF16 = 0, 1
MAX_SPLITS = 8

EXPORTS = [
    "gsplit_create", "gsplit_destroy", "gsplit_last_error", "gsplit_max_rows", "gsplit_sample_split",
    "gsplit_batch_sizes", "gsplit_batch_level", "gsplit_batch_layer", "gsplit_gather_features",
    "gsplit_sage_fwd", "gsplit_sage_bwd", "gsplit_softmax_xent", "gsplit_timing_enable",
    "gsplit_timing_read", "gsplit_presample_accumulate", "gsplit_presample_weights",
    "gsplit_gat_fwd", "gsplit_gat_bwd", "gsplit_batch_stats", "gsplit_sample_split_dev",
    "gsplit_input_counts_accumulate", "gsplit_cache_build", "gsplit_gather_features_cached",
    "gsplit_batch_shuffle", "gsplit_sage_activations", "gsplit_gat_score_terms", "gsplit_sample_split_noalloc",
    "gsplit_sample_split_multi", "gsplit_sage_step", "gsplit_gather_features_multi",
]


class GsplitError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"gsplit error {code}: {msg}")
        self.code = code


class _Graph(C.Structure):
    _fields_ = [("n_vertices", C.c_int64), ("n_edges", C.c_int64), ("d_indptr", C.c_void_p),
                ("indptr_is_64", C.c_int32), ("d_indices", C.c_void_p), ("d_pmap", C.c_void_p),
                ("n_splits", C.c_int32)]


class _Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("fanouts", C.POINTER(C.c_int32)), ("max_targets", C.c_int64),
                ("keep_edge_ids", C.c_int32), ("gat_index", C.c_int32), ("sampler_blocks_per_cu", C.c_int32),
                ("table_mode", C.c_int32)]


class _LevelView(C.Structure):
    _fields_ = [("d_local_cat", C.c_void_p), ("d_local_off", C.c_void_p)]


class _LayerView(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("d_nbr", "d_cnt", "d_mixed_cat", "d_mixed_off", "d_blk_indptr",
                                          "d_blk_src", "d_shuffle_src_row", "d_recv_cat", "d_recv_off")]


class _ShuffleView(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("d_self_row", "d_edge_row", "d_rev_ptr", "d_rev_cnt", "d_rev_list",
                                          "d_rev_eid")]


MAX_LAYERS = 8


class _BatchOut(C.Structure):
    _fields_ = [("d_local_cat", C.c_void_p * (MAX_LAYERS + 1)), ("d_local_off", C.c_void_p),
                ("d_nbr", C.c_void_p * MAX_LAYERS), ("d_cnt", C.c_void_p * MAX_LAYERS),
                ("d_mixed_cat", C.c_void_p * MAX_LAYERS), ("d_mixed_off", C.c_void_p),
                ("d_blk_indptr", C.c_void_p * MAX_LAYERS), ("d_blk_src", C.c_void_p * MAX_LAYERS),
                ("d_shuffle_src_row", C.c_void_p * MAX_LAYERS), ("d_recv_cat", C.c_void_p * MAX_LAYERS),
                ("d_recv_off", C.c_void_p)]


class _SageParams(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("dims", C.POINTER(C.c_int32)), ("d_w_self", C.POINTER(C.c_void_p)),
                ("d_w_neigh", C.POINTER(C.c_void_p)), ("d_bias", C.POINTER(C.c_void_p))]


class _GatParams(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("dims", C.POINTER(C.c_int32)), ("heads", C.POINTER(C.c_int32)),
                ("d_w", C.POINTER(C.c_void_p)), ("d_a_src", C.POINTER(C.c_void_p)),
                ("d_a_dst", C.POINTER(C.c_void_p)), ("d_bias", C.POINTER(C.c_void_p))]


_lib = None


def load_library():
    """dlopen the in-tree HIP library; never falls back to anything else."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(hipcc, gfx950) first; there is no non-HIP path")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
    L.gsplit_create.argtypes = [C.POINTER(vp), C.POINTER(_Graph), C.POINTER(_Config)]
    L.gsplit_destroy.argtypes = [vp]
    L.gsplit_last_error.argtypes = [vp]
    L.gsplit_last_error.restype = C.c_char_p
    L.gsplit_max_rows.argtypes = [vp, i32]
    L.gsplit_max_rows.restype = i64
    L.gsplit_sample_split.argtypes = [vp, vp, i64, u64, u64, vp]
    L.gsplit_sample_split_dev.argtypes = [vp, vp, i64, vp, vp]
    L.gsplit_batch_sizes.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    L.gsplit_batch_level.argtypes = [vp, i32, C.POINTER(_LevelView)]
    L.gsplit_batch_layer.argtypes = [vp, i32, C.POINTER(_LayerView)]
    L.gsplit_sample_split_multi.argtypes = [C.POINTER(vp), i32, C.POINTER(vp), C.POINTER(i64), u64, C.POINTER(u64), vp]
    L.gsplit_sample_split_noalloc.argtypes = [C.POINTER(_Graph), C.POINTER(_Config), vp, i64, u64, u64,
                                              C.POINTER(_BatchOut), vp]
    L.gsplit_batch_shuffle.argtypes = [vp, i32, C.POINTER(_ShuffleView)]
    L.gsplit_sage_activations.argtypes = [vp, i32, C.POINTER(vp)]
    L.gsplit_gat_score_terms.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    L.gsplit_gather_features.argtypes = [vp, vp, i32, i64, i64, vp, vp]
    L.gsplit_gather_features_multi.argtypes = [C.POINTER(vp), i32, vp, i32, i64, i64, C.POINTER(vp), vp]
    L.gsplit_sage_fwd.argtypes = [vp, C.POINTER(_SageParams), vp, vp, vp]
    L.gsplit_sage_bwd.argtypes = [vp, C.POINTER(_SageParams), vp, C.POINTER(vp), C.POINTER(vp),
                                  C.POINTER(vp), vp]
    L.gsplit_softmax_xent.argtypes = [vp, vp, i32, vp, vp, vp, vp]
    L.gsplit_sage_step.argtypes = [vp, C.POINTER(_SageParams), vp, vp, vp, vp, C.POINTER(vp), C.POINTER(vp),
                                   C.POINTER(vp), vp]
    L.gsplit_timing_enable.argtypes = [vp, i32]
    L.gsplit_timing_read.argtypes = [vp, C.c_char_p, i64]
    L.gsplit_timing_read.restype = i64
    L.gsplit_presample_accumulate.argtypes = [vp, vp, vp, vp]
    L.gsplit_presample_weights.argtypes = [vp, vp, i64, i64, vp, vp]
    L.gsplit_batch_stats.argtypes = [vp, vp, vp, vp]
    L.gsplit_input_counts_accumulate.argtypes = [vp, vp, vp]
    L.gsplit_cache_build.argtypes = [vp, vp, i32, i64, i64, vp, C.POINTER(i64), vp]
    L.gsplit_gather_features_cached.argtypes = [vp, vp, vp, vp, vp]
    L.gsplit_gat_fwd.argtypes = [vp, C.POINTER(_GatParams), vp, vp, vp]
    L.gsplit_gat_bwd.argtypes = [vp, C.POINTER(_GatParams), vp, vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                 C.POINTER(vp), vp]
    for name in EXPORTS:
        if name not in ("gsplit_last_error", "gsplit_max_rows", "gsplit_timing_read"):
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _view(ptr: int, n: int, device, dtype=torch.int32) -> torch.Tensor:
    """Copy n values from a raw device pointer into a fresh tensor (test/inspection only)."""
    out = torch.empty(max(n, 0), dtype=dtype, device=device)
    if n > 0:
        hip = _hip_runtime()
        rc = hip.hipMemcpy(C.c_void_p(out.data_ptr()), C.c_void_p(ptr), C.c_size_t(out.element_size() * n), 3)
        if rc != 0:
            raise GsplitError(-4, f"hipMemcpy failed ({rc})")
    return out


def _view_i32(ptr: int, n: int, device) -> torch.Tensor:
    return _view(ptr, n, device, torch.int32)


_hip = None


def _hip_runtime():
    global _hip
    if _hip is None:
        for name in ("libamdhip64.so.7", "libamdhip64.so"):   # the runtime torch already loaded
            try:
                _hip = C.CDLL(name)
                break
            except OSError:
                continue
        if _hip is None:
            raise ImportError("libamdhip64.so not found")
        _hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        _hip.hipMemcpy.restype = C.c_int
    return _hip


def noalloc_output_sizes(n_vertices: int, n_splits: int, fanouts: Sequence[int], max_targets: int) -> dict:
    """Entries of every output buffer of gsplit_sample_split_noalloc, as include/gsplit.h states them."""
    L, S = len(fanouts), n_splits
    ub = [0] * (L + 1)
    ub[L] = max_targets
    for l in range(L - 1, -1, -1):
        ub[l] = min(n_vertices, ub[l + 1] * (1 + fanouts[l]))
    return {"local_cat": ub, "local_off": (L + 1) * (S + 1), "mixed_off": L * (S + 1), "recv_off": L * (S + 1),
            "nbr": [ub[l + 1] * fanouts[l] for l in range(L)], "cnt": [ub[l + 1] for l in range(L)],
            "blk_indptr": [ub[l + 1] + 1 for l in range(L)], "blk_src": [ub[l + 1] * fanouts[l] for l in range(L)],
            "recv_cat": [ub[l + 1] * fanouts[l] for l in range(L)],
            "mixed_cat": [ub[l + 1] * (1 + fanouts[l]) for l in range(L)],
            "shuffle_src_row": [ub[l + 1] * (1 + fanouts[l]) for l in range(L)]}


def gsplit_sample_split_noalloc(indptr: torch.Tensor, indices: torch.Tensor, pmap: torch.Tensor, n_splits: int,
                                fanouts: Sequence[int], max_targets: int, targets: torch.Tensor, seed: int, it: int,
                                out: dict):
    """gsplit_sample_split without a context and without any allocation inside the library.  `out` maps
    the field names of gsplit_batch_out (without the d_ prefix) to int32 device tensors (lists of
    tensors for the per-level / per-layer fields), sized as noalloc_output_sizes says."""
    lib = load_library()
    L = len(fanouts)
    assert indptr.is_cuda and indices.is_cuda and pmap.is_cuda and targets.is_cuda
    assert indptr.dtype in (torch.int32, torch.int64) and indices.dtype == torch.int32 and pmap.dtype == torch.uint8
    assert targets.dtype == torch.int32 and targets.is_contiguous()
    want = noalloc_output_sizes(indptr.numel() - 1, n_splits, fanouts, max_targets)
    o = _BatchOut()
    for name, sizes in want.items():
        t = out[name]
        if isinstance(sizes, list):
            assert len(t) == len(sizes)
            for k, (x, n) in enumerate(zip(t, sizes)):
                assert x.is_cuda and x.dtype == torch.int32 and x.is_contiguous() and x.numel() >= n, (name, k)
                getattr(o, "d_" + name)[k] = x.data_ptr()
        else:
            assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous() and t.numel() >= sizes, name
            setattr(o, "d_" + name, t.data_ptr())
    fan = (C.c_int32 * L)(*[int(f) for f in fanouts])
    g = _Graph(indptr.numel() - 1, indices.numel(), indptr.data_ptr(), int(indptr.dtype == torch.int64),
               indices.data_ptr(), pmap.data_ptr(), int(n_splits))
    c = _Config(L, fan, int(max_targets), 0, 0, 0, 0)
    with torch.cuda.device(indptr.device):
        rc = lib.gsplit_sample_split_noalloc(C.byref(g), C.byref(c), targets.data_ptr(), targets.numel(),
                                             C.c_uint64(seed), C.c_uint64(it), C.byref(o), _stream())
    if rc != 0:
        raise GsplitError(rc, (lib.gsplit_last_error(None) or b"").decode())


def gsplit_sample_split_multi(ctxs, targets, seed: int, iters):
    """Samples targets[b] into ctxs[b] for all b in one set of launches (contexts over the same graph
    and configuration)."""
    n = len(ctxs)
    assert n >= 1 and len(targets) == n and len(iters) == n
    for t in targets:
        assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()
    hs = (C.c_void_p * n)(*[c.h.value for c in ctxs])
    tg = (C.c_void_p * n)(*[t.data_ptr() for t in targets])
    nt = (C.c_int64 * n)(*[t.numel() for t in targets])
    its = (C.c_uint64 * n)(*[int(i) for i in iters])
    for c, t in zip(ctxs, targets):
        c._targets = t
    rc = ctxs[0].lib.gsplit_sample_split_multi(hs, n, tg, nt, C.c_uint64(seed), its, _stream())
    ctxs[0]._check(rc)


def gsplit_gather_features_multi(ctxs, table: torch.Tensor, outs):
    """The loading step of ctxs[b] into outs[b] for all b in one launch."""
    n = len(ctxs)
    assert n >= 1 and len(outs) == n
    assert table.is_cuda and table.dim() == 2 and table.stride(1) == 1
    for o in outs:
        assert o.is_cuda and o.is_contiguous() and o.dtype == table.dtype and o.shape[1] == table.shape[1]
    dt = {torch.float32: GSPLIT_F32, torch.bfloat16: GSPLIT_BF16}[table.dtype]
    hs = (C.c_void_p * n)(*[c.h.value for c in ctxs])
    ps = (C.c_void_p * n)(*[o.data_ptr() for o in outs])
    rc = ctxs[0].lib.gsplit_gather_features_multi(hs, n, table.data_ptr(), dt, table.shape[1],
                                                  table.stride(0) * table.element_size(), ps, _stream())
    ctxs[0]._check(rc)


class SageParams:
    """Holds the marshalled gsplit_sage_params block (and keeps the tensors alive)."""

    def __init__(self, dims: Sequence[int], w_self: List[torch.Tensor], w_neigh: List[torch.Tensor],
                 bias: List[torch.Tensor], dtype: int = GSPLIT_F32):
        L = len(dims) - 1
        assert len(w_self) == len(w_neigh) == len(bias) == L
        for l in range(L):
            for w in (w_self[l], w_neigh[l]):
                assert w.is_cuda and w.dtype == torch.float32 and w.is_contiguous()
                assert tuple(w.shape) == (dims[l], dims[l + 1])
            assert bias[l].is_cuda and bias[l].dtype == torch.float32 and bias[l].numel() == dims[l + 1]
        self.dims = list(dims)
        self.tensors = (list(w_self), list(w_neigh), list(bias))
        self._dims = (C.c_int32 * (L + 1))(*dims)
        self._ws = (C.c_void_p * L)(*[w.data_ptr() for w in w_self])
        self._wn = (C.c_void_p * L)(*[w.data_ptr() for w in w_neigh])
        self._b = (C.c_void_p * L)(*[b.data_ptr() for b in bias])
        self.c = _SageParams(dtype, self._dims, self._ws, self._wn, self._b)
        self.dtype = dtype


class GatParams:
    """Holds the marshalled gsplit_gat_params block (and keeps the tensors alive)."""

    def __init__(self, dims: Sequence[int], heads: Sequence[int], w: List[torch.Tensor], a_src: List[torch.Tensor],
                 a_dst: List[torch.Tensor], bias: List[torch.Tensor]):
        L = len(dims) - 1
        assert len(heads) == len(w) == len(a_src) == len(a_dst) == len(bias) == L
        for l in range(L):
            width = heads[l] * dims[l + 1] if l == L - 1 else dims[l + 1]
            for t, n in ((w[l], dims[l] * width), (a_src[l], width), (a_dst[l], width), (bias[l], dims[l + 1])):
                assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == n
        self.dims, self.heads = list(dims), list(heads)
        self.widths = [heads[l] * dims[l + 1] if l == L - 1 else dims[l + 1] for l in range(L)]
        self.tensors = (list(w), list(a_src), list(a_dst), list(bias))
        self._dims = (C.c_int32 * (L + 1))(*dims)
        self._heads = (C.c_int32 * L)(*heads)
        self._ptrs = [(C.c_void_p * L)(*[t.data_ptr() for t in lst]) for lst in self.tensors]
        self.c = _GatParams(GSPLIT_F32, self._dims, self._heads, *self._ptrs)


class Context:
    """gsplit_ctx wrapper.  Methods mirror the C entry points one to one."""

    def __init__(self, indptr: torch.Tensor, indices: torch.Tensor, pmap: torch.Tensor, n_splits: int,
                 fanouts: Sequence[int], max_targets: int, keep_edge_ids: bool = False,
                 gat_index: bool = False, sampler_blocks_per_cu: int = 0, table_mode: int = 0):
        self.lib = load_library()
        assert indptr.is_cuda and indices.is_cuda and pmap.is_cuda
        assert indptr.dtype in (torch.int32, torch.int64) and indices.dtype == torch.int32
        assert pmap.dtype == torch.uint8
        assert indptr.is_contiguous() and indices.is_contiguous() and pmap.is_contiguous()
        self.device = indptr.device
        self.n_vertices = indptr.numel() - 1
        assert pmap.numel() == self.n_vertices
        self.S, self.L = int(n_splits), len(fanouts)
        self.fanouts = list(int(f) for f in fanouts)
        self._keep = (indptr, indices, pmap)
        self._fan = (C.c_int32 * self.L)(*self.fanouts)
        g = _Graph(self.n_vertices, indices.numel(), indptr.data_ptr(), int(indptr.dtype == torch.int64),
                   indices.data_ptr(), pmap.data_ptr(), self.S)
        self.n_edges = indices.numel()
        c = _Config(self.L, self._fan, int(max_targets), int(keep_edge_ids), int(gat_index), int(sampler_blocks_per_cu),
                    int(table_mode))
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            rc = self.lib.gsplit_create(C.byref(h), C.byref(g), C.byref(c))
        if rc != 0:
            raise GsplitError(rc, (self.lib.gsplit_last_error(None) or b"").decode())
        self.h = h

    # -- plumbing ------------------------------------------------------------------------
    def _check(self, rc: int):
        if rc != 0:
            raise GsplitError(rc, (self.lib.gsplit_last_error(self.h) or b"").decode())

    def close(self):
        if getattr(self, "h", None):
            self.lib.gsplit_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- entry points ----------------------------------------------------------------------
    def gsplit_max_rows(self, level: int) -> int:
        r = self.lib.gsplit_max_rows(self.h, level)
        if r < 0:
            raise GsplitError(int(r), "gsplit_max_rows")
        return int(r)

    def gsplit_sample_split(self, targets: torch.Tensor, seed: int, it: int):
        assert targets.is_cuda and targets.dtype == torch.int32 and targets.is_contiguous()
        self._targets = targets
        self._check(self.lib.gsplit_sample_split(self.h, targets.data_ptr(), targets.numel(),
                                                 C.c_uint64(seed), C.c_uint64(it), _stream()))

    def gsplit_sample_split_dev(self, targets: torch.Tensor, seed_iter: torch.Tensor):
        """seed_iter: int64 device tensor [seed, iteration] read when the kernels run."""
        assert targets.is_cuda and targets.dtype == torch.int32 and targets.is_contiguous()
        assert seed_iter.is_cuda and seed_iter.dtype == torch.int64 and seed_iter.numel() == 2
        self._check(self.lib.gsplit_sample_split_dev(self.h, targets.data_ptr(), targets.numel(),
                                                     seed_iter.data_ptr(), _stream()))

    def gsplit_batch_sizes(self):
        S, L = self.S, self.L
        nl = (C.c_int64 * ((L + 1) * S))()
        nm = (C.c_int64 * (L * S))()
        ne = (C.c_int64 * (L * S))()
        bk = (C.c_int64 * (L * S * S))()
        self._check(self.lib.gsplit_batch_sizes(self.h, nl, nm, ne, bk))
        n_local = [[nl[l * S + s] for s in range(S)] for l in range(L + 1)]
        n_mixed = [[nm[l * S + s] for s in range(S)] for l in range(L)]
        n_edges = [[ne[l * S + s] for s in range(S)] for l in range(L)]
        bucket = [[[bk[(l * S + s) * S + t] for t in range(S)] for s in range(S)] for l in range(L)]
        return n_local, n_mixed, n_edges, bucket

    def gsplit_batch_level(self, level: int) -> _LevelView:
        v = _LevelView()
        self._check(self.lib.gsplit_batch_level(self.h, level, C.byref(v)))
        return v

    def gsplit_batch_layer(self, layer: int) -> _LayerView:
        v = _LayerView()
        self._check(self.lib.gsplit_batch_layer(self.h, layer, C.byref(v)))
        return v

    def gsplit_batch_shuffle(self, layer: int) -> _ShuffleView:
        v = _ShuffleView()
        self._check(self.lib.gsplit_batch_shuffle(self.h, layer, C.byref(v)))
        return v

    def gsplit_sage_activations(self, level: int) -> int:
        """Raw device pointer of the stored activations of local_cat[level]."""
        p = C.c_void_p()
        self._check(self.lib.gsplit_sage_activations(self.h, level, C.byref(p)))
        return int(p.value or 0)

    def gsplit_gat_score_terms(self, layer: int):
        """(raw device pointer, row stride, column of the src terms, column of the dst terms)."""
        p, st, sc, dc = C.c_void_p(), C.c_int64(), C.c_int64(), C.c_int64()
        self._check(self.lib.gsplit_gat_score_terms(self.h, layer, C.byref(p), C.byref(st), C.byref(sc), C.byref(dc)))
        return int(p.value or 0), int(st.value), int(sc.value), int(dc.value)

    def gsplit_gather_features(self, table: torch.Tensor, out: torch.Tensor):
        assert table.is_cuda and out.is_cuda and table.dim() == 2 and table.stride(1) == 1
        assert out.is_contiguous() and out.dtype == table.dtype and out.shape[1] == table.shape[1]
        dt = {torch.float32: GSPLIT_F32, torch.bfloat16: GSPLIT_BF16}[table.dtype]
        self._check(self.lib.gsplit_gather_features(self.h, table.data_ptr(), dt, table.shape[1],
                                                    table.stride(0) * table.element_size(),
                                                    out.data_ptr(), _stream()))

    def gsplit_sage_fwd(self, params: SageParams, feat_local: torch.Tensor, logits: torch.Tensor):
        assert feat_local.is_cuda and feat_local.is_contiguous() and logits.is_cuda and logits.is_contiguous()
        assert logits.dtype == torch.float32
        assert feat_local.dtype == (torch.bfloat16 if params.dtype == GSPLIT_BF16 else torch.float32)
        self._fwd_keep = (params, feat_local)
        self._check(self.lib.gsplit_sage_fwd(self.h, C.byref(params.c), feat_local.data_ptr(),
                                             logits.data_ptr(), _stream()))

    def gsplit_sage_bwd(self, params: SageParams, grad_logits: torch.Tensor, gw_self, gw_neigh, gbias):
        L = self.L
        assert grad_logits.is_cuda and grad_logits.dtype == torch.float32 and grad_logits.is_contiguous()
        for lst in (gw_self, gw_neigh, gbias):
            assert len(lst) == L and all(t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
                                         for t in lst)
        a = (C.c_void_p * L)(*[t.data_ptr() for t in gw_self])
        b = (C.c_void_p * L)(*[t.data_ptr() for t in gw_neigh])
        c = (C.c_void_p * L)(*[t.data_ptr() for t in gbias])
        self._check(self.lib.gsplit_sage_bwd(self.h, C.byref(params.c), grad_logits.data_ptr(), a, b, c,
                                             _stream()))

    def gsplit_sage_step(self, params: SageParams, feat_local: torch.Tensor, labels: torch.Tensor, logits: torch.Tensor,
                         gw_self, gw_neigh, gbias, row_loss: Optional[torch.Tensor] = None):
        L = self.L
        assert feat_local.is_cuda and feat_local.is_contiguous() and logits.is_cuda and logits.is_contiguous()
        assert logits.dtype == torch.float32
        assert feat_local.dtype == (torch.bfloat16 if params.dtype == GSPLIT_BF16 else torch.float32)
        assert labels.is_cuda and labels.dtype == torch.int64 and labels.numel() == self.n_vertices
        for lst in (gw_self, gw_neigh, gbias):
            assert len(lst) == L and all(t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() for t in lst)
        if row_loss is not None:
            assert row_loss.is_cuda and row_loss.dtype == torch.float32 and row_loss.numel() >= logits.shape[0]
        a = (C.c_void_p * L)(*[t.data_ptr() for t in gw_self])
        b = (C.c_void_p * L)(*[t.data_ptr() for t in gw_neigh])
        c = (C.c_void_p * L)(*[t.data_ptr() for t in gbias])
        self._fwd_keep = (params, feat_local)
        self._check(self.lib.gsplit_sage_step(self.h, C.byref(params.c), feat_local.data_ptr(), labels.data_ptr(),
                                              logits.data_ptr(), row_loss.data_ptr() if row_loss is not None else None,
                                              a, b, c, _stream()))

    def gsplit_gat_fwd(self, params: GatParams, feat_local: torch.Tensor, logits: torch.Tensor):
        assert feat_local.is_cuda and feat_local.is_contiguous() and feat_local.dtype == torch.float32
        assert feat_local.shape[1] == params.dims[0]
        assert logits.is_cuda and logits.dtype == torch.float32 and logits.is_contiguous()
        assert logits.shape[1] == params.dims[-1]
        self._check(self.lib.gsplit_gat_fwd(self.h, C.byref(params.c), feat_local.data_ptr(), logits.data_ptr(),
                                            _stream()))

    def gsplit_gat_bwd(self, params: GatParams, feat_local: torch.Tensor, grad_logits: torch.Tensor, gw, ga_src,
                       ga_dst, gbias):
        L = self.L
        assert feat_local.is_cuda and feat_local.is_contiguous() and feat_local.dtype == torch.float32
        assert grad_logits.is_cuda and grad_logits.dtype == torch.float32 and grad_logits.is_contiguous()
        for lst in (gw, ga_src, ga_dst, gbias):
            assert len(lst) == L and all(t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() for t in lst)
        for l in range(L):
            assert gw[l].numel() == params.dims[l] * params.widths[l] and gbias[l].numel() == params.dims[l + 1]
            assert ga_src[l].numel() == params.widths[l] and ga_dst[l].numel() == params.widths[l]
        ptrs = [(C.c_void_p * L)(*[t.data_ptr() for t in lst]) for lst in (gw, ga_src, ga_dst, gbias)]
        self._check(self.lib.gsplit_gat_bwd(self.h, C.byref(params.c), feat_local.data_ptr(), grad_logits.data_ptr(),
                                            *ptrs, _stream()))

    def gsplit_softmax_xent(self, logits: torch.Tensor, labels: torch.Tensor, grad_logits: torch.Tensor,
                            row_loss: Optional[torch.Tensor] = None):
        assert logits.is_cuda and logits.dtype == torch.float32 and logits.is_contiguous()
        assert labels.is_cuda and labels.dtype == torch.int64 and labels.numel() == self.n_vertices
        assert grad_logits.is_cuda and grad_logits.dtype == torch.float32 and grad_logits.is_contiguous()
        assert grad_logits.shape == logits.shape
        if row_loss is not None:
            assert row_loss.is_cuda and row_loss.dtype == torch.float32 and row_loss.numel() >= logits.shape[0]
        self._check(self.lib.gsplit_softmax_xent(self.h, logits.data_ptr(), logits.shape[1], labels.data_ptr(),
                                                 grad_logits.data_ptr(),
                                                 row_loss.data_ptr() if row_loss is not None else None,
                                                 _stream()))

    def gsplit_presample_accumulate(self, vertex_count: Optional[torch.Tensor], edge_count: Optional[torch.Tensor]):
        # torch has no unsigned 32-bit arithmetic: int32 tensors carry the uint32 counters
        for t, n in ((vertex_count, self.n_vertices), (edge_count, self.n_edges)):
            if t is not None:
                assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous() and t.numel() == n
        self._check(self.lib.gsplit_presample_accumulate(
            self.h, vertex_count.data_ptr() if vertex_count is not None else None,
            edge_count.data_ptr() if edge_count is not None else None, _stream()))

    def gsplit_batch_stats(self, edges: torch.Tensor, cross_edges: torch.Tensor):
        # int64 tensors carry the uint64 counters
        for t in (edges, cross_edges):
            assert t.is_cuda and t.dtype == torch.int64 and t.is_contiguous() and t.numel() == self.L * self.S
        self._check(self.lib.gsplit_batch_stats(self.h, edges.data_ptr(), cross_edges.data_ptr(), _stream()))

    def gsplit_input_counts_accumulate(self, count: torch.Tensor):
        assert count.is_cuda and count.dtype == torch.int32 and count.is_contiguous() and count.numel() == self.n_vertices
        self._check(self.lib.gsplit_input_counts_accumulate(self.h, count.data_ptr(), _stream()))

    def gsplit_cache_build(self, table: torch.Tensor, cache_ids: torch.Tensor, n_cache: Sequence[int]):
        """table: [n_vertices, dim] float32 / bfloat16, on the device or in pinned host memory."""
        assert table.dim() == 2 and table.stride(1) == 1 and table.shape[0] == self.n_vertices
        assert table.dtype in (torch.float32, torch.bfloat16) and (table.is_cuda or table.is_pinned())
        assert cache_ids.is_cuda and cache_ids.dtype == torch.int32 and cache_ids.is_contiguous()
        assert len(n_cache) == self.S and sum(n_cache) == cache_ids.numel()
        self._cache_keep = (table, cache_ids)
        self._cache_dim, self._cache_dtype = table.shape[1], table.dtype
        self._check(self.lib.gsplit_cache_build(
            self.h, table.data_ptr(), GSPLIT_F32 if table.dtype == torch.float32 else GSPLIT_BF16, table.shape[1],
            table.stride(0) * table.element_size(), cache_ids.data_ptr(), (C.c_int64 * self.S)(*[int(x) for x in n_cache]),
            _stream()))

    def gsplit_gather_features_cached(self, out: torch.Tensor, hits: Optional[torch.Tensor] = None,
                                      misses: Optional[torch.Tensor] = None):
        assert out.is_cuda and out.is_contiguous() and out.dtype == self._cache_dtype and out.shape[1] == self._cache_dim
        for t in (hits, misses):      # int64 tensors carry the uint64 counters
            assert t is None or (t.is_cuda and t.dtype == torch.int64 and t.is_contiguous() and t.numel() == self.S)
        self._check(self.lib.gsplit_gather_features_cached(
            self.h, out.data_ptr(), hits.data_ptr() if hits is not None else None,
            misses.data_ptr() if misses is not None else None, _stream()))

    def gsplit_presample_weights(self, count: torch.Tensor, n_samples: int, weight: torch.Tensor):
        assert count.is_cuda and count.dtype == torch.int32 and count.is_contiguous()
        assert weight.is_cuda and weight.dtype == torch.float32 and weight.is_contiguous()
        assert weight.numel() == count.numel()
        self._check(self.lib.gsplit_presample_weights(self.h, count.data_ptr(), count.numel(), int(n_samples),
                                                      weight.data_ptr(), _stream()))

    def gsplit_timing_enable(self, enable: bool):
        self._check(self.lib.gsplit_timing_enable(self.h, int(enable)))

    def gsplit_timing_read(self) -> dict:
        """{label: (launches, total_ms)} since the last read."""
        buf = C.create_string_buffer(1 << 16)
        n = self.lib.gsplit_timing_read(self.h, buf, len(buf))
        if n < 0:
            self._check(int(n))
        out = {}
        for line in buf.value.decode().splitlines():
            name, cnt, ms = line.split()
            out[name] = (int(cnt), float(ms))
        return out

    # -- inspection helpers for tests (copies of the device views; they synchronise) -------
    def fetch_batch(self) -> dict:
        """Copies the whole current batch to torch tensors, split by split (tests only)."""
        S, L = self.S, self.L
        n_local, n_mixed, n_edges, bucket = self.gsplit_batch_sizes()
        dev = self.device
        out = {"n_local": n_local, "n_mixed": n_mixed, "n_edges": n_edges, "bucket": bucket,
               "local_front": [], "layers": []}
        for l in range(L + 1):
            v = self.gsplit_batch_level(l)
            cat = _view_i32(v.d_local_cat, sum(n_local[l]), dev)
            off = _view_i32(v.d_local_off, S + 1, dev)
            assert off.tolist() == [sum(n_local[l][:s]) for s in range(S + 1)]
            out["local_front"].append(list(torch.split(cat, n_local[l])))
        for l in range(L):
            v = self.gsplit_batch_layer(l)
            fan = self.fanouts[l]
            n_dst = sum(n_local[l + 1])
            lay = {
                "nbr": _view_i32(v.d_nbr, n_dst * fan, dev).view(n_dst, fan),
                "cnt": _view_i32(v.d_cnt, n_dst, dev),
                "mixed": list(torch.split(_view_i32(v.d_mixed_cat, sum(n_mixed[l]), dev), n_mixed[l])),
                "blk_indptr": _view_i32(v.d_blk_indptr, n_dst + 1, dev),
                "blk_src": _view_i32(v.d_blk_src, sum(n_edges[l]), dev),
                "shuffle_src_row": list(torch.split(_view_i32(v.d_shuffle_src_row, sum(n_mixed[l]), dev),
                                                    n_mixed[l])),
                "recv": _view_i32(v.d_recv_cat, sum(sum(r) for r in bucket[l]), dev),
                "recv_off": _view_i32(v.d_recv_off, S + 1, dev),
            }
            out["layers"].append(lay)
        return out

    def fetch_shuffle(self, layer: int) -> dict:
        """Copies of the composed gather side and of the scatter side of shuffle_idx[layer] (tests only)."""
        n_local, _, n_edges, _ = self.gsplit_batch_sizes()
        dev = self.device
        v = self.gsplit_batch_shuffle(layer)
        n_dst, nnz, n_lo = sum(n_local[layer + 1]), sum(n_edges[layer]), sum(n_local[layer])
        out = {"self_row": _view_i32(v.d_self_row, n_dst, dev), "edge_row": _view_i32(v.d_edge_row, nnz, dev),
               "rev_ptr": None, "rev_cnt": None, "rev_list": None, "rev_eid": None}
        if v.d_rev_list:
            out["rev_ptr"] = _view_i32(v.d_rev_ptr, n_lo, dev)
            out["rev_cnt"] = _view_i32(v.d_rev_cnt, n_lo, dev)
            out["rev_list"] = _view_i32(v.d_rev_list, n_dst + nnz, dev)
            if v.d_rev_eid:
                out["rev_eid"] = _view_i32(v.d_rev_eid, n_dst + nnz, dev)
        return out

    def fetch_sage_activations(self, level: int, width: int, dtype=torch.float32) -> torch.Tensor:
        """Copy of the stored activations of local_cat[level] as [rows, width] (tests only)."""
        n_local, _, _, _ = self.gsplit_batch_sizes()
        rows = sum(n_local[level])
        return _view(self.gsplit_sage_activations(level), rows * width, self.device, dtype).view(rows, width)

    def fetch_gat_score_terms(self, layer: int, heads: int):
        """Copies of the per-row score terms of a GAT layer: (src [rows, K], dst [rows, K]) (tests only)."""
        n_local, _, _, _ = self.gsplit_batch_sizes()
        rows = sum(n_local[layer])
        ptr, stride, sc, dc = self.gsplit_gat_score_terms(layer)
        raw = _view(ptr, rows * stride, self.device, torch.float32).view(rows, stride)
        return raw[:, sc:sc + heads].contiguous(), raw[:, dc:dc + heads].contiguous()
