// Partial feature cache aligned with the partition map f_G, and the loading step that uses it
// (paper sections 3 and 4: the input features live in host memory, every GPU statically caches
// features of vertices f_G assigns to it, and "a GPU can skip loading an input feature if it is
// already cached locally"; section 7.1: what to cache is ranked by sampling frequency).
//
// On one GPU the caches of all logical splits share one slot map (int32 per vertex: row of the
// cache or -1); since the input layer of split s only holds vertices f_G gives to s, and split s's
// part of the cache only holds vertices of s, a lookup never crosses splits.  A miss reads the row
// from the host table through the device's mapping of pinned host memory (zero copy over PCIe):
// the ids never leave the device, so the loading step needs no host round trip.
#include <algorithm>

#include "gsplit_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_fill_i32(int32_t *__restrict__ p, int64_t n, int32_t v) {
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < n; x += (int64_t)gridDim.x * blockDim.x) p[x] = v;
}

struct GroupOff { int64_t off[GS_MAXS + 1]; };

// slot_of[ids[j]] = j; flags an id outside the graph, an id f_G gives to another split than its
// group, and an id that occurs twice
__global__ __launch_bounds__(256) void k_cache_set_slots(const int32_t *__restrict__ ids, GroupOff g, int S,
                                                         const uint8_t *__restrict__ pmap, int64_t n_vertices,
                                                         int32_t *__restrict__ slot_of, int32_t *__restrict__ err) {
    const int64_t n = g.off[S];
    for (int64_t j = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; j < n; j += (int64_t)gridDim.x * blockDim.x) {
        const int v = ids[j];
        int s = 0;
        for (int k = 1; k < S; ++k) s += (g.off[k] <= j) ? 1 : 0;
        if (v < 0 || v >= n_vertices) { atomicOr(err, 1); continue; }
        if (pmap[v] != s) { atomicOr(err, 2); continue; }
        if (atomicCAS(&slot_of[v], -1, (int)j) != -1) atomicOr(err, 4);
    }
}

// rows[j, :] = table[ids[j], :] for j < n (cache fill), 16 bytes or one element per lane
template <typename VecT>
__global__ __launch_bounds__(256) void k_copy_rows(const uint8_t *__restrict__ table, int64_t row_stride_bytes,
                                                   int vec_per_row, const int32_t *__restrict__ ids, int64_t n,
                                                   int64_t n_vertices, VecT *__restrict__ out) {
    const int64_t total = n * vec_per_row;
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < total; x += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = x / vec_per_row;
        const int c = (int)(x - r * vec_per_row);
        const int64_t v = min((int64_t)max(ids[r], 0), n_vertices - 1);      // a bad id is reported by k_cache_set_slots
        out[x] = *reinterpret_cast<const VecT *>(table + v * row_stride_bytes + (int64_t)c * sizeof(VecT));
    }
}

// Loading step with the cache: row r of the input layer comes from cache row slot_of[id] when that
// is >= 0, else from the (host) table.  Same shape as the plain gather: consecutive lanes take
// consecutive 16-byte pieces, four independent loads per lane in flight; a miss simply has a longer
// latency (PCIe), which the other waves cover.
template <typename VecT, int UNROLL>
__global__ __launch_bounds__(256) void k_gather_cached(const uint8_t *__restrict__ table, int64_t row_stride_bytes,
                                                       const uint8_t *__restrict__ cache, int64_t row_bytes,
                                                       const int32_t *__restrict__ slot_of, int vec_per_row,
                                                       const int32_t *__restrict__ ids,
                                                       const GsLevelMeta *__restrict__ meta0, int S,
                                                       VecT *__restrict__ out, unsigned long long *__restrict__ hits,
                                                       unsigned long long *__restrict__ misses) {
    const int64_t n_rows = meta0->front_off[S];
    const int64_t total = n_rows * vec_per_row;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    auto source = [&](int64_t y) {
        const int64_t r = y / vec_per_row;
        const int c = (int)(y - r * vec_per_row);
        const int v = ids[r];
        const int slot = slot_of[v];
        const uint8_t *row = slot >= 0 ? cache + (int64_t)slot * row_bytes : table + (int64_t)v * row_stride_bytes;
        return reinterpret_cast<const VecT *>(row + (int64_t)c * sizeof(VecT));
    };
    int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    for (; x + (UNROLL - 1) * stride < total; x += UNROLL * stride) {
        const VecT *src[UNROLL];
        VecT v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) src[u] = source(x + u * stride);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = *src[u];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) out[x + u * stride] = v[u];
    }
    for (; x < total; x += stride) out[x] = *source(x);
    if (!hits && !misses) return;
    // hit / miss counts per split: one lane per row; the rows are ordered by split, so a wave nearly
    // always lies inside one split and adds its two ballot counts with one atomic each
    const int lane = threadIdx.x & 63;
    const int32_t *off = meta0->front_off;
    for (int64_t base = blockIdx.x * (int64_t)blockDim.x + (threadIdx.x - lane); base < n_rows; base += stride) {
        const int64_t r = base + lane;
        int s = -1;
        bool hit = false;
        if (r < n_rows) {
            s = 0;
            for (int k = 1; k < S; ++k) s += (off[k] <= r) ? 1 : 0;
            hit = slot_of[ids[r]] >= 0;
        }
        for (int k = 0; k < S; ++k) {
            const unsigned long long in_k = __ballot(s == k);
            if (in_k == 0ull) continue;
            const unsigned long long h = __ballot(s == k && hit);
            if (lane == 0) {
                const unsigned nh = (unsigned)__popcll(h), nm = (unsigned)__popcll(in_k) - nh;
                if (hits && nh) atomicAdd(&hits[k], (unsigned long long)nh);
                if (misses && nm) atomicAdd(&misses[k], (unsigned long long)nm);
            }
        }
    }
}

__global__ __launch_bounds__(256) void k_input_counts(const int32_t *__restrict__ ids, const GsLevelMeta *__restrict__ meta0,
                                                      int S, uint32_t *__restrict__ count) {
    const int64_t n = meta0->front_off[S];
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < n; x += (int64_t)gridDim.x * blockDim.x)
        atomicAdd(&count[ids[x]], 1u);
}

// the address under which the device reads `p`: device memory as it is, pinned host memory
// through its mapping; nullptr for memory the device cannot read
const void *device_view(const void *p) {
    hipPointerAttribute_t at;
    if (hipPointerGetAttributes(&at, p) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    if (at.type == hipMemoryTypeDevice || at.type == hipMemoryTypeHost || at.type == hipMemoryTypeManaged)
        return at.devicePointer ? at.devicePointer : p;
    return nullptr;
}

}  // namespace

extern "C" int gsplit_input_counts_accumulate(gsplit_ctx *ctx, uint32_t *d_count, void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    if (!d_count) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_input_counts_accumulate: NULL buffer");
    if (ctx->batch_id == 0) return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_input_counts_accumulate: no batch");
    hipStream_t st = (hipStream_t)stream;
    GsTimeScope ts(ctx, "input_counts", -1, st);
    hipLaunchKernelGGL(k_input_counts, dim3(grid_1d(ctx, ctx->ub_front[0])), dim3(256), 0, st, ctx->front[0], ctx->d_meta,
                       ctx->S, d_count);
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}

extern "C" int gsplit_cache_build(gsplit_ctx *ctx, const void *table, int32_t dtype, int64_t dim,
                                  int64_t row_stride_bytes, const int32_t *d_cache_ids, const int64_t *n_cache,
                                  void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    if (!table || !n_cache || dim <= 0 || (dtype != GSPLIT_F32 && dtype != GSPLIT_BF16))
        return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_cache_build: bad argument");
    const int64_t row_bytes = dim * (dtype == GSPLIT_F32 ? 4 : 2);
    if (row_stride_bytes < row_bytes) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_cache_build: row stride smaller than a row");
    GroupOff g{};
    for (int s = 0; s < ctx->S; ++s) {
        if (n_cache[s] < 0) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_cache_build: negative cache size");
        g.off[s + 1] = g.off[s] + n_cache[s];
    }
    const int64_t n = g.off[ctx->S];
    if (n > ctx->graph.n_vertices) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_cache_build: more cache rows than vertices");
    if (n > 0 && !d_cache_ids) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_cache_build: NULL id list");
    const void *tab = device_view(table);
    if (!tab)
        return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_cache_build: the table must be device memory or pinned host memory");
    GsFeatureCache &fc = ctx->cache;
    hipStream_t st = (hipStream_t)stream;
    // a second call replaces the cache
    fc.ready = false;
    gs_release(ctx, (void **)&fc.slot_of);
    gs_release(ctx, (void **)&fc.rows);
    int rc = gs_alloc(ctx, (void **)&fc.slot_of, sizeof(int32_t) * ctx->graph.n_vertices, "cache slot map");
    if (rc) return rc;
    rc = gs_alloc(ctx, (void **)&fc.rows, (size_t)std::max<int64_t>(n, 1) * row_bytes, "cache rows");
    if (rc) return rc;
    if (!fc.d_err) {
        rc = gs_alloc(ctx, (void **)&fc.d_err, sizeof(int32_t), "cache error flag");
        if (rc) return rc;
    }
    hipLaunchKernelGGL(k_fill_i32, dim3(grid_1d(ctx, ctx->graph.n_vertices)), dim3(256), 0, st, fc.slot_of,
                       ctx->graph.n_vertices, -1);
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(64), 0, st, fc.d_err, (int64_t)1, 0);
    if (n > 0) {
        hipLaunchKernelGGL(k_cache_set_slots, dim3(grid_1d(ctx, n)), dim3(256), 0, st, d_cache_ids, g, ctx->S,
                           (const uint8_t *)ctx->graph.d_pmap, ctx->graph.n_vertices, fc.slot_of, fc.d_err);
        const bool a16 = row_bytes % 16 == 0 && row_stride_bytes % 16 == 0 && aligned16(tab);
        const bool a4 = row_bytes % 4 == 0 && row_stride_bytes % 4 == 0 && ((uintptr_t)tab % 4) == 0;
        const int grid = grid_1d(ctx, n * gs_ceil_div(row_bytes, 16));
        if (a16)
            hipLaunchKernelGGL((k_copy_rows<u32x4>), dim3(grid), dim3(256), 0, st, (const uint8_t *)tab, row_stride_bytes,
                               (int)(row_bytes / 16), d_cache_ids, n, ctx->graph.n_vertices, (u32x4 *)fc.rows);
        else if (a4)
            hipLaunchKernelGGL((k_copy_rows<uint32_t>), dim3(grid), dim3(256), 0, st, (const uint8_t *)tab, row_stride_bytes,
                               (int)(row_bytes / 4), d_cache_ids, n, ctx->graph.n_vertices, (uint32_t *)fc.rows);
        else
            hipLaunchKernelGGL((k_copy_rows<uint16_t>), dim3(grid), dim3(256), 0, st, (const uint8_t *)tab, row_stride_bytes,
                               (int)(row_bytes / 2), d_cache_ids, n, ctx->graph.n_vertices, (uint16_t *)fc.rows);
    }
    GS_HIP(ctx, hipGetLastError());
    int32_t err = 0;
    GS_HIP(ctx, hipMemcpyAsync(&err, fc.d_err, sizeof(err), hipMemcpyDeviceToHost, st));
    GS_HIP(ctx, hipStreamSynchronize(st));
    if (err & 1) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_cache_build: a cache id lies outside the graph");
    if (err & 2) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_cache_build: a cache id is listed under a split that does not own it");
    if (err & 4) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_cache_build: a cache id is listed twice");
    fc.table = tab; fc.dtype = dtype; fc.dim = dim; fc.row_stride_bytes = row_stride_bytes; fc.n_rows = n;
    fc.ready = true;
    return GSPLIT_OK;
}

extern "C" int gsplit_gather_features_cached(gsplit_ctx *ctx, void *d_out, uint64_t *d_hits, uint64_t *d_misses,
                                             void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    if (!d_out) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_gather_features_cached: NULL buffer");
    const GsFeatureCache &fc = ctx->cache;
    if (!fc.ready) return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_gather_features_cached: no cache (gsplit_cache_build)");
    if (ctx->batch_id == 0) return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_gather_features_cached: no batch");
    hipStream_t st = (hipStream_t)stream;
    const int64_t row_bytes = fc.dim * (fc.dtype == GSPLIT_F32 ? 4 : 2);
    const int64_t ub_rows = ctx->ub_front[0];
    const int grid = (int)std::min<int64_t>((int64_t)ctx->n_cu * 32,
                                            std::max<int64_t>(1, gs_ceil_div(ub_rows * gs_ceil_div(row_bytes, 16), 256 * 4)));
    const bool a16 = row_bytes % 16 == 0 && fc.row_stride_bytes % 16 == 0 && aligned16(fc.table) && aligned16(d_out);
    const bool a4 = row_bytes % 4 == 0 && fc.row_stride_bytes % 4 == 0 && ((uintptr_t)fc.table % 4) == 0 &&
                    ((uintptr_t)d_out % 4) == 0;
    unsigned long long *h = (unsigned long long *)d_hits, *m = (unsigned long long *)d_misses;
    GsTimeScope ts(ctx, "gather_cached", -1, st);
    if (a16)
        hipLaunchKernelGGL((k_gather_cached<u32x4, 4>), dim3(grid), dim3(256), 0, st, (const uint8_t *)fc.table,
                           fc.row_stride_bytes, (const uint8_t *)fc.rows, row_bytes, fc.slot_of, (int)(row_bytes / 16),
                           ctx->front[0], ctx->d_meta, ctx->S, (u32x4 *)d_out, h, m);
    else if (a4)
        hipLaunchKernelGGL((k_gather_cached<uint32_t, 4>), dim3(grid), dim3(256), 0, st, (const uint8_t *)fc.table,
                           fc.row_stride_bytes, (const uint8_t *)fc.rows, row_bytes, fc.slot_of, (int)(row_bytes / 4),
                           ctx->front[0], ctx->d_meta, ctx->S, (uint32_t *)d_out, h, m);
    else
        hipLaunchKernelGGL((k_gather_cached<uint16_t, 4>), dim3(grid), dim3(256), 0, st, (const uint8_t *)fc.table,
                           fc.row_stride_bytes, (const uint8_t *)fc.rows, row_bytes, fc.slot_of, (int)(row_bytes / 2),
                           ctx->front[0], ctx->d_meta, ctx->S, (uint16_t *)d_out, h, m);
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}
