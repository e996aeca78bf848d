// Loading step (paper section 3): copy the feature rows of the layer-0 local frontiers from the
// HBM-resident table into a dense buffer, splits concatenated.  No arithmetic: the kernel is a
// pure HBM stream (random 256..512-byte row reads, fully coalesced writes), so it moves 16 bytes
// per lane and keeps several independent loads in flight per lane.
#include <algorithm>
#include <string>

#include "gsplit_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// one set of pointers per mini-batch of the launch (blockIdx.y = batch)
struct GatherOne { const int32_t *ids; const GsLevelMeta *meta0; void *out; };
struct GatherSet { GatherOne b[GSPLIT_MAX_MULTI]; };

template <typename VecT, int UNROLL>
__global__ __launch_bounds__(256) void k_gather_rows(const uint8_t *__restrict__ table,
                                                     int64_t row_stride_bytes, int vec_per_row,
                                                     GatherSet set, int S) {
    const int32_t *__restrict__ ids = set.b[blockIdx.y].ids;
    VecT *__restrict__ out = reinterpret_cast<VecT *>(set.b[blockIdx.y].out);
    const int64_t n_rows = set.b[blockIdx.y].meta0->front_off[S];
    const int64_t total = n_rows * vec_per_row;
    // The launch is sized from an upper bound on the rows, several times the real count.  Only as
    // many threads work as give each of them at least two pieces (the others leave at once), and
    // every round of UNROLL is complete: a piece past the end re-reads the thread's first piece (a
    // valid address) and is not stored.  So a thread fetches the ids of a round together and then
    // its rows, instead of running id -> row round trips one after the other.  (UNROLL pieces for
    // every working thread, i.e. fewer threads still, was slower for 400-byte rows.)
    const int64_t launched = (int64_t)gridDim.x * blockDim.x;
    const int64_t want = ((total + 1) / 2 + 255) & ~(int64_t)255;
    const int64_t stride = want < launched ? want : launched;
    const int64_t x0 = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (x0 >= stride) return;
    const bool narrow = total < (1ll << 31);        // (a 64-bit division costs several times a 32-bit one)
    for (int64_t x = x0; x < total; x += UNROLL * stride) {
        int64_t off[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t y = x + u * stride < total ? x + u * stride : x;
            int64_t r;
            int c;
            if (narrow) {
                const uint32_t r32 = (uint32_t)y / (uint32_t)vec_per_row;
                r = r32;
                c = (int)((uint32_t)y - r32 * (uint32_t)vec_per_row);
            } else {
                r = y / vec_per_row;
                c = (int)(y - r * vec_per_row);
            }
            off[u] = (int64_t)ids[r] * row_stride_bytes + (int64_t)c * sizeof(VecT);
        }
        VecT v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = *reinterpret_cast<const VecT *>(table + off[u]);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            if (x + u * stride < total) out[x + u * stride] = v[u];
    }
}

// the loading step of nbat contexts (same graph and configuration) in one launch
int gather_rows(gsplit_ctx *const *ctxs, int nbat, const void *d_table, int32_t dtype, int64_t dim,
                int64_t row_stride_bytes, void *const *d_outs, hipStream_t st, const char *who) {
    gsplit_ctx *ctx = ctxs[0];
    if (!d_table || dim <= 0 || (dtype != GSPLIT_F32 && dtype != GSPLIT_BF16))
        return gs_fail(ctx, GSPLIT_EINVAL, std::string(who) + ": bad argument");
    const int64_t row_bytes = dim * (dtype == GSPLIT_F32 ? 4 : 2);
    if (row_stride_bytes < row_bytes)
        return gs_fail(ctx, GSPLIT_EINVAL, std::string(who) + ": row stride smaller than a row");
    bool a16 = row_bytes % 16 == 0 && row_stride_bytes % 16 == 0 && ((uintptr_t)d_table % 16) == 0;
    bool a4 = row_bytes % 4 == 0 && row_stride_bytes % 4 == 0 && ((uintptr_t)d_table % 4) == 0;
    GatherSet set{};
    for (int b = 0; b < nbat; ++b) {
        gsplit_ctx *c = ctxs[b];
        if (!d_outs[b]) return gs_fail(ctx, GSPLIT_EINVAL, std::string(who) + ": NULL output");
        if (c->batch_id == 0) return gs_fail(ctx, GSPLIT_ESTATE, std::string(who) + ": no batch");
        a16 = a16 && ((uintptr_t)d_outs[b] % 16) == 0;
        a4 = a4 && ((uintptr_t)d_outs[b] % 4) == 0;
        set.b[b] = GatherOne{c->front[0], c->d_meta, d_outs[b]};
    }
    const int64_t ub_rows = ctx->ub_front[0];
    const int grid = (int)std::min<int64_t>(std::max<int64_t>(1, (int64_t)ctx->n_cu * 32 / nbat),
                                            std::max<int64_t>(1, gs_ceil_div(ub_rows * gs_ceil_div(row_bytes, 16), 256 * 4)));
    GsTimeScope ts(ctx, "gather_rows", -1, st);
    if (a16) {
        hipLaunchKernelGGL((k_gather_rows<u32x4, 4>), dim3(grid, nbat), dim3(256), 0, st, (const uint8_t *)d_table,
                           row_stride_bytes, (int)(row_bytes / 16), set, ctx->S);
    } else if (a4) {
        hipLaunchKernelGGL((k_gather_rows<uint32_t, 4>), dim3(grid, nbat), dim3(256), 0, st, (const uint8_t *)d_table,
                           row_stride_bytes, (int)(row_bytes / 4), set, ctx->S);
    } else {
        hipLaunchKernelGGL((k_gather_rows<uint16_t, 4>), dim3(grid, nbat), dim3(256), 0, st, (const uint8_t *)d_table,
                           row_stride_bytes, (int)(row_bytes / 2), set, ctx->S);
    }
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}

}  // namespace

extern "C" int gsplit_gather_features(gsplit_ctx *ctx, const void *d_table, int32_t dtype, int64_t dim,
                                      int64_t row_stride_bytes, void *d_out, void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    if (!d_out) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_gather_features: bad argument");
    return gather_rows(&ctx, 1, d_table, dtype, dim, row_stride_bytes, &d_out, (hipStream_t)stream,
                       "gsplit_gather_features");
}

extern "C" int gsplit_gather_features_multi(gsplit_ctx *const *ctxs, int32_t n_batches, const void *d_table,
                                            int32_t dtype, int64_t dim, int64_t row_stride_bytes,
                                            void *const *d_outs, void *stream) {
    if (!ctxs || n_batches < 1 || !ctxs[0]) return GSPLIT_EINVAL;
    gsplit_ctx *first = ctxs[0];
    if (n_batches > GSPLIT_MAX_MULTI || !d_outs)
        return gs_fail(first, GSPLIT_EINVAL, "gsplit_gather_features_multi: between 1 and GSPLIT_MAX_MULTI batches");
    for (int b = 1; b < n_batches; ++b) {
        const gsplit_ctx *c = ctxs[b];
        if (!c || c->S != first->S || c->ub_front[0] != first->ub_front[0] || c->graph.n_vertices != first->graph.n_vertices)
            return gs_fail(first, GSPLIT_EINVAL, "gsplit_gather_features_multi: contexts of one graph and configuration");
    }
    return gather_rows(ctxs, n_batches, d_table, dtype, dim, row_stride_bytes, d_outs, (hipStream_t)stream,
                       "gsplit_gather_features_multi");
}
