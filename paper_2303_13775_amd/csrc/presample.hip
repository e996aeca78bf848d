// Offline pre-sampling (paper section 4, "pre-sampling" stage): the training sampler is run for a
// number of epochs and every vertex and edge is weighted by how often it is sampled,
// w_V(v) = k_v / N, w_E(e) = k_e / N.  This file adds one sampled batch to the running counts
// k_v (appearances of v at a level l > 0) and k_e (times CSR edge e was sampled, any layer), and
// turns counts into weights.  Pure counting: 32-bit atomic increments, one launch for all levels.
#include <algorithm>

#include "gsplit_internal.h"

namespace {

struct PresampleArgs {
    const int32_t *front[GS_MAXL + 1];      // local_cat of every level
    const int64_t *epos[GS_MAXL];           // CSR position behind every slot of every sampling layer
    int fan[GS_MAXL];
    int L, S;
};

// blockIdx.y < L     : vertices of level blockIdx.y + 1 (the frontiers are duplicate-free across
//                      splits: a vertex is local to exactly one split)
// blockIdx.y >= L    : slots of sampling layer blockIdx.y - L
__global__ __launch_bounds__(256) void k_presample_accumulate(PresampleArgs a, const GsLevelMeta *__restrict__ meta,
                                                              uint32_t *__restrict__ k_v, uint32_t *__restrict__ k_e) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t x0 = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if ((int)blockIdx.y < a.L) {
        if (!k_v) return;
        const int level = blockIdx.y + 1;
        const int64_t n = meta[level].front_off[a.S];
        const int32_t *ids = a.front[level];
        for (int64_t x = x0; x < n; x += stride) atomicAdd(&k_v[ids[x]], 1u);
    } else {
        if (!k_e) return;
        const int l = blockIdx.y - a.L;
        const int64_t n = (int64_t)meta[l + 1].front_off[a.S] * a.fan[l];
        const int64_t *pos = a.epos[l];
        for (int64_t x = x0; x < n; x += stride) {
            const int64_t e = pos[x];
            if (e >= 0) atomicAdd(&k_e[e], 1u);
        }
    }
}

__global__ __launch_bounds__(256) void k_presample_weights(const uint32_t *__restrict__ count, int64_t n,
                                                           float inv_samples, float *__restrict__ w) {
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < n; x += (int64_t)gridDim.x * blockDim.x)
        w[x] = (float)count[x] * inv_samples;
}

}  // namespace

extern "C" int gsplit_presample_accumulate(gsplit_ctx *ctx, uint32_t *d_vertex_count, uint32_t *d_edge_count,
                                           void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    if (ctx->batch_id == 0) return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_presample_accumulate: no batch");
    if (d_edge_count && !ctx->keep_edge_ids)
        return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_presample_accumulate: context was created without keep_edge_ids");
    if (!d_vertex_count && !d_edge_count) return GSPLIT_OK;
    hipStream_t st = (hipStream_t)stream;
    PresampleArgs a{};
    a.L = ctx->L; a.S = ctx->S;
    int64_t ub = 1;
    for (int l = 0; l <= ctx->L; ++l) a.front[l] = ctx->front[l];
    for (int l = 0; l < ctx->L; ++l) {
        a.epos[l] = ctx->layer[l].epos;
        a.fan[l] = ctx->fan[l];
        ub = std::max<int64_t>(ub, ctx->ub_front[l + 1] * ctx->fan[l]);
    }
    const unsigned gx = (unsigned)std::max<int64_t>(1, std::min<int64_t>((int64_t)ctx->n_cu * 8, gs_ceil_div(ub, 256)));
    GsTimeScope ts(ctx, "presample_accumulate", -1, st);
    hipLaunchKernelGGL(k_presample_accumulate, dim3(gx, 2 * ctx->L), dim3(256), 0, st, a, ctx->d_meta,
                       d_vertex_count, d_edge_count);
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}

extern "C" int gsplit_presample_weights(gsplit_ctx *ctx, const uint32_t *d_count, int64_t n, int64_t n_samples,
                                        float *d_weight, void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    if (!d_count || !d_weight || n < 0 || n_samples < 1)
        return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_presample_weights: bad argument");
    if (n == 0) return GSPLIT_OK;
    hipStream_t st = (hipStream_t)stream;
    const unsigned gx = (unsigned)std::max<int64_t>(1, std::min<int64_t>((int64_t)ctx->n_cu * 8, gs_ceil_div(n, 256)));
    GsTimeScope ts(ctx, "presample_weights", -1, st);
    hipLaunchKernelGGL(k_presample_weights, dim3(gx), dim3(256), 0, st, d_count, n, 1.0f / (float)n_samples, d_weight);
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}
