// Split statistics of the current batch (paper section 7.3): per sampling layer and split, the
// edges the split computes and how many of them are cross edges (source owned by another split).
// The paper's two partitioning figures follow on the host: workload imbalance = max over splits of
// the edges at layers l > 0 over their average; communication cost = cross edges / all edges.
// Pure counting over the sampled slots (coalesced), one launch for all layers.
#include <algorithm>

#include "gsplit_internal.h"

namespace {

struct StatsArgs {
    const int32_t *nbr[GS_MAXL]; const int32_t *cnt[GS_MAXL];
    int fan[GS_MAXL];
    int L, S;
};

__global__ __launch_bounds__(256) void k_batch_stats(StatsArgs a, const uint8_t *__restrict__ pmap,
                                                     const GsLevelMeta *__restrict__ meta,
                                                     unsigned long long *__restrict__ edges,
                                                     unsigned long long *__restrict__ cross) {
    __shared__ unsigned s_e[GS_MAXS], s_c[GS_MAXS];
    const int l = blockIdx.y, S = a.S, fan = a.fan[l];
    if (threadIdx.x < GS_MAXS) s_e[threadIdx.x] = s_c[threadIdx.x] = 0u;
    __syncthreads();
    const int32_t *off = meta[l + 1].front_off;
    const int64_t n = (int64_t)off[S] * fan;
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < n; x += (int64_t)gridDim.x * blockDim.x) {
        const int i = (int)(x / fan), q = (int)(x - (int64_t)i * fan);
        if (q >= a.cnt[l][i]) continue;
        int s = 0;
        for (int k = 1; k < S; ++k) s += (off[k] <= i) ? 1 : 0;
        atomicAdd(&s_e[s], 1u);
        if (pmap[a.nbr[l][x]] != s) atomicAdd(&s_c[s], 1u);
    }
    __syncthreads();
    if ((int)threadIdx.x < S) {
        if (s_e[threadIdx.x]) atomicAdd(&edges[l * S + threadIdx.x], (unsigned long long)s_e[threadIdx.x]);
        if (s_c[threadIdx.x]) atomicAdd(&cross[l * S + threadIdx.x], (unsigned long long)s_c[threadIdx.x]);
    }
}

}  // namespace

extern "C" int gsplit_batch_stats(gsplit_ctx *ctx, uint64_t *d_edges, uint64_t *d_cross_edges, void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    if (!d_edges || !d_cross_edges) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_batch_stats: NULL buffer");
    if (ctx->batch_id == 0) return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_batch_stats: no batch");
    hipStream_t st = (hipStream_t)stream;
    StatsArgs a{};
    a.L = ctx->L; a.S = ctx->S;
    int64_t ub = 1;
    for (int l = 0; l < ctx->L; ++l) {
        a.nbr[l] = ctx->layer[l].nbr; a.cnt[l] = ctx->layer[l].cnt; a.fan[l] = ctx->fan[l];
        ub = std::max<int64_t>(ub, ctx->ub_front[l + 1] * ctx->fan[l]);
    }
    const unsigned gx = (unsigned)std::max<int64_t>(1, std::min<int64_t>((int64_t)ctx->n_cu * 8, gs_ceil_div(ub, 256)));
    GsTimeScope ts(ctx, "batch_stats", -1, st);
    hipLaunchKernelGGL(k_batch_stats, dim3(gx, ctx->L), dim3(256), 0, st, a, (const uint8_t *)ctx->graph.d_pmap,
                       ctx->d_meta, (unsigned long long *)d_edges, (unsigned long long *)d_cross_edges);
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}
