// Split statistics of the current batch (paper section 7.3): per sampling layer and split, the
// edges the split computes and how many of them are cross edges (source owned by another split).
// The paper's two partitioning figures follow on the host: workload imbalance = max over splits of
// the edges at layers l > 0 over their average; communication cost = cross edges / all edges.
// Pure counting, one launch for all layers.
#include <algorithm>

#include "gsplit_internal.h"

namespace {

struct StatsArgs {
    const int32_t *nbr[GS_MAXL]; const int32_t *cnt[GS_MAXL];
    int fan[GS_MAXL];
    int L, S;
};

// One lane per destination vertex (its sampled neighbours are `cnt` consecutive ids).  The rows of
// a level are ordered by split, so a wave nearly always sits inside one split: its counts are then
// summed across the wave and added once to the workgroup's LDS counters, which go out as one
// global atomic per workgroup and counter (atomics on one address are served one at a time).
__global__ __launch_bounds__(256) void k_batch_stats(StatsArgs a, const uint8_t *__restrict__ pmap,
                                                     const GsLevelMeta *__restrict__ meta,
                                                     unsigned long long *__restrict__ edges,
                                                     unsigned long long *__restrict__ cross) {
    __shared__ unsigned s_e[GS_MAXS], s_c[GS_MAXS];
    const int l = blockIdx.y, S = a.S, fan = a.fan[l];
    const int32_t *__restrict__ nbr = a.nbr[l];
    const int32_t *__restrict__ cnt = a.cnt[l];
    const int32_t *off = meta[l + 1].front_off;
    const int n1 = off[S];
    const int lane = threadIdx.x & 63;
    if (threadIdx.x < GS_MAXS) s_e[threadIdx.x] = s_c[threadIdx.x] = 0u;
    __syncthreads();
    for (int base = blockIdx.x * 256 + (threadIdx.x - lane); base < n1; base += gridDim.x * 256) {
        const int i = base + lane;
        int s = -1;
        unsigned ne = 0u, nc = 0u;
        if (i < n1) {
            s = 0;
            for (int k = 1; k < S; ++k) s += (off[k] <= i) ? 1 : 0;
            ne = (unsigned)cnt[i];
            const int32_t *row = nbr + (int64_t)i * fan;
            unsigned q = 0;
            for (; q + 4 <= ne; q += 4) {
                const int v0 = row[q], v1 = row[q + 1], v2 = row[q + 2], v3 = row[q + 3];
                const int o0 = pmap[v0], o1 = pmap[v1], o2 = pmap[v2], o3 = pmap[v3];
                nc += (o0 != s) + (o1 != s) + (o2 != s) + (o3 != s);
            }
            for (; q < ne; ++q) nc += pmap[row[q]] != s;
        }
        const int s0 = __builtin_amdgcn_readfirstlane(s);       // lane 0 holds the wave's lowest row
        if (__ballot(s >= 0 && s != s0) == 0ull) {
            for (int o = 32; o > 0; o >>= 1) { ne += __shfl_xor(ne, o); nc += __shfl_xor(nc, o); }
            if (lane == 0 && s0 >= 0) {
                if (ne) atomicAdd(&s_e[s0], ne);
                if (nc) atomicAdd(&s_c[s0], nc);
            }
        } else if (s >= 0) {
            if (ne) atomicAdd(&s_e[s], ne);
            if (nc) atomicAdd(&s_c[s], nc);
        }
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
        ub = std::max<int64_t>(ub, ctx->ub_front[l + 1]);
    }
    const unsigned gx = (unsigned)std::max<int64_t>(1, std::min<int64_t>((int64_t)ctx->n_cu * 4, gs_ceil_div(ub, 256)));
    GsTimeScope ts(ctx, "batch_stats", -1, st);
    hipLaunchKernelGGL(k_batch_stats, dim3(gx, ctx->L), dim3(256), 0, st, a, (const uint8_t *)ctx->graph.d_pmap,
                       ctx->d_meta, (unsigned long long *)d_edges, (unsigned long long *)d_cross_edges);
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}
