// Loading step (paper section 3): copy the feature rows of the layer-0 local frontiers from the
// HBM-resident table into a dense buffer, splits concatenated.  No arithmetic: the kernel is a
// pure HBM stream (random 256..512-byte row reads, fully coalesced writes), so it moves 16 bytes
// per lane and keeps several independent loads in flight per lane.
#include <algorithm>

#include "gsplit_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <typename VecT, int UNROLL>
__global__ __launch_bounds__(256) void k_gather_rows(const uint8_t *__restrict__ table,
                                                     int64_t row_stride_bytes, int vec_per_row,
                                                     const int32_t *__restrict__ ids,
                                                     const GsLevelMeta *__restrict__ meta0, int S,
                                                     VecT *__restrict__ out) {
    const int64_t n_rows = meta0->front_off[S];
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
    for (int64_t x = x0; x < total; x += UNROLL * stride) {
        int64_t off[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t y = x + u * stride < total ? x + u * stride : x;
            const int64_t r = y / vec_per_row;
            const int c = (int)(y - r * vec_per_row);
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

}  // namespace

extern "C" int gsplit_gather_features(gsplit_ctx *ctx, const void *d_table, int32_t dtype, int64_t dim,
                                      int64_t row_stride_bytes, void *d_out, void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    if (!d_table || !d_out || dim <= 0 || (dtype != GSPLIT_F32 && dtype != GSPLIT_BF16))
        return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_gather_features: bad argument");
    if (ctx->batch_id == 0) return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_gather_features: no batch");
    const int64_t row_bytes = dim * (dtype == GSPLIT_F32 ? 4 : 2);
    if (row_stride_bytes < row_bytes)
        return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_gather_features: row stride smaller than a row");
    hipStream_t st = (hipStream_t)stream;
    const int64_t ub_rows = ctx->ub_front[0];
    const GsLevelMeta *m0 = ctx->d_meta;
    const int grid = (int)std::min<int64_t>((int64_t)ctx->n_cu * 32,
                                            std::max<int64_t>(1, gs_ceil_div(ub_rows * gs_ceil_div(row_bytes, 16), 256 * 4)));
    const bool a16 = row_bytes % 16 == 0 && row_stride_bytes % 16 == 0 &&
                     ((uintptr_t)d_table % 16) == 0 && ((uintptr_t)d_out % 16) == 0;
    const bool a4 = row_bytes % 4 == 0 && row_stride_bytes % 4 == 0 && ((uintptr_t)d_table % 4) == 0 &&
                    ((uintptr_t)d_out % 4) == 0;
    GsTimeScope ts(ctx, "gather_rows", -1, st);
    if (a16) {
        hipLaunchKernelGGL((k_gather_rows<u32x4, 4>), dim3(grid), dim3(256), 0, st,
                           (const uint8_t *)d_table, row_stride_bytes, (int)(row_bytes / 16),
                           ctx->front[0], m0, ctx->S, (u32x4 *)d_out);
    } else if (a4) {
        hipLaunchKernelGGL((k_gather_rows<uint32_t, 4>), dim3(grid), dim3(256), 0, st,
                           (const uint8_t *)d_table, row_stride_bytes, (int)(row_bytes / 4),
                           ctx->front[0], m0, ctx->S, (uint32_t *)d_out);
    } else {
        hipLaunchKernelGGL((k_gather_rows<uint16_t, 4>), dim3(grid), dim3(256), 0, st,
                           (const uint8_t *)d_table, row_stride_bytes, (int)(row_bytes / 2),
                           ctx->front[0], m0, ctx->S, (uint16_t *)d_out);
    }
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}
