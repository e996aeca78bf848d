// GraphSAGE-mean forward and backward over the split mini-batch (paper Algorithm 2 `sp_forward`
// and the backward description after it).  The rows of all S logical splits are processed in one
// launch per step: on one GPU the training shuffle of layer l is the composition of the shuffle
// index with edges[l] (self_row / edge_row, built during sampling), so "shuffle then aggregate"
// is a gather through one index and the reverse shuffle of the backward pass is a scatter-add
// through the same index.
//
// Dense products run on the matrix cores: v_mfma_f32_32x32x2_f32 for fp32 storage.
#include <algorithm>

#include "gsplit_internal.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;

// ------------------------------------------------------------------------------------------
// mean aggregation: M[i,:] = (1/cnt_i) * sum_e H[edge_row[e],:], one lane group per destination
// row, 4 floats per lane, edges in slot order (deterministic), four row loads in flight.
// ------------------------------------------------------------------------------------------
template <int LPR>
__global__ __launch_bounds__(256) void k_mean_aggregate_f32(const float *__restrict__ H, int D,
                                                            const int32_t *__restrict__ blk_indptr,
                                                            const int32_t *__restrict__ edge_row,
                                                            const GsLevelMeta *__restrict__ meta_up,
                                                            int S, float *__restrict__ M) {
    const int n1 = meta_up->front_off[S];
    const int nvec = D >> 2;
    const int c0 = threadIdx.x % LPR;
    const int groups = (gridDim.x * blockDim.x) / LPR;
    const float4 *H4 = reinterpret_cast<const float4 *>(H);
    float4 *M4 = reinterpret_cast<float4 *>(M);
    for (int row = (blockIdx.x * blockDim.x + threadIdx.x) / LPR; row < n1; row += groups) {
        const int e0 = blk_indptr[row], e1 = blk_indptr[row + 1];
        const float cnt = (float)(e1 - e0);
        for (int c = c0; c < nvec; c += LPR) {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            int e = e0;
            for (; e + 4 <= e1; e += 4) {
                const int r0 = edge_row[e], r1 = edge_row[e + 1], r2 = edge_row[e + 2], r3 = edge_row[e + 3];
                const float4 a = H4[(int64_t)r0 * nvec + c], b = H4[(int64_t)r1 * nvec + c];
                const float4 g = H4[(int64_t)r2 * nvec + c], h = H4[(int64_t)r3 * nvec + c];
                acc.x += a.x; acc.y += a.y; acc.z += a.z; acc.w += a.w;
                acc.x += b.x; acc.y += b.y; acc.z += b.z; acc.w += b.w;
                acc.x += g.x; acc.y += g.y; acc.z += g.z; acc.w += g.w;
                acc.x += h.x; acc.y += h.y; acc.z += h.z; acc.w += h.w;
            }
            for (; e < e1; ++e) {
                const float4 a = H4[(int64_t)edge_row[e] * nvec + c];
                acc.x += a.x; acc.y += a.y; acc.z += a.z; acc.w += a.w;
            }
            if (e1 > e0) { acc.x /= cnt; acc.y /= cnt; acc.z /= cnt; acc.w /= cnt; }
            M4[(int64_t)row * nvec + c] = acc;
        }
    }
}

// scalar variant for widths that are not a multiple of 4
__global__ __launch_bounds__(256) void k_mean_aggregate_f32_any(const float *__restrict__ H, int D,
                                                                const int32_t *__restrict__ blk_indptr,
                                                                const int32_t *__restrict__ edge_row,
                                                                const GsLevelMeta *__restrict__ meta_up,
                                                                int S, float *__restrict__ M) {
    const int n1 = meta_up->front_off[S];
    const int lane = threadIdx.x & 63;
    const int waves = (gridDim.x * blockDim.x) >> 6;
    for (int row = (blockIdx.x * blockDim.x + threadIdx.x) >> 6; row < n1; row += waves) {
        const int e0 = blk_indptr[row], e1 = blk_indptr[row + 1];
        for (int c = lane; c < D; c += 64) {
            float acc = 0.f;
            for (int e = e0; e < e1; ++e) acc += H[(int64_t)edge_row[e] * D + c];
            if (e1 > e0) acc /= (float)(e1 - e0);
            M[(int64_t)row * D + c] = acc;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Tiled MFMA GEMM core.  C[M x N] = A[M x K] * B[K x N] with element functors:
//   a(m, k), b(k, n) return the operand element (0 outside the logical matrix);
//   epi(m, n, value) consumes one result element.
// Workgroup = 4 waves arranged 2 x 2 over a BM x BN tile; every wave owns (BM/2) x (BN/2) outputs
// as 32 x 32 MFMA blocks.  Tiles are staged k-major in LDS so that the 32 lanes of an MFMA operand
// read 32 consecutive words.  A_KCONTIG / B_KCONTIG say which index runs along memory, so that the
// staging loads are coalesced.
// ------------------------------------------------------------------------------------------
template <int BM, int BN, bool A_KCONTIG, bool B_KCONTIG, class AF, class BF, class EF>
__device__ __forceinline__ void gemm_tile(const int m0, const int n0, const int k_begin, const int k_end,
                                          const AF &a, const BF &b, const EF &epi) {
    constexpr int PAD = 4;
    __shared__ float As[BK][BM + PAD];
    __shared__ float Bs[BK][BN + PAD];
    constexpr int MI = BM / 64, NI = BN / 64;     // 32x32 blocks per wave in each direction
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);
    floatx16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    for (int k0 = k_begin; k0 < k_end; k0 += BK) {
        // stage A
        if (A_KCONTIG) {
#pragma unroll
            for (int r = 0; r < (BM * BK) / 256; ++r) {
                const int kk = tid % BK, mm = tid / BK + r * (256 / BK);
                As[kk][mm] = (k0 + kk < k_end) ? a(m0 + mm, k0 + kk) : 0.f;
            }
        } else {
#pragma unroll
            for (int r = 0; r < (BM * BK) / 256; ++r) {
                const int mm = tid % BM, kk = tid / BM + r * (256 / BM);
                As[kk][mm] = (k0 + kk < k_end) ? a(m0 + mm, k0 + kk) : 0.f;
            }
        }
        if (B_KCONTIG) {
#pragma unroll
            for (int r = 0; r < (BN * BK) / 256; ++r) {
                const int kk = tid % BK, nn = tid / BK + r * (256 / BK);
                Bs[kk][nn] = (k0 + kk < k_end) ? b(k0 + kk, n0 + nn) : 0.f;
            }
        } else {
#pragma unroll
            for (int r = 0; r < (BN * BK) / 256; ++r) {
                const int nn = tid % BN, kk = tid / BN + r * (256 / BN);
                Bs[kk][nn] = (k0 + kk < k_end) ? b(k0 + kk, n0 + nn) : 0.f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float av[MI], bv[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) av[i] = As[kk + (lane >> 5)][wm0 + i * 32 + (lane & 31)];
#pragma unroll
            for (int j = 0; j < NI; ++j) bv[j] = Bs[kk + (lane >> 5)][wn0 + j * 32 + (lane & 31)];
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }
    // accumulator layout of the 32x32 block: register r of lane l holds
    // row (r / 4) * 8 + (l / 32) * 4 + (r % 4), column l % 32
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                const int n = n0 + wn0 + j * 32 + (lane & 31);
                epi(m, n, acc[i][j][r]);
            }
}

// ---- operand and epilogue functors ---------------------------------------------------------
// [H_l[self] | mean] : the K = 2 * D input of a layer, row i of the destination list
struct CatIn {
    const float *H; const float *Mb; const int32_t *self_row; int D; int n1;
    __device__ __forceinline__ float operator()(int i, int c) const {
        if (i >= n1) return 0.f;
        if (c < D) return H[(int64_t)self_row[i] * D + c];
        if (c < 2 * D) return Mb[(int64_t)i * D + (c - D)];
        return 0.f;
    }
};
// same, transposed access (feature c, row i), plus a row of ones at c == 2 * D (bias gradient)
struct CatInT {
    CatIn in;
    __device__ __forceinline__ float operator()(int c, int i) const {
        if (c == 2 * in.D) return i < in.n1 ? 1.f : 0.f;
        return in(i, c);
    }
};
// [W_self; W_neigh] stacked along K
struct CatW {
    const float *Ws; const float *Wn; int D; int N;
    __device__ __forceinline__ float operator()(int k, int n) const {
        if (n >= N) return 0.f;
        if (k < D) return Ws[(int64_t)k * N + n];
        if (k < 2 * D) return Wn[(int64_t)(k - D) * N + n];
        return 0.f;
    }
};
struct CatWT {   // (n, j) -> stacked weight element (j, n)
    CatW w;
    __device__ __forceinline__ float operator()(int n, int j) const { return w(j, n); }
};
// dZ = dH' masked by the ReLU of the forward output (no mask on the last layer)
struct GradZ {
    const float *dH; const float *Hout; int N; int n1; int masked;
    __device__ __forceinline__ float operator()(int i, int n) const {
        if (i >= n1 || n >= N) return 0.f;
        const int64_t x = (int64_t)i * N + n;
        const float g = dH[x];
        return (!masked || Hout[x] > 0.f) ? g : 0.f;
    }
};
struct EpiFwd {
    float *out; const float *bias; int N; int n1; int relu;
    __device__ __forceinline__ void operator()(int m, int n, float v) const {
        if (m < n1 && n < N) {
            float z = v + bias[n];
            out[(int64_t)m * N + n] = (relu && z < 0.f) ? 0.f : z;
        }
    }
};
struct EpiGradW {
    float *gws; float *gwn; float *gb; int D; int N;
    __device__ __forceinline__ void operator()(int c, int n, float v) const {
        if (n >= N || c > 2 * D) return;
        if (c < D) atomicAdd(&gws[(int64_t)c * N + n], v);
        else if (c < 2 * D) atomicAdd(&gwn[(int64_t)(c - D) * N + n], v);
        else atomicAdd(&gb[n], v);
    }
};
// input gradients: the self part goes to the destination's own lower-layer row, the mean part is
// spread over the row's sampled sources (adjoint of the mean), both through the composed
// shuffle index -- the reverse shuffle of the backward pass.
struct EpiGradIn {
    float *g; const int32_t *self_row; const int32_t *edge_row; const int32_t *blk_indptr; int D; int n1;
    __device__ __forceinline__ void operator()(int i, int j, float v) const {
        if (i >= n1 || j >= 2 * D) return;
        if (j < D) { atomicAdd(&g[(int64_t)self_row[i] * D + j], v); return; }
        const int e0 = blk_indptr[i], e1 = blk_indptr[i + 1];
        if (e1 == e0) return;
        const float w = v / (float)(e1 - e0);
        for (int e = e0; e < e1; ++e) atomicAdd(&g[(int64_t)edge_row[e] * D + (j - D)], w);
    }
};

template <int BM, int BN>
__global__ __launch_bounds__(256) void k_sage_linear_fwd(CatIn a, CatW b, EpiFwd epi,
                                                         const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int m0 = blockIdx.x * BM;
    if (m0 >= n1) return;
    a.n1 = n1; epi.n1 = n1;
    gemm_tile<BM, BN, true, false>(m0, blockIdx.y * BN, 0, 2 * a.D, a, b, epi);
}

template <int BM, int BN>
__global__ __launch_bounds__(256) void k_sage_grad_w(CatInT a, GradZ b, EpiGradW epi, int kchunk,
                                                     const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int k_begin = blockIdx.z * kchunk;
    if (k_begin >= n1) return;
    a.in.n1 = n1; b.n1 = n1;
    const int k_end = min(n1, k_begin + kchunk);
    gemm_tile<BM, BN, false, false>(blockIdx.x * BM, blockIdx.y * BN, k_begin, k_end, a, b, epi);
}

template <int BM, int BN>
__global__ __launch_bounds__(256) void k_sage_grad_in(GradZ a, CatWT b, EpiGradIn epi,
                                                      const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int m0 = blockIdx.x * BM;
    if (m0 >= n1) return;
    a.n1 = n1; epi.n1 = n1;
    gemm_tile<BM, BN, true, true>(m0, blockIdx.y * BN, 0, a.N, a, b, epi);
}

// zero `count_rows(meta) * width` floats, or a fixed number when meta == nullptr
__global__ __launch_bounds__(256) void k_fill_zero(float *__restrict__ p, int64_t fixed_n,
                                                   const GsLevelMeta *__restrict__ meta, int S, int width) {
    const int64_t n = meta ? (int64_t)meta->front_off[S] * width : fixed_n;
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < n;
         x += (int64_t)gridDim.x * blockDim.x)
        p[x] = 0.f;
}

int grid_1d(const gsplit_ctx *ctx, int64_t upper_threads) {
    int64_t want = std::max<int64_t>(1, gs_ceil_div(upper_threads, 256));
    return (int)std::min<int64_t>(want, (int64_t)ctx->n_cu * 8);
}

int ensure_buffers(gsplit_ctx *ctx, const gsplit_sage_params *p) {
    GsSageBuf &sb = ctx->sage;
    const int L = ctx->L;
    bool same = sb.ready && sb.dtype == p->dtype;
    for (int l = 0; same && l <= L; ++l) same = sb.dims[l] == p->dims[l];
    if (same) return GSPLIT_OK;
    if (sb.ready) return gs_fail(ctx, GSPLIT_ESTATE, "sage: model shape changed; create a new context");
    for (int l = 1; l < L; ++l) {
        int rc = gs_alloc(ctx, &sb.hidden[l], sizeof(float) * ctx->ub_front[l] * p->dims[l], "hidden");
        if (rc) return rc;
        rc = gs_alloc(ctx, (void **)&sb.ghid[l], sizeof(float) * ctx->ub_front[l] * p->dims[l], "ghid");
        if (rc) return rc;
    }
    for (int l = 0; l < L; ++l) {
        int rc = gs_alloc(ctx, &sb.mean[l], sizeof(float) * ctx->ub_front[l + 1] * p->dims[l], "mean");
        if (rc) return rc;
    }
    sb.dtype = p->dtype;
    for (int l = 0; l <= L; ++l) sb.dims[l] = p->dims[l];
    sb.ready = true;
    return GSPLIT_OK;
}

int check_params(gsplit_ctx *ctx, const gsplit_sage_params *p, const char *who) {
    if (!p || !p->dims || !p->d_w_self || !p->d_w_neigh || !p->d_bias)
        return gs_fail(ctx, GSPLIT_EINVAL, std::string(who) + ": NULL parameter block");
    if (p->dtype != GSPLIT_F32)
        return gs_fail(ctx, GSPLIT_EINVAL, std::string(who) + ": only GSPLIT_F32 is available in this build");
    for (int l = 0; l <= ctx->L; ++l)
        if (p->dims[l] < 1 || p->dims[l] > 4096)
            return gs_fail(ctx, GSPLIT_EINVAL, std::string(who) + ": layer width out of range");
    for (int l = 0; l < ctx->L; ++l)
        if (!p->d_w_self[l] || !p->d_w_neigh[l] || !p->d_bias[l])
            return gs_fail(ctx, GSPLIT_EINVAL, std::string(who) + ": NULL weight pointer");
    return GSPLIT_OK;
}

void launch_aggregate(gsplit_ctx *ctx, int l, const float *hin, int D, hipStream_t st) {
    const GsLayerBuf &B = ctx->layer[l];
    const GsLevelMeta *mu = ctx->d_meta + (l + 1);
    float *M = (float *)ctx->sage.mean[l];
    const int64_t ub = ctx->ub_front[l + 1];
    if (D % 4 != 0) {
        hipLaunchKernelGGL(k_mean_aggregate_f32_any, dim3(grid_1d(ctx, ub * 64)), dim3(256), 0, st, hin, D,
                           B.blk_indptr, B.edge_row, mu, ctx->S, M);
        return;
    }
    const int nvec = D / 4;
    if (nvec <= 16)
        hipLaunchKernelGGL(k_mean_aggregate_f32<16>, dim3(grid_1d(ctx, ub * 16)), dim3(256), 0, st, hin, D,
                           B.blk_indptr, B.edge_row, mu, ctx->S, M);
    else if (nvec <= 32)
        hipLaunchKernelGGL(k_mean_aggregate_f32<32>, dim3(grid_1d(ctx, ub * 32)), dim3(256), 0, st, hin, D,
                           B.blk_indptr, B.edge_row, mu, ctx->S, M);
    else
        hipLaunchKernelGGL(k_mean_aggregate_f32<64>, dim3(grid_1d(ctx, ub * 64)), dim3(256), 0, st, hin, D,
                           B.blk_indptr, B.edge_row, mu, ctx->S, M);
}

}  // namespace

extern "C" int gsplit_sage_fwd(gsplit_ctx *ctx, const gsplit_sage_params *p, const void *d_feat_local,
                               float *d_logits, void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    int rc = check_params(ctx, p, "gsplit_sage_fwd");
    if (rc) return rc;
    if (!d_feat_local || !d_logits) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_sage_fwd: NULL buffer");
    if (ctx->batch_id == 0) return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_sage_fwd: no batch");
    rc = ensure_buffers(ctx, p);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int L = ctx->L, S = ctx->S;
    GsSageBuf &sb = ctx->sage;
    sb.hidden[0] = const_cast<void *>(d_feat_local);   // caller-owned; read again by the backward pass
    for (int l = 0; l < L; ++l) {
        const int D = p->dims[l], N = p->dims[l + 1];
        const float *hin = l == 0 ? (const float *)d_feat_local : (const float *)sb.hidden[l];
        float *hout = l == L - 1 ? d_logits : (float *)sb.hidden[l + 1];
        const GsLayerBuf &B = ctx->layer[l];
        const GsLevelMeta *mu = ctx->d_meta + (l + 1);
        launch_aggregate(ctx, l, hin, D, st);
        CatIn a{hin, (const float *)sb.mean[l], B.self_row, D, 0};
        CatW b{(const float *)p->d_w_self[l], (const float *)p->d_w_neigh[l], D, N};
        EpiFwd epi{hout, (const float *)p->d_bias[l], N, 0, l < L - 1 ? 1 : 0};
        const int64_t ub = ctx->ub_front[l + 1];
        if (N > 64) {
            dim3 grid((unsigned)gs_ceil_div(ub, 128), (unsigned)gs_ceil_div(N, 128));
            hipLaunchKernelGGL((k_sage_linear_fwd<128, 128>), grid, dim3(256), 0, st, a, b, epi, mu, S);
        } else {
            dim3 grid((unsigned)gs_ceil_div(ub, 128), 1);
            hipLaunchKernelGGL((k_sage_linear_fwd<128, 64>), grid, dim3(256), 0, st, a, b, epi, mu, S);
        }
    }
    GS_HIP(ctx, hipGetLastError());
    sb.fwd_done = true;
    sb.fwd_batch = ctx->batch_id;
    return GSPLIT_OK;
}

extern "C" int gsplit_sage_bwd(gsplit_ctx *ctx, const gsplit_sage_params *p, const float *d_grad_logits,
                               float *const *d_gw_self, float *const *d_gw_neigh, float *const *d_gbias,
                               void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    int rc = check_params(ctx, p, "gsplit_sage_bwd");
    if (rc) return rc;
    if (!d_grad_logits || !d_gw_self || !d_gw_neigh || !d_gbias)
        return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_sage_bwd: NULL buffer");
    GsSageBuf &sb = ctx->sage;
    if (!sb.ready || !sb.fwd_done || sb.fwd_batch != ctx->batch_id)
        return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_sage_bwd: needs gsplit_sage_fwd on the current batch first");
    for (int l = 0; l <= ctx->L; ++l)
        if (sb.dims[l] != p->dims[l])
            return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_sage_bwd: parameters differ from the forward pass");
    hipStream_t st = (hipStream_t)stream;
    const int L = ctx->L, S = ctx->S;
    for (int l = 0; l < L; ++l) {
        if (!d_gw_self[l] || !d_gw_neigh[l] || !d_gbias[l])
            return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_sage_bwd: NULL gradient pointer");
        const int64_t nw = (int64_t)p->dims[l] * p->dims[l + 1];
        hipLaunchKernelGGL(k_fill_zero, dim3(grid_1d(ctx, nw)), dim3(256), 0, st, d_gw_self[l], nw, nullptr, S, 0);
        hipLaunchKernelGGL(k_fill_zero, dim3(grid_1d(ctx, nw)), dim3(256), 0, st, d_gw_neigh[l], nw, nullptr, S, 0);
        hipLaunchKernelGGL(k_fill_zero, dim3(1), dim3(256), 0, st, d_gbias[l], (int64_t)p->dims[l + 1], nullptr, S, 0);
    }
    for (int l = L - 1; l >= 0; --l) {
        const int D = p->dims[l], N = p->dims[l + 1];
        const float *hin = (const float *)sb.hidden[l];
        const GsLayerBuf &B = ctx->layer[l];
        const GsLevelMeta *mu = ctx->d_meta + (l + 1);
        const float *dH = l == L - 1 ? d_grad_logits : sb.ghid[l + 1];
        const float *hout = l == L - 1 ? nullptr : (const float *)sb.hidden[l + 1];
        const int64_t ub = ctx->ub_front[l + 1];
        GradZ dz{dH, hout, N, 0, l < L - 1 ? 1 : 0};
        // weight and bias gradients, summed over all splits (layer 0 reads its input rows from the
        // caller's gathered features, which therefore must still be alive)
        CatIn in{hin, (const float *)sb.mean[l], B.self_row, D, 0};
        CatInT at{in};
        EpiGradW ew{d_gw_self[l], d_gw_neigh[l], d_gbias[l], D, N};
        const int kchunk = 1024;
        if (N > 64) {
            dim3 grid((unsigned)gs_ceil_div(2 * D + 1, 128), (unsigned)gs_ceil_div(N, 128),
                      (unsigned)gs_ceil_div(ub, kchunk));
            hipLaunchKernelGGL((k_sage_grad_w<128, 128>), grid, dim3(256), 0, st, at, dz, ew, kchunk, mu, S);
        } else {
            dim3 grid((unsigned)gs_ceil_div(2 * D + 1, 128), 1, (unsigned)gs_ceil_div(ub, kchunk));
            hipLaunchKernelGGL((k_sage_grad_w<128, 64>), grid, dim3(256), 0, st, at, dz, ew, kchunk, mu, S);
        }
        if (l > 0) {
            const GsLevelMeta *ml = ctx->d_meta + l;
            hipLaunchKernelGGL(k_fill_zero, dim3(grid_1d(ctx, ctx->ub_front[l] * D)), dim3(256), 0, st,
                               sb.ghid[l], 0, ml, S, D);
            CatW w{(const float *)p->d_w_self[l], (const float *)p->d_w_neigh[l], D, N};
            CatWT wt{w};
            EpiGradIn ei{sb.ghid[l], B.self_row, B.edge_row, B.blk_indptr, D, 0};
            dim3 grid((unsigned)gs_ceil_div(ub, 128), (unsigned)gs_ceil_div(2 * D, 128));
            hipLaunchKernelGGL((k_sage_grad_in<128, 128>), grid, dim3(256), 0, st, dz, wt, ei, mu, S);
        }
    }
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}
