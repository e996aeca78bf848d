// GAT forward and backward over the split mini-batch: the paper's second model (section 7.1; the
// layer itself is the one of Velickovic et al., ICLR 2018), run as `gnn_layer` of Algorithm 2.
//
// The linear transform commutes with the training shuffle (a shuffled row is a copy), so it runs
// once per row of local_cat[l] instead of once per row of every split's mixed frontier; the edge
// softmax and the aggregation then gather transformed rows through the composed shuffle index
// (self_row / edge_row), and the backward pass returns through its scatter side (rev_*).
//
// The attention vectors are folded into the weights: with W_ext = [W | W a_src | W a_dst] one
// product gives z and both score terms of every row, and in the backward pass
//     d h   = dz_ext W_ext^T            dz_ext = [sum alpha dagg | d e_src | d e_dst]
//     G     = h^T dz_ext                (D x (K F + 2 K), split-K on the matrix cores)
//     d W   = G_z + G_src (x) a_src + G_dst (x) a_dst,   d a_src = W^T G_src,   d a_dst = W^T G_dst
// so the per-row kernels only form dz_ext and every reduction over rows is a matrix product.
#include <algorithm>

#include "gsplit_internal.h"

namespace {

#include "gemm_f32.h"

constexpr float NEG_SLOPE = 0.2f;

// Per-layer sizes.  A wave owns one row; its 64 lanes are dealt to the heads in groups of
// lph = 64 / (K rounded up to a power of two) lanes, lane `sub` of head k holding features
// (sub + lph t) VW + 0..VW-1, t < NV, of that head.
struct GatDims {
    int K, F, HF, ZW, lph, fan;
    int64_t self_base;      // slot of destination i's self entry = self_base + i (edge slots come first)
};

struct EpiStore {
    float *out; int ld; int rows; int cols;
    __device__ __forceinline__ float col(int) const { return 0.f; }
    __device__ __forceinline__ float row(int) const { return 0.f; }
    __device__ __forceinline__ void store(int m, int n, float v, float, float) const {
        if (m < rows && n < cols) out[(int64_t)m * ld + n] = v;
    }
};

// C = A B (B_KC = false: b is K x N) or C = A B^T (B_KC = true: b is N x K) for the rows of one
// level; persistent row-block tiling
template <class T, int VA, int VB, bool B_KC>
__global__ __launch_bounds__(GNT) __attribute__((amdgpu_waves_per_eu(T::LEAN ? 6 : 2, T::LEAN ? 6 : 8)))
void k_gat_rows_gemm(MatRows a, MatRows b, EpiStore epi, const GsLevelMeta *__restrict__ meta_rows, int S) {
    const int n1 = meta_rows->front_off[S];
    const int n_out = B_KC ? b.rows : b.cols;
    const int tiles_m = (n1 + T::BM - 1) / T::BM, tiles_n = (n_out + T::BN - 1) / T::BN;
    const int total = ((tiles_m + 7) & ~7) * tiles_n;
    a.rows = n1; epi.rows = n1;
    for (int gid = blockIdx.x; gid < total; gid += gridDim.x) {
        int m0, n0;
        if (!next_tile<T>(gid, tiles_m, tiles_n, m0, n0)) continue;
        gemm_tile<T, true, B_KC, VA, VB>(m0, n0, n1, n_out, 0, a.cols, a, b, epi);
    }
}

// W_ext of every layer in one launch (blockIdx.y = layer)
struct GatPrep {
    const float *w[GS_MAXL]; const float *a_src[GS_MAXL]; const float *a_dst[GS_MAXL]; float *wext[GS_MAXL];
    int D[GS_MAXL]; int K[GS_MAXL]; int F[GS_MAXL]; int ZW[GS_MAXL];
};
__global__ __launch_bounds__(256) void k_gat_prep_weights(GatPrep p) {
    const int l = blockIdx.y;
    const int D = p.D[l], K = p.K[l], F = p.F[l], ZW = p.ZW[l], HF = K * F;
    const int64_t words = (int64_t)D * ZW;
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < words; x += (int64_t)gridDim.x * blockDim.x) {
        const int d = (int)(x / ZW), c = (int)(x % ZW);
        const float *wr = p.w[l] + (int64_t)d * HF;
        float v = 0.f;
        if (c < HF) {
            v = wr[c];
        } else if (c < HF + 2 * K) {
            const int k = (c - HF) % K;
            const float *a = (c < HF + K ? p.a_src[l] : p.a_dst[l]) + k * F;
            for (int f = 0; f < F; ++f) v += wr[k * F + f] * a[f];
        }
        p.wext[l][x] = v;
    }
}

__device__ __forceinline__ float head_sum(float v, int lph) {
    for (int o = lph >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ float head_max(float v, int lph) {
    for (int o = lph >> 1; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

// the lane's NV * VW features of head k of one row (base = row start + k F); zeros where the lane
// holds nothing
template <int VW, int NV>
__device__ __forceinline__ void load_cols(const float *__restrict__ base, int sub, int lph, int F, bool ok,
                                          float (&v)[NV * VW]) {
#pragma unroll
    for (int t = 0; t < NV; ++t) {
        const int f0 = (sub + lph * t) * VW;
        if (ok && f0 < F) {
            if (VW == 4) {
                const float4 x = *reinterpret_cast<const float4 *>(base + f0);
                v[t * 4] = x.x; v[t * 4 + 1] = x.y; v[t * 4 + 2] = x.z; v[t * 4 + 3] = x.w;
            } else {
                v[t] = base[f0];
            }
        } else {
#pragma unroll
            for (int j = 0; j < VW; ++j) v[t * VW + j] = 0.f;
        }
    }
}
template <int VW, int NV>
__device__ __forceinline__ void store_cols(float *__restrict__ base, int sub, int lph, int F, bool ok,
                                           const float (&v)[NV * VW]) {
#pragma unroll
    for (int t = 0; t < NV; ++t) {
        const int f0 = (sub + lph * t) * VW;
        if (ok && f0 < F) {
            if (VW == 4) *reinterpret_cast<float4 *>(base + f0) = make_float4(v[t * 4], v[t * 4 + 1], v[t * 4 + 2], v[t * 4 + 3]);
            else base[f0] = v[t];
        }
    }
}

struct GatFwdArgs {
    const float *zext; const int32_t *blk_indptr; const int32_t *edge_row; const int32_t *self_row;
    const float *bias; float *alpha; float *out;
};

// Edge softmax and aggregation, one wave per destination.  The entries of a destination (itself,
// then its sampled edges in slot order) are first dealt to the lanes of each head: scores, their
// maximum and sum, and the coefficients alpha, which go to HBM for the backward pass and to LDS
// for the second step, the weighted sum of the transformed rows (four row loads in flight).
template <int VW, int NV, bool LAST>
__global__ __launch_bounds__(256) void k_gat_aggregate(GatFwdArgs g, GatDims d, const GsLevelMeta *__restrict__ meta_up, int S) {
    extern __shared__ float smem[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int per_wave = (1 + d.fan) * (1 + d.K);
    int *s_row = reinterpret_cast<int *>(smem + wave * per_wave);
    float *s_val = smem + wave * per_wave + (1 + d.fan);
    const int n1 = meta_up->front_off[S];
    const int K = d.K, F = d.F, HF = d.HF, ZW = d.ZW, lph = d.lph;
    const int k = lane / lph, sub = lane % lph;
    const bool ok = k < K;
    for (int i = blockIdx.x * 4 + wave; i < n1; i += gridDim.x * 4) {
        const int e0 = g.blk_indptr[i], e1 = g.blk_indptr[i + 1];
        const int n_ent = 1 + e1 - e0;
        const int self = g.self_row[i];
        const float er = ok ? g.zext[(int64_t)self * ZW + HF + K + k] : 0.f;
        float m = -3.4e38f;
        for (int j = sub; j < n_ent; j += lph) {
            const int row = j == 0 ? self : g.edge_row[e0 + j - 1];
            if (k == 0) s_row[j] = row;
            if (ok) {
                const float raw = er + g.zext[(int64_t)row * ZW + HF + k];
                const float e = raw > 0.f ? raw : NEG_SLOPE * raw;
                s_val[j * K + k] = e;
                m = fmaxf(m, e);
            }
        }
        m = head_max(m, lph);
        float s = 0.f;
        if (ok)
            for (int j = sub; j < n_ent; j += lph) {
                const float p = expf(s_val[j * K + k] - m);
                s_val[j * K + k] = p;
                s += p;
            }
        s = head_sum(s, lph);
        if (ok)
            for (int j = sub; j < n_ent; j += lph) {
                const float a = s_val[j * K + k] / s;
                s_val[j * K + k] = a;
                const int64_t slot = j == 0 ? d.self_base + i : (int64_t)(e0 + j - 1);
                g.alpha[slot * K + k] = a;
            }
        __builtin_amdgcn_wave_barrier();
        float acc[NV * VW];
#pragma unroll
        for (int c = 0; c < NV * VW; ++c) acc[c] = 0.f;
        for (int j = 0; j < n_ent; j += 4) {
            float z[4][NV * VW], a[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool in = j + q < n_ent;
                const int row = in ? s_row[j + q] : self;
                a[q] = (in && ok) ? s_val[(j + q) * K + k] : 0.f;
                load_cols<VW, NV>(g.zext + (int64_t)row * ZW + k * F, sub, lph, F, ok, z[q]);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int c = 0; c < NV * VW; ++c) acc[c] += a[q] * z[q][c];
        }
        __builtin_amdgcn_wave_barrier();
        if (LAST) {
            // logits = mean over heads + bias: lanes with the same `sub` hold the same features
#pragma unroll
            for (int c = 0; c < NV * VW; ++c)
                for (int o = lph; o < 64; o <<= 1) acc[c] += __shfl_xor(acc[c], o);
            if (k == 0) {
#pragma unroll
                for (int t = 0; t < NV; ++t)
#pragma unroll
                    for (int jj = 0; jj < VW; ++jj) {
                        const int f = (sub + lph * t) * VW + jj;
                        if (f < F) g.out[(int64_t)i * F + f] = acc[t * VW + jj] / (float)K + g.bias[f];
                    }
            }
        } else {
#pragma unroll
            for (int t = 0; t < NV; ++t)
#pragma unroll
                for (int jj = 0; jj < VW; ++jj) {
                    const int f = (sub + lph * t) * VW + jj;
                    if (ok && f < F) {
                        const float v = acc[t * VW + jj] + g.bias[k * F + f];
                        acc[t * VW + jj] = v > 0.f ? v : expm1f(v);
                    }
                }
            store_cols<VW, NV>(g.out + (int64_t)i * HF + k * F, sub, lph, F, ok, acc);
        }
    }
}

struct GatBwdDstArgs {
    const float *zext; const int32_t *blk_indptr; const int32_t *edge_row; const int32_t *self_row;
    const float *alpha; const float *dh; const float *hout;
    float *gagg; float *de; float *der; float *bias_part; int PW;
};

// Backward over the destinations, one wave each: dagg (through the ELU, or the head mean of the
// last layer), d alpha_j = z_j . dagg per entry and head, the softmax and LeakyReLU derivatives
// (d e_j), the sum of d e_j per destination, and this workgroup's share of the bias gradient.
template <int VW, int NV, bool LAST>
__global__ __launch_bounds__(256) void k_gat_bwd_dst(GatBwdDstArgs g, GatDims d, const GsLevelMeta *__restrict__ meta_up, int S) {
    extern __shared__ float smem[];
    __shared__ float s_b[4][64 * NV * VW];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int per_wave = (1 + d.fan) * (1 + d.K);
    int *s_row = reinterpret_cast<int *>(smem + wave * per_wave);
    float *s_val = smem + wave * per_wave + (1 + d.fan);
    const int n1 = meta_up->front_off[S];
    const int K = d.K, F = d.F, HF = d.HF, ZW = d.ZW, lph = d.lph;
    const int k = lane / lph, sub = lane % lph;
    const bool ok = k < K;
    float bacc[NV * VW];
#pragma unroll
    for (int c = 0; c < NV * VW; ++c) bacc[c] = 0.f;
    for (int i = blockIdx.x * 4 + wave; i < n1; i += gridDim.x * 4) {
        float dagg[NV * VW];
#pragma unroll
        for (int t = 0; t < NV; ++t)
#pragma unroll
            for (int jj = 0; jj < VW; ++jj) {
                const int f = (sub + lph * t) * VW + jj;
                float v = 0.f;
                if (ok && f < F) {
                    if (LAST) {
                        const float dp = g.dh[(int64_t)i * F + f];
                        if (k == 0) bacc[t * VW + jj] += dp;
                        v = dp / (float)K;
                    } else {
                        const float h = g.hout[(int64_t)i * HF + k * F + f];
                        v = g.dh[(int64_t)i * HF + k * F + f] * (h > 0.f ? 1.f : h + 1.f);
                        bacc[t * VW + jj] += v;
                    }
                }
                dagg[t * VW + jj] = v;
            }
        store_cols<VW, NV>(g.gagg + (int64_t)i * HF + k * F, sub, lph, F, ok, dagg);
        const int e0 = g.blk_indptr[i], e1 = g.blk_indptr[i + 1];
        const int n_ent = 1 + e1 - e0;
        const int self = g.self_row[i];
        const float er = ok ? g.zext[(int64_t)self * ZW + HF + K + k] : 0.f;
        for (int j = 0; j < n_ent; j += 4) {
            float z[4][NV * VW], p[4];
            int rows[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int jq = j + q;
                rows[q] = (jq == 0 || jq >= n_ent) ? self : g.edge_row[e0 + jq - 1];
                load_cols<VW, NV>(g.zext + (int64_t)rows[q] * ZW + k * F, sub, lph, F, ok, z[q]);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                p[q] = 0.f;
#pragma unroll
                for (int c = 0; c < NV * VW; ++c) p[q] += z[q][c] * dagg[c];
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) p[q] = head_sum(p[q], lph);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (j + q < n_ent && sub == 0) {
                    if (ok) s_val[(j + q) * K + k] = p[q];
                    if (k == 0) s_row[j + q] = rows[q];
                }
        }
        __builtin_amdgcn_wave_barrier();
        float tsum = 0.f;
        if (ok)
            for (int j = sub; j < n_ent; j += lph) {
                const int64_t slot = j == 0 ? d.self_base + i : (int64_t)(e0 + j - 1);
                tsum += g.alpha[slot * K + k] * s_val[j * K + k];
            }
        tsum = head_sum(tsum, lph);
        float dsum = 0.f;
        if (ok)
            for (int j = sub; j < n_ent; j += lph) {
                const int64_t slot = j == 0 ? d.self_base + i : (int64_t)(e0 + j - 1);
                const float raw = er + g.zext[(int64_t)s_row[j] * ZW + HF + k];
                const float v = g.alpha[slot * K + k] * (s_val[j * K + k] - tsum) * (raw > 0.f ? 1.f : NEG_SLOPE);
                g.de[slot * K + k] = v;
                dsum += v;
            }
        dsum = head_sum(dsum, lph);
        if (ok && sub == 0) g.der[(int64_t)i * K + k] = dsum;
        __builtin_amdgcn_wave_barrier();
    }
    // bias gradient of this workgroup's rows: the four waves' sums added in wave order
#pragma unroll
    for (int c = 0; c < NV * VW; ++c) s_b[wave][c * 64 + lane] = bacc[c];
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int t = 0; t < NV; ++t)
#pragma unroll
            for (int jj = 0; jj < VW; ++jj) {
                const int c = t * VW + jj, f = (sub + lph * t) * VW + jj;
                const float v = ((s_b[0][c * 64 + lane] + s_b[1][c * 64 + lane]) + s_b[2][c * 64 + lane]) + s_b[3][c * 64 + lane];
                if (ok && f < F && (!LAST || k == 0)) g.bias_part[(int64_t)blockIdx.x * g.PW + (LAST ? f : k * F + f)] = v;
            }
    }
}

struct GatBwdSrcArgs {
    const int32_t *rev_ptr; const int32_t *rev_cnt; const int32_t *rev_list; const int32_t *rev_eid;
    const float *alpha; const float *de; const float *der; const float *gagg; float *dzext;
};

// Reverse shuffle of the backward pass as a pull, one wave per row u of local_cat[l]: over the
// destinations it fed (scatter side of the shuffle index) it sums alpha * dagg and d e_src; its own
// destination (self entry), if it has one, contributes d e_dst.  Rows that fed nothing get zeros.
template <int VW, int NV>
__global__ __launch_bounds__(256) void k_gat_bwd_src(GatBwdSrcArgs g, GatDims d, const GsLevelMeta *__restrict__ meta_lo, int S) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n0 = meta_lo->front_off[S];
    const int K = d.K, F = d.F, HF = d.HF, ZW = d.ZW, lph = d.lph;
    const int k = lane / lph, sub = lane % lph;
    const bool ok = k < K;
    for (int u = blockIdx.x * 4 + wave; u < n0; u += gridDim.x * 4) {
        const int p0 = g.rev_ptr[u], cnt = g.rev_cnt[u];
        float acc[NV * VW];
#pragma unroll
        for (int c = 0; c < NV * VW; ++c) acc[c] = 0.f;
        float dsrc = 0.f, ddst = 0.f;
        for (int x = 0; x < cnt; x += 4) {
            float gv[4][NV * VW], a[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool in = x + q < cnt;
                const int code = in ? g.rev_list[p0 + x + q] : 0;
                const int i = code >> 1;
                const int64_t slot = (code & 1) ? (int64_t)g.rev_eid[p0 + x + q] : d.self_base + i;
                a[q] = 0.f;
                if (in && ok) {
                    a[q] = g.alpha[slot * K + k];
                    dsrc += g.de[slot * K + k];
                    if (!(code & 1)) ddst = g.der[(int64_t)i * K + k];
                }
                load_cols<VW, NV>(g.gagg + (int64_t)i * HF + k * F, sub, lph, F, ok && in, gv[q]);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int c = 0; c < NV * VW; ++c) acc[c] += a[q] * gv[q][c];
        }
        float *out = g.dzext + (int64_t)u * ZW;
        store_cols<VW, NV>(out + k * F, sub, lph, F, ok, acc);
        if (ok && sub == 0) {
            out[HF + k] = dsrc;
            out[HF + K + k] = ddst;
        }
        if (lane < ZW - HF - 2 * K) out[HF + 2 * K + lane] = 0.f;
    }
}

// G = sum of the split-K slabs of h^T dz_ext in slab order, all layers in one launch
struct GatReduce {
    const float *part[GS_MAXL]; float *gmat[GS_MAXL]; int D[GS_MAXL]; int ZW[GS_MAXL]; int nchunk[GS_MAXL];
};
__global__ __launch_bounds__(256) void k_gat_reduce(GatReduce g, const GsLevelMeta *__restrict__ meta, int S) {
    const int l = blockIdx.y;
    const int n0 = meta[l].front_off[S];
    const int kchunk = grad_w_chunk_rows(n0, g.nchunk[l], GRAD_W_ROWS_MIN);
    const int chunks = (n0 + kchunk - 1) / kchunk;
    const int64_t words = (int64_t)g.D[l] * g.ZW[l], slab = (int64_t)(g.D[l] + 1) * g.ZW[l];
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < words; x += (int64_t)gridDim.x * blockDim.x) {
        const float *p = g.part[l] + x;
        float acc = 0.f;
        int z = 0;
        for (; z + 8 <= chunks; z += 8) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = p[(int64_t)(z + j) * slab];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc += v[j];
        }
        for (; z < chunks; ++z) acc += p[(int64_t)z * slab];
        g.gmat[l][x] = acc;
    }
}

// d W = G_z + G_src (x) a_src + G_dst (x) a_dst, all layers in one launch
struct GatFinish {
    const float *gmat[GS_MAXL]; const float *w[GS_MAXL]; const float *a_src[GS_MAXL]; const float *a_dst[GS_MAXL];
    const float *bias_part[GS_MAXL];
    float *gw[GS_MAXL]; float *ga_src[GS_MAXL]; float *ga_dst[GS_MAXL]; float *gb[GS_MAXL];
    int D[GS_MAXL]; int K[GS_MAXL]; int F[GS_MAXL]; int ZW[GS_MAXL]; int PW[GS_MAXL]; int slabs[GS_MAXL];
};
__global__ __launch_bounds__(256) void k_gat_finish(GatFinish g) {
    const int l = blockIdx.y;
    const int D = g.D[l], K = g.K[l], F = g.F[l], ZW = g.ZW[l], HF = K * F, PW = g.PW[l];
    const float *G = g.gmat[l];
    const int64_t tid = blockIdx.x * (int64_t)blockDim.x + threadIdx.x, nthr = (int64_t)gridDim.x * blockDim.x;
    for (int64_t x = tid; x < (int64_t)D * HF; x += nthr) {
        const int dd = (int)(x / HF), c = (int)(x % HF), k = c / F;
        const float *row = G + (int64_t)dd * ZW;
        g.gw[l][x] = row[c] + row[HF + k] * g.a_src[l][c] + row[HF + K + k] * g.a_dst[l][c];
    }
}

// d a_src = W^T G_src, d a_dst = W^T G_dst and the bias gradient (sum of the workgroup slabs of
// k_gat_bwd_dst in slab order): 64 columns per workgroup, the long sums dealt to 16 waves and
// added in wave order
__global__ __launch_bounds__(1024) void k_gat_finish_cols(GatFinish g) {
    __shared__ float red[3][16][64];
    const int l = blockIdx.y;
    const int D = g.D[l], K = g.K[l], F = g.F[l], ZW = g.ZW[l], HF = K * F, PW = g.PW[l], slabs = g.slabs[l];
    const float *G = g.gmat[l];
    const int x = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + x;
    if (blockIdx.x * 64 >= HF) return;
    float s = 0.f, t = 0.f, b = 0.f;
    if (c < HF) {
        const int k = c / F;
        for (int dd = ty; dd < D; dd += 16) {
            const float wv = g.w[l][(int64_t)dd * HF + c];
            s += wv * G[(int64_t)dd * ZW + HF + k];
            t += wv * G[(int64_t)dd * ZW + HF + K + k];
        }
    }
    if (c < PW) {
        const float *p = g.bias_part[l] + c;
        int z = ty;
        for (; z + 7 * 16 < slabs; z += 8 * 16) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = p[(int64_t)(z + 16 * j) * PW];
#pragma unroll
            for (int j = 0; j < 8; ++j) b += v[j];
        }
        for (; z < slabs; z += 16) b += p[(int64_t)z * PW];
    }
    red[0][ty][x] = s; red[1][ty][x] = t; red[2][ty][x] = b;
    __syncthreads();
    if (ty == 0) {
        s = t = b = 0.f;
        for (int j = 0; j < 16; ++j) { s += red[0][j][x]; t += red[1][j][x]; b += red[2][j][x]; }
        if (c < HF) { g.ga_src[l][c] = s; g.ga_dst[l][c] = t; }
        if (c < PW) g.gb[l][c] = b;
    }
}

// ---- host side -------------------------------------------------------------------------------
int pow2_ceil(int v) { int p = 1; while (p < v) p <<= 1; return p; }

int feat_per_head(const gsplit_ctx *ctx, const gsplit_gat_params *p, int l) {
    return l == ctx->L - 1 ? p->dims[l + 1] : p->dims[l + 1] / p->heads[l];
}
int zw_of(int K, int F) { return (K * F + 2 * K + 3) & ~3; }

GatDims dims_of(const gsplit_ctx *ctx, const gsplit_gat_params *p, int l) {
    GatDims d;
    d.K = p->heads[l]; d.F = feat_per_head(ctx, p, l); d.HF = d.K * d.F; d.ZW = zw_of(d.K, d.F);
    d.lph = 64 / pow2_ceil(d.K); d.fan = ctx->fan[l];
    d.self_base = ctx->ub_front[l + 1] * ctx->fan[l];
    return d;
}

int check_params(gsplit_ctx *ctx, const gsplit_gat_params *p, const char *who) {
    const std::string w(who);
    if (!p || !p->dims || !p->heads || !p->d_w || !p->d_a_src || !p->d_a_dst || !p->d_bias)
        return gs_fail(ctx, GSPLIT_EINVAL, w + ": NULL parameter block");
    if (p->dtype != GSPLIT_F32) return gs_fail(ctx, GSPLIT_EINVAL, w + ": dtype must be GSPLIT_F32");
    if (!ctx->gat_index) return gs_fail(ctx, GSPLIT_ESTATE, w + ": the context was created without gat_index");
    if (p->dims[0] < 1 || p->dims[0] > 4096) return gs_fail(ctx, GSPLIT_EINVAL, w + ": input width out of range");
    for (int l = 0; l < ctx->L; ++l) {
        const int K = p->heads[l];
        if (K < 1 || K > 64) return gs_fail(ctx, GSPLIT_EINVAL, w + ": heads must be in 1..64");
        if (p->dims[l + 1] < 1 || p->dims[l + 1] > 4096 || (l < ctx->L - 1 && p->dims[l + 1] % K != 0))
            return gs_fail(ctx, GSPLIT_EINVAL, w + ": a hidden width must be a positive multiple of the layer's heads");
        if (feat_per_head(ctx, p, l) > 1024 / pow2_ceil(K))
            return gs_fail(ctx, GSPLIT_EINVAL, w + ": features per head exceed 1024 / (heads rounded up to a power of two)");
        if ((int64_t)(1 + ctx->fan[l]) * (1 + K) > 3072)
            return gs_fail(ctx, GSPLIT_EINVAL, w + ": (1 + fanout) * (1 + heads) exceeds 3072");
        if (!p->d_w[l] || !p->d_a_src[l] || !p->d_a_dst[l] || !p->d_bias[l])
            return gs_fail(ctx, GSPLIT_EINVAL, w + ": NULL parameter pointer");
    }
    return GSPLIT_OK;
}

int ensure_buffers(gsplit_ctx *ctx, const gsplit_gat_params *p) {
    GsGatBuf &gb = ctx->gat;
    const int L = ctx->L;
    if (gb.ready) {
        bool same = true;
        for (int l = 0; l <= L; ++l) same = same && gb.dims[l] == p->dims[l];
        for (int l = 0; l < L; ++l) same = same && gb.heads[l] == p->heads[l];
        if (same) return GSPLIT_OK;
        return gs_fail(ctx, GSPLIT_ESTATE, "GAT layer widths or heads changed within one context");
    }
    int rc = GSPLIT_OK;
    auto A = [&](float **q, int64_t words, const char *what) {
        if (rc == GSPLIT_OK) rc = gs_alloc(ctx, (void **)q, sizeof(float) * (size_t)std::max<int64_t>(words, 4), what);
    };
    for (int l = 0; l < L; ++l) {
        const GatDims d = dims_of(ctx, p, l);
        const int D = p->dims[l];
        const int64_t n_lo = ctx->ub_front[l], n_up = ctx->ub_front[l + 1];
        A(&gb.wext[l], (int64_t)D * d.ZW, "GAT extended weights");
        A(&gb.zext[l], n_lo * d.ZW, "GAT transformed rows");
        A(&gb.dzext[l], n_lo * d.ZW, "GAT transformed-row gradients");
        A(&gb.alpha[l], (d.self_base + n_up) * d.K, "GAT attention coefficients");
        A(&gb.de[l], (d.self_base + n_up) * d.K, "GAT score gradients");
        A(&gb.der[l], n_up * d.K, "GAT destination score gradients");
        A(&gb.gagg[l], n_up * d.HF, "GAT aggregate gradients");
        if (l > 0) {
            A(&gb.hidden[l], n_lo * D, "GAT hidden activations");
            A(&gb.ghid[l], n_lo * D, "GAT hidden gradients");
        }
        const int tiles = (int)(gs_ceil_div(D, TileMid::BM) * gs_ceil_div(d.ZW, TileMid::BN));
        gb.nchunk[l] = (int)(gs_ceil_div(std::max<int64_t>(8, (int64_t)ctx->n_cu * 3 / tiles), 8) * 8);
        A(&gb.gw_part[l], (int64_t)gb.nchunk[l] * (D + 1) * d.ZW, "GAT weight-gradient partials");
        A(&gb.gmat[l], (int64_t)D * d.ZW, "GAT weight-gradient product");
        gb.bias_slabs[l] = grid_1d(ctx, n_up * 64);
        A(&gb.bias_part[l], (int64_t)gb.bias_slabs[l] * p->dims[l + 1], "GAT bias-gradient partials");
    }
    if (rc) return rc;
    for (int l = 0; l <= L; ++l) gb.dims[l] = p->dims[l];
    for (int l = 0; l < L; ++l) gb.heads[l] = p->heads[l];
    gb.ready = true;
    return GSPLIT_OK;
}

template <class T, int VA, bool B_KC>
void launch_rows_gemm_t(gsplit_ctx *ctx, hipStream_t st, int64_t ub, int n_out, const MatRows &a, const MatRows &b,
                        const EpiStore &epi, const GsLevelMeta *meta_rows) {
    hipLaunchKernelGGL((k_gat_rows_gemm<T, VA, 4, B_KC>), dim3(row_block_grid<T>(ctx, ub, n_out)), dim3(GNT), 0, st, a, b,
                       epi, meta_rows, ctx->S);
}
// b is always readable in 16-byte pieces (library buffers, widths padded to 4); va: so is a
template <bool B_KC>
void launch_rows_gemm(gsplit_ctx *ctx, hipStream_t st, int64_t ub, bool va, const MatRows &a, const MatRows &b,
                      const EpiStore &epi, const GsLevelMeta *meta_rows) {
    const int n_out = B_KC ? b.rows : b.cols;
    if (!va) launch_rows_gemm_t<TileMid, 1, B_KC>(ctx, st, ub, n_out, a, b, epi, meta_rows);
    else if (!few_rows(ub, n_out, a.cols)) launch_rows_gemm_t<TileMidLean, 4, B_KC>(ctx, st, ub, n_out, a, b, epi, meta_rows);
    else if (n_out <= 64) launch_rows_gemm_t<TileLowNarrow, 4, B_KC>(ctx, st, ub, n_out, a, b, epi, meta_rows);
    else launch_rows_gemm_t<TileLow, 4, B_KC>(ctx, st, ub, n_out, a, b, epi, meta_rows);
}

// lane layout of the per-row kernels: vector width and vectors per lane
struct RowShape { int vw, nv; };
RowShape row_shape(const GatDims &d) {
    RowShape r;
    r.vw = d.F % 4 == 0 ? 4 : 1;
    r.nv = pow2_ceil((int)gs_ceil_div(d.F, (int64_t)r.vw * d.lph));
    return r;
}

#define GAT_DISPATCH(RS, CALL)                                                        \
    do {                                                                              \
        if ((RS).vw == 4) {                                                           \
            if ((RS).nv == 1) { CALL(4, 1); } else if ((RS).nv == 2) { CALL(4, 2); } else { CALL(4, 4); } \
        } else {                                                                      \
            if ((RS).nv == 1) { CALL(1, 1); } else if ((RS).nv == 2) { CALL(1, 2); }  \
            else if ((RS).nv == 4) { CALL(1, 4); } else if ((RS).nv == 8) { CALL(1, 8); } else { CALL(1, 16); } \
        }                                                                             \
    } while (0)

}  // namespace

extern "C" int gsplit_gat_fwd(gsplit_ctx *ctx, const gsplit_gat_params *p, const void *d_feat_local, float *d_logits,
                              void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    int rc = check_params(ctx, p, "gsplit_gat_fwd");
    if (rc) return rc;
    if (!d_feat_local || !d_logits) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_gat_fwd: NULL buffer");
    if (ctx->batch_id == 0) return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_gat_fwd: no batch");
    rc = ensure_buffers(ctx, p);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int L = ctx->L, S = ctx->S;
    GsGatBuf &gb = ctx->gat;
    {
        GatPrep pp;
        int64_t wmax = 1;
        for (int l = 0; l < L; ++l) {
            const GatDims d = dims_of(ctx, p, l);
            pp.w[l] = (const float *)p->d_w[l]; pp.a_src[l] = (const float *)p->d_a_src[l];
            pp.a_dst[l] = (const float *)p->d_a_dst[l]; pp.wext[l] = gb.wext[l];
            pp.D[l] = p->dims[l]; pp.K[l] = d.K; pp.F[l] = d.F; pp.ZW[l] = d.ZW;
            wmax = std::max<int64_t>(wmax, (int64_t)p->dims[l] * d.ZW);
        }
        GsTimeScope ts(ctx, "gat_prep_weights", -1, st);
        hipLaunchKernelGGL(k_gat_prep_weights, dim3((unsigned)std::min<int64_t>(256, gs_ceil_div(wmax, 256)), L), dim3(256),
                           0, st, pp);
    }
    for (int l = 0; l < L; ++l) {
        const GatDims d = dims_of(ctx, p, l);
        const int D = p->dims[l];
        const float *hin = l == 0 ? (const float *)d_feat_local : gb.hidden[l];
        const GsLayerBuf &B = ctx->layer[l];
        {
            MatRows a{hin, 0, D};
            MatRows b{gb.wext[l], D, d.ZW};
            EpiStore epi{gb.zext[l], d.ZW, 0, d.ZW};
            GsTimeScope ts(ctx, "gat_transform", l, st);
            launch_rows_gemm<false>(ctx, st, ctx->ub_front[l], D % 4 == 0 && aligned16(hin), a, b, epi, ctx->d_meta + l);
        }
        const bool last = l == L - 1;
        GatFwdArgs fa{gb.zext[l], B.blk_indptr, B.edge_row, B.self_row, (const float *)p->d_bias[l], gb.alpha[l],
                      last ? d_logits : gb.hidden[l + 1]};
        const RowShape rs = row_shape(d);
        const dim3 grid(grid_1d(ctx, ctx->ub_front[l + 1] * 64));
        const size_t lds = sizeof(float) * 4 * (1 + d.fan) * (1 + d.K);
        GsTimeScope ts(ctx, "gat_aggregate", l, st);
#define GAT_CALL(VW, NV)                                                                                          \
    if (last) hipLaunchKernelGGL((k_gat_aggregate<VW, NV, true>), grid, dim3(256), lds, st, fa, d, ctx->d_meta + (l + 1), S); \
    else hipLaunchKernelGGL((k_gat_aggregate<VW, NV, false>), grid, dim3(256), lds, st, fa, d, ctx->d_meta + (l + 1), S)
        GAT_DISPATCH(rs, GAT_CALL);
#undef GAT_CALL
    }
    GS_HIP(ctx, hipGetLastError());
    gb.fwd_done = true;
    gb.fwd_batch = ctx->batch_id;
    return GSPLIT_OK;
}

extern "C" int gsplit_gat_bwd(gsplit_ctx *ctx, const gsplit_gat_params *p, const void *d_feat_local,
                              const float *d_grad_logits, float *const *d_gw, float *const *d_ga_src,
                              float *const *d_ga_dst, float *const *d_gbias, void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    int rc = check_params(ctx, p, "gsplit_gat_bwd");
    if (rc) return rc;
    if (!d_feat_local || !d_grad_logits || !d_gw || !d_ga_src || !d_ga_dst || !d_gbias)
        return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_gat_bwd: NULL buffer");
    GsGatBuf &gb = ctx->gat;
    if (!gb.ready || !gb.fwd_done || gb.fwd_batch != ctx->batch_id)
        return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_gat_bwd: needs gsplit_gat_fwd on the current batch first");
    const int L = ctx->L, S = ctx->S;
    for (int l = 0; l <= L; ++l)
        if (gb.dims[l] != p->dims[l] || (l < L && gb.heads[l] != p->heads[l]))
            return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_gat_bwd: parameters differ from the forward pass");
    for (int l = 0; l < L; ++l)
        if (!d_gw[l] || !d_ga_src[l] || !d_ga_dst[l] || !d_gbias[l])
            return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_gat_bwd: NULL gradient pointer");
    hipStream_t st = (hipStream_t)stream;
    for (int l = L - 1; l >= 0; --l) {
        const GatDims d = dims_of(ctx, p, l);
        const int D = p->dims[l];
        const bool last = l == L - 1;
        const GsLayerBuf &B = ctx->layer[l];
        const float *hin = l == 0 ? (const float *)d_feat_local : gb.hidden[l];
        const RowShape rs = row_shape(d);
        const size_t lds = sizeof(float) * 4 * (1 + d.fan) * (1 + d.K);
        {
            GatBwdDstArgs a{gb.zext[l], B.blk_indptr, B.edge_row, B.self_row, gb.alpha[l],
                            last ? d_grad_logits : gb.ghid[l + 1], last ? nullptr : gb.hidden[l + 1],
                            gb.gagg[l], gb.de[l], gb.der[l], gb.bias_part[l], p->dims[l + 1]};
            const dim3 grid(gb.bias_slabs[l]);
            GsTimeScope ts(ctx, "gat_bwd_dst", l, st);
#define GAT_CALL(VW, NV)                                                                                         \
    if (last) hipLaunchKernelGGL((k_gat_bwd_dst<VW, NV, true>), grid, dim3(256), lds, st, a, d, ctx->d_meta + (l + 1), S); \
    else hipLaunchKernelGGL((k_gat_bwd_dst<VW, NV, false>), grid, dim3(256), lds, st, a, d, ctx->d_meta + (l + 1), S)
            GAT_DISPATCH(rs, GAT_CALL);
#undef GAT_CALL
        }
        {
            GatBwdSrcArgs a{B.rev_ptr, B.rev_cnt, B.rev_list, B.rev_eid, gb.alpha[l], gb.de[l], gb.der[l], gb.gagg[l],
                            gb.dzext[l]};
            const dim3 grid(grid_1d(ctx, ctx->ub_front[l] * 64));
            GsTimeScope ts(ctx, "gat_bwd_src", l, st);
#define GAT_CALL(VW, NV) hipLaunchKernelGGL((k_gat_bwd_src<VW, NV>), grid, dim3(256), 0, st, a, d, ctx->d_meta + l, S)
            GAT_DISPATCH(rs, GAT_CALL);
#undef GAT_CALL
        }
        {
            // G = h^T dz_ext over the rows of level l, split-K
            MatRows in{hin, 0, D};
            MatRows dz{gb.dzext[l], 0, d.ZW};
            EpiGradW ew{gb.gw_part[l], D + 1, d.ZW, D};
            GsTimeScope ts(ctx, "gat_grad_w", l, st);
            launch_grad_w(st, gb.nchunk[l], D % 4 == 0 && aligned16(hin), true, in, dz, ew, ctx->d_meta + l, S);
        }
        if (l > 0) {
            MatRows dz{gb.dzext[l], 0, d.ZW};
            MatRows w{gb.wext[l], D, d.ZW};
            EpiStore epi{gb.ghid[l], D, 0, D};
            GsTimeScope ts(ctx, "gat_grad_in", l, st);
            launch_rows_gemm<true>(ctx, st, ctx->ub_front[l], true, dz, w, epi, ctx->d_meta + l);
        }
    }
    {
        GatReduce gr;
        int64_t wmax = 1;
        for (int l = 0; l < L; ++l) {
            const GatDims d = dims_of(ctx, p, l);
            gr.part[l] = gb.gw_part[l]; gr.gmat[l] = gb.gmat[l]; gr.D[l] = p->dims[l]; gr.ZW[l] = d.ZW;
            gr.nchunk[l] = gb.nchunk[l];
            wmax = std::max<int64_t>(wmax, (int64_t)p->dims[l] * d.ZW);
        }
        GsTimeScope ts(ctx, "gat_reduce", -1, st);
        hipLaunchKernelGGL(k_gat_reduce, dim3((unsigned)std::min<int64_t>(256, gs_ceil_div(wmax, 256)), L), dim3(256), 0, st,
                           gr, ctx->d_meta, S);
    }
    {
        GatFinish gf;
        int64_t wmax = 1;
        for (int l = 0; l < L; ++l) {
            const GatDims d = dims_of(ctx, p, l);
            gf.gmat[l] = gb.gmat[l]; gf.w[l] = (const float *)p->d_w[l]; gf.a_src[l] = (const float *)p->d_a_src[l];
            gf.a_dst[l] = (const float *)p->d_a_dst[l]; gf.bias_part[l] = gb.bias_part[l];
            gf.gw[l] = d_gw[l]; gf.ga_src[l] = d_ga_src[l]; gf.ga_dst[l] = d_ga_dst[l]; gf.gb[l] = d_gbias[l];
            gf.D[l] = p->dims[l]; gf.K[l] = d.K; gf.F[l] = d.F; gf.ZW[l] = d.ZW; gf.PW[l] = p->dims[l + 1];
            gf.slabs[l] = gb.bias_slabs[l];
            wmax = std::max<int64_t>(wmax, (int64_t)p->dims[l] * d.HF);
        }
        int hf_max = 1;
        for (int l = 0; l < L; ++l) hf_max = std::max(hf_max, gf.K[l] * gf.F[l]);
        {
            GsTimeScope ts(ctx, "gat_finish_w", -1, st);
            hipLaunchKernelGGL(k_gat_finish, dim3((unsigned)std::min<int64_t>(256, gs_ceil_div(wmax, 256)), L), dim3(256), 0,
                               st, gf);
        }
        GsTimeScope ts(ctx, "gat_finish_cols", -1, st);
        hipLaunchKernelGGL(k_gat_finish_cols, dim3((unsigned)gs_ceil_div(hf_max, 64), L), dim3(1024), 0, st, gf);
    }
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}
