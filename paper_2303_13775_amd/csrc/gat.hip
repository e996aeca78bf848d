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
//
// The bottom layer needs no input gradient and has several times more source rows than
// destinations, so (when its shapes allow) it runs in the other order: the attention-weighted sum
// is taken over the raw input rows per head, P_i^k = sum_j alpha_ij^k h_j, and the transform is a
// per-head product over the destinations only, out_i^k = P_i^k W^k.  Scores come from
// h (W a_src), h (W a_dst) (2 K columns), and the backward pass needs neither the scatter side of
// the shuffle index nor a gradient row per source:  dP^k = dagg^k W^kT,  d alpha_ij = h_j . dP_i^k,
// d W^k = P^kT dagg^k, and the columns G_src, G_dst of G are sums of d e_ij h_j over entries.
#include <algorithm>

#include "gsplit_internal.h"

namespace {

#include "gemm_f32.h"

constexpr float NEG_SLOPE = 0.2f;

// 128 x 64 tile: for products whose output is 64 wide (one head) or just past a multiple of 128
using TileTall = Tile<128, 64, 4, 2, 1, true>;
// an output width just past a multiple of 128 (K F + 2 K = 264) leaves the last 128-wide column tile
// almost empty: 64-wide column tiles then waste 21 % of the matrix-core work instead of 45 %
inline bool narrow_tail(int n_out) { return n_out > 128 && n_out % 128 > 0 && n_out % 128 <= 64; }

// Per-layer sizes.  A wave owns one row; its 64 lanes are dealt to the heads in groups of
// lph = 64 / (K rounded up to a power of two) lanes, lane `sub` of head k holding features
// (sub + lph t) VW + 0..VW-1, t < NV, of that head.
struct GatDims {
    int K, F, HF, ZW, lph, fan;
    int64_t self_base;      // slot of destination i's self entry = self_base + i (edge slots come first)
};

// plain store; with act (the ELU outputs h' at the same positions) the value is first multiplied by
// ELU'(.) = 1 for h' > 0, else h' + 1
struct EpiStore {
    float *out; int ld; int rows; int cols; const float *act;
    __device__ __forceinline__ float col(int) const { return 0.f; }
    __device__ __forceinline__ float row(int) const { return 0.f; }
    __device__ __forceinline__ void store(int m, int n, float v, float, float) const {
        if (m < rows && n < cols) {
            if (act) {
                const float hv = act[(int64_t)m * ld + n];
                v *= hv > 0.f ? 1.f : hv + 1.f;
            }
            out[(int64_t)m * ld + n] = v;
        }
    }
};

// C = A B (B_KC = false: b is K x N) or C = A B^T (B_KC = true: b is N x K) for the rows of one
// level; persistent row-block tiling
template <class T, int VA, int VB, bool B_KC>
__global__ __launch_bounds__(GNT) __attribute__((amdgpu_waves_per_eu(T::LEAN ? 2 * T::OCC : 2, T::LEAN ? 2 * T::OCC : 8)))
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

// value of another lane through the data-parallel-primitive path of the vector ALU (no LDS
// traffic): CTRL 0xB1 / 0x4E = lane ^ 1 / lane ^ 2 inside a quad, 0x141 / 0x140 = mirror inside
// 8 / 16 lanes
// 0x142 / 0x143 = lane 15 of every row of 16 lanes to the next row / lane 31 to the upper two rows;
// rows outside ROW_MASK receive zero
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_get(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, true));
}
// sum over aligned groups of lph lanes (a power of two), the same bits in every lane of a group:
// after the quad steps every lane of a quad holds the quad's sum, a mirror then pairs each lane
// with one of the other half; only groups of 32 and 64 lanes need the LDS crossbar
__device__ __forceinline__ float head_sum(float v, int lph) {
    if (lph >= 2) v += dpp_get<0xB1>(v);
    if (lph >= 4) v += dpp_get<0x4E>(v);
    if (lph >= 8) v += dpp_get<0x141>(v);
    if (lph >= 16) v += dpp_get<0x140>(v);
    if (lph >= 32) v += __shfl_xor(v, 16);
    if (lph >= 64) v += __shfl_xor(v, 32);
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
// The entries of a row were filled through an atomic cursor, in no fixed order; they are taken in
// ascending order of their codes (2 * destination, + 1 for an edge; distinct within a row), so the
// sums do not depend on it: the wave sorts (code, place) pairs across its lanes, at most 64 at a
// time; a longer row is taken in windows of ascending values whose upper ends bisection finds.
__device__ __forceinline__ unsigned long long wave_sort_pairs(unsigned long long v, int p2) {
    const int lane = threadIdx.x & 63;
    for (int k = 2; k <= p2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            const unsigned long long o = __shfl_xor(v, j);
            v = (((lane & j) == 0) == ((lane & k) == 0)) ? (v < o ? v : o) : (v > o ? v : o);
        }
    }
    return v;
}

template <int VW, int NV>
__global__ __launch_bounds__(256) void k_gat_bwd_src(GatBwdSrcArgs g, GatDims d, const GsLevelMeta *__restrict__ meta_lo, int S) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n0 = meta_lo->front_off[S];
    const int K = d.K, F = d.F, HF = d.HF, ZW = d.ZW, lph = d.lph;
    const int k = lane / lph, sub = lane % lph;
    const bool ok = k < K;
    constexpr unsigned long long PAD = ~0ull;
    for (int u = blockIdx.x * 4 + wave; u < n0; u += gridDim.x * 4) {
        const int p0 = g.rev_ptr[u], cnt = g.rev_cnt[u];
        float acc[NV * VW];
#pragma unroll
        for (int c = 0; c < NV * VW; ++c) acc[c] = 0.f;
        float dsrc = 0.f, ddst = 0.f;
        int lo = -1;
        for (int taken = 0; taken < cnt;) {
            int T = 0x7FFFFFFE;
            if (cnt > 64) {
                // largest T with at most 64 codes in (lo, T]
                int a = lo + 1, b = 0x7FFFFFFE;
                while (a < b) {
                    const int mid = a + ((b - a + 1) >> 1);
                    int inside = 0;
                    for (int t = lane; t < cnt; t += 64) {
                        const int code = g.rev_list[p0 + t];
                        inside += (code > lo && code <= mid) ? 1 : 0;
                    }
                    for (int o = 32; o > 0; o >>= 1) inside += __shfl_xor(inside, o);
                    if (inside <= 64) a = mid; else b = mid - 1;
                }
                T = a;
            }
            // the window's (code, place) pairs, one per lane, sorted by code
            unsigned long long mine = PAD;
            int m = 0;
            if (cnt <= 64) {
                if (lane < cnt) mine = ((unsigned long long)(uint32_t)g.rev_list[p0 + lane] << 32) | (uint32_t)(p0 + lane);
                m = cnt;
            } else {
                for (int t0 = 0; t0 < cnt; t0 += 64) {
                    const int t = t0 + lane;
                    const int code = t < cnt ? g.rev_list[p0 + t] : 0;
                    const bool in = t < cnt && code > lo && code <= T;
                    const unsigned long long bal = __ballot(in);
                    // hand the pair to lane `at` of the window (at most 64 in all)
                    const unsigned long long pair = ((unsigned long long)(uint32_t)code << 32) | (uint32_t)(p0 + t);
                    for (int src = 0; src < 64; ++src) {
                        const bool has = (bal >> src) & 1ull;
                        if (!has) continue;                     // uniform: bal is the same in every lane
                        const int dst = m + __popcll(bal & ((1ull << src) - 1ull));
                        const unsigned long long v = __shfl(pair, src);
                        if (lane == dst) mine = v;
                    }
                    m += __popcll(bal);
                }
                m = min(m, 64);
            }
            int p2 = 1;
            while (p2 < m) p2 <<= 1;
            const unsigned long long sorted = p2 > 1 ? wave_sort_pairs(mine, p2) : mine;
            for (int x = 0; x < m; x += 4) {
                float gv[4][NV * VW], a[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bool in = x + q < m;
                    const unsigned long long pr = __shfl(sorted, min(x + q, 63));
                    const int code = in ? (int)(uint32_t)(pr >> 32) : 0;
                    const int place = in ? (int)(uint32_t)pr : p0;
                    const int i = code >> 1;
                    const int64_t slot = (code & 1) ? (int64_t)g.rev_eid[place] : d.self_base + i;
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
            lo = T;
            taken += max(m, 1);         // (a window is never empty; the loop ends whatever the row holds)
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

// ---- bottom layer, aggregate-then-transform ---------------------------------------------------
// window of a row-major matrix: rows x cols at row stride ld (same accessor interface as MatRows)
struct MatLd {
    const float *p; int rows; int cols; int ld;
    template <int VW>
    __device__ __forceinline__ const float *at(int o, int i, bool &in) const {
        in = o < rows && i < cols;
        const int oc = min(o, rows - 1), ic = min(i, cols - VW);
        return p + (int64_t)oc * ld + ic;
    }
    __device__ __forceinline__ int tok(int i) const { return min(i, cols - 4); }
    __device__ __forceinline__ const float *km(int k, int t) const { return p + (int64_t)k * ld + t; }
};

struct EpiHeadElu {      // hidden[i, off + n] = ELU(v + bias[off + n])
    float *out; const float *bias; int ld; int rows; int cols; int off;
    __device__ __forceinline__ float col(int n) const { return n < cols ? bias[off + n] : 0.f; }
    __device__ __forceinline__ float row(int) const { return 0.f; }
    __device__ __forceinline__ void store(int m, int n, float v, float, float b) const {
        if (m < rows && n < cols) {
            const float z = v + b;
            out[(int64_t)m * ld + off + n] = z > 0.f ? z : expm1f(z);
        }
    }
};
struct EpiHeadStore {
    float *out; int ld; int rows; int cols; int off;
    __device__ __forceinline__ float col(int) const { return 0.f; }
    __device__ __forceinline__ float row(int) const { return 0.f; }
    __device__ __forceinline__ void store(int m, int n, float v, float, float) const {
        if (m < rows && n < cols) out[(int64_t)m * ld + off + n] = v;
    }
};

// one product per head over the destination rows: head k takes the window of a at column
// k * a_step, of b at column k * b_step, and writes at column k * o_step
template <class T, bool B_KC, class EF>
__global__ __launch_bounds__(GNT) __attribute__((amdgpu_waves_per_eu(4, 4)))
void k_gat0_head_gemm(MatLd a, MatLd b, EF epi, int heads, int a_step, int b_step, int o_step,
                      const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int n_out = B_KC ? b.rows : b.cols;
    const int tiles_m = (n1 + T::BM - 1) / T::BM, tiles_n = (n_out + T::BN - 1) / T::BN;
    const int per_head = ((tiles_m + 7) & ~7) * tiles_n;
    a.rows = n1; epi.rows = n1;
    for (int gid = blockIdx.x; gid < per_head * heads; gid += gridDim.x) {
        const int head = gid / per_head;
        int m0, n0;
        if (!next_tile<T>(gid - head * per_head, tiles_m, tiles_n, m0, n0)) continue;
        MatLd ah = a, bh = b;
        EF eh = epi;
        ah.p += head * a_step; bh.p += head * b_step; eh.off = head * o_step;
        gemm_tile<T, true, B_KC, 4, 4>(m0, n0, n1, n_out, 0, ah.cols, ah, bh, eh);
    }
}

// partial d W^k = P^kT dagg^k over one chunk of destination rows (split-K), slab
// [chunk][head][(D + 1) x F]; the last row of a slab holds the column sums of dagg^k (bias gradient)
template <class T>
__global__ __launch_bounds__(GNT) __attribute__((amdgpu_waves_per_eu(4, 4)))
void k_gat0_grad_w(MatLd a, MatLd dz, EpiGradW epi, int nchunk, int heads, int tiles_m, int tiles_n,
                   const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int kchunk = grad_w_chunk_rows(n1, nchunk, GRAD_W_ROWS_MIN);
    const int tiles = tiles_m * tiles_n;
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int tile = j % tiles, head = (j / tiles) % heads, chunk = (j / (tiles * heads)) * 8 + xcd;
    const int k_begin = chunk * kchunk;
    if (k_begin >= n1) return;
    a.rows = n1; dz.rows = n1;
    a.p += head * a.cols; dz.p += head * dz.cols;
    const int k_end = min(n1, k_begin + kchunk);
    epi.part += ((int64_t)chunk * heads + head) * epi.rows * epi.N;
    gemm_tile<T, false, false, 4, 4, MatLd, MatLd, EpiGradW, false, true>(
        (tile % tiles_m) * T::BM, (tile / tiles_m) * T::BN, a.cols, dz.cols, k_begin, k_end, a, dz, epi);
}

// sum over the wave without the LDS crossbar; the result is valid in lanes 48..63 only
__device__ __forceinline__ float wave_sum_top(float v) {
    v = head_sum(v, 16);                    // every lane: the sum of its row of 16
    v += dpp_get<0x142, 0xA>(v);            // rows 1 and 3 add the row below them
    v += dpp_get<0x143, 0xC>(v);            // rows 2 and 3 add lane 31 (rows 0 + 1)
    return v;
}
// lanes with the same lane % kp form a class
__device__ __forceinline__ float class_sum(float v, int kp) {
    for (int o = kp; o < 64; o <<= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ float class_max(float v, int kp) {
    for (int o = kp; o < 64; o <<= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

// score terms of every input row: s0[u, c] = h_u . wa[:, c], c < 2 K (wa = the last columns of
// W_ext: W a_src per head, then W a_dst per head).  Eight lanes per row, 16 bytes per lane and
// load, four loads in flight.
template <int KP>
__global__ __launch_bounds__(256) void k_gat0_scores(const float *__restrict__ h, int D, const float *__restrict__ wext,
                                                     int ZW, int HF, int K, float *__restrict__ s0,
                                                     const GsLevelMeta *__restrict__ meta_lo, int S) {
    extern __shared__ float s_wa[];        // [2 K][D]
    for (int x = threadIdx.x; x < 2 * K * D; x += 256) {
        const int dd = x / (2 * K), c = x - dd * 2 * K;
        s_wa[c * D + dd] = wext[(int64_t)dd * ZW + HF + c];
    }
    __syncthreads();
    const int n0 = meta_lo->front_off[S];
    const int sub = threadIdx.x & 7;
    const int nv4 = D >> 2;
    for (int u = blockIdx.x * 32 + (threadIdx.x >> 3); u < ((n0 + 31) & ~31); u += gridDim.x * 32) {
        float acc[2 * KP];
#pragma unroll
        for (int c = 0; c < 2 * KP; ++c) acc[c] = 0.f;
        if (u < n0)
            for (int v0 = sub; v0 < nv4; v0 += 32) {
                float4 x[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int v = v0 + 8 * t;
                    x[t] = v < nv4 ? *reinterpret_cast<const float4 *>(h + (int64_t)u * D + 4 * v) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int v = min(v0 + 8 * t, nv4 - 1);      // a vector past the row is zero: any weights do
#pragma unroll
                    for (int c = 0; c < 2 * KP; ++c)
                        if (c < 2 * K) {
                            const float4 w = *reinterpret_cast<const float4 *>(s_wa + c * D + 4 * v);
                            acc[c] += x[t].x * w.x + x[t].y * w.y + x[t].z * w.z + x[t].w * w.w;
                        }
                }
            }
#pragma unroll
        for (int c = 0; c < 2 * KP; ++c) acc[c] = head_sum(acc[c], 8);
        if (u < n0) {
#pragma unroll
            for (int c = 0; c < 2 * KP; ++c)
                if ((c & 7) == sub && c < 2 * K) s0[(int64_t)u * 2 * K + c] = acc[c];
        }
    }
}

struct Gat0Args {
    const float *h; const float *s0; const int32_t *blk_indptr; const int32_t *edge_row; const int32_t *self_row;
    float *alpha; float *pagg; const float *dp; float *q_part;
    int D, K, fan; int64_t self_base;
    int ch;     // input rows a wave of k_gat0_bwd stages in LDS at a time
};

// the lane's NV float4 of one input row (lane + 64 t), zeros past the row
template <int NV>
__device__ __forceinline__ void load_row4(const float *__restrict__ row, int lane, int nv4, float (&v)[NV * 4]) {
#pragma unroll
    for (int t = 0; t < NV; ++t) {
        const int c = lane + 64 * t;
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c < nv4) x = *reinterpret_cast<const float4 *>(row + 4 * c);
        v[t * 4] = x.x; v[t * 4 + 1] = x.y; v[t * 4 + 2] = x.z; v[t * 4 + 3] = x.w;
    }
}

// edge softmax of the bottom layer and P_i^k = sum_j alpha_ij^k h_j, one wave per destination:
// entry j and head k sit on lane (j KP + k) mod 64 for the softmax, then the lanes run over the
// input features and every lane keeps one accumulator per head
template <int NV, int KP>
__global__ __launch_bounds__(256) void k_gat0_aggregate(Gat0Args g, const GsLevelMeta *__restrict__ meta_up, int S) {
    extern __shared__ float smem[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int per_wave = (1 + g.fan) * (1 + KP);
    int *s_row = reinterpret_cast<int *>(smem + wave * per_wave);
    float *s_val = smem + wave * per_wave + (1 + g.fan);
    const int n1 = meta_up->front_off[S];
    const int D = g.D, K = g.K, nv4 = D >> 2;
    const int k = lane % KP;
    const bool ok = k < K;
    for (int i = blockIdx.x * 4 + wave; i < n1; i += gridDim.x * 4) {
        const int e0 = g.blk_indptr[i], e1 = g.blk_indptr[i + 1];
        const int n_ent = 1 + e1 - e0;
        const int self = g.self_row[i];
        const float er = ok ? g.s0[(int64_t)self * 2 * K + K + k] : 0.f;
        float m = -3.4e38f;
        for (int idx = lane; idx < n_ent * KP; idx += 64) {
            const int j = idx / KP;
            const int row = j == 0 ? self : g.edge_row[e0 + j - 1];
            if (k == 0) s_row[j] = row;
            if (ok) {
                const float raw = er + g.s0[(int64_t)row * 2 * K + k];
                const float e = raw > 0.f ? raw : NEG_SLOPE * raw;
                s_val[idx] = e;
                m = fmaxf(m, e);
            }
        }
        m = class_max(m, KP);
        float s = 0.f;
        if (ok)
            for (int idx = lane; idx < n_ent * KP; idx += 64) {
                const float p = expf(s_val[idx] - m);
                s_val[idx] = p;
                s += p;
            }
        s = class_sum(s, KP);
        if (ok)
            for (int idx = lane; idx < n_ent * KP; idx += 64) {
                const int j = idx / KP;
                const float a = s_val[idx] / s;
                s_val[idx] = a;
                const int64_t slot = j == 0 ? g.self_base + i : (int64_t)(e0 + j - 1);
                g.alpha[slot * K + k] = a;
            }
        __builtin_amdgcn_wave_barrier();
        float acc[KP][NV * 4];
#pragma unroll
        for (int kk = 0; kk < KP; ++kk)
#pragma unroll
            for (int c = 0; c < NV * 4; ++c) acc[kk][c] = 0.f;
        for (int j = 0; j < n_ent; j += 4) {
            float hv[4][NV * 4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row = j + q < n_ent ? s_row[j + q] : self;
                load_row4<NV>(g.h + (int64_t)row * D, lane, nv4, hv[q]);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (j + q < n_ent) {
#pragma unroll
                    for (int kk = 0; kk < KP; ++kk) {
                        const float a = kk < K ? s_val[(j + q) * KP + kk] : 0.f;
#pragma unroll
                        for (int c = 0; c < NV * 4; ++c) acc[kk][c] += a * hv[q][c];
                    }
                }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int kk = 0; kk < KP; ++kk)
            if (kk < K) {
#pragma unroll
                for (int t = 0; t < NV; ++t) {
                    const int c = lane + 64 * t;
                    if (c < nv4)
                        *reinterpret_cast<float4 *>(g.pagg + ((int64_t)i * K + kk) * D + 4 * c) =
                            make_float4(acc[kk][t * 4], acc[kk][t * 4 + 1], acc[kk][t * 4 + 2], acc[kk][t * 4 + 3]);
                }
            }
    }
}

// Backward of the bottom layer over the destinations, one wave each: d alpha_ij^k = h_j . dP_i^k,
// the softmax and LeakyReLU derivatives d e_ij^k, and the wave's running sums
//   q_src^k = sum d e_ij^k h_j   (over all entries),   q_dst^k = sum_i (sum_j d e_ij^k) h_i
// which are the columns G_src, G_dst of G once added over all waves (one slab per wave).
template <int NV, int KP>
__global__ __launch_bounds__(256) void k_gat0_bwd(Gat0Args g, const GsLevelMeta *__restrict__ meta_up, int S) {
    extern __shared__ float smem[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int D = g.D, K = g.K, nv4 = D >> 2, CH = g.ch;
    // per wave: entry rows | one value per entry and head | per-head sums | CH staged input rows
    const int w_row = (1 + g.fan + 3) & ~3, w_val = ((1 + g.fan) * KP + 3) & ~3, w_ds = (KP + 3) & ~3;
    float *base = smem + wave * (w_row + w_val + w_ds + CH * D);
    int *s_row = reinterpret_cast<int *>(base);
    float *s_val = base + w_row;
    float *s_ds = s_val + w_val;
    float *s_h = s_ds + w_ds;
    const int n1 = meta_up->front_off[S];
    const int k = lane % KP;
    const bool ok = k < K;
    // Input rows of entries [c0, c0 + nc) straight from global memory into LDS (lane L of a 16-byte
    // direct load lands at base + 16 L): every row of the chunk is in flight at once and costs no
    // registers
    auto stage = [&](int c0, int nc) {
        for (int q = 0; q < nc; ++q) {
            const float *src = g.h + (int64_t)s_row[c0 + q] * D;
#pragma unroll
            for (int t = 0; t < NV; ++t) {
                const int c = lane + 64 * t;
                if (c < nv4)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + 4 * c),
                                                     (__attribute__((address_space(3))) void *)(s_h + q * D + 256 * t), 16, 0, 0);
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_wave_barrier();
    };
    auto staged = [&](int q, float (&v)[NV * 4]) {
#pragma unroll
        for (int t = 0; t < NV; ++t) {
            const int c = lane + 64 * t;
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c < nv4) x = *reinterpret_cast<const float4 *>(s_h + q * D + 4 * c);
            v[t * 4] = x.x; v[t * 4 + 1] = x.y; v[t * 4 + 2] = x.z; v[t * 4 + 3] = x.w;
        }
    };
    float qs[KP][NV * 4], qd[KP][NV * 4];
#pragma unroll
    for (int kk = 0; kk < KP; ++kk)
#pragma unroll
        for (int c = 0; c < NV * 4; ++c) qs[kk][c] = qd[kk][c] = 0.f;
    for (int i = blockIdx.x * 4 + wave; i < n1; i += gridDim.x * 4) {
        const int e0 = g.blk_indptr[i], e1 = g.blk_indptr[i + 1];
        const int n_ent = 1 + e1 - e0;
        const int self = g.self_row[i];
        for (int j = lane; j < n_ent; j += 64) s_row[j] = j == 0 ? self : g.edge_row[e0 + j - 1];
        float dp[KP][NV * 4];
#pragma unroll
        for (int kk = 0; kk < KP; ++kk) {
            if (kk < K) load_row4<NV>(g.dp + ((int64_t)i * K + kk) * D, lane, nv4, dp[kk]);
            else {
#pragma unroll
                for (int c = 0; c < NV * 4; ++c) dp[kk][c] = 0.f;
            }
        }
        __builtin_amdgcn_wave_barrier();
        for (int c0 = 0; c0 < n_ent; c0 += CH) {
            const int nc = min(CH, n_ent - c0);
            stage(c0, nc);
            for (int q0 = 0; q0 < nc; q0 += 4) {
                float p[4][KP];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float hv[NV * 4];
                    staged(min(q0 + q, nc - 1), hv);
#pragma unroll
                    for (int kk = 0; kk < KP; ++kk) {
                        float t = 0.f;
#pragma unroll
                        for (int c = 0; c < NV * 4; ++c) t += hv[c] * dp[kk][c];
                        p[q][kk] = t;
                    }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int kk = 0; kk < KP; ++kk) p[q][kk] = wave_sum_top(p[q][kk]);
                if (lane == 63) {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (q0 + q < nc) {
#pragma unroll
                            for (int kk = 0; kk < KP; ++kk) s_val[(c0 + q0 + q) * KP + kk] = p[q][kk];
                        }
                }
            }
            __builtin_amdgcn_wave_barrier();     // the next chunk overwrites the staged rows
        }
        const float er = ok ? g.s0[(int64_t)self * 2 * K + K + k] : 0.f;
        float tsum = 0.f;
        if (ok)
            for (int idx = lane; idx < n_ent * KP; idx += 64) {
                const int j = idx / KP;
                const int64_t slot = j == 0 ? g.self_base + i : (int64_t)(e0 + j - 1);
                tsum += g.alpha[slot * K + k] * s_val[idx];
            }
        tsum = class_sum(tsum, KP);
        float dsum = 0.f;
        if (ok)
            for (int idx = lane; idx < n_ent * KP; idx += 64) {
                const int j = idx / KP;
                const int64_t slot = j == 0 ? g.self_base + i : (int64_t)(e0 + j - 1);
                const float raw = er + g.s0[(int64_t)s_row[j] * 2 * K + k];
                const float v = g.alpha[slot * K + k] * (s_val[idx] - tsum) * (raw > 0.f ? 1.f : NEG_SLOPE);
                s_val[idx] = v;
                dsum += v;
            }
        dsum = class_sum(dsum, KP);
        if (lane < KP) s_ds[lane] = dsum;
        __builtin_amdgcn_wave_barrier();
        for (int c0 = 0; c0 < n_ent; c0 += CH) {
            const int nc = min(CH, n_ent - c0);
            if (n_ent > CH) stage(c0, nc);      // a single chunk is still staged
            for (int q = 0; q < nc; ++q) {
                float hv[NV * 4];
                staged(q, hv);
#pragma unroll
                for (int kk = 0; kk < KP; ++kk) {
                    const float de = kk < K ? s_val[(c0 + q) * KP + kk] : 0.f;
#pragma unroll
                    for (int c = 0; c < NV * 4; ++c) qs[kk][c] += de * hv[c];
                }
                if (c0 + q == 0) {
#pragma unroll
                    for (int kk = 0; kk < KP; ++kk) {
                        const float ds = kk < K ? s_ds[kk] : 0.f;
#pragma unroll
                        for (int c = 0; c < NV * 4; ++c) qd[kk][c] += ds * hv[c];
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
    // one slab per workgroup: the four waves' sums added in wave order
    __shared__ float s_red[4][NV * 256];
    float *slab = g.q_part + (int64_t)blockIdx.x * 2 * K * D;
#pragma unroll
    for (int kk = 0; kk < 2 * KP; ++kk) {
        const int head = kk % KP;
        if (head >= K) continue;
        const float(&src)[NV * 4] = kk < KP ? qs[head] : qd[head];
#pragma unroll
        for (int c = 0; c < NV * 4; ++c) s_red[wave][c * 64 + lane] = src[c];
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int t = 0; t < NV; ++t) {
                const int c4 = lane + 64 * t;
                float v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int c = (t * 4 + j) * 64 + lane;
                    v[j] = ((s_red[0][c] + s_red[1][c]) + s_red[2][c]) + s_red[3][c];
                }
                if (c4 < nv4)
                    *reinterpret_cast<float4 *>(slab + ((int64_t)(kk < KP ? 0 : K) + head) * D + 4 * c4) =
                        make_float4(v[0], v[1], v[2], v[3]);
            }
        }
        __syncthreads();
    }
}

// Sum of column col0 + (tid & 15) over n_slabs slabs of `stride` floats by a workgroup of 1024: slab
// z is read by lane group z mod 64, eight loads in flight, and the 64 partial sums are added in
// group order.  Valid in threads 0..15.
__device__ __forceinline__ float slab_sum_16x64(const float *__restrict__ p, int n_cols, int64_t stride, int n_slabs,
                                                int col0, float (*red)[16]) {
    const int x = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int c = col0 + x;
    float s = 0.f;
    if (c < n_cols) {
        const float *q = p + c;
        int z = ty;
        for (; z + 7 * 64 < n_slabs; z += 8 * 64) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = q[(int64_t)(z + 64 * j) * stride];
#pragma unroll
            for (int j = 0; j < 8; ++j) s += v[j];
        }
        for (; z < n_slabs; z += 64) s += q[(int64_t)z * stride];
    }
    __syncthreads();        // red may still be read from a previous call
    red[ty][x] = s;
    __syncthreads();
    s = 0.f;
    if (ty == 0)
        for (int j = 0; j < 64; ++j) s += red[j][x];
    return s;
}

// G of the bottom layer and its bias gradient: the z columns and the bias from the split-K slabs of
// the per-head products, the G_src / G_dst columns from the workgroup slabs of k_gat0_bwd
__global__ __launch_bounds__(1024) void k_gat0_reduce(const float *__restrict__ w_part, int nchunk,
                                                      const float *__restrict__ q_part, int q_slabs, int D, int K, int F,
                                                      int ZW, float *__restrict__ gmat, float *__restrict__ gbias,
                                                      const GsLevelMeta *__restrict__ meta_up, int S) {
    __shared__ float red[64][16];
    const int HF = K * F;
    const int x = threadIdx.x & 15;
    const int n1 = meta_up->front_off[S];
    const int kchunk = grad_w_chunk_rows(n1, nchunk, GRAD_W_ROWS_MIN);
    const int chunks = (n1 + kchunk - 1) / kchunk;
    const int per_row = (F + 15) / 16;                      // workgroups per row of one head's slab
    const int n_w = K * (D + 1) * per_row;
    if ((int)blockIdx.x < n_w) {
        const int head = blockIdx.x / ((D + 1) * per_row), r = blockIdx.x % ((D + 1) * per_row);
        const int dd = r / per_row, f0 = (r % per_row) * 16;
        const float s = slab_sum_16x64(w_part + ((int64_t)head * (D + 1) + dd) * F, F, (int64_t)K * (D + 1) * F, chunks, f0,
                                       red);
        if (threadIdx.x < 16 && f0 + x < F) {
            if (dd < D) gmat[(int64_t)dd * ZW + head * F + f0 + x] = s;
            else gbias[head * F + f0 + x] = s;
        }
        return;
    }
    const int e0 = ((int)blockIdx.x - n_w) * 16;             // elements of the [2 K][D] slab
    const float s = slab_sum_16x64(q_part, 2 * K * D, (int64_t)2 * K * D, q_slabs, e0, red);
    const int e = e0 + x;
    if (threadIdx.x < 16 && e < 2 * K * D) {
        const int c = e / D, dd = e - c * D;
        gmat[(int64_t)dd * ZW + HF + c] = s;
    }
}

// G = sum of the split-K slabs of h^T dz_ext in slab order, all layers in one launch
struct GatReduce {
    const float *part[GS_MAXL]; float *gmat[GS_MAXL]; int D[GS_MAXL]; int ZW[GS_MAXL]; int nchunk[GS_MAXL];
};
__global__ __launch_bounds__(256) void k_gat_reduce(GatReduce g, const GsLevelMeta *__restrict__ meta, int S) {
    const int l = blockIdx.y;
    if (g.nchunk[l] == 0) return;      // this layer's G comes from k_gat0_reduce
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

// d a_src = W^T G_src, d a_dst = W^T G_dst and the bias gradient (sum of the bias slabs in slab
// order): 16 columns per workgroup, the long sums dealt to 64 lane groups and added in group order
__global__ __launch_bounds__(1024) void k_gat_finish_cols(GatFinish g) {
    __shared__ float red[64][16];
    const int l = blockIdx.y;
    const int D = g.D[l], K = g.K[l], F = g.F[l], ZW = g.ZW[l], HF = K * F, PW = g.PW[l];
    const float *G = g.gmat[l];
    const int x = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int c = blockIdx.x * 16 + x;
    if (blockIdx.x * 16 >= HF) return;
    float s = 0.f, t = 0.f;
    if (c < HF) {
        const int k = c / F;
        for (int dd = ty; dd < D; dd += 64) {
            const float wv = g.w[l][(int64_t)dd * HF + c];
            s += wv * G[(int64_t)dd * ZW + HF + k];
            t += wv * G[(int64_t)dd * ZW + HF + K + k];
        }
    }
    red[ty][x] = s;
    __syncthreads();
    if (ty == 0 && c < HF) {
        s = 0.f;
        for (int j = 0; j < 64; ++j) s += red[j][x];
        g.ga_src[l][c] = s;
    }
    __syncthreads();
    red[ty][x] = t;
    __syncthreads();
    if (ty == 0 && c < HF) {
        t = 0.f;
        for (int j = 0; j < 64; ++j) t += red[j][x];
        g.ga_dst[l][c] = t;
    }
    const float b = slab_sum_16x64(g.bias_part[l], PW, PW, g.slabs[l], blockIdx.x * 16, red);
    if (threadIdx.x < 16 && c < PW) g.gb[l][c] = b;
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

// vectors of four floats per lane that a bottom-layer row needs (lanes run over the input width)
int rows4_per_lane(int D) { return (int)gs_ceil_div(D, 256); }

// the bottom layer runs aggregate-then-transform when it is not also the last layer and its shapes
// fit the kernels: widths in 16-byte pieces, at most 8 heads, at most 32 accumulators per lane
bool agg_first_shapes(const gsplit_ctx *ctx, const gsplit_gat_params *p) {
    if (ctx->L < 2) return false;
    const int D = p->dims[0], K = p->heads[0], F = p->dims[1] / K;
    return D % 4 == 0 && F % 4 == 0 && K <= 8 && pow2_ceil(K) * rows4_per_lane(D) <= 8;
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
    gb.agg_first = agg_first_shapes(ctx, p);
    for (int l = 0; l < L; ++l) {
        const GatDims d = dims_of(ctx, p, l);
        const int D = p->dims[l];
        const int64_t n_lo = ctx->ub_front[l], n_up = ctx->ub_front[l + 1];
        const bool af = l == 0 && gb.agg_first;
        A(&gb.wext[l], (int64_t)D * d.ZW, "GAT extended weights");
        A(&gb.alpha[l], (d.self_base + n_up) * d.K, "GAT attention coefficients");
        if (!af) A(&gb.gagg[l], n_up * d.HF, "GAT aggregate gradients");     // else ghid[1] holds it
        A(&gb.gmat[l], (int64_t)D * d.ZW, "GAT weight-gradient product");
        if (l > 0) {
            A(&gb.hidden[l], n_lo * D, "GAT hidden activations");
            A(&gb.ghid[l], n_lo * D, "GAT hidden gradients");
        }
        if (af) {
            A(&gb.s0, n_lo * 2 * d.K, "GAT input-row scores");
            A(&gb.pagg, n_up * d.K * D, "GAT aggregated inputs");
            A(&gb.dpagg, n_up * d.K * D, "GAT aggregated-input gradients");
            // the backward row kernel keeps about a hundred registers a lane: four workgroups a compute unit
            gb.q_blocks = (int)std::min<int64_t>((int64_t)ctx->n_cu * 4, std::max<int64_t>(1, gs_ceil_div(n_up, 4)));
            A(&gb.q_part, (int64_t)gb.q_blocks * 2 * d.K * D, "GAT score-gradient sums");
            const int tiles = (int)(gs_ceil_div(D, TileTall::BM) * gs_ceil_div(d.F, TileTall::BN)) * d.K;
            gb.nchunk0 = (int)(gs_ceil_div(std::max<int64_t>(8, (int64_t)ctx->n_cu * 2 / tiles), 8) * 8);
            A(&gb.w0_part, (int64_t)gb.nchunk0 * d.K * (D + 1) * d.F, "GAT per-head weight-gradient partials");
            gb.nchunk[l] = 0;
            gb.bias_slabs[l] = 1;           // k_gat0_reduce leaves the finished sums in one slab
        } else {
            A(&gb.zext[l], n_lo * d.ZW, "GAT transformed rows");
            A(&gb.dzext[l], n_lo * d.ZW, "GAT transformed-row gradients");
            A(&gb.de[l], (d.self_base + n_up) * d.K, "GAT score gradients");
            A(&gb.der[l], n_up * d.K, "GAT destination score gradients");
            const int tiles = (int)(gs_ceil_div(D, TileMid::BM) * gs_ceil_div(d.ZW, TileMid::BN));
            gb.nchunk[l] = (int)(gs_ceil_div(std::max<int64_t>(8, (int64_t)ctx->n_cu * 3 / tiles), 8) * 8);
            A(&gb.gw_part[l], (int64_t)gb.nchunk[l] * (D + 1) * d.ZW, "GAT weight-gradient partials");
            gb.bias_slabs[l] = grid_1d(ctx, n_up * 64);
        }
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
    else if (!few_rows(ub, n_out, a.cols)) {
        if (narrow_tail(n_out)) launch_rows_gemm_t<TileTall, 4, B_KC>(ctx, st, ub, n_out, a, b, epi, meta_rows);
        // both operands k-contiguous: the unpadded direct-to-LDS tile (three workgroups a compute unit)
        else if (B_KC) launch_rows_gemm_t<TileMidDirect, 4, B_KC>(ctx, st, ub, n_out, a, b, epi, meta_rows);
        else launch_rows_gemm_t<TileMidLean, 4, B_KC>(ctx, st, ub, n_out, a, b, epi, meta_rows);
    }
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

// bottom layer: NV vectors of four floats per lane, KP = heads rounded up to a power of two
#define GAT0_DISPATCH(NVV, KPV, CALL)                                                              \
    do {                                                                                           \
        if ((NVV) == 1) {                                                                          \
            if ((KPV) == 1) { CALL(1, 1); } else if ((KPV) == 2) { CALL(1, 2); }                   \
            else if ((KPV) == 4) { CALL(1, 4); } else { CALL(1, 8); }                              \
        } else {                                                                                   \
            if ((KPV) == 1) { CALL(2, 1); } else if ((KPV) == 2) { CALL(2, 2); } else { CALL(2, 4); } \
        }                                                                                          \
    } while (0)

unsigned head_gemm_grid(const gsplit_ctx *ctx, int64_t ub, int n_out, int heads) {
    using T = TileTall;
    const int64_t want = gs_ceil_div(gs_ceil_div(ub, T::BM), 8) * 8 * gs_ceil_div(n_out, T::BN) * heads;
    return (unsigned)std::min<int64_t>(want, (int64_t)ctx->n_cu * 2 / 8 * 8);     // LDS: two workgroups a compute unit
}

void gat0_forward(gsplit_ctx *ctx, const gsplit_gat_params *p, const float *x0, hipStream_t st) {
    GsGatBuf &gb = ctx->gat;
    const GatDims d = dims_of(ctx, p, 0);
    const int D = p->dims[0], S = ctx->S, KP = pow2_ceil(d.K), NV = rows4_per_lane(D);
    const GsLayerBuf &B = ctx->layer[0];
    const GsLevelMeta *ml = ctx->d_meta, *mu = ctx->d_meta + 1;
    {
        const dim3 grid(grid_1d(ctx, ctx->ub_front[0] * 8));
        const size_t lds = sizeof(float) * 2 * d.K * D;
        GsTimeScope ts(ctx, "gat0_scores", 0, st);
#define GAT_CALL(NVV, KPV) hipLaunchKernelGGL((k_gat0_scores<KPV>), grid, dim3(256), lds, st, x0, D, gb.wext[0], d.ZW, d.HF, d.K, gb.s0, ml, S)
        GAT0_DISPATCH(1, KP, GAT_CALL);
#undef GAT_CALL
    }
    Gat0Args a{x0, gb.s0, B.blk_indptr, B.edge_row, B.self_row, gb.alpha[0], gb.pagg, nullptr, nullptr, D, d.K, d.fan, d.self_base, 0};
    {
        const dim3 grid(grid_1d(ctx, ctx->ub_front[1] * 64));
        const size_t lds = sizeof(float) * 4 * (1 + d.fan) * (1 + KP);
        GsTimeScope ts(ctx, "gat0_aggregate", 0, st);
#define GAT_CALL(NVV, KPV) hipLaunchKernelGGL((k_gat0_aggregate<NVV, KPV>), grid, dim3(256), lds, st, a, mu, S)
        GAT0_DISPATCH(NV, KP, GAT_CALL);
#undef GAT_CALL
    }
    MatLd pa{gb.pagg, 0, D, d.K * D};
    MatLd w{gb.wext[0], D, d.F, d.ZW};
    EpiHeadElu epi{gb.hidden[1], (const float *)p->d_bias[0], d.HF, 0, d.F, 0};
    GsTimeScope ts(ctx, "gat0_transform", 0, st);
    hipLaunchKernelGGL((k_gat0_head_gemm<TileTall, false, EpiHeadElu>), dim3(head_gemm_grid(ctx, ctx->ub_front[1], d.F, d.K)),
                       dim3(GNT), 0, st, pa, w, epi, d.K, D, d.F, d.F, mu, S);
}

void gat0_backward(gsplit_ctx *ctx, const gsplit_gat_params *p, const float *x0, hipStream_t st) {
    GsGatBuf &gb = ctx->gat;
    const GatDims d = dims_of(ctx, p, 0);
    const int D = p->dims[0], S = ctx->S, KP = pow2_ceil(d.K), NV = rows4_per_lane(D);
    const GsLayerBuf &B = ctx->layer[0];
    const GsLevelMeta *mu = ctx->d_meta + 1;
    // dagg of this layer: left in ghid[1] by the input-gradient product of layer 1
    const float *gagg = gb.ghid[1];
    {
        MatLd ga{gagg, 0, d.F, d.HF};
        MatLd w{gb.wext[0], D, d.F, d.ZW};
        EpiHeadStore epi{gb.dpagg, d.K * D, 0, D, 0};
        GsTimeScope ts(ctx, "gat0_grad_p", 0, st);
        hipLaunchKernelGGL((k_gat0_head_gemm<TileTall, true, EpiHeadStore>), dim3(head_gemm_grid(ctx, ctx->ub_front[1], D, d.K)),
                           dim3(GNT), 0, st, ga, w, epi, d.K, d.F, d.F, D, mu, S);
    }
    {
        const int ch = std::max(4, std::min(16, 2048 / D));      // at most 8 KiB of staged rows per wave
        Gat0Args a{x0, gb.s0, B.blk_indptr, B.edge_row, B.self_row, gb.alpha[0], gb.pagg, gb.dpagg, gb.q_part, D, d.K, d.fan,
                   d.self_base, ch};
        const dim3 grid(gb.q_blocks);
        const size_t lds = sizeof(float) * 4 * (((1 + d.fan + 3) & ~3) + (((1 + d.fan) * KP + 3) & ~3) + ((KP + 3) & ~3) + ch * D);
        GsTimeScope ts(ctx, "gat0_bwd", 0, st);
#define GAT_CALL(NVV, KPV) hipLaunchKernelGGL((k_gat0_bwd<NVV, KPV>), grid, dim3(256), lds, st, a, mu, S)
        GAT0_DISPATCH(NV, KP, GAT_CALL);
#undef GAT_CALL
    }
    const int tm = (int)gs_ceil_div(D, TileTall::BM), tn = (int)gs_ceil_div(d.F, TileTall::BN);
    {
        MatLd pa{gb.pagg, 0, D, d.K * D};
        MatLd ga{gagg, 0, d.F, d.HF};
        EpiGradW ew{gb.w0_part, D + 1, d.F, D};
        GsTimeScope ts(ctx, "gat0_grad_w", 0, st);
        hipLaunchKernelGGL((k_gat0_grad_w<TileTall>), dim3((unsigned)(gb.nchunk0 * d.K * tm * tn)), dim3(GNT), 0, st, pa, ga,
                           ew, gb.nchunk0, d.K, tm, tn, mu, S);
    }
    GsTimeScope ts(ctx, "gat0_reduce", 0, st);
    const unsigned n_w = (unsigned)(d.K * (D + 1) * gs_ceil_div(d.F, 16)), n_q = (unsigned)gs_ceil_div((int64_t)2 * d.K * D, 16);
    hipLaunchKernelGGL(k_gat0_reduce, dim3(n_w + n_q), dim3(1024), 0, st, gb.w0_part, gb.nchunk0, gb.q_part, gb.q_blocks, D,
                       d.K, d.F, d.ZW, gb.gmat[0], gb.bias_part[0], mu, S);
}

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
    if (gb.agg_first && !aligned16(d_feat_local))
        return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_gat_fwd: features must be 16-byte aligned");
    for (int l = 0; l < L; ++l) {
        const GatDims d = dims_of(ctx, p, l);
        const int D = p->dims[l];
        const float *hin = l == 0 ? (const float *)d_feat_local : gb.hidden[l];
        const GsLayerBuf &B = ctx->layer[l];
        if (l == 0 && gb.agg_first) {
            gat0_forward(ctx, p, hin, st);
            continue;
        }
        {
            MatRows a{hin, 0, D};
            MatRows b{gb.wext[l], D, d.ZW};
            EpiStore epi{gb.zext[l], d.ZW, 0, d.ZW, nullptr};
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

extern "C" int gsplit_gat_score_terms(const gsplit_ctx *ctx, int32_t layer, const float **d_terms,
                                      int64_t *row_stride, int64_t *src_col, int64_t *dst_col) {
    if (!ctx || !d_terms || !row_stride || !src_col || !dst_col || layer < 0 || layer >= ctx->L) return GSPLIT_EINVAL;
    const GsGatBuf &gb = ctx->gat;
    if (!gb.ready || !gb.fwd_done || gb.fwd_batch != ctx->batch_id) return GSPLIT_ESTATE;
    const int K = gb.heads[layer];
    if (layer == 0 && gb.agg_first) {       // [rows x 2 K]: src terms, then dst terms
        *d_terms = gb.s0; *row_stride = 2 * K; *src_col = 0; *dst_col = K;
    } else {                                // extended transformed rows: z | src terms | dst terms | padding
        const int F = layer == ctx->L - 1 ? gb.dims[layer + 1] : gb.dims[layer + 1] / K;
        *d_terms = gb.zext[layer]; *row_stride = zw_of(K, F); *src_col = K * F; *dst_col = K * F + K;
    }
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
        if (l == 0 && gb.agg_first) {
            if (!aligned16(hin)) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_gat_bwd: features must be 16-byte aligned");
            gat0_backward(ctx, p, hin, st);
            continue;
        }
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
            // (the 128 x 64 tile is no faster here: the split-K chunks are short and the slabs dominate)
            launch_grad_w(st, gb.nchunk[l], D % 4 == 0 && aligned16(hin), true, in, dz, ew, ctx->d_meta + l, S);
        }
        if (l > 0) {
            MatRows dz{gb.dzext[l], 0, d.ZW};
            MatRows w{gb.wext[l], D, d.ZW};
            // below an aggregate-then-transform bottom layer the ELU derivative is applied here: what
            // is stored is that layer's dagg
            EpiStore epi{gb.ghid[l], D, 0, D, (l == 1 && gb.agg_first) ? gb.hidden[1] : nullptr};
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
        hipLaunchKernelGGL(k_gat_finish_cols, dim3((unsigned)gs_ceil_div(hf_max, 16), L), dim3(1024), 0, st, gf);
    }
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}
