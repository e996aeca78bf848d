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

// ------------------------------------------------------------------------------------------
// Layer input assembly: for destination row i
//   X[i, 0:D]  = H[self_row[i], :]                         (its own lower-layer row)
//   X[i, D:2D] = (1/cnt_i) * sum_e H[edge_row[e], :]        (mean over its sampled sources)
// i.e. the training shuffle and the mean aggregation in one gather through the composed shuffle
// index.  One lane group per destination row, 4 floats per lane, edges in slot order
// (deterministic), four row loads in flight.  X feeds the forward product and, transposed, the
// weight-gradient product.
// ------------------------------------------------------------------------------------------
template <int LPR>
__global__ __launch_bounds__(256) void k_assemble_input_f32(const float *__restrict__ H, int D,
                                                            const int32_t *__restrict__ blk_indptr,
                                                            const int32_t *__restrict__ edge_row,
                                                            const int32_t *__restrict__ self_row,
                                                            const GsLevelMeta *__restrict__ meta_up,
                                                            int S, float *__restrict__ X) {
    const int n1 = meta_up->front_off[S];
    const int nvec = D >> 2;
    const int c0 = threadIdx.x % LPR;
    const int groups = (gridDim.x * blockDim.x) / LPR;
    const float4 *H4 = reinterpret_cast<const float4 *>(H);
    float4 *X4 = reinterpret_cast<float4 *>(X);
    for (int row = (blockIdx.x * blockDim.x + threadIdx.x) / LPR; row < n1; row += groups) {
        const int e0 = blk_indptr[row], e1 = blk_indptr[row + 1];
        const int64_t self = self_row[row];
        const float cnt = (float)(e1 - e0);
        for (int c = c0; c < nvec; c += LPR) {
            const float4 own = H4[self * nvec + c];
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
            X4[(int64_t)row * 2 * nvec + c] = own;
            X4[(int64_t)row * 2 * nvec + nvec + c] = acc;
        }
    }
}

// scalar variant for widths that are not a multiple of 4
__global__ __launch_bounds__(256) void k_assemble_input_f32_any(const float *__restrict__ H, int D,
                                                                const int32_t *__restrict__ blk_indptr,
                                                                const int32_t *__restrict__ edge_row,
                                                                const int32_t *__restrict__ self_row,
                                                                const GsLevelMeta *__restrict__ meta_up,
                                                                int S, float *__restrict__ X) {
    const int n1 = meta_up->front_off[S];
    const int lane = threadIdx.x & 63;
    const int waves = (gridDim.x * blockDim.x) >> 6;
    for (int row = (blockIdx.x * blockDim.x + threadIdx.x) >> 6; row < n1; row += waves) {
        const int e0 = blk_indptr[row], e1 = blk_indptr[row + 1];
        const int64_t self = self_row[row];
        for (int c = lane; c < D; c += 64) {
            float acc = 0.f;
            for (int e = e0; e < e1; ++e) acc += H[(int64_t)edge_row[e] * D + c];
            if (e1 > e0) acc /= (float)(e1 - e0);
            X[(int64_t)row * 2 * D + c] = H[self * D + c];
            X[(int64_t)row * 2 * D + D + c] = acc;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Tiled fp32 MFMA GEMM core:  C[M x N] = A[M x K] * B[K x N].
//
// Operands are described by accessors  at(outer, inner) -> const float* (or nullptr outside the
// logical matrix; `inner` runs along memory).  An operand is used either K-contiguous (KC: outer
// is the M or N index, inner is k) or K-major (KM: outer is k, inner is the M or N index); both
// are staged into LDS with the layout they have in memory (16-byte copies when VW == 4):
//   KC: lds[row][k]   (row stride 36 words), MFMA fragments are one 128-bit read per 8 k
//   KM: lds[k][row]   (row stride ROWS + 4), MFMA fragments are four 32-bit reads per 8 k
// v_mfma_f32_32x32x2_f32 sums two k-slots (lane / 32 selects the slot).  Within a group of 8 k the
// lower half-wave takes k = 0..3 and the upper half k = 4..7 over four consecutive MFMAs; A and B
// use the same assignment, so the sum over k is complete whatever the order.
//
// Workgroup = 4 waves as 2 x 2 over a BM x BN tile (wave tile BM/2 x BN/2, 32 x 32 blocks).
// One LDS buffer; the next k-tile is fetched into registers while the current one is multiplied.
// ------------------------------------------------------------------------------------------
constexpr int BK = 32;
constexpr int KC_LD = BK + 4;

template <int ROWS>
constexpr int lds_words() { return ROWS * KC_LD > BK * (ROWS + 4) ? ROWS * KC_LD : BK * (ROWS + 4); }

template <int ROWS, bool KC, int VW, class F>
struct Stager {
    static constexpr int NV = ROWS * BK / 4 / 256;
    float4 reg[NV];

    __device__ __forceinline__ static float4 fetch(const F &f, int outer, int inner, int inner_end) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (VW == 4) {
            if (inner < inner_end) {
                const float *p = f.at(outer, inner);
                if (p) v = *reinterpret_cast<const float4 *>(p);
            }
        } else {
            float t[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float *p = (inner + j < inner_end) ? f.at(outer, inner + j) : nullptr;
                t[j] = p ? *p : 0.f;
            }
            v = make_float4(t[0], t[1], t[2], t[3]);
        }
        return v;
    }
    // r0: first M/N index of the tile, [k0, k_end): k range still to do, r_end: matrix extent
    __device__ __forceinline__ void load(const F &f, int r0, int r_end, int k0, int k_end, int tid) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            if (KC) {
                const int kq = tid & 7, row = (tid >> 3) + 32 * v;
                reg[v] = (r0 + row < r_end) ? fetch(f, r0 + row, k0 + 4 * kq, k_end)
                                            : make_float4(0.f, 0.f, 0.f, 0.f);
            } else {
                const int x = tid % (ROWS / 4), kk = tid / (ROWS / 4) + (1024 / ROWS) * v;
                reg[v] = (k0 + kk < k_end) ? fetch(f, k0 + kk, r0 + 4 * x, r_end)
                                           : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    }
    __device__ __forceinline__ void store(float *lds, int tid) const {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            if (KC) {
                const int kq = tid & 7, row = (tid >> 3) + 32 * v;
                *reinterpret_cast<float4 *>(&lds[row * KC_LD + 4 * kq]) = reg[v];
            } else {
                const int x = tid % (ROWS / 4), kk = tid / (ROWS / 4) + (1024 / ROWS) * v;
                *reinterpret_cast<float4 *>(&lds[kk * (ROWS + 4) + 4 * x]) = reg[v];
            }
        }
    }
};

template <int ROWS, bool KC>
__device__ __forceinline__ void read_frag(const float *lds, int row, int oct, int half, float out[4]) {
    if (KC) {
        const float4 v = *reinterpret_cast<const float4 *>(&lds[row * KC_LD + oct * 8 + 4 * half]);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) out[j] = lds[(oct * 8 + 4 * half + j) * (ROWS + 4) + row];
    }
}

template <int BM, int BN, bool A_KC, bool B_KC, int VA, int VB, class AF, class BF, class EF>
__device__ __forceinline__ void gemm_tile(const int m0, const int n0, const int m_end, const int n_end,
                                          const int k_begin, const int k_end, const AF &a, const BF &b,
                                          const EF &epi) {
    __shared__ __attribute__((aligned(16))) float As[lds_words<BM>()];
    __shared__ __attribute__((aligned(16))) float Bs[lds_words<BN>()];
    constexpr int MI = BM / 64, NI = BN / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);
    floatx16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    Stager<BM, A_KC, VA, AF> sa;
    Stager<BN, B_KC, VB, BF> sb;
    sa.load(a, m0, m_end, k_begin, k_end, tid);
    sb.load(b, n0, n_end, k_begin, k_end, tid);
    for (int k0 = k_begin; k0 < k_end; k0 += BK) {
        sa.store(As, tid);
        sb.store(Bs, tid);
        __syncthreads();
        if (k0 + BK < k_end) {
            sa.load(a, m0, m_end, k0 + BK, k_end, tid);
            sb.load(b, n0, n_end, k0 + BK, k_end, tid);
        }
#pragma unroll
        for (int oct = 0; oct < BK / 8; ++oct) {
            float af[MI][4], bf[NI][4];
#pragma unroll
            for (int i = 0; i < MI; ++i) read_frag<BM, A_KC>(As, wm0 + i * 32 + l32, oct, half, af[i]);
#pragma unroll
            for (int j = 0; j < NI; ++j) read_frag<BN, B_KC>(Bs, wn0 + j * 32 + l32, oct, half, bf[j]);
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][q], bf[j][q], acc[i][j], 0, 0, 0);
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
                const int m = m0 + wm0 + i * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                const int n = n0 + wn0 + j * 32 + l32;
                epi(m, n, acc[i][j][r]);
            }
}

// ---- operand accessors and epilogues ---------------------------------------------------------
__device__ const float g_one_then_zero[4] = {1.f, 0.f, 0.f, 0.f};

// plain row-major matrix
struct MatRows {
    const float *p; int rows; int cols;
    __device__ __forceinline__ const float *at(int o, int i) const {
        return (o < rows && i < cols) ? p + (int64_t)o * cols + i : nullptr;
    }
};
// plain row-major matrix followed by one column of ones (its product with dZ is the bias gradient)
struct MatRowsOnes {
    const float *p; int rows; int cols;
    __device__ __forceinline__ const float *at(int o, int i) const {
        if (o >= rows) return nullptr;
        if (i < cols) return p + (int64_t)o * cols + i;
        return i == cols ? g_one_then_zero : nullptr;
    }
};
// [W_self; W_neigh] stacked: row k of the 2 * D x N matrix
struct CatW {
    const float *Ws; const float *Wn; int D; int N;
    __device__ __forceinline__ const float *at(int k, int n) const {
        if (n >= N) return nullptr;
        if (k < D) return Ws + (int64_t)k * N + n;
        if (k < 2 * D) return Wn + (int64_t)(k - D) * N + n;
        return nullptr;
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
// input gradients per destination row: [dH_self | dMean / cnt]; the reverse shuffle (pull through
// the scatter side of the shuffle index) follows in k_pull_input_grad
struct EpiGradIn {
    float *out; const int32_t *blk_indptr; int D; int n1;
    __device__ __forceinline__ void operator()(int i, int j, float v) const {
        if (i >= n1 || j >= 2 * D) return;
        if (j >= D) {
            const int c = blk_indptr[i + 1] - blk_indptr[i];
            v = c > 0 ? v / (float)c : 0.f;
        }
        out[(int64_t)i * 2 * D + j] = v;
    }
};

constexpr int GBM = 64, GBN = 128;

// Z = [H_self | mean] * [W_self; W_neigh] + b, ReLU except on the last layer
template <int VA, int VB>
__global__ __launch_bounds__(256) void k_sage_linear_fwd(MatRows a, CatW b, EpiFwd epi,
                                                         const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int m0 = blockIdx.x * GBM;
    if (m0 >= n1) return;
    a.rows = n1; epi.n1 = n1;
    gemm_tile<GBM, GBN, true, false, VA, VB>(m0, blockIdx.y * GBN, n1, b.N, 0, a.cols, a, b, epi);
}

// [dW_self; dW_neigh; db] += [H_self | mean | 1]^T * dZ over a chunk of destination rows
template <int VA, int VB>
__global__ __launch_bounds__(256) void k_sage_grad_w(MatRowsOnes a, MatRows dz, EpiGradW epi, int kchunk,
                                                     const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int k_begin = blockIdx.z * kchunk;
    if (k_begin >= n1) return;
    a.rows = n1; dz.rows = n1;
    const int k_end = min(n1, k_begin + kchunk);
    gemm_tile<GBM, GBN, false, false, VA, VB>(blockIdx.x * GBM, blockIdx.y * GBN, a.cols + 1, dz.cols,
                                              k_begin, k_end, a, dz, epi);
}

// [dH_self | dMean / cnt] = dZ * [W_self; W_neigh]^T per destination row
template <int VA, int VB>
__global__ __launch_bounds__(256) void k_sage_grad_in(MatRows dz, CatW w, EpiGradIn epi,
                                                      const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int m0 = blockIdx.x * GBM;
    if (m0 >= n1) return;
    dz.rows = n1; epi.n1 = n1;
    gemm_tile<GBM, GBN, true, true, VA, VB>(m0, blockIdx.y * GBN, n1, 2 * w.D, 0, dz.cols, dz, w, epi);
}

// Reverse shuffle of the backward pass as a pull: row u of local_cat[l] sums the gradient rows of
// every destination it fed (its own self term and one mean term per sampled edge), listed by the
// scatter side of the shuffle index.  The ReLU of the layer below is applied on the way out, so
// the result is that layer's dZ.  One lane group per row, 4 floats per lane; no atomics, and rows
// that fed nothing get zeros.
template <int LPR>
__global__ __launch_bounds__(256) void k_pull_input_grad(const float *__restrict__ gin, int D,
                                                         const int32_t *__restrict__ rev_ptr,
                                                         const int32_t *__restrict__ rev_cnt,
                                                         const int32_t *__restrict__ rev_list,
                                                         const float *__restrict__ hact,
                                                         const GsLevelMeta *__restrict__ meta_lo, int S,
                                                         float *__restrict__ gout) {
    const int n_lo = meta_lo->front_off[S];
    const int nvec = D >> 2;
    const int c0 = threadIdx.x % LPR;
    const int groups = (gridDim.x * blockDim.x) / LPR;
    const float4 *G4 = reinterpret_cast<const float4 *>(gin);
    const float4 *A4 = reinterpret_cast<const float4 *>(hact);
    float4 *O4 = reinterpret_cast<float4 *>(gout);
    for (int u = (blockIdx.x * blockDim.x + threadIdx.x) / LPR; u < n_lo; u += groups) {
        const int e0 = rev_ptr[u], e1 = e0 + rev_cnt[u];
        for (int c = c0; c < nvec; c += LPR) {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            int e = e0;
            for (; e + 2 <= e1; e += 2) {
                const int k0 = rev_list[e], k1 = rev_list[e + 1];
                const float4 a = G4[(int64_t)(k0 >> 1) * 2 * nvec + (k0 & 1) * nvec + c];
                const float4 b = G4[(int64_t)(k1 >> 1) * 2 * nvec + (k1 & 1) * nvec + c];
                acc.x += a.x; acc.y += a.y; acc.z += a.z; acc.w += a.w;
                acc.x += b.x; acc.y += b.y; acc.z += b.z; acc.w += b.w;
            }
            if (e < e1) {
                const int k0 = rev_list[e];
                const float4 a = G4[(int64_t)(k0 >> 1) * 2 * nvec + (k0 & 1) * nvec + c];
                acc.x += a.x; acc.y += a.y; acc.z += a.z; acc.w += a.w;
            }
            const float4 h = A4[(int64_t)u * nvec + c];
            acc.x = h.x > 0.f ? acc.x : 0.f; acc.y = h.y > 0.f ? acc.y : 0.f;
            acc.z = h.z > 0.f ? acc.z : 0.f; acc.w = h.w > 0.f ? acc.w : 0.f;
            O4[(int64_t)u * nvec + c] = acc;
        }
    }
}

__global__ __launch_bounds__(256) void k_pull_input_grad_any(const float *__restrict__ gin, int D,
                                                             const int32_t *__restrict__ rev_ptr,
                                                             const int32_t *__restrict__ rev_cnt,
                                                             const int32_t *__restrict__ rev_list,
                                                             const float *__restrict__ hact,
                                                             const GsLevelMeta *__restrict__ meta_lo, int S,
                                                             float *__restrict__ gout) {
    const int n_lo = meta_lo->front_off[S];
    const int lane = threadIdx.x & 63;
    const int waves = (gridDim.x * blockDim.x) >> 6;
    for (int u = (blockIdx.x * blockDim.x + threadIdx.x) >> 6; u < n_lo; u += waves) {
        const int e0 = rev_ptr[u], e1 = e0 + rev_cnt[u];
        for (int c = lane; c < D; c += 64) {
            float acc = 0.f;
            for (int e = e0; e < e1; ++e) {
                const int k = rev_list[e];
                acc += gin[(int64_t)(k >> 1) * 2 * D + (k & 1) * D + c];
            }
            gout[(int64_t)u * D + c] = hact[(int64_t)u * D + c] > 0.f ? acc : 0.f;
        }
    }
}

// Mean softmax cross-entropy of the target rows and its gradient w.r.t. the logits: one wave per
// target; the label of row r is labels[local_cat[L][r]].
__global__ __launch_bounds__(256) void k_softmax_xent(const float *__restrict__ logits, int C,
                                                      const int64_t *__restrict__ labels,
                                                      const int32_t *__restrict__ front_top,
                                                      const GsLevelMeta *__restrict__ meta_top, int S,
                                                      float *__restrict__ grad, float *__restrict__ row_loss) {
    const int n = meta_top->front_off[S];
    const int lane = threadIdx.x & 63;
    const int waves = (gridDim.x * blockDim.x) >> 6;
    for (int r = (blockIdx.x * blockDim.x + threadIdx.x) >> 6; r < n; r += waves) {
        const float *z = logits + (int64_t)r * C;
        float mx = -3.4e38f;
        for (int c = lane; c < C; c += 64) mx = fmaxf(mx, z[c]);
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        float sum = 0.f;
        for (int c = lane; c < C; c += 64) sum += __expf(z[c] - mx);
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        const int y = (int)labels[front_top[r]];
        const float inv = 1.f / sum, invn = 1.f / (float)n;
        for (int c = lane; c < C; c += 64) {
            const float p = __expf(z[c] - mx) * inv;
            grad[(int64_t)r * C + c] = (p - (c == y ? 1.f : 0.f)) * invn;
        }
        if (row_loss && lane == 0) row_loss[r] = (y >= 0 && y < C) ? (logf(sum) + mx - z[y]) : 0.f;
    }
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// zero up to 3 * GS_MAXL caller buffers in one launch (blockIdx.y selects the buffer)
struct ZeroList {
    float *p[3 * GS_MAXL];
    int64_t n[3 * GS_MAXL];
};
__global__ __launch_bounds__(256) void k_zero_buffers(ZeroList z) {
    float *p = z.p[blockIdx.y];
    const int64_t n = z.n[blockIdx.y];
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
        int rc = gs_alloc(ctx, &sb.xin[l], sizeof(float) * ctx->ub_front[l + 1] * 2 * p->dims[l], "layer input");
        if (rc) return rc;
    }
    int64_t gtmp_words = 1;
    for (int l = 1; l < L; ++l) gtmp_words = std::max<int64_t>(gtmp_words, ctx->ub_front[l + 1] * 2 * p->dims[l]);
    {
        int rc = gs_alloc(ctx, (void **)&sb.gtmp, sizeof(float) * gtmp_words, "input gradients");
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

void launch_assemble(gsplit_ctx *ctx, int l, const float *hin, int D, hipStream_t st) {
    const GsLayerBuf &B = ctx->layer[l];
    const GsLevelMeta *mu = ctx->d_meta + (l + 1);
    float *X = (float *)ctx->sage.xin[l];
    const int64_t ub = ctx->ub_front[l + 1];
    GsTimeScope ts(ctx, "assemble_input", l, st);
    if (D % 4 != 0 || !aligned16(hin)) {
        hipLaunchKernelGGL(k_assemble_input_f32_any, dim3(grid_1d(ctx, ub * 64)), dim3(256), 0, st, hin, D,
                           B.blk_indptr, B.edge_row, B.self_row, mu, ctx->S, X);
        return;
    }
    const int nvec = D / 4;
    if (nvec <= 16)
        hipLaunchKernelGGL(k_assemble_input_f32<16>, dim3(grid_1d(ctx, ub * 16)), dim3(256), 0, st, hin, D,
                           B.blk_indptr, B.edge_row, B.self_row, mu, ctx->S, X);
    else if (nvec <= 32)
        hipLaunchKernelGGL(k_assemble_input_f32<32>, dim3(grid_1d(ctx, ub * 32)), dim3(256), 0, st, hin, D,
                           B.blk_indptr, B.edge_row, B.self_row, mu, ctx->S, X);
    else
        hipLaunchKernelGGL(k_assemble_input_f32<64>, dim3(grid_1d(ctx, ub * 64)), dim3(256), 0, st, hin, D,
                           B.blk_indptr, B.edge_row, B.self_row, mu, ctx->S, X);
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
    for (int l = 0; l < L; ++l) {
        const int D = p->dims[l], N = p->dims[l + 1];
        const float *hin = l == 0 ? (const float *)d_feat_local : (const float *)sb.hidden[l];
        float *hout = l == L - 1 ? d_logits : (float *)sb.hidden[l + 1];
        const GsLayerBuf &B = ctx->layer[l];
        const GsLevelMeta *mu = ctx->d_meta + (l + 1);
        launch_assemble(ctx, l, hin, D, st);
        MatRows a{(const float *)sb.xin[l], 0, 2 * D};
        CatW b{(const float *)p->d_w_self[l], (const float *)p->d_w_neigh[l], D, N};
        EpiFwd epi{hout, (const float *)p->d_bias[l], N, 0, l < L - 1 ? 1 : 0};
        dim3 grid((unsigned)gs_ceil_div(ctx->ub_front[l + 1], GBM), (unsigned)gs_ceil_div(N, GBN));
        const bool va = D % 2 == 0;   // rows of the assembled input are 2 * D floats: 16-byte aligned
        const bool vb = N % 4 == 0 && aligned16(p->d_w_self[l]) && aligned16(p->d_w_neigh[l]);
        GsTimeScope ts(ctx, "linear_fwd", l, st);
        if (va && vb) hipLaunchKernelGGL((k_sage_linear_fwd<4, 4>), grid, dim3(256), 0, st, a, b, epi, mu, S);
        else if (va) hipLaunchKernelGGL((k_sage_linear_fwd<4, 1>), grid, dim3(256), 0, st, a, b, epi, mu, S);
        else if (vb) hipLaunchKernelGGL((k_sage_linear_fwd<1, 4>), grid, dim3(256), 0, st, a, b, epi, mu, S);
        else hipLaunchKernelGGL((k_sage_linear_fwd<1, 1>), grid, dim3(256), 0, st, a, b, epi, mu, S);
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
    ZeroList zl;
    int64_t zmax = 1;
    for (int l = 0; l < L; ++l) {
        if (!d_gw_self[l] || !d_gw_neigh[l] || !d_gbias[l])
            return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_sage_bwd: NULL gradient pointer");
        const int64_t nw = (int64_t)p->dims[l] * p->dims[l + 1];
        zl.p[3 * l] = d_gw_self[l];      zl.n[3 * l] = nw;
        zl.p[3 * l + 1] = d_gw_neigh[l]; zl.n[3 * l + 1] = nw;
        zl.p[3 * l + 2] = d_gbias[l];    zl.n[3 * l + 2] = p->dims[l + 1];
        zmax = std::max(zmax, nw);
    }
    {
    GsTimeScope ts(ctx, "zero_grads", -1, st);
    hipLaunchKernelGGL(k_zero_buffers, dim3((unsigned)std::min<int64_t>(64, gs_ceil_div(zmax, 1024)), 3 * L),
                       dim3(256), 0, st, zl);
    }
    for (int l = L - 1; l >= 0; --l) {
        const int D = p->dims[l], N = p->dims[l + 1];
        const GsLayerBuf &B = ctx->layer[l];
        const GsLevelMeta *mu = ctx->d_meta + (l + 1);
        const float *dH = l == L - 1 ? d_grad_logits : sb.ghid[l + 1];
        const int64_t ub = ctx->ub_front[l + 1];
        MatRows dz{dH, 0, N};
        // weight and bias gradients, summed over all splits: [X | 1]^T dZ with the layer input X
        // assembled by the forward pass
        MatRowsOnes in{(const float *)sb.xin[l], 0, 2 * D};
        EpiGradW ew{d_gw_self[l], d_gw_neigh[l], d_gbias[l], D, N};
        const bool vin = D % 2 == 0;
        const bool vdz = N % 4 == 0 && aligned16(dH);
        const bool vw = N % 4 == 0 && aligned16(p->d_w_self[l]) && aligned16(p->d_w_neigh[l]);
        {
            const int kchunk = 512;
            dim3 grid((unsigned)gs_ceil_div(2 * D + 1, GBM), (unsigned)gs_ceil_div(N, GBN),
                      (unsigned)gs_ceil_div(ub, kchunk));
            GsTimeScope ts(ctx, "grad_w", l, st);
            if (vin && vdz) hipLaunchKernelGGL((k_sage_grad_w<4, 4>), grid, dim3(256), 0, st, in, dz, ew, kchunk, mu, S);
            else if (vin) hipLaunchKernelGGL((k_sage_grad_w<4, 1>), grid, dim3(256), 0, st, in, dz, ew, kchunk, mu, S);
            else if (vdz) hipLaunchKernelGGL((k_sage_grad_w<1, 4>), grid, dim3(256), 0, st, in, dz, ew, kchunk, mu, S);
            else hipLaunchKernelGGL((k_sage_grad_w<1, 1>), grid, dim3(256), 0, st, in, dz, ew, kchunk, mu, S);
        }
        if (l > 0) {
            const GsLevelMeta *ml = ctx->d_meta + l;
            CatW w{(const float *)p->d_w_self[l], (const float *)p->d_w_neigh[l], D, N};
            EpiGradIn ei{sb.gtmp, B.blk_indptr, D, 0};
            dim3 grid((unsigned)gs_ceil_div(ub, GBM), (unsigned)gs_ceil_div(2 * D, GBN));
            {
            GsTimeScope ts(ctx, "grad_in", l, st);
            if (vdz && vw) hipLaunchKernelGGL((k_sage_grad_in<4, 4>), grid, dim3(256), 0, st, dz, w, ei, mu, S);
            else if (vdz) hipLaunchKernelGGL((k_sage_grad_in<4, 1>), grid, dim3(256), 0, st, dz, w, ei, mu, S);
            else if (vw) hipLaunchKernelGGL((k_sage_grad_in<1, 4>), grid, dim3(256), 0, st, dz, w, ei, mu, S);
            else hipLaunchKernelGGL((k_sage_grad_in<1, 1>), grid, dim3(256), 0, st, dz, w, ei, mu, S);
            }
            GsTimeScope ts(ctx, "pull_input_grad", l, st);
            // reverse shuffle + ReLU of the layer below: dZ of layer l-1
            const float *hact = (const float *)sb.hidden[l];
            const int64_t ubl = ctx->ub_front[l];
            if (D % 4 != 0) {
                hipLaunchKernelGGL(k_pull_input_grad_any, dim3(grid_1d(ctx, ubl * 64)), dim3(256), 0, st,
                                   sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, hact, ml, S, sb.ghid[l]);
            } else if (D / 4 <= 16) {
                hipLaunchKernelGGL(k_pull_input_grad<16>, dim3(grid_1d(ctx, ubl * 16)), dim3(256), 0, st,
                                   sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, hact, ml, S, sb.ghid[l]);
            } else if (D / 4 <= 32) {
                hipLaunchKernelGGL(k_pull_input_grad<32>, dim3(grid_1d(ctx, ubl * 32)), dim3(256), 0, st,
                                   sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, hact, ml, S, sb.ghid[l]);
            } else {
                hipLaunchKernelGGL(k_pull_input_grad<64>, dim3(grid_1d(ctx, ubl * 64)), dim3(256), 0, st,
                                   sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, hact, ml, S, sb.ghid[l]);
            }
        }
    }
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}

extern "C" int gsplit_softmax_xent(gsplit_ctx *ctx, const float *d_logits, int32_t n_classes,
                                   const int64_t *d_labels, float *d_grad_logits, float *d_row_loss,
                                   void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    if (!d_logits || !d_labels || !d_grad_logits || n_classes < 1)
        return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_softmax_xent: bad argument");
    if (ctx->batch_id == 0) return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_softmax_xent: no batch");
    hipStream_t st = (hipStream_t)stream;
    const int L = ctx->L;
    GsTimeScope ts(ctx, "softmax_xent", -1, st);
    hipLaunchKernelGGL(k_softmax_xent, dim3(grid_1d(ctx, ctx->ub_front[L] * 64)), dim3(256), 0, st, d_logits,
                       n_classes, d_labels, ctx->front[L], ctx->d_meta + L, ctx->S, d_grad_logits, d_row_loss);
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}
