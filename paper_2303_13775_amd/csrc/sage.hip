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
                                                            int S, float *__restrict__ X,
                                                            float *__restrict__ inv_cnt) {
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
        if (c0 == 0) inv_cnt[row] = e1 > e0 ? 1.f / cnt : 0.f;
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
                                                                int S, float *__restrict__ X,
                                                                float *__restrict__ inv_cnt) {
    const int n1 = meta_up->front_off[S];
    const int lane = threadIdx.x & 63;
    const int waves = (gridDim.x * blockDim.x) >> 6;
    for (int row = (blockIdx.x * blockDim.x + threadIdx.x) >> 6; row < n1; row += waves) {
        const int e0 = blk_indptr[row], e1 = blk_indptr[row + 1];
        const int64_t self = self_row[row];
        if (lane == 0) inv_cnt[row] = e1 > e0 ? 1.f / (float)(e1 - e0) : 0.f;
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
// Workgroup = 8 waves as 2 x 4 over a BM x BN tile (32 x 32 MFMA blocks per wave).
// ------------------------------------------------------------------------------------------
constexpr int BK = 32;
constexpr int KC_LD = BK + 4;
// workgroup = GWM x GWN waves; two waves share each SIMD, so one wave's LDS traffic and barrier
// waits overlap the other's MFMAs
constexpr int GWM = 2, GWN = 4, GNT = 64 * GWM * GWN;

template <int ROWS>
constexpr int lds_words() { return ROWS * KC_LD > BK * (ROWS + 4) ? ROWS * KC_LD : BK * (ROWS + 4); }

__device__ __forceinline__ uint16_t f2bf(float f) {          // round to nearest, ties to even
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(uint32_t h) { return __uint_as_float(h << 16); }

// SRC_H: the source matrix holds bfloat16; the raw halves travel through the registers and are
// widened to float (exactly) when the tile is written to LDS.
template <int ROWS, bool KC, int VW, int NT, class F, bool SRC_H = false>
struct Stager {
    static constexpr int NV = ROWS * BK / 4 / NT;
    static_assert(NV >= 1 && NV <= 8, "tile too small or too large for the workgroup");
    float4 reg[NV];
    unsigned keep;   // 4 bits per register: which of its words exist in the matrix

    // Loads are unconditional (the accessor clamps the address into the matrix); words outside the
    // matrix are zeroed only when the registers are written to LDS, so nothing depends on a load
    // before that point and the loads of two k-tiles stay in flight.
    __device__ __forceinline__ void fetch(int v, const F &f, int outer, int inner, int inner_end, bool ok) {
        if (VW == 4) {
            bool in;
            if (SRC_H) {
                const uint2 raw = *reinterpret_cast<const uint2 *>(f.template at<4>(outer, inner, in));
                reg[v].x = __uint_as_float(raw.x);
                reg[v].y = __uint_as_float(raw.y);
            } else {
                reg[v] = *reinterpret_cast<const float4 *>(f.template at<4>(outer, inner, in));
            }
            keep |= (in && ok && inner < inner_end) ? (0xFu << (4 * v)) : 0u;
        } else {
            float t[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bool in;
                if (SRC_H) t[j] = __uint_as_float((uint32_t)*reinterpret_cast<const uint16_t *>(f.template at<1>(outer, inner + j, in)));
                else t[j] = *reinterpret_cast<const float *>(f.template at<1>(outer, inner + j, in));
                keep |= (in && ok && inner + j < inner_end) ? (1u << (4 * v + j)) : 0u;
            }
            reg[v] = make_float4(t[0], t[1], t[2], t[3]);
        }
    }
    // r0: first M/N index of the tile, [k0, k_end): k range still to do, r_end: matrix extent
    __device__ __forceinline__ void load(const F &f, int r0, int r_end, int k0, int k_end, int tid) {
        keep = 0u;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            if (KC) {
                const int kq = tid & 7, row = (tid >> 3) + (NT / 8) * v;
                fetch(v, f, r0 + row, k0 + 4 * kq, k_end, r0 + row < r_end);
            } else {
                const int x = tid % (ROWS / 4), kk = tid / (ROWS / 4) + (4 * NT / ROWS) * v;
                fetch(v, f, k0 + kk, r0 + 4 * x, r_end, k0 + kk < k_end);
            }
        }
    }
    __device__ __forceinline__ void store(float *lds, int tid) const {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            float4 w = reg[v];
            if (SRC_H) {
                if (VW == 4) {
                    const uint32_t lo = __float_as_uint(reg[v].x), hi = __float_as_uint(reg[v].y);
                    w = make_float4(bf2f(lo & 0xFFFFu), bf2f(lo >> 16), bf2f(hi & 0xFFFFu), bf2f(hi >> 16));
                } else {
                    w = make_float4(bf2f(__float_as_uint(reg[v].x)), bf2f(__float_as_uint(reg[v].y)),
                                    bf2f(__float_as_uint(reg[v].z)), bf2f(__float_as_uint(reg[v].w)));
                }
            }
            w.x = (keep >> (4 * v)) & 1u ? w.x : 0.f;
            w.y = (keep >> (4 * v + 1)) & 1u ? w.y : 0.f;
            w.z = (keep >> (4 * v + 2)) & 1u ? w.z : 0.f;
            w.w = (keep >> (4 * v + 3)) & 1u ? w.w : 0.f;
            if (KC) {
                const int kq = tid & 7, row = (tid >> 3) + (NT / 8) * v;
                *reinterpret_cast<float4 *>(&lds[row * KC_LD + 4 * kq]) = w;
            } else {
                const int x = tid % (ROWS / 4), kk = tid / (ROWS / 4) + (4 * NT / ROWS) * v;
                *reinterpret_cast<float4 *>(&lds[kk * (ROWS + 4) + 4 * x]) = w;
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

template <int BM, int BN, bool A_KC, bool B_KC, int VA, int VB, class AF, class BF, class EF, bool A_H = false>
__device__ __forceinline__ void gemm_tile(const int m0, const int n0, const int m_end, const int n_end,
                                          const int k_begin, const int k_end, const AF &a, const BF &b,
                                          const EF &epi) {
    // two LDS stages and two register stages: k-tile t is multiplied out of LDS while tile t+1
    // sits in the other LDS stage and tile t+2 is in flight into registers, so a global load has
    // two iterations to land (an HBM round trip is longer than one k-tile of MFMA work)
    __shared__ __attribute__((aligned(16))) float As0[lds_words<BM>()];
    __shared__ __attribute__((aligned(16))) float As1[lds_words<BM>()];
    __shared__ __attribute__((aligned(16))) float Bs0[lds_words<BN>()];
    __shared__ __attribute__((aligned(16))) float Bs1[lds_words<BN>()];
    constexpr int MI = BM / (32 * GWM), NI = BN / (32 * GWN);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int wm0 = (wave / GWN) * (BM / GWM), wn0 = (wave % GWN) * (BN / GWN);
    floatx16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    using SA = Stager<BM, A_KC, VA, GNT, AF, A_H>;
    using SB = Stager<BN, B_KC, VB, GNT, BF>;
    SA sa0, sa1;
    SB sb0, sb1;

    // The fragments of the next group of 8 k are read from LDS while the MFMAs of the current group
    // execute (an MFMA occupies the matrix pipe for 64 cycles but not the issue slot), so only the
    // first LDS read of a k-tile is exposed.
    auto multiply = [&](const float *As, const float *Bs) {
        float af[2][MI][4], bf[2][NI][4];
#pragma unroll
        for (int i = 0; i < MI; ++i) read_frag<BM, A_KC>(As, wm0 + i * 32 + l32, 0, half, af[0][i]);
#pragma unroll
        for (int j = 0; j < NI; ++j) read_frag<BN, B_KC>(Bs, wn0 + j * 32 + l32, 0, half, bf[0][j]);
#pragma unroll
        for (int oct = 0; oct < BK / 8; ++oct) {
            if (oct + 1 < BK / 8) {
#pragma unroll
                for (int i = 0; i < MI; ++i)
                    read_frag<BM, A_KC>(As, wm0 + i * 32 + l32, oct + 1, half, af[(oct + 1) & 1][i]);
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    read_frag<BN, B_KC>(Bs, wn0 + j * 32 + l32, oct + 1, half, bf[(oct + 1) & 1][j]);
            }
            __builtin_amdgcn_sched_barrier(0);   // reads of the next group stay ahead of these MFMAs
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[oct & 1][i][q], bf[oct & 1][j][q], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // one k-tile: fetch tile k0 + 2 BK into the registers that held tile k0, multiply tile k0,
    // move tile k0 + BK from registers to the other LDS stage
    auto step = [&](SA &ra_cur, SB &rb_cur, SA &ra_nxt, SB &rb_nxt, const float *As_cur, const float *Bs_cur,
                    float *As_nxt, float *Bs_nxt, int k0) {
        if (k0 + 2 * BK < k_end) {
            ra_cur.load(a, m0, m_end, k0 + 2 * BK, k_end, tid);
            rb_cur.load(b, n0, n_end, k0 + 2 * BK, k_end, tid);
        }
        multiply(As_cur, Bs_cur);
        if (k0 + BK < k_end) {
            ra_nxt.store(As_nxt, tid);
            rb_nxt.store(Bs_nxt, tid);
        }
        __syncthreads();
    };

    sa0.load(a, m0, m_end, k_begin, k_end, tid);
    sb0.load(b, n0, n_end, k_begin, k_end, tid);
    if (k_begin + BK < k_end) {
        sa1.load(a, m0, m_end, k_begin + BK, k_end, tid);
        sb1.load(b, n0, n_end, k_begin + BK, k_end, tid);
    }
    sa0.store(As0, tid);
    sb0.store(Bs0, tid);
    __syncthreads();
    for (int k0 = k_begin; k0 < k_end; k0 += 2 * BK) {
        step(sa0, sb0, sa1, sb1, As0, Bs0, As1, Bs1, k0);
        if (k0 + BK < k_end) step(sa1, sb1, sa0, sb0, As1, Bs1, As0, Bs0, k0 + BK);
    }
    // accumulator layout of the 32x32 block: register r of lane l holds
    // row (r / 4) * 8 + (l / 32) * 4 + (r % 4), column l % 32.
    // Per-column and per-row side inputs of the epilogue (bias, 1/count) are fetched up front so
    // that their latencies overlap instead of adding up in front of every store.
    float colv[NI], rowv[MI][16];
#pragma unroll
    for (int j = 0; j < NI; ++j) colv[j] = epi.col(n0 + wn0 + j * 32 + l32);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            rowv[i][r] = epi.row(m0 + wm0 + i * 32 + (r >> 2) * 8 + half * 4 + (r & 3));
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm0 + i * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                const int n = n0 + wn0 + j * 32 + l32;
                epi.store(m, n, acc[i][j][r], rowv[i][r], colv[j]);
            }
}

// ---- operand accessors and epilogues ---------------------------------------------------------
__device__ const float g_one_then_zero[4] = {1.f, 0.f, 0.f, 0.f};
__device__ const uint16_t g_one_then_zero_h[4] __attribute__((aligned(8))) = {0x3F80, 0, 0, 0};   // bf16 1, 0, 0, 0

// Accessors return an address that is always safe to read VW floats from (indices are clamped into
// the matrix; matrices have at least one row and VW columns) and say whether the element exists.
// plain row-major matrix
struct MatRows {
    const float *p; int rows; int cols;
    template <int VW>
    __device__ __forceinline__ const float *at(int o, int i, bool &in) const {
        in = o < rows && i < cols;
        const int oc = min(o, rows - 1), ic = min(i, cols - VW);
        return p + (int64_t)oc * cols + ic;
    }
};
// plain row-major matrix followed by one column of ones (its product with dZ is the bias gradient)
struct MatRowsOnes {
    const float *p; int rows; int cols;
    template <int VW>
    __device__ __forceinline__ const float *at(int o, int i, bool &in) const {
        in = o < rows && i <= cols;
        const int oc = min(o, rows - 1), ic = min(i, cols - VW);
        const float *q = p + (int64_t)oc * cols + ic;
        return i == cols ? g_one_then_zero : q;
    }
};
// [W_self; W_neigh] stacked: row k of the 2 * D x N matrix
struct CatW {
    const float *Ws; const float *Wn; int D; int N;
    template <int VW>
    __device__ __forceinline__ const float *at(int k, int n, bool &in) const {
        in = k < 2 * D && n < N;
        const int nc = min(n, N - VW);
        const int kc = min(k, 2 * D - 1);
        const float *base = kc < D ? Ws : Wn;
        const int kr = kc < D ? kc : kc - D;
        return base + (int64_t)kr * N + nc;
    }
};
struct EpiFwd {
    float *out; const float *bias; int N; int n1; int relu;
    __device__ __forceinline__ float col(int n) const { return n < N ? bias[n] : 0.f; }
    __device__ __forceinline__ float row(int) const { return 0.f; }
    __device__ __forceinline__ void store(int m, int n, float v, float, float b) const {
        if (m < n1 && n < N) {
            const float z = v + b;
            out[(int64_t)m * N + n] = (relu && z < 0.f) ? 0.f : z;
        }
    }
};
// partial [dW_self; dW_neigh; db] of one chunk of destination rows, written to the chunk's slab
struct EpiGradW {
    float *part; int rows; int N;     // rows = 2 * D + 1
    __device__ __forceinline__ float col(int) const { return 0.f; }
    __device__ __forceinline__ float row(int) const { return 0.f; }
    __device__ __forceinline__ void store(int c, int n, float v, float, float) const {
        if (n < N && c < rows) part[(int64_t)c * N + n] = v;
    }
};
// input gradients per destination row: [dH_self | dMean / cnt]; the reverse shuffle (pull through
// the scatter side of the shuffle index) follows in k_pull_input_grad
struct EpiGradIn {
    float *out; const float *inv_cnt; int D; int n1;
    __device__ __forceinline__ float col(int) const { return 0.f; }
    __device__ __forceinline__ float row(int i) const { return i < n1 ? inv_cnt[i] : 0.f; }
    __device__ __forceinline__ void store(int i, int j, float v, float w, float) const {
        if (i >= n1 || j >= 2 * D) return;
        out[(int64_t)i * 2 * D + j] = j < D ? v : v * w;
    }
};

constexpr int GBM = 64, GBN = 128;

// Z = [H_self | mean] * [W_self; W_neigh] + b, ReLU except on the last layer
template <int VA, int VB>
__global__ __launch_bounds__(GNT) void k_sage_linear_fwd(MatRows a, CatW b, EpiFwd epi,
                                                         const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int m0 = blockIdx.x * GBM;
    if (m0 >= n1) return;
    a.rows = n1; epi.n1 = n1;
    gemm_tile<GBM, GBN, true, false, VA, VB>(m0, blockIdx.y * GBN, n1, b.N, 0, a.cols, a, b, epi);
}

// Partial [dW_self; dW_neigh; db] = [X | 1]^T * dZ over one chunk of destination rows (split-K).
// The output tiles of one chunk read the same slabs of X and dZ; the launch is one-dimensional and
// the workgroup id is decoded so that all tiles of a chunk land on the same XCD (workgroups are
// dealt round-robin to the 8 XCDs) and share its L2.  Partials go to a per-chunk slab; a
// fixed-order reduction follows (deterministic, no atomics).
template <int VA, int VB>
__global__ __launch_bounds__(GNT) void k_sage_grad_w(MatRowsOnes a, MatRows dz, EpiGradW epi, int kchunk,
                                                     int tiles_m, int tiles_n,
                                                     const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int tiles = tiles_m * tiles_n;
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int tile = j % tiles, chunk = (j / tiles) * 8 + xcd;
    const int k_begin = chunk * kchunk;
    if (k_begin >= n1) return;
    a.rows = n1; dz.rows = n1;
    const int k_end = min(n1, k_begin + kchunk);
    epi.part += (int64_t)chunk * epi.rows * epi.N;
    gemm_tile<GBM, GBN, false, false, VA, VB>((tile % tiles_m) * GBM, (tile / tiles_m) * GBN, a.cols + 1,
                                              dz.cols, k_begin, k_end, a, dz, epi);
}

// Sum the per-chunk partials in chunk order into the caller's gradient buffers, all layers in one
// launch (blockIdx.y = layer).
struct GradReduce {
    const float *part[GS_MAXL]; float *gws[GS_MAXL]; float *gwn[GS_MAXL]; float *gb[GS_MAXL];
    int D[GS_MAXL]; int N[GS_MAXL]; int kchunk[GS_MAXL];
};
__global__ __launch_bounds__(256) void k_reduce_grads(GradReduce g, const GsLevelMeta *__restrict__ meta, int S) {
    const int l = blockIdx.y;
    const int n1 = meta[l + 1].front_off[S];
    const int chunks = (n1 + g.kchunk[l] - 1) / g.kchunk[l];
    const int D = g.D[l], N = g.N[l];
    const int64_t words = (int64_t)(2 * D + 1) * N;
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < words;
         x += (int64_t)gridDim.x * blockDim.x) {
        float acc = 0.f;
        const float *p = g.part[l] + x;
        int z = 0;
        for (; z + 4 <= chunks; z += 4) {
            const float v0 = p[(int64_t)z * words], v1 = p[(int64_t)(z + 1) * words];
            const float v2 = p[(int64_t)(z + 2) * words], v3 = p[(int64_t)(z + 3) * words];
            acc += v0; acc += v1; acc += v2; acc += v3;
        }
        for (; z < chunks; ++z) acc += p[(int64_t)z * words];
        const int64_t wn = (int64_t)D * N;
        if (x < wn) g.gws[l][x] = acc;
        else if (x < 2 * wn) g.gwn[l][x - wn] = acc;
        else g.gb[l][x - 2 * wn] = acc;
    }
}

// [dH_self | dMean / cnt] = dZ * [W_self; W_neigh]^T per destination row
template <int VA, int VB>
__global__ __launch_bounds__(GNT) void k_sage_grad_in(MatRows dz, CatW w, EpiGradIn epi,
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
template <int LPR, bool HACT_H>
__global__ __launch_bounds__(256) void k_pull_input_grad(const float *__restrict__ gin, int D,
                                                         const int32_t *__restrict__ rev_ptr,
                                                         const int32_t *__restrict__ rev_cnt,
                                                         const int32_t *__restrict__ rev_list,
                                                         const void *__restrict__ hact,
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
            float4 h;
            if (HACT_H) {
                const uint2 raw = reinterpret_cast<const uint2 *>(hact)[(int64_t)u * nvec + c];
                h = make_float4(bf2f(raw.x & 0xFFFFu), bf2f(raw.x >> 16), bf2f(raw.y & 0xFFFFu), bf2f(raw.y >> 16));
            } else {
                h = A4[(int64_t)u * nvec + c];
            }
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

#include "sage_bf16.h"

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

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
    const size_t esz = p->dtype == GSPLIT_BF16 ? 2 : 4;
    for (int l = 1; l < L; ++l) {
        int rc = gs_alloc(ctx, &sb.hidden[l], esz * ctx->ub_front[l] * p->dims[l], "hidden");
        if (rc) return rc;
        rc = gs_alloc(ctx, (void **)&sb.ghid[l], sizeof(float) * ctx->ub_front[l] * p->dims[l], "ghid");
        if (rc) return rc;
    }
    for (int l = 0; l < L; ++l) {
        int rc = gs_alloc(ctx, &sb.xin[l], esz * ctx->ub_front[l + 1] * 2 * p->dims[l], "layer input");
        if (rc) return rc;
        if (p->dtype == GSPLIT_BF16) {
            const int64_t np = (p->dims[l + 1] + 7) & ~7;
            rc = gs_alloc(ctx, (void **)&sb.wstack[l], 2 * (size_t)(2 * p->dims[l]) * np, "bf16 weights");
            if (rc) return rc;
            rc = gs_alloc(ctx, (void **)&sb.wtrans[l], 2 * (size_t)p->dims[l + 1] * 2 * p->dims[l], "bf16 weights^T");
        }
        if (rc) return rc;
        rc = gs_alloc(ctx, (void **)&sb.inv_cnt[l], sizeof(float) * ctx->ub_front[l + 1], "inverse counts");
        if (rc) return rc;
    }
    for (int l = 0; l < L; ++l) {
        // split-K geometry of the weight-gradient product: about 1024 workgroups at the upper bound
        const int tiles = (int)(gs_ceil_div(2 * p->dims[l] + 1, GBM) * gs_ceil_div(p->dims[l + 1], GBN));
        const int64_t ub = ctx->ub_front[l + 1];
        int64_t chunks = std::max<int64_t>(8, 1024 / tiles);
        int64_t kchunk = std::max<int64_t>(64, gs_ceil_div(gs_ceil_div(ub, chunks), 32) * 32);
        chunks = gs_ceil_div(gs_ceil_div(ub, kchunk), 8) * 8;
        sb.kchunk[l] = (int)kchunk;
        sb.nchunk[l] = (int)chunks;
        int rc = gs_alloc(ctx, (void **)&sb.gw_part[l],
                          sizeof(float) * chunks * (2 * p->dims[l] + 1) * p->dims[l + 1], "weight-gradient partials");
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
    if (p->dtype != GSPLIT_F32 && p->dtype != GSPLIT_BF16)
        return gs_fail(ctx, GSPLIT_EINVAL, std::string(who) + ": dtype must be GSPLIT_F32 or GSPLIT_BF16");
    if (p->dtype == GSPLIT_BF16)
        for (int l = 0; l < ctx->L; ++l)
            if (p->dims[l] % 4 != 0)
                return gs_fail(ctx, GSPLIT_EINVAL, std::string(who) + ": GSPLIT_BF16 needs input and hidden widths "
                                                                      "that are multiples of 4");
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
                           B.blk_indptr, B.edge_row, B.self_row, mu, ctx->S, X, ctx->sage.inv_cnt[l]);
        return;
    }
    const int nvec = D / 4;
    if (nvec <= 16)
        hipLaunchKernelGGL(k_assemble_input_f32<16>, dim3(grid_1d(ctx, ub * 16)), dim3(256), 0, st, hin, D,
                           B.blk_indptr, B.edge_row, B.self_row, mu, ctx->S, X, ctx->sage.inv_cnt[l]);
    else if (nvec <= 32)
        hipLaunchKernelGGL(k_assemble_input_f32<32>, dim3(grid_1d(ctx, ub * 32)), dim3(256), 0, st, hin, D,
                           B.blk_indptr, B.edge_row, B.self_row, mu, ctx->S, X, ctx->sage.inv_cnt[l]);
    else
        hipLaunchKernelGGL(k_assemble_input_f32<64>, dim3(grid_1d(ctx, ub * 64)), dim3(256), 0, st, hin, D,
                           B.blk_indptr, B.edge_row, B.self_row, mu, ctx->S, X, ctx->sage.inv_cnt[l]);
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
    if (p->dtype == GSPLIT_BF16) {
        if (!aligned16(d_feat_local)) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_sage_fwd: features must be 16-byte aligned");
        WeightPrep wp;
        int64_t wmax = 1;
        for (int l = 0; l < L; ++l) {
            wp.ws[l] = (const float *)p->d_w_self[l]; wp.wn[l] = (const float *)p->d_w_neigh[l];
            wp.stacked[l] = sb.wstack[l]; wp.transposed[l] = sb.wtrans[l];
            wp.D[l] = p->dims[l]; wp.N[l] = p->dims[l + 1];
            wmax = std::max<int64_t>(wmax, (int64_t)2 * p->dims[l] * ((p->dims[l + 1] + 7) & ~7));
        }
        {
            GsTimeScope ts(ctx, "prep_weights", -1, st);
            hipLaunchKernelGGL(k_prep_weights_h, dim3((unsigned)std::min<int64_t>(128, gs_ceil_div(wmax, 256)), L),
                               dim3(256), 0, st, wp);
        }
        for (int l = 0; l < L; ++l) {
            const int D = p->dims[l], N = p->dims[l + 1];
            const uint16_t *hin = l == 0 ? (const uint16_t *)d_feat_local : (const uint16_t *)sb.hidden[l];
            const GsLayerBuf &B = ctx->layer[l];
            const GsLevelMeta *mu = ctx->d_meta + (l + 1);
            const int64_t ub = ctx->ub_front[l + 1];
            {
                GsTimeScope ts(ctx, "assemble_input", l, st);
                uint16_t *X = (uint16_t *)sb.xin[l];
                if (D / 4 <= 16)
                    hipLaunchKernelGGL(k_assemble_input_h<16>, dim3(grid_1d(ctx, ub * 16)), dim3(256), 0, st, hin, D,
                                       B.blk_indptr, B.edge_row, B.self_row, mu, S, X, sb.inv_cnt[l]);
                else if (D / 4 <= 32)
                    hipLaunchKernelGGL(k_assemble_input_h<32>, dim3(grid_1d(ctx, ub * 32)), dim3(256), 0, st, hin, D,
                                       B.blk_indptr, B.edge_row, B.self_row, mu, S, X, sb.inv_cnt[l]);
                else
                    hipLaunchKernelGGL(k_assemble_input_h<64>, dim3(grid_1d(ctx, ub * 64)), dim3(256), 0, st, hin, D,
                                       B.blk_indptr, B.edge_row, B.self_row, mu, S, X, sb.inv_cnt[l]);
            }
            MatRowsH x{(const uint16_t *)sb.xin[l], 0, 2 * D};
            MatRowsH wt{sb.wtrans[l], N, 2 * D};
            EpiFwdH epi{l == L - 1 ? (void *)d_logits : sb.hidden[l + 1], (const float *)p->d_bias[l], N, 0,
                        l < L - 1 ? 1 : 0, l == L - 1 ? 1 : 0};
            dim3 grid((unsigned)gs_ceil_div(ub, GBM), (unsigned)gs_ceil_div(N, GBN));
            GsTimeScope ts(ctx, "linear_fwd", l, st);
            hipLaunchKernelGGL(k_sage_linear_fwd_h, grid, dim3(GNT), 0, st, x, wt, epi, mu, S);
        }
        GS_HIP(ctx, hipGetLastError());
        sb.fwd_done = true;
        sb.fwd_batch = ctx->batch_id;
        return GSPLIT_OK;
    }
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
        if (va && vb) hipLaunchKernelGGL((k_sage_linear_fwd<4, 4>), grid, dim3(GNT), 0, st, a, b, epi, mu, S);
        else if (va) hipLaunchKernelGGL((k_sage_linear_fwd<4, 1>), grid, dim3(GNT), 0, st, a, b, epi, mu, S);
        else if (vb) hipLaunchKernelGGL((k_sage_linear_fwd<1, 4>), grid, dim3(GNT), 0, st, a, b, epi, mu, S);
        else hipLaunchKernelGGL((k_sage_linear_fwd<1, 1>), grid, dim3(GNT), 0, st, a, b, epi, mu, S);
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
        if (sb.dims[l] != p->dims[l] || sb.dtype != p->dtype)
            return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_sage_bwd: parameters differ from the forward pass");
    hipStream_t st = (hipStream_t)stream;
    const int L = ctx->L, S = ctx->S;
    for (int l = 0; l < L; ++l)
        if (!d_gw_self[l] || !d_gw_neigh[l] || !d_gbias[l])
            return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_sage_bwd: NULL gradient pointer");
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
        EpiGradW ew{sb.gw_part[l], 2 * D + 1, N};
        const bool vin = D % 2 == 0;
        const bool vdz = N % 4 == 0 && aligned16(dH);
        const bool vw = N % 4 == 0 && aligned16(p->d_w_self[l]) && aligned16(p->d_w_neigh[l]);
        const bool h16 = p->dtype == GSPLIT_BF16;
        {
            const int kchunk = sb.kchunk[l];
            const int tm = (int)gs_ceil_div(2 * D + 1, GBM), tn = (int)gs_ceil_div(N, GBN);
            dim3 grid((unsigned)(sb.nchunk[l] * tm * tn));
            GsTimeScope ts(ctx, "grad_w", l, st);
            MatRowsOnesH inh{(const uint16_t *)sb.xin[l], 0, 2 * D};
            if (h16 && vdz) hipLaunchKernelGGL((k_sage_grad_w_h<4, 4>), grid, dim3(GNT), 0, st, inh, dz, ew, kchunk, tm, tn, mu, S);
            else if (h16) hipLaunchKernelGGL((k_sage_grad_w_h<4, 1>), grid, dim3(GNT), 0, st, inh, dz, ew, kchunk, tm, tn, mu, S);
            else if (vin && vdz) hipLaunchKernelGGL((k_sage_grad_w<4, 4>), grid, dim3(GNT), 0, st, in, dz, ew, kchunk, tm, tn, mu, S);
            else if (vin) hipLaunchKernelGGL((k_sage_grad_w<4, 1>), grid, dim3(GNT), 0, st, in, dz, ew, kchunk, tm, tn, mu, S);
            else if (vdz) hipLaunchKernelGGL((k_sage_grad_w<1, 4>), grid, dim3(GNT), 0, st, in, dz, ew, kchunk, tm, tn, mu, S);
            else hipLaunchKernelGGL((k_sage_grad_w<1, 1>), grid, dim3(GNT), 0, st, in, dz, ew, kchunk, tm, tn, mu, S);
        }
        if (l > 0) {
            const GsLevelMeta *ml = ctx->d_meta + l;
            CatW w{(const float *)p->d_w_self[l], (const float *)p->d_w_neigh[l], D, N};
            EpiGradIn ei{sb.gtmp, sb.inv_cnt[l], D, 0};
            dim3 grid((unsigned)gs_ceil_div(ub, GBM), (unsigned)gs_ceil_div(2 * D, GBN));
            {
            GsTimeScope ts(ctx, "grad_in", l, st);
            MatRowsH wsk{sb.wstack[l], 2 * D, (N + 7) & ~7};
            if (h16 && vdz) hipLaunchKernelGGL((k_sage_grad_in_h<4>), grid, dim3(GNT), 0, st, dz, wsk, ei, mu, S);
            else if (h16) hipLaunchKernelGGL((k_sage_grad_in_h<1>), grid, dim3(GNT), 0, st, dz, wsk, ei, mu, S);
            else if (vdz && vw) hipLaunchKernelGGL((k_sage_grad_in<4, 4>), grid, dim3(GNT), 0, st, dz, w, ei, mu, S);
            else if (vdz) hipLaunchKernelGGL((k_sage_grad_in<4, 1>), grid, dim3(GNT), 0, st, dz, w, ei, mu, S);
            else if (vw) hipLaunchKernelGGL((k_sage_grad_in<1, 4>), grid, dim3(GNT), 0, st, dz, w, ei, mu, S);
            else hipLaunchKernelGGL((k_sage_grad_in<1, 1>), grid, dim3(GNT), 0, st, dz, w, ei, mu, S);
            }
            GsTimeScope ts(ctx, "pull_input_grad", l, st);
            // reverse shuffle + ReLU of the layer below: dZ of layer l-1
            const void *hact = sb.hidden[l];
            const int64_t ubl = ctx->ub_front[l];
            if (h16) {
                if (D / 4 <= 16)
                    hipLaunchKernelGGL((k_pull_input_grad<16, true>), dim3(grid_1d(ctx, ubl * 16)), dim3(256), 0, st,
                                       sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, hact, ml, S, sb.ghid[l]);
                else if (D / 4 <= 32)
                    hipLaunchKernelGGL((k_pull_input_grad<32, true>), dim3(grid_1d(ctx, ubl * 32)), dim3(256), 0, st,
                                       sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, hact, ml, S, sb.ghid[l]);
                else
                    hipLaunchKernelGGL((k_pull_input_grad<64, true>), dim3(grid_1d(ctx, ubl * 64)), dim3(256), 0, st,
                                       sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, hact, ml, S, sb.ghid[l]);
            } else if (D % 4 != 0) {
                hipLaunchKernelGGL(k_pull_input_grad_any, dim3(grid_1d(ctx, ubl * 64)), dim3(256), 0, st,
                                   sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, (const float *)hact, ml, S, sb.ghid[l]);
            } else if (D / 4 <= 16) {
                hipLaunchKernelGGL((k_pull_input_grad<16, false>), dim3(grid_1d(ctx, ubl * 16)), dim3(256), 0, st,
                                   sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, hact, ml, S, sb.ghid[l]);
            } else if (D / 4 <= 32) {
                hipLaunchKernelGGL((k_pull_input_grad<32, false>), dim3(grid_1d(ctx, ubl * 32)), dim3(256), 0, st,
                                   sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, hact, ml, S, sb.ghid[l]);
            } else {
                hipLaunchKernelGGL((k_pull_input_grad<64, false>), dim3(grid_1d(ctx, ubl * 64)), dim3(256), 0, st,
                                   sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, hact, ml, S, sb.ghid[l]);
            }
        }
    }
    {
        GradReduce gr;
        int64_t wmax = 1;
        for (int l = 0; l < L; ++l) {
            gr.part[l] = sb.gw_part[l]; gr.gws[l] = d_gw_self[l]; gr.gwn[l] = d_gw_neigh[l]; gr.gb[l] = d_gbias[l];
            gr.D[l] = p->dims[l]; gr.N[l] = p->dims[l + 1]; gr.kchunk[l] = sb.kchunk[l];
            wmax = std::max<int64_t>(wmax, (int64_t)(2 * p->dims[l] + 1) * p->dims[l + 1]);
        }
        GsTimeScope ts(ctx, "reduce_grads", -1, st);
        hipLaunchKernelGGL(k_reduce_grads, dim3((unsigned)std::min<int64_t>(256, gs_ceil_div(wmax, 256)), L), dim3(256),
                           0, st, gr, ctx->d_meta, S);
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

