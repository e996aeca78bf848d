// bfloat16 storage path of the GraphSAGE layers (included by sage.hip, inside its anonymous
// namespace): features, activations, assembled layer inputs and weights are held in bfloat16 and
// fed to v_mfma_f32_32x32x16_bf16 with float accumulation; biases, logits and all gradients stay
// float.  dZ is rounded to bfloat16 where it enters a matrix product (both operands of a bf16 MFMA
// are bf16).
#pragma once

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int BKH = 64;          // k per tile
constexpr int H_LD16 = 9;        // LDS row stride in 16-byte units: 64 bf16 + 8 padding = 144 bytes

// ------------------------------------------------------------------------------------------
// weights: float [D x N] pairs -> bf16 stacked [2D x Npad] (rows j, for dZ * W^T) and transposed
// [N x 2D] (rows n, for X * W), all layers in one launch (blockIdx.y = layer).  Npad = N rounded
// up to 8, padding columns are zero.
// ------------------------------------------------------------------------------------------
struct WeightPrep {
    const float *ws[GS_MAXL]; const float *wn[GS_MAXL];
    uint16_t *stacked[GS_MAXL]; uint16_t *transposed[GS_MAXL];
    int D[GS_MAXL]; int N[GS_MAXL];
};
__global__ __launch_bounds__(256) void k_prep_weights_h(WeightPrep w) {
    const int l = blockIdx.y;
    const int D = w.D[l], N = w.N[l], Np = (N + 7) & ~7;
    const int64_t total = (int64_t)2 * D * Np;
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < total;
         x += (int64_t)gridDim.x * blockDim.x) {
        const int j = (int)(x / Np), n = (int)(x - (int64_t)j * Np);
        uint16_t h = 0;
        if (n < N) {
            const float v = j < D ? w.ws[l][(int64_t)j * N + n] : w.wn[l][(int64_t)(j - D) * N + n];
            h = f2bf(v);
            w.transposed[l][(int64_t)n * 2 * D + j] = h;
        }
        w.stacked[l][x] = h;
    }
}

// ------------------------------------------------------------------------------------------
// layer input assembly, bf16 rows: X[i] = [H[self_row[i]] | bf16(mean of H[edge_row[e]])], the
// mean accumulated in float in slot order; 4 halves (8 bytes) per lane.
// ------------------------------------------------------------------------------------------
template <int LPR>
__global__ __launch_bounds__(256) void k_assemble_input_h(const uint16_t *__restrict__ H, int D,
                                                          const int32_t *__restrict__ blk_indptr,
                                                          const int32_t *__restrict__ edge_row,
                                                          const int32_t *__restrict__ self_row,
                                                          const GsLevelMeta *__restrict__ meta_up, int S,
                                                          uint16_t *__restrict__ X, float *__restrict__ inv_cnt) {
    const int n1 = meta_up->front_off[S];
    const int nvec = D >> 2;
    const int c0 = threadIdx.x % LPR;
    const int groups = (gridDim.x * blockDim.x) / LPR;
    const uint2 *H2 = reinterpret_cast<const uint2 *>(H);
    uint2 *X2 = reinterpret_cast<uint2 *>(X);
    for (int row = (blockIdx.x * blockDim.x + threadIdx.x) / LPR; row < n1; row += groups) {
        const int e0 = blk_indptr[row], e1 = blk_indptr[row + 1];
        const int64_t self = self_row[row];
        const float cnt = (float)(e1 - e0);
        if (c0 == 0) inv_cnt[row] = e1 > e0 ? 1.f / cnt : 0.f;
        for (int c = c0; c < nvec; c += LPR) {
            const uint2 own = H2[self * nvec + c];
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
            int e = e0;
            for (; e + 2 <= e1; e += 2) {
                const uint2 p = H2[(int64_t)edge_row[e] * nvec + c], q = H2[(int64_t)edge_row[e + 1] * nvec + c];
                a0 += bf2f(p.x & 0xFFFFu); a1 += bf2f(p.x >> 16); a2 += bf2f(p.y & 0xFFFFu); a3 += bf2f(p.y >> 16);
                a0 += bf2f(q.x & 0xFFFFu); a1 += bf2f(q.x >> 16); a2 += bf2f(q.y & 0xFFFFu); a3 += bf2f(q.y >> 16);
            }
            if (e < e1) {
                const uint2 p = H2[(int64_t)edge_row[e] * nvec + c];
                a0 += bf2f(p.x & 0xFFFFu); a1 += bf2f(p.x >> 16); a2 += bf2f(p.y & 0xFFFFu); a3 += bf2f(p.y >> 16);
            }
            if (e1 > e0) { a0 /= cnt; a1 /= cnt; a2 /= cnt; a3 /= cnt; }
            uint2 m;
            m.x = (uint32_t)f2bf(a0) | ((uint32_t)f2bf(a1) << 16);
            m.y = (uint32_t)f2bf(a2) | ((uint32_t)f2bf(a3) << 16);
            X2[(int64_t)row * 2 * nvec + c] = own;
            X2[(int64_t)row * 2 * nvec + nvec + c] = m;
        }
    }
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA GEMM core: C[M x N] = A[M x K] * B[K x N], both operands K-contiguous in memory
// (A rows m, B rows n), staged as lds[row][k] with 144-byte rows; a fragment is one 128-bit LDS
// read (8 consecutive k of one row), v_mfma_f32_32x32x16_bf16 consumes k = 8 * (lane / 32) .. + 7
// of a 16-k step.  Same 8-wave workgroup, two LDS stages and two register stages as the float
// core.  A may be a float matrix (dZ), converted when written to LDS.
// ------------------------------------------------------------------------------------------
struct MatRowsH {            // bf16 row-major matrix, cols % 8 == 0
    const uint16_t *p; int rows; int cols;
    __device__ __forceinline__ const uint16_t *at8(int o, int i, bool &in) const {
        in = o < rows && i < cols;
        const int oc = min(o, rows - 1), ic = min(i, cols - 8);
        return p + (int64_t)oc * cols + ic;
    }
};

template <int ROWS, int NT, class F>
struct StagerH {             // bf16 source
    static constexpr int NV = ROWS * BKH / 8 / NT;
    static_assert(NV >= 1 && NV <= 8, "tile does not fit the workgroup");
    uint4 reg[NV];
    unsigned keep;
    __device__ __forceinline__ void load(const F &f, int r0, int r_end, int k0, int k_end, int tid) {
        keep = 0u;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int kq = tid & 7, row = (tid >> 3) + (NT / 8) * v;
            bool in;
            reg[v] = *reinterpret_cast<const uint4 *>(f.at8(r0 + row, k0 + 8 * kq, in));
            keep |= (in && r0 + row < r_end && k0 + 8 * kq < k_end) ? (1u << v) : 0u;
        }
    }
    __device__ __forceinline__ void store(uint4 *lds, int tid) const {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int kq = tid & 7, row = (tid >> 3) + (NT / 8) * v;
            uint4 w = reg[v];
            if (!((keep >> v) & 1u)) w = make_uint4(0u, 0u, 0u, 0u);
            lds[row * H_LD16 + kq] = w;
        }
    }
};

template <int ROWS, int NT, int VW, class F>
struct StagerF2H {           // float source (accessor of the float core), VW = 4 or 1
    static constexpr int NV = ROWS * BKH / 8 / NT;
    float4 reg[2 * NV];
    unsigned keep;           // 8 bits per chunk
    __device__ __forceinline__ void load(const F &f, int r0, int r_end, int k0, int k_end, int tid) {
        keep = 0u;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int kq = tid & 7, row = (tid >> 3) + (NT / 8) * v;
            const int k = k0 + 8 * kq;
            const bool rok = r0 + row < r_end;
            if (VW == 4) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    bool in;
                    reg[2 * v + h] = *reinterpret_cast<const float4 *>(f.template at<4>(r0 + row, k + 4 * h, in));
                    keep |= (in && rok && k + 4 * h < k_end) ? (0xFu << (8 * v + 4 * h)) : 0u;
                }
            } else {
                float t[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    bool in;
                    t[j] = *reinterpret_cast<const float *>(f.template at<1>(r0 + row, k + j, in));
                    keep |= (in && rok && k + j < k_end) ? (1u << (8 * v + j)) : 0u;
                }
                reg[2 * v] = make_float4(t[0], t[1], t[2], t[3]);
                reg[2 * v + 1] = make_float4(t[4], t[5], t[6], t[7]);
            }
        }
    }
    __device__ __forceinline__ void store(uint4 *lds, int tid) const {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int kq = tid & 7, row = (tid >> 3) + (NT / 8) * v;
            const float4 a = reg[2 * v], b = reg[2 * v + 1];
            const float t[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            uint32_t h[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) h[j] = ((keep >> (8 * v + j)) & 1u) ? (uint32_t)f2bf(t[j]) : 0u;
            lds[row * H_LD16 + kq] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16),
                                                h[6] | (h[7] << 16));
        }
    }
};

template <int BM, int BN, class SA, class SB, class AF, class BF, class EF>
__device__ __forceinline__ void gemm_tile_h(const int m0, const int n0, const int m_end, const int n_end,
                                            const int k_end, const AF &a, const BF &b, const EF &epi) {
    __shared__ uint4 As0[BM * H_LD16], As1[BM * H_LD16], Bs0[BN * H_LD16], Bs1[BN * H_LD16];
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
    SA sa0, sa1;
    SB sb0, sb1;

    auto multiply = [&](const uint4 *As, const uint4 *Bs) {
        uint4 af[BKH / 16][MI], bf[BKH / 16][NI];
#pragma unroll
        for (int ks = 0; ks < BKH / 16; ++ks) {
#pragma unroll
            for (int i = 0; i < MI; ++i) af[ks][i] = As[(wm0 + i * 32 + l32) * H_LD16 + 2 * ks + half];
#pragma unroll
            for (int j = 0; j < NI; ++j) bf[ks][j] = Bs[(wn0 + j * 32 + l32) * H_LD16 + 2 * ks + half];
        }
#pragma unroll
        for (int ks = 0; ks < BKH / 16; ++ks)
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[ks][i]),
                                                                        __builtin_bit_cast(bf16x8, bf[ks][j]),
                                                                        acc[i][j], 0, 0, 0);
    };
    auto step = [&](SA &ra_cur, SB &rb_cur, SA &ra_nxt, SB &rb_nxt, const uint4 *As_cur, const uint4 *Bs_cur,
                    uint4 *As_nxt, uint4 *Bs_nxt, int k0) {
        if (k0 + 2 * BKH < k_end) {
            ra_cur.load(a, m0, m_end, k0 + 2 * BKH, k_end, tid);
            rb_cur.load(b, n0, n_end, k0 + 2 * BKH, k_end, tid);
        }
        multiply(As_cur, Bs_cur);
        if (k0 + BKH < k_end) {
            ra_nxt.store(As_nxt, tid);
            rb_nxt.store(Bs_nxt, tid);
        }
        __syncthreads();
    };
    sa0.load(a, m0, m_end, 0, k_end, tid);
    sb0.load(b, n0, n_end, 0, k_end, tid);
    if (BKH < k_end) {
        sa1.load(a, m0, m_end, BKH, k_end, tid);
        sb1.load(b, n0, n_end, BKH, k_end, tid);
    }
    sa0.store(As0, tid);
    sb0.store(Bs0, tid);
    __syncthreads();
    // steady state without conditions around the loads (every tile a round fetches exists), so that
    // the compiler waits only for the loads a step is about to store and the younger ones stay in
    // flight; the general loop takes the last tiles
    int k0 = 0;
    {
        auto whole_step = [&](SA &ra_cur, SB &rb_cur, SA &ra_nxt, SB &rb_nxt, const uint4 *As_cur,
                              const uint4 *Bs_cur, uint4 *As_nxt, uint4 *Bs_nxt, int kk) {
            ra_cur.load(a, m0, m_end, kk + 2 * BKH, k_end, tid);
            rb_cur.load(b, n0, n_end, kk + 2 * BKH, k_end, tid);
            multiply(As_cur, Bs_cur);
            ra_nxt.store(As_nxt, tid);
            rb_nxt.store(Bs_nxt, tid);
            __syncthreads();
        };
        for (; k0 + 3 * BKH < k_end; k0 += 2 * BKH) {
            whole_step(sa0, sb0, sa1, sb1, As0, Bs0, As1, Bs1, k0);
            whole_step(sa1, sb1, sa0, sb0, As1, Bs1, As0, Bs0, k0 + BKH);
        }
    }
    for (; k0 < k_end; k0 += 2 * BKH) {
        step(sa0, sb0, sa1, sb1, As0, Bs0, As1, Bs1, k0);
        if (k0 + BKH < k_end) step(sa1, sb1, sa0, sb0, As1, Bs1, As0, Bs0, k0 + BKH);
    }
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

// forward epilogue: + bias, ReLU, bf16 activations (float logits on the last layer)
struct EpiFwdH {
    void *out; const float *bias; int N; int n1; int relu; int out_is_float;
    __device__ __forceinline__ float col(int n) const { return n < N ? bias[n] : 0.f; }
    __device__ __forceinline__ float row(int) const { return 0.f; }
    __device__ __forceinline__ void store(int m, int n, float v, float, float b) const {
        if (m < n1 && n < N) {
            float z = v + b;
            z = (relu && z < 0.f) ? 0.f : z;
            if (out_is_float) reinterpret_cast<float *>(out)[(int64_t)m * N + n] = z;
            else reinterpret_cast<uint16_t *>(out)[(int64_t)m * N + n] = f2bf(z);
        }
    }
};

// Z = X * [W_self; W_neigh] + b with X bf16 [n1 x 2D] and the transposed bf16 weights [N x 2D].
// Persistent launch like the float row-block products (tiles gid, gid + gridDim.x, ...).
__global__ __launch_bounds__(GNT) void k_sage_linear_fwd_h(MatRowsH x, MatRowsH wt, EpiFwdH epi,
                                                           const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int tiles_m = (n1 + GBM - 1) / GBM, tiles_n = (wt.rows + GBN - 1) / GBN;
    const int total = ((tiles_m + 7) & ~7) * tiles_n;
    x.rows = n1; epi.n1 = n1;
    for (int gid = blockIdx.x; gid < total; gid += gridDim.x) {
        int m0, n0;
        if (!next_tile<TileMid>(gid, tiles_m, tiles_n, m0, n0)) continue;
        gemm_tile_h<GBM, GBN, StagerH<GBM, GNT, MatRowsH>, StagerH<GBN, GNT, MatRowsH>>(
            m0, n0, n1, wt.rows, x.cols, x, wt, epi);
    }
}

// [dH_self | dMean / cnt] = dZ * [W_self; W_neigh]^T with dZ float [n1 x N] (converted on the way
// into LDS) and the stacked bf16 weights [2D x Npad]
template <int VW>
__global__ __launch_bounds__(GNT) void k_sage_grad_in_h(MatRows dz, MatRowsH wstack, EpiGradIn epi,
                                                        const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int tiles_m = (n1 + GBM - 1) / GBM, tiles_n = (wstack.rows + GBN - 1) / GBN;
    const int total = ((tiles_m + 7) & ~7) * tiles_n;
    dz.rows = n1; epi.n1 = n1;
    for (int gid = blockIdx.x; gid < total; gid += gridDim.x) {
        int m0, n0;
        if (!next_tile<TileMid>(gid, tiles_m, tiles_n, m0, n0)) continue;
        gemm_tile_h<GBM, GBN, StagerF2H<GBM, GNT, VW, MatRows>, StagerH<GBN, GNT, MatRowsH>>(
            m0, n0, n1, wstack.rows, dz.cols, dz, wstack, epi);
    }
}

// the same with dZ already held in bf16 (levels below the top one, width a multiple of 8)
__global__ __launch_bounds__(GNT) void k_sage_grad_in_hh(MatRowsH dz, MatRowsH wstack, EpiGradIn epi,
                                                         const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int tiles_m = (n1 + GBM - 1) / GBM, tiles_n = (wstack.rows + GBN - 1) / GBN;
    const int total = ((tiles_m + 7) & ~7) * tiles_n;
    dz.rows = n1; epi.n1 = n1;
    for (int gid = blockIdx.x; gid < total; gid += gridDim.x) {
        int m0, n0;
        if (!next_tile<TileMid>(gid, tiles_m, tiles_n, m0, n0)) continue;
        gemm_tile_h<GBM, GBN, StagerH<GBM, GNT, MatRowsH>, StagerH<GBN, GNT, MatRowsH>>(
            m0, n0, n1, wstack.rows, dz.cols, dz, wstack, epi);
    }
}

// bf16 matrix followed by a column of ones, read by the float weight-gradient product
struct MatRowsOnesH {
    const uint16_t *p; int rows; int cols;
    template <int VW>
    __device__ __forceinline__ const uint16_t *at(int o, int i, bool &in) const {
        in = o < rows && i <= cols;
        const int oc = min(o, rows - 1), ic = min(i, cols - VW);
        const uint16_t *q = p + (int64_t)oc * cols + ic;
        return i == cols ? g_one_then_zero_h : q;
    }
    __device__ __forceinline__ int tok(int i) const { return i >= cols ? -1 : min(i, cols - 4); }
    __device__ __forceinline__ const uint16_t *km(int k, int t) const {
        return t < 0 ? g_one_then_zero_h : p + (int64_t)k * cols + t;
    }
};

// ------------------------------------------------------------------------------------------
// Weight gradients on the bf16 matrix cores: C[m][n] = sum_k [X | 1][k][m] * bf16(dZ[k][n]) over
// one chunk of destination rows k (split-K as in the float path, same slabs and reduction).
// Both operands are k-major in memory while a fragment of v_mfma_f32_32x32x16_bf16 holds 8
// consecutive k of one m (or n), so tiles are transposed on the way into LDS: a thread loads a
// 2 (k) x 4 (m or n) patch with coalesced 8- or 16-byte reads, pairs the two k of each column into
// one 32-bit word and writes four words.  LDS rows are 64 k = 128 bytes without padding; the
// eight 16-byte granules of row r sit at granule ^ ((r ^ (r >> 2)) & 7), which spreads both the
// transposed 32-bit writes (lanes along r in steps of 4) and the 128-bit fragment reads (lanes
// along consecutive r) over all banks.
// ------------------------------------------------------------------------------------------
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {     // round to nearest even
    floatx2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ int t_swz(int r) { return (r ^ (r >> 2)) & 7; }
// 32-bit word of k pair kp (0..31) of row r in a transposed [rows][64 k] bf16 tile
__device__ __forceinline__ int t_word(int r, int kp) { return r * 32 + ((((kp >> 2) ^ t_swz(r)) << 2) | (kp & 3)); }

// dZ: plain float matrix read k-major; VW = 4 needs N % 4 == 0 and a 16-byte aligned base
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));

// dZ: plain float matrix read k-major; VW = 4 needs N % 4 == 0 and a 16-byte aligned base
template <int VW>
struct PatchDz {
    floatx4 r00, r01, r10, r11;     // r<pass><k of the pair>
    static __device__ __forceinline__ floatx4 fetch(const MatRows &dz, int n, int k, int k_end, bool full) {
        const int kr = min(k, dz.rows - 1);
        floatx4 v;
        if (VW == 4) {
            v = *reinterpret_cast<const floatx4 *>(dz.p + (int64_t)kr * dz.cols + min(n, dz.cols - 4));
        } else {
            const float *q = dz.p + (int64_t)kr * dz.cols;
            v.x = q[min(n, dz.cols - 1)]; v.y = q[min(n + 1, dz.cols - 1)];
            v.z = q[min(n + 2, dz.cols - 1)]; v.w = q[min(n + 3, dz.cols - 1)];
        }
        const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
        return (full || k < k_end) ? v : zero;
    }
    __device__ __forceinline__ void load(const MatRows &dz, int n0, int k, int k_end, int x, bool full) {
        r00 = fetch(dz, n0 + 4 * x, k, k_end, full);
        r01 = fetch(dz, n0 + 4 * x, k + 1, k_end, full);
        r10 = fetch(dz, n0 + 4 * (x + 16), k, k_end, full);
        r11 = fetch(dz, n0 + 4 * (x + 16), k + 1, k_end, full);
    }
    __device__ __forceinline__ void store(uint32_t *lds, int x, int kp) const {
        int row = 4 * x;
        lds[t_word(row, kp)] = pack_bf16(r00.x, r01.x);
        lds[t_word(row + 1, kp)] = pack_bf16(r00.y, r01.y);
        lds[t_word(row + 2, kp)] = pack_bf16(r00.z, r01.z);
        lds[t_word(row + 3, kp)] = pack_bf16(r00.w, r01.w);
        row = 4 * (x + 16);
        lds[t_word(row, kp)] = pack_bf16(r10.x, r11.x);
        lds[t_word(row + 1, kp)] = pack_bf16(r10.y, r11.y);
        lds[t_word(row + 2, kp)] = pack_bf16(r10.z, r11.z);
        lds[t_word(row + 3, kp)] = pack_bf16(r10.w, r11.w);
    }
};
// dZ already held in bf16 (cols % 4 == 0)
struct PatchDzH {
    uintx2 r00, r01, r10, r11;     // r<pass><k of the pair>
    static __device__ __forceinline__ uintx2 fetch(const MatRowsH &dz, int n, int k, int k_end, bool full) {
        const uintx2 v = *reinterpret_cast<const uintx2 *>(dz.p + (int64_t)min(k, dz.rows - 1) * dz.cols + min(n, dz.cols - 4));
        const uintx2 zero = {0u, 0u};
        return (full || k < k_end) ? v : zero;
    }
    __device__ __forceinline__ void load(const MatRowsH &dz, int n0, int k, int k_end, int x, bool full) {
        r00 = fetch(dz, n0 + 4 * x, k, k_end, full);
        r01 = fetch(dz, n0 + 4 * x, k + 1, k_end, full);
        r10 = fetch(dz, n0 + 4 * (x + 16), k, k_end, full);
        r11 = fetch(dz, n0 + 4 * (x + 16), k + 1, k_end, full);
    }
    static __device__ __forceinline__ void put(uint32_t *lds, int row, int kp, uintx2 a, uintx2 b) {
        lds[t_word(row, kp)] = (a.x & 0xFFFFu) | (b.x << 16);
        lds[t_word(row + 1, kp)] = (a.x >> 16) | (b.x & 0xFFFF0000u);
        lds[t_word(row + 2, kp)] = (a.y & 0xFFFFu) | (b.y << 16);
        lds[t_word(row + 3, kp)] = (a.y >> 16) | (b.y & 0xFFFF0000u);
    }
    __device__ __forceinline__ void store(uint32_t *lds, int x, int kp) const {
        put(lds, 4 * x, kp, r00, r01);
        put(lds, 4 * (x + 16), kp, r10, r11);
    }
};
// [X | 1]: bf16 matrix with its column of ones, read k-major
struct PatchX {
    uintx2 r0, r1;
    static __device__ __forceinline__ uintx2 fetch(const MatRowsOnesH &a, int tok, int k, int k_end, bool full) {
        const uintx2 v = *reinterpret_cast<const uintx2 *>(a.km(min(k, a.rows - 1), tok));
        const uintx2 zero = {0u, 0u};
        return (full || k < k_end) ? v : zero;
    }
    __device__ __forceinline__ void load(const MatRowsOnesH &a, int tok, int k, int k_end, bool full) {
        r0 = fetch(a, tok, k, k_end, full);
        r1 = fetch(a, tok, k + 1, k_end, full);
    }
    __device__ __forceinline__ void store(uint32_t *lds, int x, int kp) const {
        const int row = 4 * x;
        lds[t_word(row, kp)] = (r0.x & 0xFFFFu) | (r1.x << 16);
        lds[t_word(row + 1, kp)] = (r0.x >> 16) | (r1.x & 0xFFFF0000u);
        lds[t_word(row + 2, kp)] = (r0.y & 0xFFFFu) | (r1.y << 16);
        lds[t_word(row + 3, kp)] = (r0.y >> 16) | (r1.y & 0xFFFF0000u);
    }
};

// PDZ / DZ: PatchDz<4 or 1> with a float dZ (MatRows), PatchDzH with a bf16 dZ (MatRowsH)
template <class PDZ, class DZ>
__global__ __launch_bounds__(GNT) void k_sage_grad_w_h(MatRowsOnesH a, DZ dz, EpiGradW epi, int nchunk,
                                                       int rows_min, int tiles_m, int tiles_n,
                                                       const GsLevelMeta *__restrict__ meta_up, int S, int leave_from) {
    const int n1 = meta_up->front_off[S];
    if (leave_from > 0 && n1 >= leave_from) return;      // a level this large is the streaming kernel's
    const int kchunk = grad_w_chunk_rows(n1, nchunk, rows_min);
    const int tiles = tiles_m * tiles_n;
    const int xcd = blockIdx.x & 7, jb = blockIdx.x >> 3;
    const int tile = jb % tiles, chunk = (jb / tiles) * 8 + xcd;
    const int k_begin = chunk * kchunk;
    if (k_begin >= n1) return;
    a.rows = n1; dz.rows = n1;
    const int k_end = min(n1, k_begin + kchunk);
    epi.part += (int64_t)chunk * epi.rows * epi.N;
    const int m0 = (tile % tiles_m) * GBM, n0 = (tile / tiles_m) * GBN;

    // [stage][A rows then B rows][32 words]
    __shared__ __attribute__((aligned(16))) uint32_t lds[2][(GBM + GBN) * 32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int wm0 = (wave / GWN) * 32, wn0 = (wave % GWN) * 32;
    const int x = tid & 15, kp = (tid >> 4);          // patch: rows 4x.., k pair kp (0..31)
    const int tok = a.tok(m0 + 4 * x);
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    PatchX pa0, pa1;
    PDZ pb0, pb1;

    auto load_tile = [&](PatchX &pa, PDZ &pb, int k0) {
        const bool full = k0 + BKH <= k_end;
        pa.load(a, tok, k0 + 2 * kp, k_end, full);
        pb.load(dz, n0, k0 + 2 * kp, k_end, x, full);
    };
    auto store_tile = [&](const PatchX &pa, const PDZ &pb, uint32_t *buf) {
        pa.store(buf, x, kp);
        pb.store(buf + GBM * 32, x, kp);
    };
    auto multiply = [&](const uint32_t *buf) {
        const uint4 *As = reinterpret_cast<const uint4 *>(buf);
        const uint4 *Bs = reinterpret_cast<const uint4 *>(buf + GBM * 32);
        const int ra = wm0 + l32, rb = wn0 + l32;
        uint4 af[BKH / 16], bf[BKH / 16];
#pragma unroll
        for (int ks = 0; ks < BKH / 16; ++ks) {
            af[ks] = As[ra * 8 + ((2 * ks + half) ^ t_swz(ra))];
            bf[ks] = Bs[rb * 8 + ((2 * ks + half) ^ t_swz(rb))];
        }
#pragma unroll
        for (int ks = 0; ks < BKH / 16; ++ks)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[ks]),
                                                          __builtin_bit_cast(bf16x8, bf[ks]), acc, 0, 0, 0);
    };
    // one k-tile: the registers that held tile k0 (now in LDS) are refilled with tile k0 + 2 BKH,
    // tile k0 is multiplied, tile k0 + BKH moves from the other registers to the other LDS stage
    auto step = [&](PatchX &pa_cur, PDZ &pb_cur, const PatchX &pa_nxt, const PDZ &pb_nxt,
                    const uint32_t *buf_cur, uint32_t *buf_nxt, int k0) {
        if (k0 + 2 * BKH < k_end) load_tile(pa_cur, pb_cur, k0 + 2 * BKH);
        multiply(buf_cur);
        if (k0 + BKH < k_end) store_tile(pa_nxt, pb_nxt, buf_nxt);
        __syncthreads();
    };

    load_tile(pa0, pb0, k_begin);
    if (k_begin + BKH < k_end) load_tile(pa1, pb1, k_begin + BKH);
    store_tile(pa0, pb0, lds[0]);
    __syncthreads();
    // steady state without conditions around the loads: whole tiles that exist (see the row-block
    // product above)
    int k0 = k_begin;
    {
        auto whole_step = [&](PatchX &pa_cur, PDZ &pb_cur, const PatchX &pa_nxt, const PDZ &pb_nxt,
                              const uint32_t *buf_cur, uint32_t *buf_nxt, int kk) {
            pa_cur.load(a, tok, kk + 2 * BKH + 2 * kp, k_end, true);
            pb_cur.load(dz, n0, kk + 2 * BKH + 2 * kp, k_end, x, true);
            multiply(buf_cur);
            store_tile(pa_nxt, pb_nxt, buf_nxt);
            __syncthreads();
        };
        for (; k0 + 4 * BKH <= k_end; k0 += 2 * BKH) {
            whole_step(pa0, pb0, pa1, pb1, lds[0], lds[1], k0);
            whole_step(pa1, pb1, pa0, pb0, lds[1], lds[0], k0 + BKH);
        }
    }
    for (; k0 < k_end; k0 += 2 * BKH) {
        step(pa0, pb0, pa1, pb1, lds[0], lds[1], k0);
        if (k0 + BKH < k_end) step(pa1, pb1, pa0, pb0, lds[1], lds[0], k0 + BKH);
    }
    // accumulator layout of the 32x32 block: register r of lane l holds
    // row (r / 4) * 8 + (l / 32) * 4 + (r % 4), column l % 32
#pragma unroll
    for (int r = 0; r < 16; ++r)
        epi.store(m0 + wm0 + (r >> 2) * 8 + half * 4 + (r & 3), n0 + wn0 + l32, acc[r], 0.f, 0.f);
}
