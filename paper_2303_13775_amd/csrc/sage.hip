// GraphSAGE-mean forward and backward over the split mini-batch (paper Algorithm 2 `sp_forward`
// and the backward description after it).  The rows of all S logical splits are processed in one
// launch per step: on one GPU the training shuffle of layer l is the composition of the shuffle
// index with edges[l] (self_row / edge_row, built during sampling), so "shuffle then aggregate"
// is a gather through one index and the reverse shuffle of the backward pass is a scatter-add
// through the same index.
//
// Dense products run on the matrix cores: v_mfma_f32_32x32x2_f32 for fp32 storage.
#include <algorithm>
#include <cstdlib>
#include <type_traits>

#include "gsplit_internal.h"

namespace {

#include "gemm_f32.h"

// [W_self; W_neigh] stacked into one 2 D x Npad matrix (Npad = N rounded up to 4, padding zeroed):
// every product then reads the weights as one plain matrix in 16-byte pieces whatever N is.  All
// layers are stacked by one launch: a launch of its own (blockIdx.y = layer), or, riding on the
// bottom layer's input assembly, the workgroups behind that kernel's own (it needs the stacked
// weights no earlier than the product that follows).
struct WeightStack {
    const float *ws[GS_MAXL]; const float *wn[GS_MAXL]; float *stacked[GS_MAXL]; int D[GS_MAXL]; int N[GS_MAXL];
};
__device__ __forceinline__ void stack_weights(const WeightStack &w, int l, int block, int n_blocks) {
    const int D = w.D[l], N = w.N[l], np = (N + 3) & ~3;
    const int64_t words = (int64_t)2 * D * np;
    for (int64_t x = block * (int64_t)blockDim.x + threadIdx.x; x < words; x += (int64_t)n_blocks * blockDim.x) {
        const int k = (int)(x / np), n = (int)(x % np);
        float v = 0.f;
        if (n < N) v = k < D ? w.ws[l][(int64_t)k * N + n] : w.wn[l][(int64_t)(k - D) * N + n];
        w.stacked[l][x] = v;
    }
}
__global__ __launch_bounds__(256) void k_stack_weights(WeightStack w) {
    stack_weights(w, blockIdx.y, blockIdx.x, gridDim.x);
}

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
                                                            int S, int fan, float *__restrict__ X,
                                                            float *__restrict__ inv_cnt, int n_main,
                                                            WeightStack wstack, int n_stack) {
    if ((int)blockIdx.x >= n_main) {        // the workgroups behind the kernel's own stack the weights
        const int b = (int)blockIdx.x - n_main;
        stack_weights(wstack, b / n_stack, b % n_stack, n_stack);
        return;
    }
    const int n1 = meta_up->front_off[S];
    const int nvec = D >> 2;
    const int c0 = threadIdx.x % LPR;
    const int groups = (n_main * blockDim.x) / LPR;
    const int n_c = (nvec + LPR - 1) / LPR;      // column rounds, the same for every lane of a group
    const float4 *H4 = reinterpret_cast<const float4 *>(H);
    float4 *X4 = reinterpret_cast<float4 *>(X);
    // A row is a chain of dependent accesses (offsets -> source rows of its edges -> their values), and
    // the kernel's time is the length of that chain, not its bytes.  So the lanes of a group fetch the
    // source rows of up to LPR edges with one load (lane u takes edge u, the others get it by shuffle)
    // and keep the values of sixteen edges in flight; the sum still runs in edge order.  Edges a row
    // does not have are read from its own row (a valid address) and not added.
    for (int row = (blockIdx.x * blockDim.x + threadIdx.x) / LPR; row < n1; row += groups) {
        const int e0 = blk_indptr[row];
        const int m = blk_indptr[row + 1] - e0;
        const int64_t self = self_row[row];
        const float cnt = (float)m;
        if (c0 == 0) inv_cnt[row] = m > 0 ? 1.f / cnt : 0.f;
        for (int ci = 0; ci < n_c; ++ci) {
            const int c = c0 + ci * LPR;
            const bool cv = c < nvec;
            const int cc = cv ? c : 0;
            const float4 own = H4[self * nvec + cc];
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int chunk = 0; chunk < fan; chunk += LPR) {
                const int mine = chunk + c0 < m ? edge_row[e0 + chunk + c0] : -1;
#pragma unroll
                for (int half = 0; half < LPR; half += 16) {
                    // wave-uniform: does any row of this wave reach this far?
                    if (__ballot(chunk + half < m) == 0ull) break;
                    float4 v[16];
                    unsigned have = 0u;
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        const int r = __shfl(mine, half + u, LPR);
                        have |= (r >= 0 ? 1u : 0u) << u;
                        v[u] = H4[(r >= 0 ? (int64_t)r : self) * nvec + cc];
                    }
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        if ((have >> u) & 1u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
                    }
                }
            }
            if (m > 0) { acc.x /= cnt; acc.y /= cnt; acc.z /= cnt; acc.w /= cnt; }
            if (cv) {
                X4[(int64_t)row * 2 * nvec + c] = own;
                X4[(int64_t)row * 2 * nvec + nvec + c] = acc;
            }
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

// ---- operand accessors and epilogues ---------------------------------------------------------
__device__ const uint16_t g_one_then_zero_h[4] __attribute__((aligned(8))) = {0x3F80, 0, 0, 0};   // bf16 1, 0, 0, 0

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

// tile of the bf16 kernels
constexpr int GBM = 64, GBN = 128, GWM = 2, GWN = 4;

// Z = [H_self | mean] * [W_self; W_neigh] + b, ReLU except on the last layer; b is the stacked
// weight matrix, its columns padded to a multiple of 4
template <class T, int VA, int VB>
__global__ __launch_bounds__(GNT) __attribute__((amdgpu_waves_per_eu(T::LEAN ? 6 : 2, T::LEAN ? 6 : 8))) void k_sage_linear_fwd(MatRows a, MatRows b, EpiFwd epi,
                                                         const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int tiles_m = (n1 + T::BM - 1) / T::BM, tiles_n = (b.cols + T::BN - 1) / T::BN;
    const int total = ((tiles_m + 7) & ~7) * tiles_n;
    a.rows = n1; epi.n1 = n1;
    for (int gid = blockIdx.x; gid < total; gid += gridDim.x) {
        int m0, n0;
        if (!next_tile<T>(gid, tiles_m, tiles_n, m0, n0)) continue;
        gemm_tile<T, true, false, VA, VB>(m0, n0, n1, b.cols, 0, a.cols, a, b, epi);
    }
}

// Sum the per-chunk partials in chunk order into the caller's gradient buffers, all layers in one
// launch (blockIdx.y = layer).
struct GradReduce {
    const float *part[GS_MAXL]; float *gws[GS_MAXL]; float *gwn[GS_MAXL]; float *gb[GS_MAXL];
    int D[GS_MAXL]; int N[GS_MAXL]; int nchunk[GS_MAXL]; int rows_min[GS_MAXL];
    int fixed_chunks[GS_MAXL];      // > 0: the layer's slabs were written by that many workgroups, all of them
    // a level of at least stream_rows rows (> 0) had its slabs written by the streaming bf16 kernel,
    // whose chunks follow (stream_nchunk, stream_rows_min)
    int stream_rows[GS_MAXL]; int stream_nchunk[GS_MAXL]; int stream_rows_min[GS_MAXL];
};
__global__ __launch_bounds__(256) void k_reduce_grads(GradReduce g, const GsLevelMeta *__restrict__ meta, int S) {
    const int l = blockIdx.y;
    const int n1 = meta[l + 1].front_off[S];
    const bool streamed = g.stream_rows[l] > 0 && n1 >= g.stream_rows[l];
    const int kchunk = streamed ? grad_w_chunk_rows(n1, g.stream_nchunk[l], g.stream_rows_min[l])
                                : grad_w_chunk_rows(n1, g.nchunk[l], g.rows_min[l]);
    const int chunks = g.fixed_chunks[l] > 0 ? g.fixed_chunks[l] : (n1 + kchunk - 1) / kchunk;
    const int D = g.D[l], N = g.N[l];
    const int64_t words = (int64_t)(2 * D + 1) * N;
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < words;
         x += (int64_t)gridDim.x * blockDim.x) {
        float acc = 0.f;
        const float *p = g.part[l] + x;
        int z = 0;
        for (; z + 16 <= chunks; z += 16) {     // sixteen loads in flight, added in chunk order
            float v[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) v[j] = p[(int64_t)(z + j) * words];
#pragma unroll
            for (int j = 0; j < 16; ++j) acc += v[j];
        }
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

// [dH_self | dMean / cnt] = dZ * [W_self; W_neigh]^T per destination row; w is the stacked weight
// matrix (2 D rows, columns padded to a multiple of 4), n_k the true number of columns
template <class T, int VA, int VB>
__global__ __launch_bounds__(GNT) __attribute__((amdgpu_waves_per_eu(T::LEAN ? 6 : 2, T::LEAN ? 6 : 8))) void k_sage_grad_in(MatRows dz, MatRows w, EpiGradIn epi,
                                                      const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int tiles_m = (n1 + T::BM - 1) / T::BM, tiles_n = (w.rows + T::BN - 1) / T::BN;
    const int total = ((tiles_m + 7) & ~7) * tiles_n;
    dz.rows = n1; epi.n1 = n1;
    for (int gid = blockIdx.x; gid < total; gid += gridDim.x) {
        int m0, n0;
        if (!next_tile<T>(gid, tiles_m, tiles_n, m0, n0)) continue;
        gemm_tile<T, true, true, VA, VB>(m0, n0, n1, w.rows, 0, dz.cols, dz, w, epi);
    }
}

// Reverse shuffle of the backward pass as a pull: row u of local_cat[l] sums the gradient rows of
// every destination it fed (its own self term and one mean term per sampled edge), listed by the
// scatter side of the shuffle index.  The ReLU of the layer below is applied on the way out, so
// the result is that layer's dZ.  No atomics; rows that fed nothing get zeros.
//
// The entries of a row sit in its segment in the order an atomic cursor handed them out, which
// differs from run to run; a float sum in that order would too.  So the sum runs in ascending order
// of the entry codes (2 * destination [+ 1]), whatever the segment's order: one wave per row, one
// entry per lane, sorted across the wave with a bitonic network of shuffles (21 exchange steps, no
// memory traffic); then LPR lanes cover a gradient row 4 floats each, the 64 / LPR lane groups of
// the wave take every (64 / LPR)-th entry of the sorted list, and their partial sums are added in
// a fixed tree.  A row with up to 256 entries keeps four per lane (the same network over registers and
// lanes).  Gradients are bit-reproducible.
// A row with more than 256 entries (a hub: tens of thousands of destinations can sample the same
// vertex) is left to the workgroups behind the launch's own (blockIdx.x >= n_main), which walk the
// list of such rows that the sampler made: codes sorted in LDS (bitonic, up to PULL_LONG_CAP at a
// time: a longer row in windows of ascending values), the four waves sum a quarter of the sorted
// window each, partial sums added in wave order, windows in ascending order.
constexpr int PULL_LONG_CAP = 2048;
constexpr int PULL_LONG_BLOCKS = 1024;

// workgroups of 256 threads of a kernel that one compute unit holds at once (asked once per kernel)
template <class K>
int resident_blocks(K kernel) {
    static const int blocks = [kernel] {
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kernel, 256, 0) != hipSuccess || nb < 1) nb = 4;
        return std::min(nb, 8);
    }();
    return blocks;
}

// Bitonic sort across a wave, ascending, of the first p2 lanes' values (p2 a power of two; the lanes
// behind hold INT_MAX padding and stay where they are): log2(p2) * (log2(p2) + 1) / 2 exchange steps, so
// the common rows with two or three entries cost one or three shuffles, not the 21 of a full wave.
__device__ __forceinline__ int wave_sort_ascending(int v, int p2) {
    const int lane = threadIdx.x & 63;
    for (int k = 2; k <= p2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            const int o = __shfl_xor(v, j);
            v = (((lane & j) == 0) == ((lane & k) == 0)) ? min(v, o) : max(v, o);
        }
    }
    return v;
}

// The same for 256 values, four per lane: element r * 64 + lane lives in v[r].  Exchanges at a distance
// of 64 or 128 elements are between registers of one lane, the others between lanes.
__device__ __forceinline__ void wave_sort4_ascending(int (&v)[4]) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 2; k <= 256; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            if (j >= 64) {
                const int jr = j >> 6;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if ((r & jr) == 0) {
                        const bool asc = ((r * 64 + lane) & k) == 0;
                        const int a = v[r], b = v[r | jr];
                        if ((a > b) == asc) { v[r] = b; v[r | jr] = a; }
                    }
                }
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int o = __shfl_xor(v[r], j);
                    const bool asc = ((r * 64 + lane) & k) == 0;
                    v[r] = (((lane & j) == 0) == asc) ? min(v[r], o) : max(v[r], o);
                }
            }
        }
    }
}

template <bool HACT_H>
__device__ __forceinline__ float4 load_act4(const void *__restrict__ hact, int64_t idx) {
    if (HACT_H) {
        const uint2 raw = reinterpret_cast<const uint2 *>(hact)[idx];
        return make_float4(bf2f(raw.x & 0xFFFFu), bf2f(raw.x >> 16), bf2f(raw.y & 0xFFFFu), bf2f(raw.y >> 16));
    }
    return reinterpret_cast<const float4 *>(hact)[idx];
}

template <bool OUT_H>
__device__ __forceinline__ void store_masked4(void *__restrict__ gout, int64_t idx, float4 acc, float4 h) {
    acc.x = h.x > 0.f ? acc.x : 0.f; acc.y = h.y > 0.f ? acc.y : 0.f;
    acc.z = h.z > 0.f ? acc.z : 0.f; acc.w = h.w > 0.f ? acc.w : 0.f;
    // bf16 storage: dZ is kept as the bf16 value that both backward products consume
    if (OUT_H)
        reinterpret_cast<uint2 *>(gout)[idx] = make_uint2((uint32_t)f2bf(acc.x) | ((uint32_t)f2bf(acc.y) << 16),
                                                          (uint32_t)f2bf(acc.z) | ((uint32_t)f2bf(acc.w) << 16));
    else
        reinterpret_cast<float4 *>(gout)[idx] = acc;
}

__device__ __forceinline__ void add4(float4 &a, const float4 &b) { a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w; }

template <int LPR, bool HACT_H, bool OUT_H = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(OUT_H ? 8 : 4, 8))) void k_pull_input_grad(const float *__restrict__ gin, int D,
                                                         const int32_t *__restrict__ rev_ptr,
                                                         const int32_t *__restrict__ rev_cnt,
                                                         const int32_t *__restrict__ rev_list,
                                                         const int32_t *__restrict__ rev_long,
                                                         const void *__restrict__ hact,
                                                         const GsLevelMeta *__restrict__ meta_lo, int S,
                                                         void *__restrict__ gout, int n_main) {
    const int n_lo = meta_lo->front_off[S];
    const int nvec = D >> 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float4 *G4 = reinterpret_cast<const float4 *>(gin);
    if ((int)blockIdx.x >= n_main) {
        // ---- long rows: one workgroup per row
        __shared__ int s_code[PULL_LONG_CAP];
        __shared__ float4 s_part[4][64];
        __shared__ int s_cnt;
        const int n_long = meta_lo->n_long;
        for (int i = (int)blockIdx.x - n_main; i < n_long; i += (int)gridDim.x - n_main) {
            const int u = rev_long[i];
            const int n = rev_cnt[u], e0 = rev_ptr[u];
            for (int cb = 0; cb < nvec; cb += 64) {
                const int c = cb + lane;
                const bool cv = c < nvec;
                const float4 h = cv ? load_act4<HACT_H>(hact, (int64_t)u * nvec + c) : make_float4(0.f, 0.f, 0.f, 0.f);
                float4 total = make_float4(0.f, 0.f, 0.f, 0.f);
                // A row of at most PULL_LONG_CAP entries is one window.  A longer one is taken in windows of
                // values (lo, T]: the codes of a row are distinct, so the largest T with at most
                // PULL_LONG_CAP codes inside (found by bisection over the values, one counting pass over
                // the row per step) yields the next PULL_LONG_CAP codes in ascending order whatever
                // order the row was filled in.
                int lo = -1;
                for (int taken = 0; taken < n;) {
                    int T = 0x7FFFFFFE;
                    if (n > PULL_LONG_CAP) {
                        int a = lo + 1, b = 0x7FFFFFFE;
                        while (a < b) {
                            const int mid = a + ((b - a + 1) >> 1);
                            __syncthreads();
                            if (threadIdx.x == 0) s_cnt = 0;
                            __syncthreads();
                            int cnt = 0;
                            for (int t = threadIdx.x; t < n; t += 256) {
                                const int code = rev_list[e0 + t];
                                cnt += (code > lo && code <= mid) ? 1 : 0;
                            }
                            for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o);
                            if (lane == 0 && cnt) atomicAdd(&s_cnt, cnt);
                            __syncthreads();
                            if (s_cnt <= PULL_LONG_CAP) a = mid; else b = mid - 1;
                        }
                        T = a;
                    }
                    __syncthreads();
                    if (threadIdx.x == 0) s_cnt = 0;
                    __syncthreads();
                    if (n > PULL_LONG_CAP) {
                        for (int t = threadIdx.x; t < n; t += 256) {
                            const int code = rev_list[e0 + t];
                            if (code > lo && code <= T) {
                                const int at = atomicAdd(&s_cnt, 1);
                                if (at < PULL_LONG_CAP) s_code[at] = code;
                            }
                        }
                    } else {
                        for (int t = threadIdx.x; t < n; t += 256) s_code[t] = rev_list[e0 + t];
                        if (threadIdx.x == 0) s_cnt = n;
                    }
                    __syncthreads();
                    const int m = min(s_cnt, PULL_LONG_CAP);
                    int p2 = 64;
                    while (p2 < m) p2 <<= 1;
                    for (int t = m + threadIdx.x; t < p2; t += 256) s_code[t] = 0x7FFFFFFF;
                    __syncthreads();
                    lo = T;
                    taken += max(m, 1);         // (a window is never empty; the loop ends whatever the row holds)
                    for (int k = 2; k <= p2; k <<= 1) {
                        for (int j = k >> 1; j > 0; j >>= 1) {
                            for (int t = threadIdx.x; t < (p2 >> 1); t += 256) {
                                const int ia = ((t & ~(j - 1)) << 1) | (t & (j - 1)), ib = ia | j;
                                const int x = s_code[ia], y = s_code[ib];
                                const bool asc = (ia & k) == 0;
                                if ((x > y) == asc) { s_code[ia] = y; s_code[ib] = x; }
                            }
                            __syncthreads();
                        }
                    }
                    // the four waves sum a quarter of the sorted codes each, eight gradient rows in flight
                    const int q = (m + 3) >> 2;
                    const int jb = wave * q, je = min(m, jb + q);
                    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
                    for (int j = jb; j < je; j += 8) {
                        float4 v[8];
#pragma unroll
                        for (int x = 0; x < 8; ++x) {
                            const int code = s_code[min(j + x, je - 1)];
                            v[x] = cv ? G4[(int64_t)(code >> 1) * 2 * nvec + (code & 1) * nvec + c] : make_float4(0.f, 0.f, 0.f, 0.f);
                        }
#pragma unroll
                        for (int x = 0; x < 8; ++x)
                            if (j + x < je) add4(acc, v[x]);
                    }
                    s_part[wave][lane] = acc;
                    __syncthreads();
                    if (wave == 0) {
                        float4 t = s_part[0][lane];
                        add4(t, s_part[1][lane]); add4(t, s_part[2][lane]); add4(t, s_part[3][lane]);
                        add4(total, t);
                    }
                }
                if (wave == 0 && cv) store_masked4<OUT_H>(gout, (int64_t)u * nvec + c, total, h);
            }
        }
        return;
    }
    constexpr int G = 64 / LPR;                 // lane groups of a wave: entries summed side by side
    const int sub = lane / LPR, c0 = lane % LPR;
    const int waves = (n_main * (int)blockDim.x) >> 6;
    const int n_c = (nvec + LPR - 1) / LPR;      // column rounds, the same for every lane
    // A row is a chain of three dependent accesses (segment -> codes -> gradient rows), and with one
    // row per wave at a time the kernel runs at the rate of that chain, not of the memory.  So a wave
    // looks two rows ahead: while it sums row u it already holds the codes of its next row and the
    // segment of the one after, and only the gradient rows themselves are waited for.
    const int u_first = (int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    int n_a = 0, e_a = 0, n_b = 0, e_b = 0, code_a = 0x7FFFFFFF;
    if (u_first < n_lo) { n_a = rev_cnt[u_first]; e_a = rev_ptr[u_first]; }
    if (u_first + waves < n_lo) { n_b = rev_cnt[u_first + waves]; e_b = rev_ptr[u_first + waves]; }
    if (lane < min(n_a, 64)) code_a = rev_list[e_a + lane];
    for (int u = u_first; u < n_lo; u += waves) {
        int n_c2 = 0, e_c2 = 0, code_b = 0x7FFFFFFF;
        if (u + 2 * waves < n_lo) { n_c2 = rev_cnt[u + 2 * waves]; e_c2 = rev_ptr[u + 2 * waves]; }
        if (u + waves < n_lo && lane < min(n_b, 64)) code_b = rev_list[e_b + lane];
        const int n = n_a, e0 = e_a;
        int v4[4];
        v4[0] = code_a;
        n_a = n_b; e_a = e_b; n_b = n_c2; e_b = e_c2; code_a = code_b;
        if (n > GS_REV_LONG) continue;          // a workgroup behind the launch's own takes it
        // the row's codes in registers, sorted: entry j of the sorted list is v[j / 64] of lane j % 64
        const int n_reg = (n + 63) >> 6;          // registers in use (uniform)
        if (n <= 64) {
            if (n > 1) {
                int p2 = 2;
                while (p2 < n) p2 <<= 1;
                v4[0] = wave_sort_ascending(v4[0], p2);
            }
        } else {
#pragma unroll
            for (int r = 1; r < 4; ++r) v4[r] = r * 64 + lane < n ? rev_list[e0 + r * 64 + lane] : 0x7FFFFFFF;
            wave_sort4_ascending(v4);
        }
        for (int ci = 0; ci < n_c; ++ci) {
            const int c = c0 + ci * LPR;
            const bool cv = c < nvec;
            // the activation that gates the result does not depend on the sum: fetched first, it
            // travels while the gradient rows are fetched
            const float4 h = cv ? load_act4<HACT_H>(hact, (int64_t)u * nvec + c) : make_float4(0.f, 0.f, 0.f, 0.f);
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (r >= n_reg) break;
                const int code = v4[r];
                const int m = min(64, n - r * 64);
                for (int j0 = 0; j0 < m; j0 += 4 * G) {
                    float4 v[4];
                    bool have[4];
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const int j = j0 + x * G + sub;
                        const int k = __shfl(code, j < 64 ? j : 63);
                        have[x] = j < m && cv;
                        v[x] = have[x] ? G4[(int64_t)(k >> 1) * 2 * nvec + (k & 1) * nvec + c] : make_float4(0.f, 0.f, 0.f, 0.f);
                    }
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        if (have[x]) add4(acc, v[x]);
                }
            }
            // the lane groups' partial sums, added in a fixed tree
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) {
                acc.x += __shfl_xor(acc.x, o); acc.y += __shfl_xor(acc.y, o);
                acc.z += __shfl_xor(acc.z, o); acc.w += __shfl_xor(acc.w, o);
            }
            if (sub == 0 && cv) store_masked4<OUT_H>(gout, (int64_t)u * nvec + c, acc, h);
        }
    }
}

// widths that are not a multiple of 4: one wave per row, one float per lane; entries in ascending
// code order when the row has at most 64 of them (longer rows of such a model: in list order, i.e.
// not reproducibly in the last bits)
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
        const int e0 = rev_ptr[u], n = rev_cnt[u];
        int code = lane < n ? rev_list[e0 + lane] : 0x7FFFFFFF;
        if (n > 1 && n <= 64) {
            int p2 = 2;
            while (p2 < n) p2 <<= 1;
            code = wave_sort_ascending(code, p2);
        }
        const int n_c = (D + 63) >> 6;
        for (int ci = 0; ci < n_c; ++ci) {
            const int c = lane + 64 * ci;
            float acc = 0.f;
            if (n <= 64) {
                for (int j = 0; j < n; ++j) {
                    const int k = __shfl(code, j);
                    if (c < D) acc += gin[(int64_t)(k >> 1) * 2 * D + (k & 1) * D + c];
                }
            } else if (c < D) {
                for (int e = e0; e < e0 + n; ++e) {
                    const int k = rev_list[e];
                    acc += gin[(int64_t)(k >> 1) * 2 * D + (k & 1) * D + c];
                }
            }
            if (c < D) gout[(int64_t)u * D + c] = hact[(int64_t)u * D + c] > 0.f ? acc : 0.f;
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

// ------------------------------------------------------------------------------------------
// The top layer of a training step in one launch.  Its products are tiny (n_targets x 2 D x classes:
// 49 MFLOP each for 1024 targets, 512 inputs, 47 classes) and as separate launches the chain
//   input assembly -> forward product -> loss -> weight-gradient product -> input-gradient product
// is five kernel boundaries around a few microseconds of work.  Here a workgroup takes TOP_R
// destination rows at a time through all of it: the assembled rows [H_self | mean] and dZ stay in LDS, the
// stacked weights (at most 2 D x 64 floats) are read from the L2 by every workgroup, the
// weight-gradient partial of the workgroup goes to its own slab (summed in slab order by
// k_reduce_grads: deterministic, no atomics).  Plain FMAs: at these sizes the matrix cores would
// idle on the launch edges anyway.
// ------------------------------------------------------------------------------------------
// Destination rows a workgroup takes per round.  The kernel's arithmetic is bound by the FMA rate of
// the compute units it occupies, so fewer rows per workgroup (more workgroups) shorten it, while
// every workgroup costs one weight-gradient slab that k_reduce_grads has to read: measured on 1024
// targets x 512 x 47, kernel + reduction 16 rows 40 + 9 us, 8 rows 25 + 10 us, 4 rows 22 + 14 us.
constexpr int TOP_ROWS = 8;
constexpr int TOP_NMAX = 64;       // classes the kernel takes (one lane per class)
constexpr int TOP_DMAX = 384;      // input width it takes (TOP_R x 2 D floats of LDS)

struct TopArgs {
    const float *H; int D; int N; int Npad;
    const int32_t *blk_indptr; const int32_t *edge_row; const int32_t *self_row;
    const float *W; const float *bias;
    const int64_t *labels; const int32_t *front_top;
    float *logits; float *row_loss;
    float *gin; float *part;
    const GsLevelMeta *meta_up; int S;
};

constexpr int TOP_W = 8;           // waves of a workgroup
constexpr int TOP_T = 64 * TOP_W;

// LDS of the kernel in 4-byte words: rows, per-wave partial logits, dZ, edge rows, per-row scalars
__host__ __device__ inline size_t top_lds_words(int D, int R) {
    return (size_t)R * 2 * D + (size_t)TOP_W * R * 64 + (size_t)R * 64 + (size_t)R * 64 + 4 * R;
}

template <int TOP_R>
__global__ __launch_bounds__(TOP_T) void k_sage_top_fused(TopArgs a) {
    extern __shared__ __attribute__((aligned(16))) float s_mem[];
    const int D = a.D, N = a.N, Npad = a.Npad, D2 = 2 * D, nvec = D >> 2;
    float *s_x = s_mem;                                         // [TOP_R][2 D]
    float *s_p = s_x + (size_t)TOP_R * D2;                      // [TOP_W][TOP_R][64]
    float *s_dz = s_p + TOP_W * TOP_R * 64;                     // [TOP_R][64]
    int *s_e = reinterpret_cast<int *>(s_dz + TOP_R * 64);      // [TOP_R][64]
    int *s_e0 = s_e + TOP_R * 64, *s_m = s_e0 + TOP_R, *s_self = s_m + TOP_R;
    float *s_inv = reinterpret_cast<float *>(s_self + TOP_R);
    const int n1 = a.meta_up->front_off[a.S];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float4 *H4 = reinterpret_cast<const float4 *>(a.H);
    const float inv_n = n1 > 0 ? 1.f / (float)n1 : 0.f;
    float *slab = a.part + (int64_t)blockIdx.x * (D2 + 1) * N;
    // Every phase is one or two round trips to memory for the whole workgroup: what a thread needs is
    // fetched with independent loads, never one after the other.
    int round = 0;
    for (int r0 = blockIdx.x * TOP_R; round == 0 || r0 < n1; r0 += gridDim.x * TOP_R, ++round) {
        const int rows = max(0, min(TOP_R, n1 - r0));
        __syncthreads();                           // the previous round has finished with the LDS
        // (1) layer input: own lower-layer row | mean over the sampled sources, edges in slot order
        if ((int)threadIdx.x < rows) {
            const int row = r0 + threadIdx.x;
            const int e0 = a.blk_indptr[row], m = min(64, a.blk_indptr[row + 1] - e0);
            s_e0[threadIdx.x] = e0; s_m[threadIdx.x] = m; s_self[threadIdx.x] = a.self_row[row];
            s_inv[threadIdx.x] = m > 0 ? 1.f / (float)m : 0.f;
        }
        __syncthreads();
        for (int idx = threadIdx.x; idx < TOP_R * 64; idx += TOP_T) {
            const int r = idx >> 6, e = idx & 63;
            if (r < rows && e < s_m[r]) s_e[idx] = a.edge_row[s_e0[r] + e];
        }
        __syncthreads();
        for (int r = wave; r < rows; r += TOP_W) {
            const int m = s_m[r];
            const int64_t self = s_self[r];
            for (int c = lane; c < nvec; c += 64) {
                const float4 own = H4[self * nvec + c];
                float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
                for (int e = 0; e < m; e += 8) {
                    float4 v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = H4[(int64_t)(e + u < m ? s_e[r * 64 + e + u] : (int)self) * nvec + c];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (e + u < m) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
                }
                if (m > 0) { const float cnt = (float)m; acc.x /= cnt; acc.y /= cnt; acc.z /= cnt; acc.w /= cnt; }
                float4 *x4 = reinterpret_cast<float4 *>(s_x + (size_t)r * D2);
                x4[c] = own;
                x4[nvec + c] = acc;
            }
        }
        __syncthreads();
        // (2) logits: the contraction is dealt to the waves (2 D / 8 inputs each, lane = class); the
        // partial sums meet in LDS and are added in wave order
        {
            float acc[TOP_R];
#pragma unroll
            for (int r = 0; r < TOP_R; ++r) acc[r] = 0.f;
            const int per = ((D2 / TOP_W + 3) >> 2) << 2;      // a multiple of 4: 16-byte aligned LDS reads below
            const int nn = lane < Npad ? lane : 0;
            const float *wcol = a.W + nn;
            const int kend = min(D2, (wave + 1) * per);
            for (int k0 = wave * per; k0 < kend; k0 += 32) {
                float w[32];
#pragma unroll
                for (int u = 0; u < 32; ++u) w[u] = wcol[(int64_t)(k0 + u < kend ? k0 + u : k0) * Npad];
                // (the rows are read from LDS four inputs at a time: one LDS instruction per four FMAs)
#pragma unroll
                for (int u = 0; u < 32; u += 4) {
                    if (k0 + u + 3 < kend) {
#pragma unroll
                        for (int r = 0; r < TOP_R; ++r) {
                            const float4 x = *reinterpret_cast<const float4 *>(s_x + (size_t)r * D2 + k0 + u);
                            acc[r] += x.x * w[u] + x.y * w[u + 1] + x.z * w[u + 2] + x.w * w[u + 3];
                        }
                    }       // (k0, kend and 2 D are multiples of 4: there are no partial groups)
                }
            }
#pragma unroll
            for (int r = 0; r < TOP_R; ++r) s_p[(wave * TOP_R + r) * 64 + lane] = acc[r];
        }
        __syncthreads();
        for (int r = wave; r < TOP_R; r += TOP_W) {
            const bool live = r < rows;
            float zsum = lane < N ? a.bias[lane] : 0.f;
            if (live) {
#pragma unroll
                for (int w = 0; w < TOP_W; ++w) zsum += s_p[(w * TOP_R + r) * 64 + lane];
            }
            const float z = (live && lane < N) ? zsum : -3.4e38f;
            float mx = z;
            for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
            const float e = (live && lane < N) ? __expf(z - mx) : 0.f;
            float sum = e;
            for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
            float dz = 0.f;
            if (live) {
                const int row = r0 + r;
                const int y = (int)a.labels[a.front_top[row]];
                if (lane < N) {
                    a.logits[(int64_t)row * N + lane] = z;
                    dz = (e / sum - (lane == y ? 1.f : 0.f)) * inv_n;
                }
                const float zy = __shfl(z, (y >= 0 && y < N) ? y : 0);
                if (lane == 0 && a.row_loss) a.row_loss[row] = (y >= 0 && y < N) ? (logf(sum) + mx - zy) : 0.f;
            }
            s_dz[r * 64 + lane] = dz;
        }
        __syncthreads();
        // (3a) input gradients of the rows: [dH_self | dMean / cnt] = dZ W^T, one input k per thread
        for (int k = threadIdx.x; k < D2; k += TOP_T) {
            float w[TOP_NMAX];
            const float4 *w4 = reinterpret_cast<const float4 *>(a.W + (int64_t)k * Npad);
#pragma unroll
            for (int q = 0; q < TOP_NMAX / 4; ++q) {
                const float4 v = 4 * q < Npad ? w4[q] : make_float4(0.f, 0.f, 0.f, 0.f);
                w[4 * q] = v.x; w[4 * q + 1] = v.y; w[4 * q + 2] = v.z; w[4 * q + 3] = v.w;
            }
            for (int r = 0; r < rows; ++r) {
                float sacc = 0.f;
#pragma unroll
                for (int n = 0; n < TOP_NMAX; n += 4) {
                    const float4 d = *reinterpret_cast<const float4 *>(s_dz + r * 64 + n);
                    sacc += d.x * w[n] + d.y * w[n + 1] + d.z * w[n + 2] + d.w * w[n + 3];
                }
                a.gin[(int64_t)(r0 + r) * D2 + k] = k < D ? sacc : sacc * s_inv[r];
            }
        }
        // (3b) this workgroup's share of X^T dZ and of the column sums of dZ, into its slab
        if (lane < N) {
            float dzr[TOP_R];
#pragma unroll
            for (int r = 0; r < TOP_R; ++r) dzr[r] = r < rows ? s_dz[r * 64 + lane] : 0.f;
            // four inputs per thread and step, read from LDS with one instruction per row
            for (int k = 4 * wave; k < D2; k += 4 * TOP_W) {
                float4 sacc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int r = 0; r < TOP_R; ++r) {
                    if (r < rows) {
                        const float4 x = *reinterpret_cast<const float4 *>(s_x + (size_t)r * D2 + k);
                        sacc.x += x.x * dzr[r]; sacc.y += x.y * dzr[r]; sacc.z += x.z * dzr[r]; sacc.w += x.w * dzr[r];
                    }
                }
                float *dst = slab + (int64_t)k * N + lane;
                if (round == 0) { dst[0] = sacc.x; dst[N] = sacc.y; dst[2 * N] = sacc.z; dst[3 * N] = sacc.w; }
                else { dst[0] += sacc.x; dst[N] += sacc.y; dst[2 * N] += sacc.z; dst[3 * N] += sacc.w; }
            }
            if (wave == 0) {                       // column sums of dZ: the bias gradient
                float sacc = 0.f;
#pragma unroll
                for (int r = 0; r < TOP_R; ++r) sacc += dzr[r];
                float *dst = slab + (int64_t)D2 * N + lane;
                *dst = round == 0 ? sacc : *dst + sacc;
            }
        }
    }
}

#include "sage_bf16.h"
#include "gemm_bf16_rows.h"

// The streaming bf16 row-block kernel takes a product when the contraction is 256 or 512, the output
// rows are whole 16-byte granules and the level is large enough (by its bound) to fill the chip.
constexpr int64_t RB_MIN_ROWS = 32768;
constexpr int RB_FWD_STAGES = 4;        // (six stages fit beside the forward product's bf16 patch and measured the same: 197 against 198 us)
bool rows_gemm_fits(int64_t ub_rows, int K, int NB, int granule) {
    return (K == 256 || K == 512) && NB % granule == 0 && ub_rows >= RB_MIN_ROWS;
}
// weight gradients of layer l through the streaming kernel: dZ held in bf16 (a level below the top
// one whose width allows 16-byte rows), whole 16-byte column groups, a level that fills the chip
bool grad_w_streams(const gsplit_sage_params *p, int l, int L, int64_t ub_rows) {
    const int D = p->dims[l], N = p->dims[l + 1];
    return p->dtype == GSPLIT_BF16 && l < L - 1 && N % 8 == 0 && N >= 128 && (2 * D) % 8 == 0 && 2 * D >= 128 &&
           ub_rows >= RB_MIN_ROWS;
}
// one workgroup per compute unit, a multiple of (8 XCDs x column blocks)
unsigned rows_gemm_grid(const gsplit_ctx *ctx, int NB, int BN) {
    const int nb = (NB + BN - 1) / BN;
    return (unsigned)(std::max(1, ctx->n_cu / (8 * nb)) * 8 * nb);
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
        if (p->dtype == GSPLIT_F32) {
            const int64_t np = (p->dims[l + 1] + 3) & ~3;
            rc = gs_alloc(ctx, (void **)&sb.wstack32[l], sizeof(float) * 2 * p->dims[l] * np, "stacked weights");
        } else {
            const int64_t np = (p->dims[l + 1] + 7) & ~7;
            rc = gs_alloc(ctx, (void **)&sb.wstack[l], 2 * (size_t)(2 * p->dims[l]) * np, "bf16 weights");
            if (rc) return rc;
            rc = gs_alloc(ctx, (void **)&sb.wtrans[l], 2 * (size_t)p->dims[l + 1] * 2 * p->dims[l], "bf16 weights^T");
        }
        if (rc) return rc;
        rc = gs_alloc(ctx, (void **)&sb.inv_cnt[l], sizeof(float) * (ctx->ub_front[l + 1] + RB_BM), "inverse counts");
        if (rc) return rc;
    }
    for (int l = 0; l < L; ++l) {
        // split-K geometry of the weight-gradient product: about as many workgroups as the chip
        // holds at once (three per compute unit); how many of the chunks are used is decided on
        // the device from the actual row count
        const int m_rows = 2 * p->dims[l] + (p->dtype == GSPLIT_BF16 ? 1 : 0);    // bf16: plus the row of ones
        const int tiles = (int)(gs_ceil_div(m_rows, TileMid::BM) * gs_ceil_div(p->dims[l + 1], TileMid::BN));
        int64_t chunks = gs_ceil_div(std::max<int64_t>(8, (int64_t)ctx->n_cu * 3 / tiles), 8) * 8;
        sb.nchunk[l] = (int)chunks;
        // a bf16 level below the top one that can reach GWH_MIN_ROWS rows: when it does (decided on the
        // device), one workgroup per compute unit forms a whole 256 x 256 block over its chunk of rows
        if (l == 0) {
            sb.stream_rows = GWH_MIN_ROWS;
            if (const char *e = std::getenv("GSPLIT_GRADW_STREAM_ROWS")) {
                const long v = std::strtol(e, nullptr, 10);
                if (v >= 64 && v <= (1l << 30)) sb.stream_rows = (int)v;
            }
        }
        sb.gw_stream[l] = grad_w_streams(p, l, L, ctx->ub_front[l + 1]);
        sb.stream_nchunk[l] = 0;
        if (sb.gw_stream[l]) {
            const int big = (int)(gs_ceil_div(2 * p->dims[l], GWH_B) * gs_ceil_div(p->dims[l + 1], GWH_B));
            sb.stream_nchunk[l] = std::max(8, ctx->n_cu / big / 8 * 8);
            chunks = std::max<int64_t>(chunks, sb.stream_nchunk[l]);
        }
        // the fused top-layer kernel writes one slab per workgroup: TOP_R rows each, at most 256 of them
        int64_t slabs = chunks;
        if (l == L - 1) {
            sb.top_chunks = (int)std::min<int64_t>(256, std::max<int64_t>(32, gs_ceil_div(ctx->ub_front[L], TOP_ROWS)));
            slabs = std::max<int64_t>(slabs, sb.top_chunks);
        }
        int rc = gs_alloc(ctx, (void **)&sb.gw_part[l],
                          sizeof(float) * slabs * (2 * p->dims[l] + 1) * p->dims[l + 1], "weight-gradient partials");
        if (rc) return rc;
    }
    {
        int rc = gs_alloc(ctx, (void **)&sb.glog, sizeof(float) * ctx->ub_front[L] * p->dims[L], "loss gradient");
        if (rc) return rc;
    }
    int64_t gtmp_words = 1;
    for (int l = 1; l < L; ++l) gtmp_words = std::max<int64_t>(gtmp_words, ctx->ub_front[l + 1] * 2 * p->dims[l]);
    {
        int rc = gs_alloc(ctx, (void **)&sb.gtmp, sizeof(float) * gtmp_words, "input gradients");
        if (rc) return rc;
    }
    // the fused top-layer kernel takes up to 89 KiB of dynamic LDS (a gfx950 workgroup may use all 160 KiB)
    GS_HIP(ctx, hipFuncSetAttribute((const void *)k_sage_top_fused<TOP_ROWS>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)(sizeof(float) * top_lds_words(TOP_DMAX, TOP_ROWS))));
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

// ---- tile choice and launches of the fp32 products ------------------------------------------
// The tile is chosen from what the host knows: the upper bound on the rows, the output width and
// the length of the contraction.  The middle tile serves products with enough rows to fill the
// chip; when even the upper bound gives at most about one workgroup per compute unit, the low
// tiles with their k split give more and shorter workgroups (a long contraction walked by few
// workgroups is a chain of dependent k-tiles, not a throughput problem).  Operands that cannot be
// read in 16-byte pieces take the middle tile with scalar loads.
template <class T, int VA, int VB>
void launch_fwd_t(gsplit_ctx *ctx, hipStream_t st, int64_t ub, const MatRows &a, const MatRows &b, const EpiFwd &epi,
                  const GsLevelMeta *mu) {
    hipLaunchKernelGGL((k_sage_linear_fwd<T, VA, VB>), dim3(row_block_grid<T>(ctx, ub, b.cols)), dim3(GNT), 0, st, a, b,
                       epi, mu, ctx->S);
}
// b: stacked weights, always readable in 16-byte pieces
void launch_fwd(gsplit_ctx *ctx, hipStream_t st, int64_t ub, bool va, const MatRows &a, const MatRows &b,
                const EpiFwd &epi, const GsLevelMeta *mu) {
    if (!va) launch_fwd_t<TileMid, 1, 4>(ctx, st, ub, a, b, epi, mu);
    else if (!few_rows(ub, epi.N, a.cols)) launch_fwd_t<TileMidLean, 4, 4>(ctx, st, ub, a, b, epi, mu);
    else if (epi.N <= 64) launch_fwd_t<TileLowNarrow, 4, 4>(ctx, st, ub, a, b, epi, mu);
    else launch_fwd_t<TileLow, 4, 4>(ctx, st, ub, a, b, epi, mu);
}

template <class T, int VA, int VB>
void launch_grad_in_t(gsplit_ctx *ctx, hipStream_t st, int64_t ub, const MatRows &dz, const MatRows &w,
                      const EpiGradIn &epi, const GsLevelMeta *mu) {
    hipLaunchKernelGGL((k_sage_grad_in<T, VA, VB>), dim3(row_block_grid<T>(ctx, ub, w.rows)), dim3(GNT), 0, st, dz, w,
                       epi, mu, ctx->S);
}
void launch_grad_in(gsplit_ctx *ctx, hipStream_t st, int64_t ub, bool vdz, const MatRows &dz, const MatRows &w,
                    const EpiGradIn &epi, const GsLevelMeta *mu) {
    const bool few = few_rows(ub, w.rows, dz.cols);
    if (!vdz) {
        if (few) launch_grad_in_t<TileLow, 1, 4>(ctx, st, ub, dz, w, epi, mu);
        else launch_grad_in_t<TileMid, 1, 4>(ctx, st, ub, dz, w, epi, mu);
    } else if (!few) launch_grad_in_t<TileMidDirect, 4, 4>(ctx, st, ub, dz, w, epi, mu);
    else if (w.rows <= 64) launch_grad_in_t<TileLowNarrow, 4, 4>(ctx, st, ub, dz, w, epi, mu);
    else launch_grad_in_t<TileLow, 4, 4>(ctx, st, ub, dz, w, epi, mu);
}

// ws (may be NULL): weights to stack behind the assembly's own workgroups.  Returns false if they
// were not stacked (the scalar variant does not carry them).
bool launch_assemble(gsplit_ctx *ctx, int l, const float *hin, int D, hipStream_t st, const WeightStack *ws,
                     int64_t stack_words) {
    const GsLayerBuf &B = ctx->layer[l];
    const GsLevelMeta *mu = ctx->d_meta + (l + 1);
    float *X = (float *)ctx->sage.xin[l];
    const int64_t ub = ctx->ub_front[l + 1];
    GsTimeScope ts(ctx, "assemble_input", l, st);
    if (D % 4 != 0 || !aligned16(hin)) {
        hipLaunchKernelGGL(k_assemble_input_f32_any, dim3(grid_1d(ctx, ub * 64)), dim3(256), 0, st, hin, D,
                           B.blk_indptr, B.edge_row, B.self_row, mu, ctx->S, X, ctx->sage.inv_cnt[l]);
        return false;
    }
    const int nvec = D / 4;
    const int n_stack = ws ? (int)std::min<int64_t>(128, gs_ceil_div(stack_words, 256)) : 0;
    const WeightStack none{};
    const WeightStack &w = ws ? *ws : none;
    const int extra = n_stack * ctx->L;
#define GS_ASSEMBLE(LPR)                                                                                     \
    do {                                                                                                     \
        const int n_main = grid_1d(ctx, ub * LPR);                                                           \
        hipLaunchKernelGGL(k_assemble_input_f32<LPR>, dim3(n_main + extra), dim3(256), 0, st, hin, D,        \
                           B.blk_indptr, B.edge_row, B.self_row, mu, ctx->S, ctx->fan[l], X,                 \
                           ctx->sage.inv_cnt[l], n_main, w, n_stack);                                        \
    } while (0)
    if (nvec <= 16) GS_ASSEMBLE(16);
    else if (nvec <= 32) GS_ASSEMBLE(32);
    else GS_ASSEMBLE(64);
#undef GS_ASSEMBLE
    return ws != nullptr;
}

}  // namespace

namespace {

// forward layers 0 .. l_end - 1 (l_end = L: the whole pass, logits included)
int sage_forward(gsplit_ctx *ctx, const gsplit_sage_params *p, const void *d_feat_local, float *d_logits,
                 hipStream_t st, int l_end) {
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
        for (int l = 0; l < l_end; ++l) {
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
            GsTimeScope ts(ctx, "linear_fwd", l, st);
            if (l < L - 1 && rows_gemm_fits(ub, 2 * D, N, 8)) {
                RbEpi re{sb.hidden[l + 1], N, (const float *)p->d_bias[l], nullptr, 0, 1};
                if (2 * D == 256)
                    hipLaunchKernelGGL((k_rows_gemm_hb<16, false, RB_FWD_STAGES>), dim3(rows_gemm_grid(ctx, N, 256)), dim3(GNT), 0, st,
                                       x.p, wt.p, N, re, mu, S);
                else
                    hipLaunchKernelGGL((k_rows_gemm_hb<32, false, RB_FWD_STAGES>), dim3(rows_gemm_grid(ctx, N, 128)), dim3(GNT), 0, st,
                                       x.p, wt.p, N, re, mu, S);
            } else {
                dim3 grid(row_block_grid<TileMid>(ctx, ub, N));
                hipLaunchKernelGGL(k_sage_linear_fwd_h, grid, dim3(GNT), 0, st, x, wt, epi, mu, S);
            }
        }
        GS_HIP(ctx, hipGetLastError());
        sb.fwd_done = l_end == L;
        sb.fwd_batch = ctx->batch_id;
        return GSPLIT_OK;
    }
    WeightStack ws{};
    int64_t stack_words = 1;
    {
        int64_t wmax = 1;
        for (int l = 0; l < L; ++l) {
            ws.ws[l] = (const float *)p->d_w_self[l]; ws.wn[l] = (const float *)p->d_w_neigh[l];
            ws.stacked[l] = sb.wstack32[l]; ws.D[l] = p->dims[l]; ws.N[l] = p->dims[l + 1];
            wmax = std::max<int64_t>(wmax, (int64_t)2 * p->dims[l] * ((p->dims[l + 1] + 3) & ~3));
        }
        stack_words = wmax;
    }
    for (int l = 0; l < l_end; ++l) {
        const int D = p->dims[l], N = p->dims[l + 1];
        const float *hin = l == 0 ? (const float *)d_feat_local : (const float *)sb.hidden[l];
        float *hout = l == L - 1 ? d_logits : (float *)sb.hidden[l + 1];
        const GsLevelMeta *mu = ctx->d_meta + (l + 1);
        // the stacked weights are first needed by the bottom layer's product: the bottom layer's
        // input assembly carries the stacking; if it cannot, a launch of its own does it
        const bool stacked = launch_assemble(ctx, l, hin, D, st, l == 0 ? &ws : nullptr, stack_words);
        if (l == 0 && !stacked) {
            GsTimeScope ts(ctx, "stack_weights", -1, st);
            hipLaunchKernelGGL(k_stack_weights, dim3((unsigned)std::min<int64_t>(128, gs_ceil_div(stack_words, 256)), L),
                               dim3(256), 0, st, ws);
        }
        MatRows a{(const float *)sb.xin[l], 0, 2 * D};
        MatRows b{sb.wstack32[l], 2 * D, (N + 3) & ~3};
        EpiFwd epi{hout, (const float *)p->d_bias[l], N, 0, l < L - 1 ? 1 : 0};
        const bool va = D % 2 == 0;   // rows of the assembled input are 2 * D floats: 16-byte aligned
        GsTimeScope ts(ctx, "linear_fwd", l, st);
        launch_fwd(ctx, st, ctx->ub_front[l + 1], va, a, b, epi, mu);
    }
    GS_HIP(ctx, hipGetLastError());
    sb.fwd_done = l_end == L;
    sb.fwd_batch = ctx->batch_id;
    return GSPLIT_OK;
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
    return sage_forward(ctx, p, d_feat_local, d_logits, (hipStream_t)stream, ctx->L);
}


namespace {

// backward pass, top layer down.  top_chunks > 0: the fused top-layer kernel has already left the top
// layer's input gradients in gtmp and its weight-gradient partials in that many slabs.
int sage_backward(gsplit_ctx *ctx, const gsplit_sage_params *p, const float *d_grad_logits, float *const *d_gw_self,
                  float *const *d_gw_neigh, float *const *d_gbias, hipStream_t st, int top_chunks) {
    GsSageBuf &sb = ctx->sage;
    const int L = ctx->L, S = ctx->S;
    for (int l = L - 1; l >= 0; --l) {
        const int D = p->dims[l], N = p->dims[l + 1];
        const GsLayerBuf &B = ctx->layer[l];
        const GsLevelMeta *mu = ctx->d_meta + (l + 1);
        const float *dH = l == L - 1 ? d_grad_logits : sb.ghid[l + 1];
        const int64_t ub = ctx->ub_front[l + 1];
        const bool h16 = p->dtype == GSPLIT_BF16;
        // bf16 storage: below the top level dZ is held in bf16 when its width allows 16-byte rows
        const bool dz_h = h16 && l < L - 1 && N % 8 == 0;
        MatRows dz{dH, 0, N};
        MatRowsH dzh{(const uint16_t *)dH, 0, N};
        // weight and bias gradients, summed over all splits: X^T dZ with the layer input X
        // assembled by the forward pass
        MatRows in{(const float *)sb.xin[l], 0, 2 * D};
        EpiGradW ew{sb.gw_part[l], 2 * D + 1, N, h16 ? 2 * D + 1 : 2 * D};
        const bool vin = D % 2 == 0;
        const bool vdz = N % 4 == 0 && aligned16(dH);
        const bool done_above = top_chunks > 0 && l == L - 1;
        if (!done_above) {
            GsTimeScope ts(ctx, "grad_w", l, st);
            if (h16) {
                MatRowsOnesH inh{(const uint16_t *)sb.xin[l], 0, 2 * D};
                const int tm = (int)gs_ceil_div(ew.rows, GBM), tn = (int)gs_ceil_div(ew.N, GBN);
                dim3 grid((unsigned)(sb.nchunk[l] * tm * tn));
                if (sb.gw_stream[l]) {
                    // two launches, one of which finds the level on its side of GWH_MIN_ROWS and works
                    const int bm = (int)gs_ceil_div(2 * D, GWH_B), bn = (int)gs_ceil_div(N, GWH_B);
                    hipLaunchKernelGGL(k_grad_w_hb, dim3((unsigned)(sb.stream_nchunk[l] * bm * bn)), dim3(GWH_NT), 0, st, inh.p,
                                       2 * D, dzh.p, N, sb.gw_part[l], sb.stream_nchunk[l], GWH_ROWS_MIN, bm, bn, mu, S,
                                       sb.stream_rows);
                }
                if (dz_h)
                    hipLaunchKernelGGL((k_sage_grad_w_h<PatchDzH, MatRowsH>), grid, dim3(GNT), 0, st, inh, dzh, ew,
                                       sb.nchunk[l], GRAD_W_ROWS_MIN, tm, tn, mu, S, sb.gw_stream[l] ? sb.stream_rows : 0);
                else if (vdz)
                    hipLaunchKernelGGL((k_sage_grad_w_h<PatchDz<4>, MatRows>), grid, dim3(GNT), 0, st, inh, dz, ew,
                                       sb.nchunk[l], GRAD_W_ROWS_MIN, tm, tn, mu, S, 0);
                else
                    hipLaunchKernelGGL((k_sage_grad_w_h<PatchDz<1>, MatRows>), grid, dim3(GNT), 0, st, inh, dz, ew,
                                       sb.nchunk[l], GRAD_W_ROWS_MIN, tm, tn, mu, S, 0);
            } else {
                launch_grad_w(st, sb.nchunk[l], vin, vdz, in, dz, ew, mu, S);
            }
        }
        if (l > 0) {
            const GsLevelMeta *ml = ctx->d_meta + l;
            EpiGradIn ei{sb.gtmp, sb.inv_cnt[l], D, 0};
            if (!done_above) {
                GsTimeScope ts(ctx, "grad_in", l, st);
                if (h16) {
                    dim3 grid(row_block_grid<TileMid>(ctx, ub, 2 * D));
                    MatRowsH wsk{sb.wstack[l], 2 * D, (N + 7) & ~7};
                    if (dz_h && rows_gemm_fits(ub, N, 2 * D, 4)) {
                        RbEpi re{sb.gtmp, 2 * D, nullptr, sb.inv_cnt[l], D, 0};
                        if (N == 256)
                            hipLaunchKernelGGL((k_rows_gemm_hb<16, true, 4>), dim3(rows_gemm_grid(ctx, 2 * D, 256)), dim3(GNT), 0,
                                               st, dzh.p, wsk.p, 2 * D, re, mu, S);
                        else
                            hipLaunchKernelGGL((k_rows_gemm_hb<32, true, 4>), dim3(rows_gemm_grid(ctx, 2 * D, 128)), dim3(GNT), 0,
                                               st, dzh.p, wsk.p, 2 * D, re, mu, S);
                    } else if (dz_h) hipLaunchKernelGGL(k_sage_grad_in_hh, grid, dim3(GNT), 0, st, dzh, wsk, ei, mu, S);
                    else if (vdz) hipLaunchKernelGGL((k_sage_grad_in_h<4>), grid, dim3(GNT), 0, st, dz, wsk, ei, mu, S);
                    else hipLaunchKernelGGL((k_sage_grad_in_h<1>), grid, dim3(GNT), 0, st, dz, wsk, ei, mu, S);
                } else {
                    MatRows w{sb.wstack32[l], 2 * D, (N + 3) & ~3};
                    launch_grad_in(ctx, st, ub, vdz, dz, w, ei, mu);
                }
            }
            GsTimeScope ts(ctx, "pull_input_grad", l, st);
            // reverse shuffle + ReLU of the layer below: dZ of layer l-1
            const void *hact = sb.hidden[l];
            const int64_t ubl = ctx->ub_front[l];
            // one wave per row of the level, and no more workgroups than stay resident at once: the waves
            // stride over the rows, and workgroups that had to queue behind the resident ones would run
            // their whole share after them on a nearly empty chip
#define GS_PULL(LPR, HH, OH)                                                                                     \
    do {                                                                                                         \
        const int n_main = (int)std::min<int64_t>(grid_1d(ctx, ubl * 64),                                        \
                                                  (int64_t)ctx->n_cu * resident_blocks(k_pull_input_grad<LPR, HH, OH>)); \
        hipLaunchKernelGGL((k_pull_input_grad<LPR, HH, OH>), dim3(n_main + PULL_LONG_BLOCKS), dim3(256), 0, st,  \
                           sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, B.rev_long, hact, ml, S,                \
                           (void *)sb.ghid[l], n_main);                                                          \
    } while (0)
#define GS_PULL_W(HH, OH)                                                                                        \
    do {                                                                                                         \
        if (D / 4 <= 16) GS_PULL(16, HH, OH);                                                                    \
        else if (D / 4 <= 32) GS_PULL(32, HH, OH);                                                               \
        else GS_PULL(64, HH, OH);                                                                                \
    } while (0)
            if (h16) {
                // the level's dZ is held in bf16 under the same condition its consumers test (dz_h)
                if (D % 8 == 0) GS_PULL_W(true, true);
                else GS_PULL_W(true, false);
            } else if (D % 4 != 0) {
                hipLaunchKernelGGL(k_pull_input_grad_any, dim3(grid_1d(ctx, ubl * 64)), dim3(256), 0, st,
                                   sb.gtmp, D, B.rev_ptr, B.rev_cnt, B.rev_list, (const float *)hact, ml, S, sb.ghid[l]);
            } else {
                GS_PULL_W(false, false);
            }
#undef GS_PULL_W
#undef GS_PULL
        }
    }
    {
        GradReduce gr;
        int64_t wmax = 1;
        for (int l = 0; l < L; ++l) {
            gr.part[l] = sb.gw_part[l]; gr.gws[l] = d_gw_self[l]; gr.gwn[l] = d_gw_neigh[l]; gr.gb[l] = d_gbias[l];
            gr.D[l] = p->dims[l]; gr.N[l] = p->dims[l + 1]; gr.nchunk[l] = sb.nchunk[l]; gr.rows_min[l] = GRAD_W_ROWS_MIN;
            gr.stream_rows[l] = sb.gw_stream[l] ? sb.stream_rows : 0; gr.stream_nchunk[l] = sb.stream_nchunk[l];
            gr.stream_rows_min[l] = GWH_ROWS_MIN;
            gr.fixed_chunks[l] = l == L - 1 ? top_chunks : 0;
            wmax = std::max<int64_t>(wmax, (int64_t)(2 * p->dims[l] + 1) * p->dims[l + 1]);
        }
        GsTimeScope ts(ctx, "reduce_grads", -1, st);
        hipLaunchKernelGGL(k_reduce_grads, dim3((unsigned)std::min<int64_t>(256, gs_ceil_div(wmax, 256)), L), dim3(256),
                           0, st, gr, ctx->d_meta, S);
    }
    GS_HIP(ctx, hipGetLastError());
    return GSPLIT_OK;
}

int check_grad_outputs(gsplit_ctx *ctx, float *const *d_gw_self, float *const *d_gw_neigh, float *const *d_gbias,
                       const char *who) {
    if (!d_gw_self || !d_gw_neigh || !d_gbias) return gs_fail(ctx, GSPLIT_EINVAL, std::string(who) + ": NULL buffer");
    for (int l = 0; l < ctx->L; ++l)
        if (!d_gw_self[l] || !d_gw_neigh[l] || !d_gbias[l])
            return gs_fail(ctx, GSPLIT_EINVAL, std::string(who) + ": NULL gradient pointer");
    return GSPLIT_OK;
}

// can the top layer of this model run as k_sage_top_fused?
bool top_fusable(const gsplit_ctx *ctx, const gsplit_sage_params *p, const void *top_input) {
    const int L = ctx->L;
    if (p->dtype != GSPLIT_F32 || L < 2) return false;
    const int D = p->dims[L - 1], N = p->dims[L];
    return N <= TOP_NMAX && D % 4 == 0 && D <= TOP_DMAX && aligned16(top_input);
}

}  // namespace

extern "C" int gsplit_sage_bwd(gsplit_ctx *ctx, const gsplit_sage_params *p, const float *d_grad_logits,
                               float *const *d_gw_self, float *const *d_gw_neigh, float *const *d_gbias,
                               void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    int rc = check_params(ctx, p, "gsplit_sage_bwd");
    if (rc) return rc;
    if (!d_grad_logits) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_sage_bwd: NULL buffer");
    rc = check_grad_outputs(ctx, d_gw_self, d_gw_neigh, d_gbias, "gsplit_sage_bwd");
    if (rc) return rc;
    GsSageBuf &sb = ctx->sage;
    if (!sb.ready || !sb.fwd_done || sb.fwd_batch != ctx->batch_id)
        return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_sage_bwd: needs gsplit_sage_fwd on the current batch first");
    for (int l = 0; l <= ctx->L; ++l)
        if (sb.dims[l] != p->dims[l] || sb.dtype != p->dtype)
            return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_sage_bwd: parameters differ from the forward pass");
    return sage_backward(ctx, p, d_grad_logits, d_gw_self, d_gw_neigh, d_gbias, (hipStream_t)stream, 0);
}

extern "C" int gsplit_sage_step(gsplit_ctx *ctx, const gsplit_sage_params *p, const void *d_feat_local,
                                const int64_t *d_labels, float *d_logits, float *d_row_loss, float *const *d_gw_self,
                                float *const *d_gw_neigh, float *const *d_gbias, void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    int rc = check_params(ctx, p, "gsplit_sage_step");
    if (rc) return rc;
    if (!d_feat_local || !d_labels || !d_logits) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_sage_step: NULL buffer");
    rc = check_grad_outputs(ctx, d_gw_self, d_gw_neigh, d_gbias, "gsplit_sage_step");
    if (rc) return rc;
    if (ctx->batch_id == 0) return gs_fail(ctx, GSPLIT_ESTATE, "gsplit_sage_step: no batch");
    rc = ensure_buffers(ctx, p);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    GsSageBuf &sb = ctx->sage;
    const int L = ctx->L, S = ctx->S;
    const int N = p->dims[L];
    if (!top_fusable(ctx, p, sb.hidden[L - 1])) {
        // the three steps one after the other, the loss gradient in the context's own buffer
        rc = sage_forward(ctx, p, d_feat_local, d_logits, st, L);
        if (rc) return rc;
        {
            GsTimeScope ts(ctx, "softmax_xent", -1, st);
            hipLaunchKernelGGL(k_softmax_xent, dim3(grid_1d(ctx, ctx->ub_front[L] * 64)), dim3(256), 0, st, d_logits, N,
                               d_labels, ctx->front[L], ctx->d_meta + L, S, sb.glog, d_row_loss);
        }
        rc = sage_backward(ctx, p, sb.glog, d_gw_self, d_gw_neigh, d_gbias, st, 0);
        sb.fwd_done = false;
        return rc;
    }
    rc = sage_forward(ctx, p, d_feat_local, d_logits, st, L - 1);
    if (rc) return rc;
    const int l = L - 1, D = p->dims[l];
    const GsLayerBuf &B = ctx->layer[l];
    const int chunks = sb.top_chunks;
    {
        TopArgs ta{(const float *)sb.hidden[l], D, N, (N + 3) & ~3, B.blk_indptr, B.edge_row, B.self_row, sb.wstack32[l],
                   (const float *)p->d_bias[l], d_labels, ctx->front[L], d_logits, d_row_loss, sb.gtmp, sb.gw_part[l],
                   ctx->d_meta + L, S};
        GsTimeScope ts(ctx, "top_fused", l, st);
        hipLaunchKernelGGL(k_sage_top_fused<TOP_ROWS>, dim3(chunks), dim3(TOP_T), sizeof(float) * top_lds_words(D, TOP_ROWS),
                           st, ta);
    }
    rc = sage_backward(ctx, p, nullptr, d_gw_self, d_gw_neigh, d_gbias, st, chunks);
    sb.fwd_done = false;        // the step is complete: a separate backward call needs a forward call of its own
    return rc;
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

