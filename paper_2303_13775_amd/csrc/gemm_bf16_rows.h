// Row-block products of the bf16 path for layers with many rows and a short contraction (included
// by sage.hip, inside its anonymous namespace): C[n1 x NB] = A[n1 x K] * B^T with A bf16 row-major
// (K = 256 or 512 contiguous), B given by rows of output columns (NB x K, K contiguous).
//
// Such a product moves far more bytes than it has flops for (a layer of GraphSAGE, paper section 2:
// 961k x 256 x 256 is 0.98 GB of rows in and out against 50 us of matrix-core time), so the kernel
// is laid out around the memory system:
//   * one workgroup of 8 waves per compute unit, persistent: it owns one block of 128 * NI output
//     columns and walks over row tiles of 64;
//   * B stays in registers for the whole launch: a wave's 32 * NI columns x K are 128 VGPRs, loaded
//     once in the fragment layout of v_mfma_f32_32x32x16_bf16 (8 consecutive k of one column per lane);
//   * A streams through LDS in units of 64 rows x 128 k (16 KiB) that go straight from global
//     memory into one of four or six stages (global_load_lds_dwordx4, 16 bytes a lane, two instructions
//     a wave and unit), three or five units ahead of the one being multiplied.  The 16-byte granules of a row
//     are stored at granule ^ (row & 15): 16 consecutive rows of one granule column then fall into
//     16 different bank groups and a fragment read (one 128-bit read per lane) is conflict-free;
//   * a finished tile leaves the accumulators through a wave-private LDS patch (bias / ReLU /
//     bfloat16 or the 1 / count scaling applied on the way in) and is written to global memory at
//     the top of the next step with 16-byte stores of whole row segments, so the stores have a
//     whole step to drain before the next wait.
// Waiting: a wave waits until at most four (eight with six stages) of its vector-memory operations
// are outstanding, i.e. (they complete in order) everything but the units it issued last, then the workgroup meets
// at a barrier; after it every wave may read the unit and the stage of the unit before is free.
// The prefetch is issued unconditionally (past the end it re-reads the last unit into a free
// stage), so the last operations before a wait are always those loads.
#pragma once

constexpr int RB_BM = 64;                  // rows of a tile
constexpr int RB_UK = 128;                 // k of a unit
constexpr int RB_UNIT4 = RB_BM * RB_UK * 2 / 16;   // 16-byte words of a unit: 1024

struct RbEpi {
    void *out;               // [n1 x ldo] bf16 (forward) or float (input gradient)
    int ldo;                 // output columns
    const float *bias;       // forward: per column
    const float *inv_cnt;    // input gradient: per row, applied to columns >= D; readable up to a whole tile past n1
    int D;
    int relu;
};

template <class F, int... I>
__device__ __forceinline__ void rb_for_each(F &&f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
constexpr int rb_lcm(int a, int b) { int x = a; while (x % b) x += a; return x; }

// NS: LDS stages (4 or 6): NS - 1 units are in flight ahead of the one being multiplied
template <int KS16, bool OUT_F32, int NS>
__global__ __launch_bounds__(GNT) void k_rows_gemm_hb(const uint16_t *__restrict__ A, const uint16_t *__restrict__ Bt,
                                                      int NB, RbEpi epi, const GsLevelMeta *__restrict__ meta_up, int S) {
    constexpr int NI = 32 / KS16, BN = 128 * NI, UPT = KS16 / 8, K = KS16 * 16;
    static_assert(KS16 == 16 || KS16 == 32, "contraction of 256 or 512");
    static_assert(GNT == 512, "eight waves");
    static_assert(NS == 4 || NS == 6, "four or six stages");
    __shared__ __attribute__((aligned(16))) uint4 st0[RB_UNIT4], st1[RB_UNIT4], st2[RB_UNIT4], st3[RB_UNIT4];
    __shared__ __attribute__((aligned(16))) uint4 st4[NS > 4 ? RB_UNIT4 : 1], st5[NS > 4 ? RB_UNIT4 : 1];
    constexpr int PITCH = OUT_F32 ? (32 * NI + 4) * 4 : (32 * NI + 8) * 2;     // bytes of a patch row
    __shared__ __attribute__((aligned(16))) unsigned char patches[8 * 32 * PITCH];

    const int n1 = meta_up->front_off[S];
    const int tiles_m = (n1 + RB_BM - 1) / RB_BM;
    const int nb = (NB + BN - 1) / BN;
    const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
    const int cb = q % nb, walker = (q / nb) * 8 + xcd, nwalk = ((int)gridDim.x / 8 / nb) * 8;
    if (walker >= tiles_m || walker >= nwalk) return;
    const int nt = (tiles_m - walker + nwalk - 1) / nwalk;
    const int nu = nt * UPT;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int n0 = cb * BN, wn0 = (wave & 3) * 32 * NI, wm0 = (wave >> 2) * 32;
    unsigned char *const patch = patches + wave * 32 * PITCH;

    // ---- B fragments, once
    uint4 bq[NI][KS16];
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int n = n0 + wn0 + 32 * j + l32;
        const uint4 *src = reinterpret_cast<const uint4 *>(Bt + (int64_t)min(n, NB - 1) * K + 8 * half);
#pragma unroll
        for (int ks = 0; ks < KS16; ++ks) {
            uint4 v = src[2 * ks];
            if (n >= NB) v = make_uint4(0u, 0u, 0u, 0u);
            bq[j][ks] = v;
        }
    }
    float colv[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int n = n0 + wn0 + 32 * j + l32;
        colv[j] = (!OUT_F32 && n < NB) ? epi.bias[n] : 0.f;
    }

    // ---- the two pieces of a unit this wave loads: piece p = 4 rows, lane -> (row, stored granule)
    int prow[2], pgran[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        const int p = wave + 8 * x;
        prow[x] = 4 * p + (lane >> 4);
        pgran[x] = ((lane & 15) ^ (prow[x] & 15)) * 8;       // element offset of the global granule that lands here
    }
    auto issue = [&](uint4 *stage, int v) __attribute__((always_inline)) {
        v = min(v, nu - 1);
        const int tile = walker + (v / UPT) * nwalk, kp = v % UPT;
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const int row = min(tile * RB_BM + prow[x], n1 - 1);
            const uint16_t *src = A + (int64_t)row * K + kp * RB_UK + pgran[x];
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                             (__attribute__((address_space(3))) void *)(stage + (wave + 8 * x) * 64), 16, 0, 0);
        }
    };

    floatx16 acc[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    const int arow = wm0 + l32, abase = arow * 16, asw = arow & 15;
    auto multiply = [&](const uint4 *stage, auto kp_c) __attribute__((always_inline)) {
        constexpr int KP = decltype(kp_c)::value;
#pragma unroll
        for (int k8 = 0; k8 < 8; ++k8) {
            const uint4 af = stage[abase + ((2 * k8 + half) ^ asw)];
#pragma unroll
            for (int j = 0; j < NI; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af),
                                                                 __builtin_bit_cast(bf16x8, bq[j][KP * 8 + k8]), acc[j], 0, 0, 0);
        }
    };

    // ---- epilogue halves
    float4 inv[4];                       // 1 / count of the lane's 16 accumulator rows (input gradient)
    auto load_inv = [&](int m0) __attribute__((always_inline)) {
        if (OUT_F32) {
#pragma unroll
            for (int g = 0; g < 4; ++g)
                inv[g] = *reinterpret_cast<const float4 *>(epi.inv_cnt + m0 + wm0 + 8 * g + 4 * half);
        }
    };
    auto to_patch = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int n = n0 + wn0 + 32 * j + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = (r >> 2) * 8 + half * 4 + (r & 3);
                float v = acc[j][r];
                if (OUT_F32) {
                    const float4 w4 = inv[r >> 2];
                    const float w = (r & 3) == 0 ? w4.x : (r & 3) == 1 ? w4.y : (r & 3) == 2 ? w4.z : w4.w;
                    v = n >= epi.D ? v * w : v;
                    *reinterpret_cast<float *>(patch + row * PITCH + (32 * j + l32) * 4) = v;
                } else {
                    v += colv[j];
                    v = (epi.relu && v < 0.f) ? 0.f : v;
                    *reinterpret_cast<uint16_t *>(patch + row * PITCH + (32 * j + l32) * 2) = f2bf(v);
                }
                acc[j][r] = 0.f;
            }
        }
    };
    constexpr int GPR = (OUT_F32 ? 8 : 4) * NI;          // 16-byte granules of a patch row
    constexpr int RPI = 64 / GPR;                        // rows a wave stores with one instruction
    constexpr int EPG = OUT_F32 ? 4 : 8;                 // elements of a granule
    auto from_patch = [&](int m0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int row = RPI * i + lane / GPR, gr = lane % GPR;
            const uint4 v = *reinterpret_cast<const uint4 *>(patch + row * PITCH + gr * 16);
            const int m = m0 + wm0 + row, n = n0 + wn0 + EPG * gr;
            if (m < n1 && n < NB) {
                if (OUT_F32) *reinterpret_cast<uint4 *>(reinterpret_cast<float *>(epi.out) + (int64_t)m * epi.ldo + n) = v;
                else *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(epi.out) + (int64_t)m * epi.ldo + n) = v;
            }
        }
    };

    // One step = one unit.  cur: the stage that holds unit u; free: the stage unit u - 1 was in.
    int m_done = -1;                      // first row of the tile waiting in the patch, -1: none
    auto step = [&](const uint4 *cur, uint4 *free_stage, int u, auto kp_c) __attribute__((always_inline)) {
        constexpr int KP = decltype(kp_c)::value;
        // all but the youngest NS - 2 units (two loads each) have landed: that includes unit u
        if (NS == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        const int m0 = (walker + (u / UPT) * nwalk) * RB_BM;
        if (KP == 0) {
            if (m_done >= 0) from_patch(m_done);
            load_inv(m0);
        }
        issue(free_stage, u + NS - 1);
        multiply(cur, kp_c);
        if (KP == UPT - 1) {
            to_patch();
            m_done = m0;
        }
    };
    auto stage = [&](auto ic) __attribute__((always_inline)) -> uint4 * {
        constexpr int x = decltype(ic)::value;
        if constexpr (x == 0) return st0;
        else if constexpr (x == 1) return st1;
        else if constexpr (x == 2) return st2;
        else if constexpr (x == 3) return st3;
        else if constexpr (x == 4) return st4;
        else return st5;
    };
    // a round: as many steps as bring both the stages and the units of a tile back to where they started
    constexpr int ROUND = rb_lcm(NS, UPT);
    rb_for_each([&](auto ic) __attribute__((always_inline)) { issue(stage(ic), decltype(ic)::value); }, std::make_integer_sequence<int, NS - 1>{});
    int u = 0;
    for (; u + ROUND <= nu; u += ROUND)
        rb_for_each([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            step(stage(std::integral_constant<int, i % NS>{}), stage(std::integral_constant<int, (i + NS - 1) % NS>{}), u + i,
                 std::integral_constant<int, i % UPT>{});
        }, std::make_integer_sequence<int, ROUND>{});
    if (u < nu) {                          // the tiles of an incomplete round
        const int left = nu - u;
        rb_for_each([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            if (i < left)
                step(stage(std::integral_constant<int, i % NS>{}), stage(std::integral_constant<int, (i + NS - 1) % NS>{}),
                     u + i, std::integral_constant<int, i % UPT>{});
        }, std::make_integer_sequence<int, ROUND>{});
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (m_done >= 0) from_patch(m_done);
}

// ------------------------------------------------------------------------------------------
// Weight gradients of such a layer: G[M2 x N] = X^T dZ over a chunk of destination rows (split-K,
// the slabs and the fixed-order reduction of the other weight-gradient kernels), X bf16 [n1 x M2],
// dZ bf16 [n1 x N].  One workgroup of 16 waves forms a whole 256 x 256 block of G (64 accumulator
// registers a lane), so a chunk's rows of X and dZ are read once (twice where M2 or N exceeds 256),
// not once per 64 x 128 output tile.
// Both operands are k-major in memory while a fragment holds 8 consecutive k of one column, so a
// k-tile (64 rows) is transposed in registers on its way into LDS: waves 0-7 take X, waves 8-15 dZ;
// a thread loads an 8 (k) x 4 (columns) patch as eight 8-byte row pieces (a wave reads one whole
// 512-byte row segment per instruction), regroups the 32 halves with byte permutes into four
// 16-byte fragments (8 k of one column each) and writes those with 128-bit LDS stores.
// LDS tile: [8 granules of 8 k][256 columns]; granule kg of column c sits at kg * 256 + p(c) with
//     p(c) = (c & ~15) | ((c & 15) ^ ((c >> 4) & 3)),
// a permutation inside every aligned group of 16 columns: the 16 lanes of a fragment read (16
// consecutive columns of one granule row) still cover 256 contiguous bytes, the 16 lanes of a
// transposed store (columns 4 apart) fall into 16 different bank groups, and the four k steps of a
// tile are constant offsets from one address per fragment.
// The bias gradient (column sums of dZ) is taken by the dZ threads of the first tile row from the
// values they load, summed over the k groups in LDS in a fixed order.
// ------------------------------------------------------------------------------------------
constexpr int GWH_B = 256;                 // columns of an operand tile (rows / columns of the output block)
constexpr int GWH_TILE4 = GWH_B * 8;       // 16-byte words of an operand tile: 2048 (32 KiB)
constexpr int GWH_NT = 1024;               // threads of a workgroup
constexpr int GWH_ROWS_MIN = 1024;
constexpr int GWH_MIN_ROWS = 131072;       // levels with fewer rows leave too few chunks of that size: the tiled kernel takes them
                                           // (default; the environment variable GSPLIT_GRADW_STREAM_ROWS overrides it)

__device__ __forceinline__ int gwh_word(int c, int kg) {
    return kg * GWH_B + ((c & ~15) | ((c & 15) ^ ((c >> 4) & 3)));
}

__global__ __launch_bounds__(GWH_NT) void k_grad_w_hb(const uint16_t *__restrict__ X, int M2,
                                                      const uint16_t *__restrict__ dZ, int N, float *__restrict__ part,
                                                      int nchunk, int rows_min, int tiles_m, int tiles_n,
                                                      const GsLevelMeta *__restrict__ meta_up, int S, int take_from) {
    __shared__ __attribute__((aligned(16))) uint4 sA0[GWH_TILE4], sB0[GWH_TILE4], sA1[GWH_TILE4], sB1[GWH_TILE4];
    const int n1 = meta_up->front_off[S];
    if (n1 < take_from) return;                          // a smaller level is the tiled kernel's
    const int kchunk = grad_w_chunk_rows(n1, nchunk, rows_min);
    const int tiles = tiles_m * tiles_n;
    const int xcd = blockIdx.x & 7, jb = blockIdx.x >> 3;
    const int tile = jb % tiles, chunk = (jb / tiles) * 8 + xcd;
    const int k_begin = chunk * kchunk;
    if (k_begin >= n1) return;
    const int k_end = min(n1, k_begin + kchunk);
    part += (int64_t)chunk * (M2 + 1) * N;
    const int tm = tile % tiles_m, m0 = tm * GWH_B, n0 = (tile / tiles_m) * GWH_B;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int wm0 = (wave >> 2) * 64, wn0 = (wave & 3) * 64;
    // loader role: waves 0-7 X (columns m), waves 8-15 dZ (columns n); cg = group of 4 columns, kg = group of 8 k
    const bool is_b = wave >= 8;
    const int cg = lane, kg = wave & 7;
    const uint16_t *src = is_b ? dZ : X;
    const int ld = is_b ? N : M2;
    const int c_first = (is_b ? n0 : m0) + 4 * cg;
    const uint16_t *src_col = src + min(c_first, ld - 4);        // a group past the edge re-reads the last one; never stored
    const bool want_cs = is_b && tm == 0;

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    float cs[4] = {0.f, 0.f, 0.f, 0.f};

    uint2 in[8];
    auto load = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int k = k0 + 8 * kg + i;
            uint2 v = *reinterpret_cast<const uint2 *>(src_col + (int64_t)min(k, n1 - 1) * ld);
            if (k >= k_end) v = make_uint2(0u, 0u);
            in[i] = v;
        }
    };
    auto land = [&](uint4 *tA, uint4 *tB) {
        uint4 *t = is_b ? tB : tA;
        if (want_cs) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                cs[0] += bf2f(in[i].x & 0xFFFFu); cs[1] += bf2f(in[i].x >> 16);
                cs[2] += bf2f(in[i].y & 0xFFFFu); cs[3] += bf2f(in[i].y >> 16);
            }
        }
        // o[c] = the 8 k of column c: word w holds k = 2 w (low half) and 2 w + 1 (high half)
        uint4 o0, o1, o2, o3;
        o0.x = __builtin_amdgcn_perm(in[1].x, in[0].x, 0x05040100u); o1.x = __builtin_amdgcn_perm(in[1].x, in[0].x, 0x07060302u);
        o0.y = __builtin_amdgcn_perm(in[3].x, in[2].x, 0x05040100u); o1.y = __builtin_amdgcn_perm(in[3].x, in[2].x, 0x07060302u);
        o0.z = __builtin_amdgcn_perm(in[5].x, in[4].x, 0x05040100u); o1.z = __builtin_amdgcn_perm(in[5].x, in[4].x, 0x07060302u);
        o0.w = __builtin_amdgcn_perm(in[7].x, in[6].x, 0x05040100u); o1.w = __builtin_amdgcn_perm(in[7].x, in[6].x, 0x07060302u);
        o2.x = __builtin_amdgcn_perm(in[1].y, in[0].y, 0x05040100u); o3.x = __builtin_amdgcn_perm(in[1].y, in[0].y, 0x07060302u);
        o2.y = __builtin_amdgcn_perm(in[3].y, in[2].y, 0x05040100u); o3.y = __builtin_amdgcn_perm(in[3].y, in[2].y, 0x07060302u);
        o2.z = __builtin_amdgcn_perm(in[5].y, in[4].y, 0x05040100u); o3.z = __builtin_amdgcn_perm(in[5].y, in[4].y, 0x07060302u);
        o2.w = __builtin_amdgcn_perm(in[7].y, in[6].y, 0x05040100u); o3.w = __builtin_amdgcn_perm(in[7].y, in[6].y, 0x07060302u);
        t[gwh_word(4 * cg, kg)] = o0;
        t[gwh_word(4 * cg + 1, kg)] = o1;
        t[gwh_word(4 * cg + 2, kg)] = o2;
        t[gwh_word(4 * cg + 3, kg)] = o3;
    };
    const int ra[2] = {gwh_word(wm0 + l32, half), gwh_word(wm0 + 32 + l32, half)};
    const int rb[2] = {gwh_word(wn0 + l32, half), gwh_word(wn0 + 32 + l32, half)};
    auto multiply = [&](const uint4 *tA, const uint4 *tB) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            uint4 af[2], bfr[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) af[i] = tA[ra[i] + 2 * ks * GWH_B];
#pragma unroll
            for (int j = 0; j < 2; ++j) bfr[j] = tB[rb[j] + 2 * ks * GWH_B];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[i]),
                                                                        __builtin_bit_cast(bf16x8, bfr[j]), acc[i][j], 0, 0, 0);
        }
    };

    load(k_begin);
    land(sA0, sB0);
    __syncthreads();
    const int nt = (k_end - k_begin + 63) >> 6;
    // every step fetches the next tile while it multiplies the current one; the fetch behind the last
    // tile finds no rows (k >= k_end reads as zero) and lands in the stage nobody reads any more
    for (int t = 0; t < nt; ++t) {
        const bool odd = t & 1;
        load(k_begin + 64 * (t + 1));
        multiply(odd ? sA1 : sA0, odd ? sB1 : sB0);
        land(odd ? sA0 : sA1, odd ? sB0 : sB1);
        __syncthreads();
    }

    // accumulator layout of a 32 x 32 block: register r of lane l holds row (r / 4) * 8 + (l / 32) * 4 + (r % 4), column l % 32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm0 + 32 * i + (r >> 2) * 8 + half * 4 + (r & 3), n = n0 + wn0 + 32 * j + l32;
                if (m < M2 && n < N) part[(int64_t)m * N + n] = acc[i][j][r];
            }
    if (tm == 0) {
        // column sums: [8 k groups][256 columns], added in k-group order
        __syncthreads();
        float *red = reinterpret_cast<float *>(sA0);
        if (is_b) {
#pragma unroll
            for (int c = 0; c < 4; ++c) red[kg * GWH_B + 4 * cg + c] = cs[c];
        }
        __syncthreads();
        if (tid < GWH_B) {
            float s = 0.f;
#pragma unroll
            for (int g = 0; g < 8; ++g) s += red[g * GWH_B + tid];
            if (n0 + tid < N) part[(int64_t)M2 * N + n0 + tid] = s;
        }
    }
}
