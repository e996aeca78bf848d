// fp32 MFMA GEMM core shared by the GraphSAGE and GAT translation units (included inside their
// anonymous namespaces): tile templates, operand staging, the k loop, the plain row-major operand
// accessor, persistent row-block tiling, and the split-K weight-gradient kernel with its launch.
#pragma once

typedef float floatx16 __attribute__((ext_vector_type(16)));

// ------------------------------------------------------------------------------------------
// Tiled fp32 MFMA GEMM core:  C[M x N] = A[M x K] * B[K x N].
//
// Operands are described by accessors  at(outer, inner) -> const float* (clamped into the matrix;
// `inner` runs along memory).  An operand is used either K-contiguous (KC: outer is the M or N
// index, inner is k) or K-major (KM: outer is k, inner is the M or N index); both are staged into
// LDS with the layout they have in memory, without padding, so that a tile is a run of 1-KiB
// pieces each of which one wave can load straight from global memory into LDS (lane L of a
// global_load_lds_dwordx4 lands at base + 16 L):
//   KC: lds[row][32 k], the eight 16-byte granules of a row stored at granule ^ ((row >> 1) & 7)
//       (a lane simply loads the granule that belongs where it writes); MFMA fragments are one
//       128-bit read per 8 k
//   KM: lds[k][ROWS], the two 32-word halves of a row swapped when (k >> 2) is odd; MFMA fragments
//       are four 32-bit reads per 8 k
// Both permutations are for the 64 LDS banks: sixteen consecutive rows of a KC tile, and the k
// rows that the two halves of a wave read from a KM tile, fall on different banks.
// v_mfma_f32_32x32x2_f32 sums two k-slots (lane / 32 selects the slot).  Within a group of 8 k the
// lower half-wave takes k = 0..3 and the upper half k = 4..7 over four consecutive MFMAs; A and B
// use the same assignment, so the sum over k is complete whatever the order.
//
// A workgroup always has 8 waves.  Tile<BM, BN, WM, WN, KS> lays them out WM x WN over a BM x BN
// output tile and KS-fold over k: with KS > 1 the groups of 8 k inside every k-tile are dealt to KS
// wave groups whose accumulators are added through LDS at the end.  Products with few rows use a
// small tile with KS > 1, which shortens the dependent chain of k-tiles a workgroup walks and
// yields more workgroups.
// ------------------------------------------------------------------------------------------
constexpr int BK = 32;
constexpr int GNT = 512;

template <int BM_, int BN_, int WM_, int WN_, int KS_, bool LEAN_ = false, bool DIRECT_ = false>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, KS = KS_;
    // DIRECT (lean tiles only): unpadded, permuted LDS layouts and k-tiles loaded straight from
    // global memory into LDS; otherwise padded layouts filled through registers
    static constexpr bool DIRECT = DIRECT_;
    static_assert(!DIRECT_ || LEAN_, "direct loads belong to the lean schedule");
    // LEAN: one register stage and no fragment double-buffering, so that three workgroups fit a
    // compute unit (80 registers a lane); latency is then hidden by the other workgroups' waves
    static constexpr bool LEAN = LEAN_;
    static constexpr int MI = BM / (32 * WM), NI = BN / (32 * WN);
    static constexpr int NO = BK / 8 / KS;      // groups of 8 k per k-tile and wave
    // workgroups one compute unit holds (registers for the full schedule, LDS for a padded lean tile
    // of 128 rows: two stages of 128 x 36 + 32 x 68 words are 54 KiB)
    static constexpr int OCC = (BM * BN >= 8192 && !LEAN) ? 2 : (LEAN && !DIRECT && BM >= 128) ? 2 : 3;
    static_assert(WM * WN * KS * 64 == GNT, "a workgroup has 8 waves");
    static_assert(MI >= 1 && NI >= 1 && MI * 32 * WM == BM && NI * 32 * WN == BN, "32 x 32 MFMA blocks");
    static_assert(KS == 1 || KS == 2 || KS == 4, "k split");
};
using TileMid = Tile<64, 128, 2, 4, 1>;
using TileMidLean = Tile<64, 128, 2, 4, 1, true>;
using TileMidDirect = Tile<64, 128, 2, 4, 1, true, true>;
using TileLow = Tile<32, 128, 1, 4, 2>;
using TileLowNarrow = Tile<32, 64, 1, 2, 4>;

// PAD: row strides of 36 (KC) and ROWS + 4 (KM) words instead of the permutations
template <int ROWS, bool KC, bool PAD>
constexpr int lds_words() { return PAD ? (KC ? ROWS * (BK + 4) : BK * (ROWS + 4)) : ROWS * BK; }
template <bool PAD>
__device__ __forceinline__ int kc_word(int row, int granule) {
    return PAD ? row * (BK + 4) + (granule << 2) : row * BK + ((granule ^ ((row >> 1) & 7)) << 2);
}
template <int ROWS, bool PAD>
__device__ __forceinline__ int km_word(int k, int col) {
    return PAD ? k * (ROWS + 4) + col : k * ROWS + (ROWS >= 64 ? col ^ (((k >> 2) & 1) << 5) : col);
}

__device__ __forceinline__ uint16_t f2bf(float f) {          // round to nearest, ties to even
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(uint32_t h) { return __uint_as_float(h << 16); }

// SRC_H: the source matrix holds bfloat16; the raw halves travel through the registers and are
// widened to float (exactly) when the tile is written to LDS.
template <int ROWS, bool KC, int VW, int NT, class F, bool SRC_H = false, bool PAD = true>
struct Stager {
    static constexpr int TOT = ROWS * BK / 4;                 // 4-word pieces of one tile
    static constexpr int NV = (TOT + NT - 1) / NT;
    static_assert(NV >= 1 && NV <= 8, "tile too large for the workgroup");
    typedef typename std::conditional<SRC_H, uint16_t, float>::type E;
    float4 reg[NV];
    unsigned keep;   // 4 bits per register: which of its words exist in the matrix
    // what does not change along k, prepared once (16-byte path): the row of a KC piece, the
    // clamped M/N index of a KM piece
    const E *fixed_row[KC ? NV : 1];
    int fixed_tok[KC ? 1 : NV];

    // piece v of thread tid: (row, k / 4) for KC, (k, row / 4) for KM; false if the tile has no such piece
    static __device__ __forceinline__ bool piece(int tid, int v, int &outer, int &inner4) {
        if (KC) {
            inner4 = tid & (BK / 4 - 1); outer = tid / (BK / 4) + (NT / (BK / 4)) * v;
            return TOT % NT == 0 || outer < ROWS;
        }
        inner4 = tid % (ROWS / 4); outer = tid / (ROWS / 4) + (4 * NT / ROWS) * v;
        return TOT % NT == 0 || outer < BK;
    }
    __device__ __forceinline__ void init(const F &f, int r0, int tid) {
        if (VW != 4) return;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int o, i4;
            piece(tid, v, o, i4);
            bool in;
            if (KC) fixed_row[v] = f.template at<4>(r0 + o, 0, in);
            else fixed_tok[v] = f.tok(r0 + 4 * i4);
        }
    }
    __device__ __forceinline__ void take(int v, const E *src) {
        if (SRC_H) {
            const uint2 raw = *reinterpret_cast<const uint2 *>(src);
            reg[v].x = __uint_as_float(raw.x);
            reg[v].y = __uint_as_float(raw.y);
        } else {
            reg[v] = *reinterpret_cast<const float4 *>(src);
        }
    }
    // A k-tile that lies wholly inside [k_begin, k_end) needs no masking at all: M/N indices past
    // the matrix read a clamped (valid) address and only feed outputs that are never stored.
    __device__ __forceinline__ void load_full(const F &f, int k0, int tid) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int o, i4;
            if (!piece(tid, v, o, i4)) continue;
            if (KC) take(v, fixed_row[v] + k0 + 4 * i4);
            else take(v, f.km(k0 + o, fixed_tok[v]));
        }
    }
    // General form: loads are unconditional (the accessor clamps the address into the matrix);
    // words outside the matrix are zeroed only when the registers are written to LDS, so nothing
    // depends on a load before that point and the loads of two k-tiles stay in flight.
    __device__ __forceinline__ void fetch(int v, const F &f, int outer, int inner, int inner_end, bool ok) {
        if (VW == 4) {
            bool in;
            take(v, f.template at<4>(outer, inner, in));
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
            int o, i4;
            if (!piece(tid, v, o, i4)) continue;
            if (KC) fetch(v, f, r0 + o, k0 + 4 * i4, k_end, r0 + o < r_end);
            else fetch(v, f, k0 + o, r0 + 4 * i4, r_end, k0 + o < k_end);
        }
    }
    __device__ __forceinline__ float4 widened(int v) const {
        if (!SRC_H) return reg[v];
        if (VW == 4) {
            const uint32_t lo = __float_as_uint(reg[v].x), hi = __float_as_uint(reg[v].y);
            return make_float4(bf2f(lo & 0xFFFFu), bf2f(lo >> 16), bf2f(hi & 0xFFFFu), bf2f(hi >> 16));
        }
        return make_float4(bf2f(__float_as_uint(reg[v].x)), bf2f(__float_as_uint(reg[v].y)),
                           bf2f(__float_as_uint(reg[v].z)), bf2f(__float_as_uint(reg[v].w)));
    }
    template <bool MASKED>
    __device__ __forceinline__ void store(float *lds, int tid) const {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int o, i4;
            if (!piece(tid, v, o, i4)) continue;
            float4 w = widened(v);
            if (MASKED) {
                w.x = (keep >> (4 * v)) & 1u ? w.x : 0.f;
                w.y = (keep >> (4 * v + 1)) & 1u ? w.y : 0.f;
                w.z = (keep >> (4 * v + 2)) & 1u ? w.z : 0.f;
                w.w = (keep >> (4 * v + 3)) & 1u ? w.w : 0.f;
            }
            if (KC) *reinterpret_cast<float4 *>(&lds[kc_word<PAD>(o, i4)]) = w;
            else *reinterpret_cast<float4 *>(&lds[km_word<ROWS, PAD>(o, 4 * i4)]) = w;
        }
    }
};

// Global memory straight into LDS for a k-tile that needs no masking: the tile is ROWS / 8 pieces
// of 1 KiB, piece j loaded by wave j mod 8 with one global_load_lds_dwordx4 (16 bytes a lane).
template <int ROWS, bool KC, class F>
struct Direct {
    static constexpr int PIECES = ROWS / 8;
    static constexpr int PER = (PIECES + 7) / 8;      // pieces per wave
    const float *fixed_row[KC ? PER : 1];             // KC: row pointer plus the lane's (swizzled) granule
    int fixed_tok[KC ? 1 : PER];                      // KM: clamped M/N index
    int fixed_k[KC ? 1 : PER];                        // KM: k row inside the tile
    __device__ __forceinline__ void init(const F &f, int r0, int wave, int lane) {
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int j = wave + 8 * p;
            if (KC) {
                const int row = 8 * j + (lane >> 3);
                bool in;
                fixed_row[p] = f.template at<4>(r0 + row, 0, in) + 4 * ((lane & 7) ^ ((row >> 1) & 7));
            } else {
                constexpr int LPK = ROWS / 4;         // lanes per k row
                fixed_k[p] = j * (64 / LPK) + lane / LPK;
                // the lane fills position 4 * (lane % LPK) of row k: it loads the column stored there
                fixed_tok[p] = f.tok(r0 + (km_word<ROWS, false>(fixed_k[p], 4 * (lane % LPK)) - fixed_k[p] * ROWS));
            }
        }
    }
    __device__ __forceinline__ void issue(const F &f, float *stage, int k0, int wave) const {
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int j = wave + 8 * p;
            if (PIECES % 8 != 0 && j >= PIECES) continue;
            const float *src = KC ? fixed_row[p] + k0 : f.km(k0 + fixed_k[p], fixed_tok[p]);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                             (__attribute__((address_space(3))) void *)(stage + j * 256), 16, 0, 0);
        }
    }
};

template <int ROWS, bool KC, bool PAD>
__device__ __forceinline__ void read_frag(const float *lds, int row, int oct, int half, float out[4]) {
    if (KC) {
        const float4 v = *reinterpret_cast<const float4 *>(&lds[kc_word<PAD>(row, oct * 2 + half)]);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) out[j] = lds[km_word<ROWS, PAD>(oct * 8 + 4 * half + j, row)];
    }
}

// COLSUM: the workgroups of the first tile row (m0 == 0) also sum the columns of B over their k
// range, from the tiles they stage in LDS anyway, and hand the sums to epi.colsum(): the
// weight-gradient product gets the bias gradient without a row of ones in A.
template <class T, bool A_KC, bool B_KC, int VA, int VB, class AF, class BF, class EF, bool A_H = false,
          bool COLSUM = false>
__device__ __forceinline__ void gemm_tile(const int m0, const int n0, const int m_end, const int n_end,
                                          const int k_begin, const int k_end, const AF &a, const BF &b,
                                          const EF &epi) {
    constexpr int BM = T::BM, BN = T::BN, MI = T::MI, NI = T::NI, KS = T::KS, NO = T::NO;
    // two LDS stages and RS (two or four) register stages: k-tile t is multiplied out of LDS while
    // tile t+1 sits in the other LDS stage and tiles t+2 .. t+RS are in flight into registers, so a
    // global load has RS iterations to land (an HBM round trip is longer than one k-tile of MFMA work)
    constexpr bool PAD = !T::DIRECT;
    constexpr int AW = lds_words<BM, A_KC, PAD>(), BW = lds_words<BN, B_KC, PAD>();
    constexpr int RED = (KS - 1) * T::WM * T::WN * MI * NI * 1024;   // accumulators handed over at the end
    static_assert(RED <= 2 * (AW + BW), "k-split hand-over does not fit the staging area");
    // A direct tile keeps its four stages in separate LDS objects: the compiler then knows that a
    // straight-to-LDS load into one stage does not alias the fragment reads of the other and does
    // not make the reads wait for the load.
    constexpr bool SPLIT = T::DIRECT;
    __shared__ __attribute__((aligned(16))) float lds[SPLIT ? (COLSUM ? GNT : 4) : 2 * (AW + BW)];
    __shared__ __attribute__((aligned(16))) float stA0[SPLIT ? AW : 4], stA1[SPLIT ? AW : 4];
    __shared__ __attribute__((aligned(16))) float stB0[SPLIT ? BW : 4], stB1[SPLIT ? BW : 4];
    float *const As0 = SPLIT ? stA0 : lds, *const As1 = SPLIT ? stA1 : lds + AW;
    float *const Bs0 = SPLIT ? stB0 : lds + 2 * AW, *const Bs1 = SPLIT ? stB1 : lds + 2 * AW + BW;
    static_assert(!T::LEAN || KS == 1, "a lean tile has no k split");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int kg = wave / (T::WM * T::WN), wv = wave % (T::WM * T::WN);
    const int wm0 = (wv / T::WN) * (BM / T::WM), wn0 = (wv % T::WN) * (BN / T::WN);
    floatx16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    using SA = Stager<BM, A_KC, VA, GNT, AF, A_H, PAD>;
    using SB = Stager<BN, B_KC, VB, GNT, BF, false, PAD>;
    // register stages of the full schedule.  A 32-row tile belongs to a product with few rows: the
    // launch has about one workgroup per compute unit, nobody else hides its loads, and its k loop
    // is a chain of global-load latencies (an iteration holds 0.2 us of MFMA work); four tiles in
    // flight instead of two shorten every link of that chain.
    constexpr int RS = (!T::LEAN && BM <= 32) ? 4 : 2;
    SA sa[RS];
    SB sb[RS];
    SA &sa0 = sa[0];
    SB &sb0 = sb[0];

    static_assert(!COLSUM || (!B_KC && KS == 1 && GNT % BN == 0 && BK % (GNT / BN) == 0), "column sums need a k-major B");
    constexpr int CS_KPG = COLSUM ? BK / (GNT / BN) : 1;    // k rows of a tile per thread
    const bool want_cs = COLSUM && m0 == 0;
    float csum = 0.f;
    auto colsum_tile = [&](const float *Bs) {
        if (!want_cs) return;
        const int n = tid % BN, g = tid / BN;
#pragma unroll
        for (int j = 0; j < CS_KPG; ++j) csum += Bs[km_word<BN, PAD>(g * CS_KPG + j, n)];
    };

    // The fragments of the next group of 8 k are read from LDS while the MFMAs of the current group
    // execute (an MFMA occupies the matrix pipe for 64 cycles but not the issue slot), so only the
    // first LDS read of a k-tile is exposed.
    // kv: k values of the tile that lie inside the k range.  The last tile of a range may hold
    // fewer than BK, and a group of 8 k that lies wholly outside contributes nothing: it is skipped
    // (a contraction of 200 runs 25 groups instead of 28, one of 100 runs 13 instead of 16).
    auto multiply = [&](const float *As, const float *Bs, int kv) {
        if (T::LEAN) {
            float af[MI][4], bf[NI][4];
#pragma unroll
            for (int t = 0; t < NO; ++t) {
                if (t > 0 && 8 * (kg + KS * t) >= kv) break;        // uniform over the wave
#pragma unroll
                for (int i = 0; i < MI; ++i) read_frag<BM, A_KC, PAD>(As, wm0 + i * 32 + l32, kg + KS * t, half, af[i]);
#pragma unroll
                for (int j = 0; j < NI; ++j) read_frag<BN, B_KC, PAD>(Bs, wn0 + j * 32 + l32, kg + KS * t, half, bf[j]);
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int i = 0; i < MI; ++i)
#pragma unroll
                        for (int j = 0; j < NI; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][q], bf[j][q], acc[i][j], 0, 0, 0);
            }
            return;
        }
        float af[2][MI][4], bf[2][NI][4];
#pragma unroll
        for (int i = 0; i < MI; ++i) read_frag<BM, A_KC, PAD>(As, wm0 + i * 32 + l32, kg, half, af[0][i]);
#pragma unroll
        for (int j = 0; j < NI; ++j) read_frag<BN, B_KC, PAD>(Bs, wn0 + j * 32 + l32, kg, half, bf[0][j]);
#pragma unroll
        for (int t = 0; t < NO; ++t) {
            if (t + 1 < NO) {
#pragma unroll
                for (int i = 0; i < MI; ++i)
                    read_frag<BM, A_KC, PAD>(As, wm0 + i * 32 + l32, kg + KS * (t + 1), half, af[(t + 1) & 1][i]);
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    read_frag<BN, B_KC, PAD>(Bs, wn0 + j * 32 + l32, kg + KS * (t + 1), half, bf[(t + 1) & 1][j]);
            }
            __builtin_amdgcn_sched_barrier(0);   // reads of the next group stay ahead of these MFMAs
            if (t == 0 || 8 * (kg + KS * t) < kv) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int i = 0; i < MI; ++i)
#pragma unroll
                        for (int j = 0; j < NI; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t & 1][i][q], bf[t & 1][j][q], acc[i][j], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // A k-tile wholly inside the k range takes the unmasked 16-byte path; only the last tile of a
    // range can be partial (and every tile is treated so when an operand needs scalar loads).
    auto load_tile = [&](SA &ra, SB &rb, int k0) {
        const bool full = k0 + BK <= k_end;
        if (VA == 4 && full) ra.load_full(a, k0, tid);
        else ra.load(a, m0, m_end, k0, k_end, tid);
        if (VB == 4 && full) rb.load_full(b, k0, tid);
        else rb.load(b, n0, n_end, k0, k_end, tid);
    };
    auto store_tile = [&](const SA &ra, const SB &rb, float *As, float *Bs, int k0) {
        const bool full = k0 + BK <= k_end;
        if (VA == 4 && full) ra.template store<false>(As, tid);
        else ra.template store<true>(As, tid);
        if (VB == 4 && full) rb.template store<false>(Bs, tid);
        else rb.template store<true>(Bs, tid);
    };
    // one k-tile: fetch tile k0 + RS BK into the registers that held tile k0, multiply tile k0,
    // move tile k0 + BK from registers to the other LDS stage
    auto step = [&](SA &ra_cur, SB &rb_cur, SA &ra_nxt, SB &rb_nxt, const float *As_cur, const float *Bs_cur,
                    float *As_nxt, float *Bs_nxt, int k0) {
        if (k0 + RS * BK < k_end) load_tile(ra_cur, rb_cur, k0 + RS * BK);
        multiply(As_cur, Bs_cur, k_end - k0);
        colsum_tile(Bs_cur);
        if (k0 + BK < k_end) store_tile(ra_nxt, rb_nxt, As_nxt, Bs_nxt, k0 + BK);
        __syncthreads();
    };

    if (T::LEAN) {
        // one k-tile ahead: tile k0 + BK goes straight from global memory into the other LDS stage
        // while tile k0 is multiplied (no staging registers, no LDS store instructions); a masked
        // or scalar-loaded tile takes the register path into the same layout
        constexpr bool DA = T::DIRECT && VA == 4 && !A_H, DB = T::DIRECT && VB == 4;
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);
        Direct<BM, A_KC, AF> da;
        Direct<BN, B_KC, BF> db;
        if (DA) da.init(a, m0, wave_u, lane); else sa0.init(a, m0, tid);
        if (DB) db.init(b, n0, wave_u, lane); else sb0.init(b, n0, tid);
        auto fetch_tile = [&](float *As, float *Bs, int k0) {
            const bool full = k0 + BK <= k_end;
            if (DA && full) da.issue(a, As, k0, wave_u);
            else if (VA == 4 && full) sa0.load_full(a, k0, tid);
            else sa0.load(a, m0, m_end, k0, k_end, tid);
            if (DB && full) db.issue(b, Bs, k0, wave_u);
            else if (VB == 4 && full) sb0.load_full(b, k0, tid);
            else sb0.load(b, n0, n_end, k0, k_end, tid);
        };
        auto land_tile = [&](float *As, float *Bs, int k0) {
            const bool full = k0 + BK <= k_end;
            if (!(DA && full)) {
                if (VA == 4 && full) sa0.template store<false>(As, tid); else sa0.template store<true>(As, tid);
            }
            if (!(DB && full)) {
                if (VB == 4 && full) sb0.template store<false>(Bs, tid); else sb0.template store<true>(Bs, tid);
            }
        };
        fetch_tile(As0, Bs0, k_begin);
        land_tile(As0, Bs0, k_begin);
        __syncthreads();
        auto lean_step = [&](const float *As_cur, const float *Bs_cur, float *As_nxt, float *Bs_nxt, int k0) {
            if (k0 + BK < k_end) fetch_tile(As_nxt, Bs_nxt, k0 + BK);
            multiply(As_cur, Bs_cur, k_end - k0);
            colsum_tile(Bs_cur);
            if (k0 + BK < k_end) land_tile(As_nxt, Bs_nxt, k0 + BK);
            __syncthreads();
        };
        int k0 = k_begin;
        // steady state without conditions: the tile fetched by each step is a whole tile that exists
        if (VA == 4 && VB == 4) {
            auto whole_step = [&](const float *As_cur, const float *Bs_cur, float *As_nxt, float *Bs_nxt, int kk) {
                if (DA) da.issue(a, As_nxt, kk + BK, wave_u); else sa0.load_full(a, kk + BK, tid);
                if (DB) db.issue(b, Bs_nxt, kk + BK, wave_u); else sb0.load_full(b, kk + BK, tid);
                multiply(As_cur, Bs_cur, BK);
                colsum_tile(Bs_cur);
                if (!DA) sa0.template store<false>(As_nxt, tid);
                if (!DB) sb0.template store<false>(Bs_nxt, tid);
                __syncthreads();
            };
            for (; k0 + 3 * BK <= k_end; k0 += 2 * BK) {
                whole_step(As0, Bs0, As1, Bs1, k0);
                whole_step(As1, Bs1, As0, Bs0, k0 + BK);
            }
        }
        for (; k0 < k_end; k0 += 2 * BK) {
            lean_step(As0, Bs0, As1, Bs1, k0);
            if (k0 + BK < k_end) lean_step(As1, Bs1, As0, Bs0, k0 + BK);
        }
    } else {
#pragma unroll
    for (int u = 0; u < RS; ++u) {
        sa[u].init(a, m0, tid);
        sb[u].init(b, n0, tid);
        if (k_begin + u * BK < k_end) load_tile(sa[u], sb[u], k_begin + u * BK);
    }
    store_tile(sa[0], sb[0], As0, Bs0, k_begin);
    __syncthreads();
    int k0 = k_begin;
    // Steady state, free of conditions: every tile a round touches is a whole tile that exists.
    // Only then does the compiler know how many loads are younger than the ones a step is about
    // to store to LDS, and waits for those alone; a condition around a load makes it wait for
    // every load in flight, which puts a full memory latency into each iteration.
    if (VA == 4 && VB == 4) {
        auto whole_step = [&](SA &ra_cur, SB &rb_cur, SA &ra_nxt, SB &rb_nxt, const float *As_cur,
                              const float *Bs_cur, float *As_nxt, float *Bs_nxt, int kk) {
            ra_cur.load_full(a, kk + RS * BK, tid);
            rb_cur.load_full(b, kk + RS * BK, tid);
            multiply(As_cur, Bs_cur, BK);
            colsum_tile(Bs_cur);
            ra_nxt.template store<false>(As_nxt, tid);
            rb_nxt.template store<false>(Bs_nxt, tid);
            __syncthreads();
        };
        for (; k0 + 2 * RS * BK <= k_end; k0 += RS * BK) {
#pragma unroll
            for (int u = 0; u < RS; ++u) {
                if (u & 1) whole_step(sa[u], sb[u], sa[(u + 1) % RS], sb[(u + 1) % RS], As1, Bs1, As0, Bs0, k0 + u * BK);
                else whole_step(sa[u], sb[u], sa[(u + 1) % RS], sb[(u + 1) % RS], As0, Bs0, As1, Bs1, k0 + u * BK);
            }
        }
    }
    for (; k0 < k_end; k0 += RS * BK) {
#pragma unroll
        for (int u = 0; u < RS; ++u) {
            if (k0 + u * BK >= k_end) break;            // uniform over the workgroup
            if (u & 1) step(sa[u], sb[u], sa[(u + 1) % RS], sb[(u + 1) % RS], As1, Bs1, As0, Bs0, k0 + u * BK);
            else step(sa[u], sb[u], sa[(u + 1) % RS], sb[(u + 1) % RS], As0, Bs0, As1, Bs1, k0 + u * BK);
        }
    }
    }
    if constexpr (COLSUM) {
        if (want_cs) {
            // every wave is past its last LDS read (the k loop ends on a barrier)
            lds[tid] = csum;
            __syncthreads();
            if (tid < BN) {
                float sum = 0.f;
#pragma unroll
                for (int g = 0; g < GNT / BN; ++g) sum += lds[g * BN + tid];
                epi.colsum(n0 + tid, sum);
            }
        }
    }
    if (KS > 1) {
        // every wave is past its last LDS read (the k loop ends on a barrier): wave groups 1.. hand
        // their accumulators to group 0, which adds them in group order
        constexpr int PER_WAVE = MI * NI * 1024;
        if (kg > 0) {
            float *dst = lds + ((kg - 1) * T::WM * T::WN + wv) * PER_WAVE + lane;
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) dst[((i * NI + j) * 16 + r) * 64] = acc[i][j][r];
        }
        __syncthreads();
        if (kg == 0) {
#pragma unroll
            for (int g = 1; g < KS; ++g) {
                const float *src = lds + ((g - 1) * T::WM * T::WN + wv) * PER_WAVE + lane;
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[i][j][r] += src[((i * NI + j) * 16 + r) * 64];
            }
        }
    }
    // accumulator layout of the 32x32 block: register r of lane l holds
    // row (r / 4) * 8 + (l / 32) * 4 + (r % 4), column l % 32.
    // Per-column and per-row side inputs of the epilogue (bias, 1/count) are fetched up front so
    // that their latencies overlap instead of adding up in front of every store.
    if (kg == 0) {
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
    // the staging area is reused by the caller's next tile
    if (KS > 1) __syncthreads();
}

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
    // K-major use, 16-byte pieces: tok() clamps the M/N index once, km() addresses row k < rows
    __device__ __forceinline__ int tok(int i) const { return min(i, cols - 4); }
    __device__ __forceinline__ const float *km(int k, int t) const { return p + (int64_t)k * cols + t; }
};
// partial [dW_self; dW_neigh; db] of one chunk of destination rows, written to the chunk's slab
struct EpiGradW {
    // rows = 2 * D + 1: the slab's last row holds the bias gradient.  It arrives through colsum()
    // (own_rows = 2 * D: the product has no row of ones) or as an ordinary row (own_rows = rows)
    float *part; int rows; int N; int own_rows;
    __device__ __forceinline__ void colsum(int n, float v) const { if (n < N) part[(int64_t)(rows - 1) * N + n] = v; }
    __device__ __forceinline__ float col(int) const { return 0.f; }
    __device__ __forceinline__ float row(int) const { return 0.f; }
    __device__ __forceinline__ void store(int c, int n, float v, float, float) const {
        if (n < N && c < own_rows) part[(int64_t)c * N + n] = v;
    }
};
// Row-block products run as persistent workgroups: the launch has at most as many workgroups as the
// chip holds at once (the host only knows an upper bound on the rows; workgroups without a tile
// would otherwise queue behind the working ones and drain after them) and each walks the tiles
// gid = blockIdx.x, + gridDim.x, ...  The id is decoded so that the column tiles of one row block
// run on the same XCD (workgroups are dealt round-robin to the 8 XCDs) and share its L2.
template <class T>
__device__ __forceinline__ bool next_tile(int gid, int tiles_m, int tiles_n, int &m0, int &n0) {
    const int xcd = gid & 7, j = gid >> 3;
    const int tm = (j / tiles_n) * 8 + xcd;
    m0 = tm * T::BM; n0 = (j % tiles_n) * T::BN;
    return tm < tiles_m;
}

// Split-K geometry of the weight-gradient product, decided on the device from the actual number
// of destination rows n1: as many chunks (a multiple of 8, at most nchunk) as keep rows_min rows
// in each, every chunk a multiple of the k-tile.
__device__ __forceinline__ int grad_w_chunk_rows(int n1, int nchunk, int rows_min) {
    const int want = min(nchunk, max(8, ((n1 + rows_min - 1) / rows_min + 7) & ~7));
    const int per = (n1 + want - 1) / want;
    return max(BK, (per + BK - 1) & ~(BK - 1));
}

// Partial [dW_self; dW_neigh] = X^T * dZ and db = column sums of dZ over one chunk of destination
// rows (split-K).
// The output tiles of one chunk read the same slabs of X and dZ; the launch is one-dimensional and
// the workgroup id is decoded so that all tiles of a chunk land on the same XCD (workgroups are
// dealt round-robin to the 8 XCDs) and share its L2.  Partials go to a per-chunk slab; a
// fixed-order reduction follows (deterministic, no atomics).
template <class T, int VA, int VB>
__global__ __launch_bounds__(GNT) __attribute__((amdgpu_waves_per_eu(T::LEAN ? 6 : 2, T::LEAN ? 6 : 8))) void k_sage_grad_w(MatRows a, MatRows dz, EpiGradW epi, int nchunk,
                                                     int rows_min, int tiles_m, int tiles_n,
                                                     const GsLevelMeta *__restrict__ meta_up, int S) {
    const int n1 = meta_up->front_off[S];
    const int kchunk = grad_w_chunk_rows(n1, nchunk, rows_min);
    const int tiles = tiles_m * tiles_n;
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int tile = j % tiles, chunk = (j / tiles) * 8 + xcd;
    const int k_begin = chunk * kchunk;
    if (k_begin >= n1) return;
    a.rows = n1; dz.rows = n1;
    const int k_end = min(n1, k_begin + kchunk);
    epi.part += (int64_t)chunk * epi.rows * epi.N;
    gemm_tile<T, false, false, VA, VB, MatRows, MatRows, EpiGradW, false, true>(
        (tile % tiles_m) * T::BM, (tile / tiles_m) * T::BN, a.cols, dz.cols, k_begin, k_end, a, dz, epi);
}

constexpr int GRAD_W_ROWS_MIN = 256;

inline bool few_rows(int64_t ub, int n_out, int k) {
    return ub * gs_ceil_div(n_out, 128) <= 16384 && (k >= 384 || k <= 64);
}

// persistent launch: no more workgroups than the chip holds, a multiple of 8
template <class T>
unsigned row_block_grid(const gsplit_ctx *ctx, int64_t ub, int n_out) {
    const int64_t want = gs_ceil_div(gs_ceil_div(ub, T::BM), 8) * 8 * gs_ceil_div(n_out, T::BN);
    return (unsigned)std::min<int64_t>(want, (int64_t)ctx->n_cu * T::OCC / 8 * 8);
}
// vin / vdz: rows of the layer input / of dZ can be read in 16-byte pieces
template <class T, int VA, int VB>
void launch_grad_w_t(hipStream_t st, int nchunk, const MatRows &in, const MatRows &dz, const EpiGradW &ew,
                     const GsLevelMeta *mu, int S) {
    const int tm = (int)gs_ceil_div(ew.own_rows, T::BM), tn = (int)gs_ceil_div(ew.N, T::BN);
    hipLaunchKernelGGL((k_sage_grad_w<T, VA, VB>), dim3((unsigned)(nchunk * tm * tn)), dim3(GNT), 0, st, in, dz,
                       ew, nchunk, GRAD_W_ROWS_MIN, tm, tn, mu, S);
}
template <class T = TileMidLean>
void launch_grad_w(hipStream_t st, int nchunk, bool vin, bool vdz, const MatRows &in, const MatRows &dz,
                   const EpiGradW &ew, const GsLevelMeta *mu, int S) {
    if (vin && vdz) launch_grad_w_t<T, 4, 4>(st, nchunk, in, dz, ew, mu, S);
    else if (vin) launch_grad_w_t<T, 4, 1>(st, nchunk, in, dz, ew, mu, S);
    else if (vdz) launch_grad_w_t<T, 1, 4>(st, nchunk, in, dz, ew, mu, S);
    else launch_grad_w_t<T, 1, 1>(st, nchunk, in, dz, ew, mu, S);
}

