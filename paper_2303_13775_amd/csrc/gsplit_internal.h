// Internal definitions shared by the HIP translation units of libgsplit (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "gsplit.h"

// a row of the reverse index with more entries than one wave holds in registers (four per lane) is a
// "long" row: the backward pass hands those to whole workgroups
#define GS_REV_LONG 256
#define GS_MAXS GSPLIT_MAX_SPLITS
// a sampling layer with at least this many slots (by its bound) is "wide": its relabelling runs as two
// launches, which cuts the dependent random accesses per slot from three to one
#define GS_WIDE_SLOTS (1ll << 20)
#define GS_MAXL GSPLIT_MAX_LAYERS

// Device-resident bookkeeping of one level l (0..L) of the current batch.  Every kernel reads its
// problem sizes from here, so a whole iteration is enqueued without a host round trip.
//   front_off : split offsets of local_cat[l]            (front_off[S] = |local_cat[l]|)
// and, for sampling layer l (expanding level l+1 into level l):
//   mixed_off : split offsets of the concatenated mixed frontiers
//   recv_off  : receiver offsets of the concatenated received buckets
//   bucket_start: where bucket[s->t] starts inside recv, at [s * GS_MAXS + t] (senders with an
//               empty mixed frontier are not written)
//   nnz       : number of sampled edges of the layer
struct GsLevelMeta {
    int32_t front_off[GS_MAXS + 1];
    int32_t mixed_off[GS_MAXS + 1];
    int32_t recv_off[GS_MAXS + 1];
    int32_t bucket_start[GS_MAXS * GS_MAXS];
    int32_t nnz;
    int32_t error;      // set non-zero by a kernel that hit an impossible state (probe overflow)
    int32_t rev_cursor; // allocation cursor of the reverse (scatter) index
    int32_t n_long;     // rows of the level with more than GS_REV_LONG entries in the reverse index
    uint32_t batches;   // (level 0 only) batches sampled by this context so far: the source of the direct tables' stamps
    int32_t pad[3];
};

// Dedup table in HBM, in one of two forms.
//   hashed: open addressing, entry = key << 32 | smallest position seen.  One table of
//   (vertex, split) keys, hashed by the vertex (tab_mixed; tab_local has a row array only).
//   direct (pos != nullptr): one 64-bit entry per possible key, indexed by the key itself: an insert
//   is a single atomic min, no probing, no key compare, and nothing is ever reset: the entry is
//   stamp << 32 | smallest position seen, where the stamp of a (batch, layer) is smaller than every
//   stamp before it, so whatever an older layer left behind loses against the first insert of the
//   current one.  Takes 8 bytes per key of the key space (|V| * S keys).
// row: the final row of a key, kept at the position of the key's first occurrence in the slot
// stream (one entry per element of the largest layer, whatever the form of the table).
struct GsTable {
    unsigned long long *slot;
    int32_t            *row;
    unsigned long long *pos;
};

struct GsLayerBuf {            // sampling layer l
    int32_t *nbr = nullptr;        // [ub_dst * fan]
    int64_t *epos = nullptr;       // [ub_dst * fan]  CSR position behind every slot (keep_edge_ids only)
    int32_t *cnt = nullptr;        // [ub_dst]
    int32_t *mixed = nullptr;      // [ub_dst * (1 + fan)]
    int32_t *blk_indptr = nullptr; // [ub_dst + 1]
    int32_t *blk_src = nullptr;    // [ub_dst * fan]
    int32_t *recv = nullptr;       // [ub_dst * fan]
    int32_t *src_row = nullptr;    // [ub_dst * (1 + fan)]
    int32_t *self_row = nullptr;   // [ub_dst]        row of local_cat[l] of each destination vertex
    int32_t *edge_row = nullptr;   // [ub_dst * fan]  row of local_cat[l] of each edge's source
    // reverse (scatter) index for the backward pass, layers l >= 1 only: for every row u of
    // local_cat[l] the destination rows whose input it feeds, as 2 * i (self) or 2 * i + 1 (edge)
    int32_t *rev_cnt = nullptr;    // [ub_front[l]]
    int32_t *rev_ptr = nullptr;    // [ub_front[l]]
    int32_t *rev_fill = nullptr;   // [ub_front[l]]
    int32_t *rev_list = nullptr;   // [ub_dst * (1 + fan)]
    int32_t *rev_eid = nullptr;    // [ub_dst * (1 + fan)]  edge number of an edge entry, -1 for a self entry (gat_index only)
    int32_t *rev_long = nullptr;   // [ub_dst * (1 + fan) / GS_REV_LONG + 1]  rows with more than GS_REV_LONG entries
};

struct GsSageBuf {             // activations kept between forward and backward
    bool     ready = false;
    int32_t  dtype = -1;
    int32_t  dims[GS_MAXL + 1] = {0};
    void    *hidden[GS_MAXL + 1] = {nullptr};   // local_cat activations of level 1..L-1
    void    *xin[GS_MAXL] = {nullptr};          // assembled layer inputs [rows x 2*dims[l]]: self | mean
    float   *ghid[GS_MAXL + 1] = {nullptr};     // d loss / d hidden of level 1..L
    float   *gtmp = nullptr;                    // [rows x 2*dim] input gradients before the reverse shuffle
    float   *inv_cnt[GS_MAXL] = {nullptr};      // 1 / (sampled neighbours) per destination row
    float   *wstack32[GS_MAXL] = {nullptr};     // fp32 [2D x Npad] stacked weights, Npad = N rounded up to 4
    uint16_t *wstack[GS_MAXL] = {nullptr};      // bf16 [2D x Npad] stacked weights (bf16 mode)
    uint16_t *wtrans[GS_MAXL] = {nullptr};      // bf16 [N x 2D] transposed stacked weights
    float   *gw_part[GS_MAXL] = {nullptr};      // per-chunk partial weight gradients
    int      nchunk[GS_MAXL] = {0};             // slabs of gw_part (multiple of 8)
    int      stream_nchunk[GS_MAXL] = {0};      // chunks of the streaming weight-gradient kernel
    int      stream_rows = 0;                   // rows of a level from which that kernel takes the weight gradients
    bool     gw_stream[GS_MAXL] = {false};      // the layer's weight gradients take the streaming bf16 kernel
    int      top_chunks = 0;                    // workgroups (= slabs) of the fused top-layer kernel
    float   *glog = nullptr;                    // [n_targets x classes] loss gradient of gsplit_sage_step
    bool     fwd_done = false;
    uint64_t fwd_batch = 0;
};

struct GsGatBuf {              // GAT: what the forward pass keeps for the backward pass, and scratch
    bool     ready = false;
    int32_t  dims[GS_MAXL + 1] = {0};
    int32_t  heads[GS_MAXL] = {0};
    float   *wext[GS_MAXL] = {nullptr};      // [D x ZW]  W | W a_src | W a_dst | zero padding
    float   *zext[GS_MAXL] = {nullptr};      // [rows of level l x ZW]  z | a_src . z | a_dst . z | padding
    float   *alpha[GS_MAXL] = {nullptr};     // [(ub_dst * fan + ub_dst) x K]  edge slots, then self slots
    float   *de[GS_MAXL] = {nullptr};        // same shape: d loss / d (score before the LeakyReLU)
    float   *der[GS_MAXL] = {nullptr};       // [ub_dst x K]  sum of de over a destination's entries
    float   *gagg[GS_MAXL] = {nullptr};      // [ub_dst x K F]  d loss / d (aggregated heads)
    float   *dzext[GS_MAXL] = {nullptr};     // [rows of level l x ZW]  gradient of zext
    float   *hidden[GS_MAXL + 1] = {nullptr};
    float   *ghid[GS_MAXL + 1] = {nullptr};
    float   *gw_part[GS_MAXL] = {nullptr};   // split-K slabs of X^T dzext
    int      nchunk[GS_MAXL] = {0};
    float   *gmat[GS_MAXL] = {nullptr};      // [D x ZW]  X^T dzext
    float   *bias_part[GS_MAXL] = {nullptr}; // [bias_slabs x dims[l+1]]
    int      bias_slabs[GS_MAXL] = {0};
    // bottom layer run as aggregate-then-transform (no zext / dzext / de / der / gw_part for layer 0)
    bool     agg_first = false;
    float   *s0 = nullptr;                   // [rows of level 0 x 2 K]  h . (W a_src) | h . (W a_dst)
    float   *pagg = nullptr;                 // [ub_dst x K x D]  sum_j alpha_ij^k h_j
    float   *dpagg = nullptr;                // [ub_dst x K x D]  its gradient
    float   *q_part = nullptr;               // [q_slabs x 2 K x D]  per-wave sums of d e h
    int      q_blocks = 0;
    float   *w0_part = nullptr;              // [nchunk0 x K x D x F]  split-K slabs of P^kT dagg^k
    int      nchunk0 = 0;
    bool     fwd_done = false;
    uint64_t fwd_batch = 0;
};

struct GsFeatureCache {        // static input-feature cache aligned with f_G
    bool        ready = false;
    const void *table = nullptr;   // full table as the device reads it (pinned host or device memory)
    int32_t     dtype = 0;
    int64_t     dim = 0, row_stride_bytes = 0, n_rows = 0;
    int32_t    *slot_of = nullptr; // [n_vertices]  cache row of the vertex, or -1
    void       *rows = nullptr;    // [n_rows x dim]
    int32_t    *d_err = nullptr;
};

// Optional per-kernel device timing: when enabled, every kernel launch is bracketed by two events
// on its stream; gsplit_timing_read() waits for them and reports totals per label.
struct GsTimer {
    struct Rec { int label; hipEvent_t a, b; };
    bool enabled = false;
    double overhead_ms = -1.0;     // what an event pair adds to a bracketed kernel; < 0: not measured yet
    std::vector<std::string> names;
    std::vector<double> total_ms;
    std::vector<int64_t> count;
    std::vector<Rec> pending;
    std::vector<hipEvent_t> pool;
};

struct gsplit_ctx {
    gsplit_graph graph;
    int32_t  L = 0, S = 0;
    int32_t  fan[GS_MAXL] = {0};
    int64_t  max_targets = 0;
    bool     keep_edge_ids = false;
    bool     gat_index = false;
    int      sampler_blocks_per_cu = 8;    // cap on the grids of the sampling and index kernels
    bool     direct_tables = false;    // dedup tables indexed by the key itself (see GsTable)
    int      rev_from = 1;             // lowest sampling layer with a reverse index (0 with gat_index)
    int64_t  ub_front[GS_MAXL + 1] = {0};   // upper bounds on |local_cat[l]|
    int      n_cu = 256;

    int32_t     *front[GS_MAXL + 1] = {nullptr};
    int32_t     *target_perm = nullptr;
    GsLayerBuf   layer[GS_MAXL];
    GsLevelMeta *d_meta = nullptr;          // [L + 1]
    GsLevelMeta  h_meta[GS_MAXL + 1];
    bool         h_meta_valid = false;
    GsTable      tab_local, tab_mixed;
    int64_t      tab_cap = 0;
    // per-element scratch of the current sampling layer (sized for the largest layer):
    int32_t     *ent_mixed = nullptr;       // tab_mixed entry of each destination / slot
    int32_t     *ent_local = nullptr;       // tab_local entry of each destination / received id
    int32_t     *mixed_ent = nullptr;       // tab_local entry of each mixed-frontier row
    uint32_t    *cls = nullptr;             // class mask left by a count pass for its scatter pass
    // wide layers only (contexts that have one): per position of a key's first occurrence the pair
    // (row in the split's mixed frontier, row in local_cat), and per mixed-frontier row that position
    int32_t     *pos_pair = nullptr;        // [2 * max_items]
    int32_t     *mixed_pos = nullptr;       // [max_items]
    int64_t      wide_slots = GS_WIDE_SLOTS; // the bar in force (GSPLIT_WIDE_SLOTS in the environment moves it: tests)
    int32_t     *part_hist = nullptr;       // partition scratch
    int32_t     *part_base = nullptr;

    uint64_t     batch_id = 0;
    bool         captured = false;          // the current batch was enqueued under stream capture
    int64_t      n_targets = 0;
    hipStream_t  last_stream = nullptr;
    hipEvent_t   sample_done = nullptr;

    GsSageBuf    sage;
    GsGatBuf     gat;
    GsFeatureCache cache;
    GsTimer      timer;
    std::vector<void *> allocs;
    std::string  err;
};

int gs_fail(gsplit_ctx *ctx, int code, const std::string &msg);
int gs_alloc(gsplit_ctx *ctx, void **p, size_t bytes, const char *what);
void gs_release(gsplit_ctx *ctx, void **p);

#define GS_HIP(ctx, call)                                                                  \
    do {                                                                                   \
        hipError_t e__ = (call);                                                           \
        if (e__ != hipSuccess)                                                             \
            return gs_fail((ctx), GSPLIT_EHIP, std::string(#call) + ": " + hipGetErrorString(e__)); \
    } while (0)

// brackets the launches issued during its lifetime (exactly one kernel per scope) when timing is on
struct GsTimeScope {
    gsplit_ctx *ctx; hipStream_t st; int label; hipEvent_t a;
    GsTimeScope(gsplit_ctx *c, const char *name, int layer, hipStream_t s) : ctx(c), st(s), label(-1), a(nullptr) {
        if (!c->timer.enabled || c->captured) return;
        GsTimer &t = c->timer;
        std::string full = layer >= 0 ? std::string(name) + ".l" + std::to_string(layer) : std::string(name);
        for (size_t i = 0; i < t.names.size(); ++i)
            if (t.names[i] == full) { label = (int)i; break; }
        if (label < 0) {
            label = (int)t.names.size();
            t.names.push_back(full); t.total_ms.push_back(0.0); t.count.push_back(0);
        }
        a = take();
        if (a) (void)hipEventRecord(a, st);
    }
    ~GsTimeScope() {
        if (label < 0 || !a) return;
        hipEvent_t b = take();
        if (!b) return;
        (void)hipEventRecord(b, st);
        ctx->timer.pending.push_back({label, a, b});
    }
    hipEvent_t take() {
        GsTimer &t = ctx->timer;
        if (!t.pool.empty()) { hipEvent_t e = t.pool.back(); t.pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
};

static inline int64_t gs_ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

static inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// one-dimensional grid of 256-thread workgroups for grid-stride kernels: enough for upper_threads,
// at most eight workgroups per compute unit
static inline int grid_1d(const gsplit_ctx *ctx, int64_t upper_threads) {
    const int64_t want = gs_ceil_div(upper_threads, 256);
    const int64_t cap = (int64_t)ctx->n_cu * 8;
    return (int)(want < 1 ? 1 : want > cap ? cap : want);
}
