// Context life cycle, workspace sizing and the read-only views of the current batch.
#include <algorithm>
#include <cstdlib>
#include <cstring>

#include "gsplit_internal.h"

static thread_local std::string g_create_error;

int gs_fail(gsplit_ctx *ctx, int code, const std::string &msg) {
    if (ctx) ctx->err = msg;
    else g_create_error = msg;
    return code;
}

int gs_alloc(gsplit_ctx *ctx, void **p, size_t bytes, const char *what) {
    *p = nullptr;
    if (bytes == 0) bytes = 256;
    hipError_t e = hipMalloc(p, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return gs_fail(ctx, GSPLIT_ENOMEM, std::string("hipMalloc failed for ") + what + " (" +
                                               std::to_string(bytes) + " bytes)");
    }
    ctx->allocs.push_back(*p);
    return GSPLIT_OK;
}

// Gives one of the context's buffers back (hipFree waits for the device, so no kernel still uses it).
void gs_release(gsplit_ctx *ctx, void **p) {
    if (!*p) return;
    auto it = std::find(ctx->allocs.begin(), ctx->allocs.end(), *p);
    if (it != ctx->allocs.end()) ctx->allocs.erase(it);
    (void)hipFree(*p);
    *p = nullptr;
}

static void free_all(gsplit_ctx *ctx) {
    for (auto &r : ctx->timer.pending) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (hipEvent_t e : ctx->timer.pool) (void)hipEventDestroy(e);
    ctx->timer.pending.clear();
    ctx->timer.pool.clear();
    for (void *p : ctx->allocs) (void)hipFree(p);
    ctx->allocs.clear();
    if (ctx->sample_done) (void)hipEventDestroy(ctx->sample_done);
    ctx->sample_done = nullptr;
}

// Direct tables take 8 bytes per key of the whole key space; the hashed ones 8 bytes per entry of a
// table sized for the largest layer.  Measured: direct tables shorten the sampler of a layer (one atomic
// per insert, no probing) as long as their key space stays inside the memory-side cache (256 MB); over a
// key space of GBs every lookup of the later passes misses it, and the hashed tables, which are
// compact, win.
static bool direct_tables_pay(int64_t keys_m, int64_t tab_cap) {
    (void)tab_cap;
    return keys_m * 8 <= (128ll << 20);
}

static int64_t pow2_at_least(int64_t x) {
    int64_t p = 1024;
    while (p < x) p <<= 1;
    return p;
}

extern "C" int gsplit_create(gsplit_ctx **out, const gsplit_graph *g, const gsplit_config *c) {
    if (!out || !g || !c) return gs_fail(nullptr, GSPLIT_EINVAL, "gsplit_create: NULL argument");
    if (g->n_vertices <= 0 || g->n_vertices >= (1ll << 31) || g->n_edges < 0 || !g->d_indptr ||
        (g->n_edges > 0 && !g->d_indices) || !g->d_pmap)
        return gs_fail(nullptr, GSPLIT_EINVAL, "gsplit_create: bad graph");
    if (g->n_splits < 1 || g->n_splits > GSPLIT_MAX_SPLITS)
        return gs_fail(nullptr, GSPLIT_EINVAL, "gsplit_create: n_splits out of range");
    if ((unsigned long long)g->n_vertices * (unsigned long long)g->n_splits >= 0xFFFFFFFFull)
        return gs_fail(nullptr, GSPLIT_ECAPACITY, "gsplit_create: n_vertices * n_splits must be < 2^32 - 1");
    if (c->n_layers < 1 || c->n_layers > GSPLIT_MAX_LAYERS || !c->fanouts || c->max_targets < 1)
        return gs_fail(nullptr, GSPLIT_EINVAL, "gsplit_create: bad config");
    for (int l = 0; l < c->n_layers; ++l)
        if (c->fanouts[l] < 1 || c->fanouts[l] > GSPLIT_MAX_FANOUT)
            return gs_fail(nullptr, GSPLIT_EINVAL, "gsplit_create: fanout out of range");
    if (c->max_targets > g->n_vertices)
        return gs_fail(nullptr, GSPLIT_EINVAL, "gsplit_create: max_targets exceeds n_vertices");

    gsplit_ctx *ctx = new (std::nothrow) gsplit_ctx();
    if (!ctx) return gs_fail(nullptr, GSPLIT_ENOMEM, "gsplit_create: host allocation failed");
    ctx->graph = *g;
    ctx->L = c->n_layers;
    ctx->S = g->n_splits;
    ctx->max_targets = c->max_targets;
    ctx->keep_edge_ids = c->keep_edge_ids != 0;
    ctx->gat_index = c->gat_index != 0;
    ctx->sampler_blocks_per_cu = c->sampler_blocks_per_cu > 0 ? std::min(c->sampler_blocks_per_cu, 8) : 8;
    ctx->rev_from = ctx->gat_index ? 0 : 1;
    for (int l = 0; l < ctx->L; ++l) ctx->fan[l] = c->fanouts[l];

    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        delete ctx;
        return gs_fail(nullptr, GSPLIT_EHIP, "gsplit_create: no HIP device");
    }
    ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

    // no-dedup upper bounds on the frontier sizes
    const int L = ctx->L;
    ctx->ub_front[L] = c->max_targets;
    int64_t tab_cap = 1024, max_items = 1024;
    for (int l = L - 1; l >= 0; --l) {
        const int64_t grown = ctx->ub_front[l + 1] * (1 + ctx->fan[l]);
        max_items = std::max(max_items, grown);
        ctx->ub_front[l] = std::min<int64_t>(g->n_vertices, grown);
        if (grown >= (1ll << 29)) {
            delete ctx;
            return gs_fail(nullptr, GSPLIT_ECAPACITY, "gsplit_create: frontier bound exceeds 2^29 slots");
        }
        tab_cap = std::max(tab_cap, pow2_at_least(2 * grown));
    }
    ctx->tab_cap = tab_cap;

    int rc = GSPLIT_OK;
    auto A = [&](void **p, size_t bytes, const char *what) {
        if (rc == GSPLIT_OK) rc = gs_alloc(ctx, p, bytes, what);
    };
    for (int l = 0; l <= L; ++l) A((void **)&ctx->front[l], sizeof(int32_t) * ctx->ub_front[l], "front");
    A((void **)&ctx->target_perm, sizeof(int32_t) * ctx->ub_front[L], "target_perm");
    for (int l = 0; l < L; ++l) {
        GsLayerBuf &B = ctx->layer[l];
        const int64_t nd = ctx->ub_front[l + 1], f = ctx->fan[l];
        A((void **)&B.nbr, sizeof(int32_t) * nd * f, "nbr");
        if (ctx->keep_edge_ids) A((void **)&B.epos, sizeof(int64_t) * nd * f, "edge positions");
        A((void **)&B.cnt, sizeof(int32_t) * nd, "cnt");
        A((void **)&B.mixed, sizeof(int32_t) * nd * (1 + f), "mixed");
        A((void **)&B.blk_indptr, sizeof(int32_t) * (nd + 1), "blk_indptr");
        A((void **)&B.blk_src, sizeof(int32_t) * nd * f, "blk_src");
        A((void **)&B.recv, sizeof(int32_t) * nd * f, "recv");
        A((void **)&B.src_row, sizeof(int32_t) * nd * (1 + f), "src_row");
        A((void **)&B.self_row, sizeof(int32_t) * nd, "self_row");
        A((void **)&B.edge_row, sizeof(int32_t) * nd * f, "edge_row");
        if (l >= ctx->rev_from) {
            if (ctx->gat_index) A((void **)&B.rev_eid, sizeof(int32_t) * nd * (1 + f), "rev_eid");
            A((void **)&B.rev_cnt, sizeof(int32_t) * ctx->ub_front[l], "rev_cnt");
            A((void **)&B.rev_ptr, sizeof(int32_t) * ctx->ub_front[l], "rev_ptr");
            A((void **)&B.rev_fill, sizeof(int32_t) * ctx->ub_front[l], "rev_fill");
            A((void **)&B.rev_list, sizeof(int32_t) * nd * (1 + f), "rev_list");
            A((void **)&B.rev_long, sizeof(int32_t) * (nd * (1 + f) / GS_REV_LONG + 1), "rev_long");
        }
    }
    A((void **)&ctx->d_meta, sizeof(GsLevelMeta) * (L + 1), "meta");
    // one split: the (vertex, split) key is the vertex key (direct form: one table under both names)
    const int64_t keys_m = g->n_vertices * (int64_t)g->n_splits;
    int table_mode = c->table_mode;
    if (table_mode == 0) {      // (GSPLIT_TABLE_MODE in the environment decides where the configuration leaves the choice open)
        if (const char *e = std::getenv("GSPLIT_TABLE_MODE")) {
            const long v = std::strtol(e, nullptr, 10);
            if (v == 1 || v == 2) table_mode = (int)v;
        }
    }
    ctx->direct_tables = table_mode == 2 || (table_mode == 0 && direct_tables_pay(keys_m, tab_cap));
    if (ctx->direct_tables && keys_m >= (1ll << 30)) ctx->direct_tables = false;     // entry indices are 31-bit
    for (GsTable *t : {&ctx->tab_mixed, &ctx->tab_local}) {
        if (t == &ctx->tab_local && ctx->S == 1 && ctx->direct_tables) {
            *t = ctx->tab_mixed;
            break;
        }
        t->slot = nullptr; t->row = nullptr; t->pos = nullptr;
        if (ctx->direct_tables) {
            // (vertex, split) keys only: the entries of a vertex lie side by side, which answers the
            // questions a table keyed by the vertex alone would
            if (t == &ctx->tab_mixed) A((void **)&t->pos, sizeof(unsigned long long) * keys_m, "direct table entries");
        } else if (t == &ctx->tab_mixed) {
            // hashed by the vertex: the keys of a vertex share lines, which answers the same questions
            A((void **)&t->slot, sizeof(unsigned long long) * tab_cap, "table entries");
        }
        // rows are handed out by position in the slot stream, not by table entry
        A((void **)&t->row, sizeof(int32_t) * max_items, "rows by position");
    }
    A((void **)&ctx->ent_mixed, sizeof(int32_t) * max_items, "ent_mixed");
    A((void **)&ctx->ent_local, sizeof(int32_t) * max_items, "ent_local");
    A((void **)&ctx->mixed_ent, sizeof(int32_t) * max_items, "mixed_ent");
    A((void **)&ctx->cls, sizeof(uint32_t) * max_items, "class masks");
    if (const char *e = std::getenv("GSPLIT_WIDE_SLOTS")) {
        const long long v = std::strtoll(e, nullptr, 10);
        if (v >= 1) ctx->wide_slots = v;
    }
    bool any_wide = false;
    for (int l = 0; l < L; ++l) any_wide = any_wide || ctx->ub_front[l + 1] * ctx->fan[l] >= ctx->wide_slots;
    if (any_wide) {
        A((void **)&ctx->pos_pair, sizeof(int32_t) * 2 * max_items, "row pairs by position");
        A((void **)&ctx->mixed_pos, sizeof(int32_t) * max_items, "positions of mixed rows");
    }
    A((void **)&ctx->part_hist, sizeof(int32_t) * 1024 * 25, "partition histogram");
    A((void **)&ctx->part_base, sizeof(int32_t) * 1024 * 25, "partition bases");
    if (rc == GSPLIT_OK && hipMemset(ctx->d_meta, 0, sizeof(GsLevelMeta) * (L + 1)) != hipSuccess)
        rc = gs_fail(ctx, GSPLIT_EHIP, "gsplit_create: hipMemset failed");
    // every table entry empty (all bits set): a batch starts on clean tables, and leaves them so
    for (GsTable *t : {&ctx->tab_mixed, &ctx->tab_local}) {
        if (rc != GSPLIT_OK) break;
        if (ctx->direct_tables ? !t->pos : !t->slot) continue;
        if (t == &ctx->tab_local && t->slot == ctx->tab_mixed.slot && t->pos == ctx->tab_mixed.pos) continue;   // one split: one table
        const hipError_t e = ctx->direct_tables ? hipMemset(t->pos, 0xFF, sizeof(unsigned long long) * keys_m)
                                                : hipMemset(t->slot, 0xFF, sizeof(unsigned long long) * tab_cap);
        if (e != hipSuccess) rc = gs_fail(ctx, GSPLIT_EHIP, "gsplit_create: hipMemset failed");
    }
    if (rc == GSPLIT_OK && hipEventCreateWithFlags(&ctx->sample_done, hipEventDisableTiming) != hipSuccess)
        rc = gs_fail(ctx, GSPLIT_EHIP, "gsplit_create: hipEventCreate failed");
    if (rc != GSPLIT_OK) {
        g_create_error = ctx->err;
        free_all(ctx);
        delete ctx;
        return rc;
    }
    std::memset(ctx->h_meta, 0, sizeof(ctx->h_meta));
    *out = ctx;
    return GSPLIT_OK;
}

extern "C" int gsplit_destroy(gsplit_ctx *ctx) {
    if (!ctx) return GSPLIT_OK;
    (void)hipDeviceSynchronize();
    free_all(ctx);
    delete ctx;
    return GSPLIT_OK;
}

extern "C" const char *gsplit_last_error(const gsplit_ctx *ctx) {
    return ctx ? ctx->err.c_str() : g_create_error.c_str();
}

extern "C" int64_t gsplit_max_rows(const gsplit_ctx *ctx, int32_t level) {
    if (!ctx || level < 0 || level > ctx->L) return GSPLIT_EINVAL;
    return ctx->ub_front[level];
}

static int fetch_meta(gsplit_ctx *ctx) {
    if (ctx->h_meta_valid) return GSPLIT_OK;
    if (ctx->batch_id == 0) return gs_fail(ctx, GSPLIT_ESTATE, "no batch has been sampled yet");
    // a captured batch has no event and changes with every replay of its graph: wait for the device
    // and read the sizes again on every call
    if (ctx->captured) GS_HIP(ctx, hipDeviceSynchronize());
    else GS_HIP(ctx, hipEventSynchronize(ctx->sample_done));
    GS_HIP(ctx, hipMemcpy(ctx->h_meta, ctx->d_meta, sizeof(GsLevelMeta) * (ctx->L + 1),
                          hipMemcpyDeviceToHost));
    if (ctx->h_meta[ctx->L].error != 0)
        return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_sample_split: a target id lies outside the graph");
    for (int l = 0; l < ctx->L; ++l)
        if (ctx->h_meta[l].error != 0)
            return gs_fail(ctx, GSPLIT_ESTATE, "internal: hash table probe failed at layer " +
                                                   std::to_string(l));
    ctx->h_meta_valid = !ctx->captured;
    return GSPLIT_OK;
}

extern "C" int gsplit_batch_sizes(gsplit_ctx *ctx, int64_t *n_local, int64_t *n_mixed,
                                  int64_t *n_edges, int64_t *bucket) {
    if (!ctx) return GSPLIT_EINVAL;
    int rc = fetch_meta(ctx);
    if (rc != GSPLIT_OK) return rc;
    const int S = ctx->S, L = ctx->L;
    std::vector<int32_t> indptr_at;  // block CSR offsets at the split boundaries
    for (int l = 0; l <= L; ++l)
        for (int s = 0; s < S; ++s)
            if (n_local) n_local[l * S + s] = ctx->h_meta[l].front_off[s + 1] - ctx->h_meta[l].front_off[s];
    for (int l = 0; l < L; ++l) {
        for (int s = 0; s < S; ++s) {
            if (n_mixed) n_mixed[l * S + s] = ctx->h_meta[l].mixed_off[s + 1] - ctx->h_meta[l].mixed_off[s];
            if (bucket) {
                // bucket[s->t] runs from its start to the start of the next non-empty sender
                const GsLevelMeta &m = ctx->h_meta[l];
                const bool empty = m.mixed_off[s + 1] == m.mixed_off[s];
                int nxt = s + 1;
                while (nxt < S && m.mixed_off[nxt + 1] == m.mixed_off[nxt]) ++nxt;
                for (int t = 0; t < S; ++t) {
                    const int end = nxt < S ? m.bucket_start[nxt * GS_MAXS + t] : m.recv_off[t + 1];
                    bucket[(l * S + s) * S + t] = empty ? 0 : end - m.bucket_start[s * GS_MAXS + t];
                }
            }
        }
        if (n_edges) {
            int32_t cut[GS_MAXS + 1];
            for (int s = 0; s <= S; ++s)
                GS_HIP(ctx, hipMemcpy(&cut[s], ctx->layer[l].blk_indptr + ctx->h_meta[l + 1].front_off[s],
                                      sizeof(int32_t), hipMemcpyDeviceToHost));
            for (int s = 0; s < S; ++s) n_edges[l * S + s] = cut[s + 1] - cut[s];
        }
    }
    return GSPLIT_OK;
}

extern "C" int gsplit_batch_level(const gsplit_ctx *ctx, int32_t level, gsplit_level_view *out) {
    if (!ctx || !out || level < 0 || level > ctx->L) return GSPLIT_EINVAL;
    out->d_local_cat = ctx->front[level];
    out->d_local_off = ctx->d_meta[level].front_off;
    return GSPLIT_OK;
}

extern "C" int gsplit_batch_layer(const gsplit_ctx *ctx, int32_t layer, gsplit_layer_view *out) {
    if (!ctx || !out || layer < 0 || layer >= ctx->L) return GSPLIT_EINVAL;
    const GsLayerBuf &B = ctx->layer[layer];
    out->d_nbr = B.nbr;
    out->d_cnt = B.cnt;
    out->d_mixed_cat = B.mixed;
    out->d_mixed_off = ctx->d_meta[layer].mixed_off;
    out->d_blk_indptr = B.blk_indptr;
    out->d_blk_src = B.blk_src;
    out->d_shuffle_src_row = B.src_row;
    out->d_recv_cat = B.recv;
    out->d_recv_off = ctx->d_meta[layer].recv_off;
    return GSPLIT_OK;
}

extern "C" int gsplit_batch_shuffle(const gsplit_ctx *ctx, int32_t layer, gsplit_shuffle_view *out) {
    if (!ctx || !out || layer < 0 || layer >= ctx->L) return GSPLIT_EINVAL;
    const GsLayerBuf &B = ctx->layer[layer];
    out->d_self_row = B.self_row;
    out->d_edge_row = B.edge_row;
    out->d_rev_ptr = B.rev_ptr;
    out->d_rev_cnt = B.rev_cnt;
    out->d_rev_list = B.rev_list;
    out->d_rev_eid = B.rev_eid;
    return GSPLIT_OK;
}

extern "C" int gsplit_sage_activations(const gsplit_ctx *ctx, int32_t level, const void **d_act) {
    if (!ctx || !d_act || level < 1 || level >= ctx->L) return GSPLIT_EINVAL;
    const GsSageBuf &sb = ctx->sage;
    // (the activations below the top level are there after a forward pass or a whole step on this batch)
    if (!sb.ready || sb.fwd_batch != ctx->batch_id) return GSPLIT_ESTATE;
    *d_act = sb.hidden[level];
    return GSPLIT_OK;
}

extern "C" int gsplit_timing_enable(gsplit_ctx *ctx, int32_t enable) {
    if (!ctx) return GSPLIT_EINVAL;
    ctx->timer.enabled = enable != 0;
    return GSPLIT_OK;
}

// about 20 us of waiting on the 100 MHz wall clock (the loop is bounded by its iteration count too)
__global__ void k_timing_probe(int ticks) {
    const long long t0 = wall_clock64();
    for (int i = 0; i < 100000 && wall_clock64() - t0 < ticks; ++i) __builtin_amdgcn_s_sleep(8);
}

// What an event pair adds to the kernel it brackets: (a bracketed kernel) - (the same kernel at
// back-to-back rate), for a kernel about as long as the ones that matter (part of the event's own
// processing hides behind a running kernel, so an empty kernel would overstate it).  Measured once
// per context, on the stream of the last batch.
static double timing_overhead_ms(gsplit_ctx *ctx) {
    GsTimer &t = ctx->timer;
    if (t.overhead_ms >= 0.0) return t.overhead_ms;
    hipStream_t st = ctx->last_stream;
    hipEvent_t a = nullptr, b = nullptr;
    double ovh = 0.0;
    if (hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess) {
        const int reps = 16, burst = 32, ticks = 2000;
        double bracket = 0.0;
        int got = 0;
        hipLaunchKernelGGL(k_timing_probe, dim3(1), dim3(64), 0, st, ticks);
        for (int i = 0; i < reps; ++i) {
            float ms = 0.f;
            (void)hipEventRecord(a, st);
            hipLaunchKernelGGL(k_timing_probe, dim3(1), dim3(64), 0, st, ticks);
            (void)hipEventRecord(b, st);
            if (hipEventSynchronize(b) == hipSuccess && hipEventElapsedTime(&ms, a, b) == hipSuccess) { bracket += ms; ++got; }
        }
        float total = 0.f;
        (void)hipEventRecord(a, st);
        for (int i = 0; i < burst; ++i) hipLaunchKernelGGL(k_timing_probe, dim3(1), dim3(64), 0, st, ticks);
        (void)hipEventRecord(b, st);
        if (got == reps && hipEventSynchronize(b) == hipSuccess && hipEventElapsedTime(&total, a, b) == hipSuccess) {
            bracket /= reps;
            const double each = (total - bracket) / (burst - 1);
            ovh = std::min(0.01, std::max(0.0, bracket - each));
        }
    }
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
    (void)hipGetLastError();
    t.overhead_ms = ovh;
    return ovh;
}

extern "C" int64_t gsplit_timing_read(gsplit_ctx *ctx, char *buf, int64_t buf_bytes) {
    if (!ctx || !buf || buf_bytes < 1) return GSPLIT_EINVAL;
    GsTimer &t = ctx->timer;
    const double ovh = t.pending.empty() ? 0.0 : timing_overhead_ms(ctx);
    for (auto &r : t.pending) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
            t.total_ms[r.label] += std::max(0.0, (double)ms - ovh);
            t.count[r.label] += 1;
        }
        t.pool.push_back(r.a);
        t.pool.push_back(r.b);
    }
    t.pending.clear();
    std::string out;
    for (size_t i = 0; i < t.names.size(); ++i) {
        out += t.names[i] + " " + std::to_string(t.count[i]) + " " + std::to_string(t.total_ms[i]) + "\n";
        t.total_ms[i] = 0.0;
        t.count[i] = 0;
    }
    if ((int64_t)out.size() + 1 > buf_bytes) return gs_fail(ctx, GSPLIT_ECAPACITY, "gsplit_timing_read: buffer too small");
    std::memcpy(buf, out.c_str(), out.size() + 1);
    return (int64_t)out.size();
}
