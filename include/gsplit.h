/*
 * gsplit.h -- C ABI of the MI355X (gfx950) split-parallel mini-batch hot path.
 *
 * One GPU's share of a GSplit training iteration (paper sections 3-5): fanout neighbour sampling
 * layer by layer, online splitting of every sampled vertex through the precomputed global
 * partition function f_G, per-split dedup/relabel and shuffle-index construction
 * (Algorithm 1, `sp_sample`), loading of the layer-0 input features (section 3, "loading step"),
 * and the GraphSAGE forward and backward passes over the split mini-batch (Algorithm 2,
 * `sp_forward`, and the backward description after it).  The S splits that the paper places on S
 * GPUs are S *logical* splits on this one GPU; the per-layer all-to-all shuffles become index
 * permutations between them.
 *
 * Conventions
 *  - Every `d_*` pointer is a DEVICE pointer owned by the CALLER.  The library never frees or
 *    reallocates caller memory; caller memory must stay valid until the stream work that uses it
 *    has completed.  Pointers without the prefix are HOST pointers.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *    enqueued on it; calls return without waiting unless stated otherwise.
 *  - Every function returns 0 (GSPLIT_OK) or a negative error code.  No exceptions, no abort,
 *    nothing printed.  After an error the outputs are unspecified, the context stays usable, and
 *    gsplit_last_error() describes what went wrong.
 *  - A context is not thread-safe; calls on one context must be issued from one thread at a
 *    time and on one stream at a time.
 *  - Layer numbering follows Algorithm 1: local_front[L] are the targets, sampling layer l
 *    (l = L-1 .. 0) expands local_front[l+1] into layer l using fanouts[l]; forward layer l
 *    (l = 0 .. L-1) maps width dims[l] to dims[l+1].
 *  - "cat" arrays hold the S splits one after the other in split order.
 */
#ifndef GSPLIT_H
#define GSPLIT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GSPLIT_API __attribute__((visibility("default")))

#define GSPLIT_OK          0
#define GSPLIT_EINVAL     -1   /* bad argument */
#define GSPLIT_ENOMEM     -2   /* device or host allocation failed */
#define GSPLIT_ECAPACITY  -3   /* input larger than what the context was created for */
#define GSPLIT_EHIP       -4   /* a HIP runtime call failed */
#define GSPLIT_ESTATE     -5   /* call out of order (e.g. backward without forward) */

#define GSPLIT_MAX_SPLITS  8
#define GSPLIT_MAX_LAYERS  8
#define GSPLIT_MAX_FANOUT  64
#define GSPLIT_MAX_MULTI   8    /* mini-batches one gsplit_sample_split_multi call can take */

#define GSPLIT_F32   0
#define GSPLIT_BF16  1

typedef struct gsplit_ctx gsplit_ctx;

/* The graph G(V_G, E_G) and the global partition function f_G (section 4).  Row v of the CSR
 * lists the vertices v aggregates from; rows must be free of duplicates.  All arrays stay
 * caller-owned and must outlive the context. */
typedef struct {
    int64_t        n_vertices;      /* |V_G|;  n_vertices * n_splits must be < 2^32 - 1 */
    int64_t        n_edges;         /* number of CSR entries, < 2^40 */
    const void    *d_indptr;        /* [n_vertices + 1], int32 or int64 */
    int32_t        indptr_is_64;    /* 0: int32 indptr, 1: int64 indptr */
    const int32_t *d_indices;       /* [n_edges] */
    const uint8_t *d_pmap;          /* f_G: [n_vertices], values in [0, n_splits) */
    int32_t        n_splits;        /* S, 1 .. GSPLIT_MAX_SPLITS */
} gsplit_graph;

typedef struct {
    int32_t        n_layers;        /* L, 1 .. GSPLIT_MAX_LAYERS */
    const int32_t *fanouts;         /* HOST array [L]; fanouts[l] in 1 .. GSPLIT_MAX_FANOUT */
    int64_t        max_targets;     /* largest n_targets any gsplit_sample_split call will pass */
    int32_t        keep_edge_ids;   /* 1: the sampler also records the CSR position of every sampled
                                       edge (8 bytes per slot), which gsplit_presample_accumulate needs */
    int32_t        gat_index;       /* 1: the scatter side of the shuffle index is also built for the bottom
                                       layer and carries edge ids, which gsplit_gat_bwd needs */
    int32_t        sampler_blocks_per_cu; /* 0 or 1..8: workgroups per compute unit the sampling and index
                                       kernels may occupy (default 8 = all wave slots: fastest alone).  A caller
                                       that overlaps sampling with training on another stream does better with
                                       2: the latency-bound sampling kernels then leave room for the training
                                       kernels' workgroups */
    int32_t        table_mode;      /* dedup tables of the split step: 0 = the library chooses, 1 = hashed (open
                                       addressing, sized for the largest layer), 2 = direct (indexed by the key
                                       itself: 8 bytes per vertex and split, one atomic per
                                       insert; needs n_vertices * n_splits < 2^30).  Same results either way */
} gsplit_config;

/* Creates a context on the current HIP device and allocates its workspace, sized from the
 * no-dedup upper bounds |F_l| <= min(|V|, |F_{l+1}| * (1 + fanouts[l])).  ENOMEM if it does not
 * fit.  *out is set only on success. */
GSPLIT_API int gsplit_create(gsplit_ctx **out, const gsplit_graph *graph, const gsplit_config *config);

/* Waits for the device, then frees everything the context owns.  NULL is accepted. */
GSPLIT_API int gsplit_destroy(gsplit_ctx *ctx);

/* Message for the most recent error on this context (context-owned, valid until the next call);
 * with ctx == NULL, the message of the most recent failed gsplit_create on this thread. */
GSPLIT_API const char *gsplit_last_error(const gsplit_ctx *ctx);

/* Upper bound on the number of rows of local_cat[level] (level 0 .. L) that any batch of this
 * context can have; callers size gather and activation buffers with it.  Returns the bound or a
 * negative error code. */
GSPLIT_API int64_t gsplit_max_rows(const gsplit_ctx *ctx, int32_t level);

/* Algorithm 1 for all S splits at once.
 *   d_targets [n_targets]: DISTINCT vertex ids of the mini-batch (all splits' local_targets
 *   together; the library separates them by f_G keeping the given order).
 * For l = L-1 .. 0: sample_layer on every local frontier (without replacement, all neighbours in
 * CSR order when degree <= fanout; random choices are a pure function of
 * (seed, iter, l, vertex id), so a vertex draws the same neighbours in any split), then split():
 * dedup into each split's mixed frontier (first-occurrence order, destination vertices first),
 * edges[l] relabelled to mixed-frontier rows, the sampled part of each mixed frontier bucketed by
 * owner (stable) and handed to the owners, next local frontiers by first-occurrence dedup of
 * (own destination vertices, then buckets in sender order), and shuffle_idx[l].
 * The result (the "batch") lives in the context until the next call.  Asynchronous.
 * EINVAL for n_targets < 0 or NULL pointers, ECAPACITY for n_targets > max_targets. */
GSPLIT_API int gsplit_sample_split(gsplit_ctx *ctx, const int32_t *d_targets, int64_t n_targets,
                        uint64_t seed, uint64_t iter, void *stream);

/* Algorithm 1 for several mini-batches in one set of launches.  Sampling depends on the graph, the
 * targets and the random stream, not on the model's weights, so the mini-batches of the next steps
 * can be sampled ahead of the training steps that consume them; n_batches of them go through the
 * same kernels together (one launch serves all of them), which hides the chains of dependent
 * memory accesses that a single small mini-batch consists of.  ctxs: HOST array of n_batches
 * DISTINCT contexts created for the same graph arrays and the same configuration (1 ..
 * GSPLIT_MAX_MULTI); batch b is sampled into ctxs[b] from d_targets[b] (HOST array of DEVICE
 * pointers), n_targets[b] and iters[b] (HOST arrays) exactly as gsplit_sample_split(ctxs[b],
 * d_targets[b], n_targets[b], seed, iters[b], stream) would: every output is bit-equal.
 * Afterwards each context holds its batch and is used on its own.  Errors are reported on
 * ctxs[0].  Asynchronous. */
GSPLIT_API int gsplit_sample_split_multi(gsplit_ctx *const *ctxs, int32_t n_batches,
                                         const int32_t *const *d_targets, const int64_t *n_targets,
                                         uint64_t seed, const uint64_t *iters, void *stream);

/* The same with the seed and the iteration counter read from DEVICE memory when the kernels run
 * (d_seed_iter[0] = seed, d_seed_iter[1] = iter), for steps that are captured into a HIP graph
 * and replayed for successive iterations.
 *
 * Stream capture: every asynchronous entry point only enqueues kernels on `stream`, with launch
 * shapes that depend on the context's upper bounds alone (the sizes of a batch stay in device
 * memory), so a whole step (this call, gsplit_gather_features, forward, loss, backward) can be
 * captured with hipStreamBeginCapture / hipStreamEndCapture and replayed.  Before capturing, run the
 * same step once eagerly: the first forward/backward call sizes the context's internal buffers
 * (allocation is not possible under capture).  Under capture no timing is taken, and the
 * host-side queries of a captured batch (gsplit_batch_sizes) wait for the whole device and read the
 * sizes anew on every call. */
GSPLIT_API int gsplit_sample_split_dev(gsplit_ctx *ctx, const int32_t *d_targets, int64_t n_targets,
                                       const uint64_t *d_seed_iter, void *stream);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): gsplit_sample_split without a context.  The graph, the configuration and the
 * targets are passed as to gsplit_create / gsplit_sample_split (keep_edge_ids and gat_index must be
 * 0); the outputs are the caller's DEVICE buffers; every piece of working memory (hash tables, entry
 * indices, class masks, histograms, level bookkeeping) comes out of one static device array of
 * GSPLIT_NOALLOC_SCRATCH_MIB MiB that every GPU the library runs on holds until the process ends.  The
 * call allocates nothing, frees nothing and enqueues only kernels on `stream`.
 *
 * Capacity: with B = max_l max_targets * prod_{k >= l} (1 + fanouts[k]) (the no-dedup bound on the
 * destinations plus slots of a layer) the call needs 32 bytes per element of B
 * plus 8 bytes per entry of its table, which has the next power of two above 2 * B entries.  ECAPACITY, with the figures in gsplit_last_error(NULL), when that exceeds
 * the array (1024 targets with fanouts [10, 5] take 4.1 MiB and fit; with [15, 10, 5] they would take
 * about 65 MiB and do not).
 *
 * Output sizes (entries, with ub[L] = max_targets, ub[l] = min(n_vertices, ub[l+1] * (1 + fanouts[l]))):
 *   d_local_cat[l] ub[l] (l = 0 .. L);  d_nbr[l], d_blk_src[l], d_recv_cat[l] ub[l+1] * fanouts[l];
 *   d_cnt[l] ub[l+1];  d_blk_indptr[l] ub[l+1] + 1;  d_mixed_cat[l], d_shuffle_src_row[l]
 *   ub[l+1] * (1 + fanouts[l]);  d_local_off (L+1) * (S+1);  d_mixed_off, d_recv_off L * (S+1).
 * Contents are those of gsplit_batch_level / gsplit_batch_layer after gsplit_sample_split with the
 * same arguments, bit for bit; d_local_off[l * (S+1) + s] etc. are the split offsets (the live sizes:
 * rows past them are not written).
 *
 * All calls on one GPU share that GPU's array, which keeps what the last call left (this call clears
 * what it needs first): calls that overlap in time on one GPU race, also from different threads or
 * streams; run them one after the other.  Errors are reported through gsplit_last_error(NULL). */
#define GSPLIT_NOALLOC_SCRATCH_MIB 16

typedef struct {
    int32_t *d_local_cat[GSPLIT_MAX_LAYERS + 1];
    int32_t *d_local_off;
    int32_t *d_nbr[GSPLIT_MAX_LAYERS];
    int32_t *d_cnt[GSPLIT_MAX_LAYERS];
    int32_t *d_mixed_cat[GSPLIT_MAX_LAYERS];
    int32_t *d_mixed_off;
    int32_t *d_blk_indptr[GSPLIT_MAX_LAYERS];
    int32_t *d_blk_src[GSPLIT_MAX_LAYERS];
    int32_t *d_shuffle_src_row[GSPLIT_MAX_LAYERS];
    int32_t *d_recv_cat[GSPLIT_MAX_LAYERS];
    int32_t *d_recv_off;
} gsplit_batch_out;

GSPLIT_API int gsplit_sample_split_noalloc(const gsplit_graph *graph, const gsplit_config *config,
                                           const int32_t *d_targets, int64_t n_targets, uint64_t seed,
                                           uint64_t iter, const gsplit_batch_out *out, void *stream);

/* Host-visible sizes of the current batch.  The first call after a gsplit_sample_split waits for
 * `stream` work of that call to finish (one device-to-host copy); later calls are free.
 *   n_local  [(L+1) * S]: |local_front[l]_s| at [l * S + s]
 *   n_mixed  [L * S]    : |mixed_front_s[l]|
 *   n_edges  [L * S]    : entries of edges[l] held by split s
 *   bucket   [L * S * S]: ids split s sends to split t at sampling layer l, at [(l*S + s)*S + t]
 * Any of the four may be NULL. */
GSPLIT_API int gsplit_batch_sizes(gsplit_ctx *ctx, int64_t *n_local, int64_t *n_mixed, int64_t *n_edges,
                       int64_t *bucket);

/* Device views of the current batch (context-owned, valid until the next gsplit_sample_split).
 * No synchronisation; sizes come from gsplit_batch_sizes. */
typedef struct {
    const int32_t *d_local_cat;     /* local_front[level] of all splits, global ids */
    const int32_t *d_local_off;     /* [S+1] device-side split offsets into d_local_cat */
} gsplit_level_view;

typedef struct {
    const int32_t *d_nbr;           /* [n_dst_total * fanout] sampled global ids, -1 padded      */
    const int32_t *d_cnt;           /* [n_dst_total] min(degree, fanout)                         */
    const int32_t *d_mixed_cat;     /* mixed frontiers of all splits, global ids                 */
    const int32_t *d_mixed_off;     /* [S+1] device-side offsets into d_mixed_cat                */
    const int32_t *d_blk_indptr;    /* [n_dst_total + 1] offsets into d_blk_src (whole layer)    */
    const int32_t *d_blk_src;       /* edges[l]: row of the owning split's mixed frontier        */
    const int32_t *d_shuffle_src_row;/* [sum n_mixed] row of local_cat[l] holding that vertex    */
    const int32_t *d_recv_cat;      /* received buckets: for t, for s: bucket[s->t] (global ids) */
    const int32_t *d_recv_off;      /* [S+1] device-side offsets of each receiver in d_recv_cat  */
} gsplit_layer_view;

GSPLIT_API int gsplit_batch_level(const gsplit_ctx *ctx, int32_t level, gsplit_level_view *out);
GSPLIT_API int gsplit_batch_layer(const gsplit_ctx *ctx, int32_t layer, gsplit_layer_view *out);

/* The shuffle index as the training passes use it (section 3: the shuffle index "consists of gather
 * and scatter indexes"; Algorithm 2 and the backward description after it).  Gather side, composed
 * with edges[l]: for destination row i of sampling layer `layer` (a row of local_cat[layer + 1]) and
 * for each of its sampled edges e (numbered d_blk_indptr[i] .. d_blk_indptr[i + 1] - 1), the row of
 * local_cat[layer] that holds the vertex.  Scatter side (the transpose, which the backward shuffle
 * follows): for every row u of local_cat[layer], d_rev_cnt[u] entries starting at
 * d_rev_list[d_rev_ptr[u]]; an entry is 2 * i for "u is destination i's own row" and 2 * i + 1 for
 * "u is the source of one sampled edge of destination i"; d_rev_eid holds the edge number of such an
 * entry (-1 for a self entry).  The entries of a row come in no particular order, and neither do
 * the segments of different rows.
 * The scatter side exists for layers >= 1, and for layer 0 too in a context created with
 * gat_index = 1 (which alone has d_rev_eid); pointers of absent parts are NULL.
 * Views are context-owned, valid until the next gsplit_sample_split; no synchronisation. */
typedef struct {
    const int32_t *d_self_row;      /* [n_dst_total]                                   */
    const int32_t *d_edge_row;      /* [number of sampled edges of the layer]          */
    const int32_t *d_rev_ptr;       /* [rows of local_cat[layer]]                      */
    const int32_t *d_rev_cnt;       /* [rows of local_cat[layer]]                      */
    const int32_t *d_rev_list;      /* [n_dst_total + number of sampled edges]         */
    const int32_t *d_rev_eid;       /* like d_rev_list, or NULL                        */
} gsplit_shuffle_view;

GSPLIT_API int gsplit_batch_shuffle(const gsplit_ctx *ctx, int32_t layer, gsplit_shuffle_view *out);

/* Loading step (section 3): d_out[r, :] = d_table[local_cat[0][r], :] for every row r of the
 * current batch's layer-0 local frontiers (splits concatenated).  A pure row copy of
 * dim * sizeof(dtype) bytes; rows of d_out are dense.  d_out must hold gsplit_max_rows(ctx, 0)
 * rows (or the exact count from gsplit_batch_sizes).  row_stride_bytes >= row bytes.
 * dtype: GSPLIT_F32 or GSPLIT_BF16.  Asynchronous. */
GSPLIT_API int gsplit_gather_features(gsplit_ctx *ctx, const void *d_table, int32_t dtype, int64_t dim,
                           int64_t row_stride_bytes, void *d_out, void *stream);

/* The loading step (section 3) of up to GSPLIT_MAX_MULTI contexts of one graph and configuration in
 * one launch (the companion of gsplit_sample_split_multi): d_outs[b] (HOST array of device
 * pointers) receives the rows of ctxs[b]'s current batch, exactly as gsplit_gather_features would
 * write them.  One table for all.  Errors are reported on ctxs[0].  Asynchronous. */
GSPLIT_API int gsplit_gather_features_multi(gsplit_ctx *const *ctxs, int32_t n_batches, const void *d_table,
                                            int32_t dtype, int64_t dim, int64_t row_stride_bytes,
                                            void *const *d_outs, void *stream);

/* GraphSAGE-mean model: layer l computes, for the destination vertices of every split,
 *   H_{l+1} = act( H_l[self] * W_self[l] + mean_{u in sampled N(v)} H_l[u] * W_neigh[l] + b[l] ),
 * act = ReLU except on the last layer; an empty neighbourhood has mean 0.  Weights are row-major
 * [dims[l] x dims[l+1]] float32 (HOST arrays of DEVICE pointers), biases [dims[l+1]] float32.
 * dtype selects how activations are stored and multiplied: GSPLIT_F32 (fp32 storage, fp32 MFMA) or
 * GSPLIT_BF16: features, activations between layers, the assembled layer inputs and a converted
 * copy of the weights are bfloat16 (round to nearest even) and the forward and input-gradient
 * products run on the bf16 matrix cores with float accumulation; the weight-gradient product,
 * biases, logits and all gradients stay float.  GSPLIT_BF16 needs dims[0..L-1] to be multiples
 * of 4 and d_feat_local to hold bfloat16 rows. */
typedef struct {
    int32_t             dtype;
    const int32_t      *dims;        /* HOST [L+1] */
    const void *const  *d_w_self;    /* HOST [L] of device pointers */
    const void *const  *d_w_neigh;
    const void *const  *d_bias;
} gsplit_sage_params;

/* Algorithm 2 on the current batch.  d_feat_local = output of gsplit_gather_features (dtype as in
 * params).  d_logits [n_targets x dims[L]] float32; row r belongs to local_cat[L][r], i.e. the
 * targets grouped by split in the order given (gsplit_batch_level(ctx, L) shows the ids).
 * Keeps the activations needed by the backward pass inside the context.  Asynchronous. */
GSPLIT_API int gsplit_sage_fwd(gsplit_ctx *ctx, const gsplit_sage_params *params, const void *d_feat_local,
                    float *d_logits, void *stream);

/* Backward pass, top layer down, from d_grad_logits [n_targets x dims[L]] (same row order as
 * d_logits).  Gradients of rows held by other splits travel back through the reversed shuffle
 * index; weight gradients are summed over all splits (the gradient aggregation of section 2).
 * Outputs (HOST arrays of DEVICE pointers, each buffer overwritten): d_gw_self[l], d_gw_neigh[l]
 * [dims[l] x dims[l+1]] float32, d_gbias[l] [dims[l+1]] float32.  No gradient is formed for the
 * input features.  Needs a preceding gsplit_sage_fwd on the same batch with the same params,
 * else ESTATE.  Asynchronous. */
GSPLIT_API int gsplit_sage_bwd(gsplit_ctx *ctx, const gsplit_sage_params *params, const float *d_grad_logits,
                    float *const *d_gw_self, float *const *d_gw_neigh, float *const *d_gbias,
                    void *stream);

/* The model part of one training step in one call: Algorithm 2's forward pass, the mean softmax
 * cross-entropy of the targets (as gsplit_softmax_xent: the label of row r is d_labels[vertex of
 * row r], int64, one entry per graph vertex) and the backward pass.  Same inputs and outputs as
 * gsplit_sage_fwd + gsplit_softmax_xent + gsplit_sage_bwd in this order, within float rounding of
 * them (sums run in another order); d_row_loss may be NULL.  With float32 storage, at least two
 * layers, at most 64 classes and a top-layer input width that is a multiple of 4 and at most 384,
 * the top layer's input assembly, forward product, loss and both backward products run as one
 * kernel (they are a few microseconds of work behind five kernel boundaries otherwise); other
 * shapes run the three steps one after the other.  Asynchronous.  A separate gsplit_sage_bwd
 * afterwards needs a gsplit_sage_fwd of its own (ESTATE). */
GSPLIT_API int gsplit_sage_step(gsplit_ctx *ctx, const gsplit_sage_params *params, const void *d_feat_local,
                                const int64_t *d_labels, float *d_logits, float *d_row_loss,
                                float *const *d_gw_self, float *const *d_gw_neigh, float *const *d_gbias,
                                void *stream);

/* View of the activations the last gsplit_sage_fwd (or gsplit_sage_step) stored for local_cat[level], level 1 .. L-1:
 * [rows of that level x dims[level]], float32 or bfloat16 as the forward pass's dtype says, after the
 * ReLU.  The backward pass of layer level - 1 multiplies by [activation > 0] (Algorithm 2's layers in
 * reverse): a parity check reads from this view which way the device decided a ReLU whose argument is
 * zero to rounding.  Context-owned, valid until the next forward pass; no synchronisation.  ESTATE
 * without a forward pass on the current batch, EINVAL for a level outside 1 .. L-1. */
GSPLIT_API int gsplit_sage_activations(const gsplit_ctx *ctx, int32_t level, const void **d_act);

/* GAT layer on the split mini-batch: the paper's second model (section 7.1), the layer of
 * Velickovic et al. (ICLR 2018) that it cites, run as `gnn_layer` of Algorithm 2.  Layer l, head k,
 * destination i with neighbourhood N(i) = {i} + its sampled neighbours:
 *     z_j = h_j W^k,   e_ij = LeakyReLU_0.2(a_dst^k . z_i + a_src^k . z_j),
 *     alpha_ij = softmax_j e_ij,   out_i^k = sum_j alpha_ij z_j
 *     hidden layers: h'_i = ELU(concat_k out_i^k + b);   last layer: logits_i = mean_k out_i^k + b
 * F_l = features per head.  dims[0] = input width; dims[l+1] = heads[l] * F_l for hidden layers,
 * F_l for the last one.  All parameters float32 in DEVICE memory:
 *   d_w[l]      [dims[l] x heads[l] * F_l] row-major, head k in columns k F_l .. (k+1) F_l - 1
 *   d_a_src[l], d_a_dst[l]  [heads[l] * F_l]
 *   d_bias[l]   [dims[l+1]]
 * Limits: heads[l] <= 64; F_l <= 1024 / p with p = heads[l] rounded up to a power of two;
 * (1 + fanouts[l]) * (1 + heads[l]) <= 3072.
 * Needs a context created with gat_index = 1 (else ESTATE). */
typedef struct gsplit_gat_params {
    int32_t             dtype;       /* GSPLIT_F32 */
    const int32_t      *dims;        /* HOST [L+1] */
    const int32_t      *heads;       /* HOST [L] */
    const void *const  *d_w;         /* HOST [L] of device pointers */
    const void *const  *d_a_src;
    const void *const  *d_a_dst;
    const void *const  *d_bias;
} gsplit_gat_params;

/* Forward pass on the current batch.  d_feat_local = output of gsplit_gather_features (float32,
 * [rows of level 0 x dims[0]]).  d_logits [n_targets x dims[L]] float32, rows as in
 * gsplit_sage_fwd.  Keeps the transformed rows, the attention coefficients and the activations
 * inside the context for the backward pass.  Asynchronous. */
GSPLIT_API int gsplit_gat_fwd(gsplit_ctx *ctx, const gsplit_gat_params *params, const void *d_feat_local,
                              float *d_logits, void *stream);

/* Backward pass from d_grad_logits [n_targets x dims[L]], top layer down; gradients of rows held
 * by other splits travel back through the reversed shuffle index, parameter gradients are summed
 * over all splits.  d_feat_local: the buffer the forward pass read, unchanged.  Outputs (HOST
 * arrays of DEVICE pointers, each buffer overwritten, float32): d_gw[l] like d_w[l], d_ga_src[l],
 * d_ga_dst[l] [heads[l] * F_l], d_gbias[l] [dims[l+1]].  No gradient for the input features.  Needs
 * a preceding gsplit_gat_fwd on the same batch with the same params (ESTATE).  Asynchronous. */
GSPLIT_API int gsplit_gat_bwd(gsplit_ctx *ctx, const gsplit_gat_params *params, const void *d_feat_local,
                              const float *d_grad_logits, float *const *d_gw, float *const *d_ga_src,
                              float *const *d_ga_dst, float *const *d_gbias, void *stream);

/* View of the two score terms the last gsplit_gat_fwd stored per row of local_cat[layer] and head k:
 *   a_src^k . z_r^k at d_terms[r * row_stride + src_col + k],  a_dst^k . z_r^k at [... + dst_col + k]
 * (float32).  Both passes form the argument of the LeakyReLU of an entry (destination i, source j) as
 * the float32 sum of i's dst term and j's src term, so a parity check can tell from this view which
 * slope the device took where that argument is zero to rounding.  Context-owned, valid until the next
 * forward pass; no synchronisation.  ESTATE without a forward pass on the current batch. */
GSPLIT_API int gsplit_gat_score_terms(const gsplit_ctx *ctx, int32_t layer, const float **d_terms,
                                      int64_t *row_stride, int64_t *src_col, int64_t *dst_col);

/* Diagnostics: per-kernel device time.  While enabled, every kernel the library launches is
 * bracketed by two events on the stream it runs on (this adds a little host work per launch).
 * gsplit_timing_read waits for the recorded events, writes one line per kernel label
 * ("<label> <launches> <total milliseconds>\n", labels carry the layer as ".l<k>") into buf as a
 * NUL-terminated string, resets the totals, and returns the string length; ECAPACITY if buf_bytes is
 * too small.  An event pair adds a few microseconds to what it brackets; the library measures that
 * once per context (a bracketed 20-microsecond kernel against the same kernel launched back to
 * back) and subtracts it, so the totals are kernel durations.  For callers that profile (benchmarks); never
 * needed for results. */
GSPLIT_API int gsplit_timing_enable(gsplit_ctx *ctx, int32_t enable);
GSPLIT_API int64_t gsplit_timing_read(gsplit_ctx *ctx, char *buf, int64_t buf_bytes);

/* Offline pre-sampling (section 4, "pre-sampling" stage; analysis after Eq. 2): adds the current
 * batch to running counts from which the weighted graph G_w is built.
 *   d_vertex_count [n_vertices], uint32: += 1 for every level l > 0 (level L holds the targets,
 *       level 0, the input layer, does not count) whose frontier holds the vertex            (k_v)
 *   d_edge_count   [n_edges], uint32   : += 1 for every time CSR edge e was sampled, at any
 *       layer of this batch                                                                  (k_e)
 * Either pointer may be NULL (that count is skipped).  The counts do not depend on the number of
 * splits the context was created with.  Needs keep_edge_ids = 1 for d_edge_count (else ESTATE) and
 * a batch (ESTATE).  Counters wrap at 2^32.  Asynchronous. */
GSPLIT_API int gsplit_presample_accumulate(gsplit_ctx *ctx, uint32_t *d_vertex_count, uint32_t *d_edge_count,
                                           void *stream);

/* Split statistics (section 7.3, evaluation of the splitting algorithm): adds the current batch to
 *   d_edges       [L * S], uint64: += edges of sampling layer l computed by split s, at [l * S + s]
 *   d_cross_edges [L * S], uint64: += those of them whose source vertex another split owns
 * From the sums the paper's figures follow: workload imbalance = max over s of the edges at layers
 * l > 0 divided by their average over s; communication cost = cross edges / all edges.  A
 * data-parallel micro-batch (Table 1) is a context with one split; its edge total and its
 * level-0 row count (gsplit_batch_sizes) are the "edges computed" and "features loaded" columns.
 * EINVAL for NULL pointers, ESTATE without a batch.  Asynchronous. */
GSPLIT_API int gsplit_batch_stats(gsplit_ctx *ctx, uint64_t *d_edges, uint64_t *d_cross_edges, void *stream);

/* Partial feature cache aligned with f_G, and the host-memory miss path (sections 3 and 4: the
 * features live in host memory, f_G also decides on which GPU a vertex's input features are
 * statically cached, and the loading step skips what is cached; section 7.1: what to cache is
 * ranked by sampling frequency).
 *
 * gsplit_input_counts_accumulate: d_count[v] += 1 (uint32) for every vertex of the current batch's
 * input layer (level 0): run over some epochs of sampling it is the ranking criterion.  The
 * choice of what to cache from the counts is the caller's (an offline step, like the partition
 * map).  ESTATE without a batch.  Asynchronous.
 *
 * gsplit_cache_build: `table` is the full feature table [n_vertices x dim] (dtype, row stride as
 * in gsplit_gather_features) in memory the device can read: pinned HOST memory (hipHostMalloc,
 * torch pin_memory) or device memory; it must stay valid and unchanged in the rows that are not
 * cached for as long as the cache is used.  d_cache_ids (DEVICE) lists the vertices to cache,
 * grouped by split: first n_cache[0] ids that f_G gives to split 0, then n_cache[1] of split 1, ...
 * (n_cache: HOST [S]).  Cache row j holds a copy of table row d_cache_ids[j] in HBM.  EINVAL for
 * an id outside the graph, listed under a split that does not own it, or listed twice, and for a
 * table the device cannot read.  Synchronises with `stream` (a set-up call).  One cache per
 * context; building again replaces it (the old buffers are freed first, which waits for the device).
 *
 * gsplit_gather_features_cached: the loading step: d_out[r, :] = the cached copy if the vertex of
 * row r (local_cat[0][r]) is cached, else the row of `table`, read over the host link without a
 * host round trip.  d_out as in gsplit_gather_features.  d_hits / d_misses (may be NULL): DEVICE
 * [S] uint64, += rows of split s served by the cache / by the table.  ESTATE without a cache or a
 * batch.  Asynchronous. */
GSPLIT_API int gsplit_input_counts_accumulate(gsplit_ctx *ctx, uint32_t *d_count, void *stream);
GSPLIT_API int gsplit_cache_build(gsplit_ctx *ctx, const void *table, int32_t dtype, int64_t dim,
                                  int64_t row_stride_bytes, const int32_t *d_cache_ids, const int64_t *n_cache,
                                  void *stream);
GSPLIT_API int gsplit_gather_features_cached(gsplit_ctx *ctx, void *d_out, uint64_t *d_hits, uint64_t *d_misses,
                                             void *stream);

/* w[i] = count[i] / n_samples for i < n (w_V = k_v / N, w_E = k_e / N).  EINVAL for NULL pointers,
 * n < 0 or n_samples < 1.  Asynchronous. */
GSPLIT_API int gsplit_presample_weights(gsplit_ctx *ctx, const uint32_t *d_count, int64_t n, int64_t n_samples,
                                        float *d_weight, void *stream);

/* Loss between forward and backward.  The paper only says that the target features "are used to
 * calculate the loss" (section 2); this is the usual choice for node classification: mean softmax
 * cross-entropy over the targets.  Row r of d_logits / d_grad_logits belongs to local_cat[L][r];
 * its label is d_labels[that vertex id] (int64, one entry per graph vertex, values in
 * [0, n_classes)).  d_grad_logits [n_targets x n_classes] receives d loss / d logits;
 * d_row_loss (may be NULL) [n_targets] receives the per-target loss terms, whose mean is the loss.
 * Asynchronous. */
GSPLIT_API int gsplit_softmax_xent(gsplit_ctx *ctx, const float *d_logits, int32_t n_classes,
                                   const int64_t *d_labels, float *d_grad_logits, float *d_row_loss,
                                   void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GSPLIT_H */
