// Split-parallel sampling for all S logical splits at once (paper Algorithm 1, `sp_sample`, with
// the online splitting of section 4): neighbour sampling, mixed-frontier dedup/relabel, owner
// buckets, next local frontiers and the shuffle index.  Every kernel takes its problem size from
// device memory (GsLevelMeta), so one iteration is enqueued without any host synchronisation and
// the launch shapes depend only on the context's upper bounds.
//
// Per sampling layer (4 launches):
//   1 sample_layer       + insert (vertex, split) keys of destinations and slots into tab_mixed
//                        and vertex keys into tab_local
//   2 partition: count     one multi-class pass over the slots: per split its mixed frontier, per
//   3 partition: scatter   owner its bucket (= received ids) and its new local-frontier members,
//                          and the edge numbers; + block CSR offsets, destination vertices at the
//                          head of both frontiers; + the reverse index of the layer above
//   4 shuffle index (+ its composition with edges[l] for the forward/backward passes, + edges[l]
//                          relabelled to mixed-frontier rows, + reset of both tables for the next
//                          layer)
// (One workgroup doing count and scatter of a small partition in a single launch was tried for the
// top layer: its chains of dependent accesses have nobody to overlap with, 85 us against 21 us
// for 5120 slots.  The targets themselves, one lookup each, do take a single workgroup when there
// are at most 1024 of them.)
// The scatter side of the shuffle index (for every row of local_cat[l], the destination rows it
// feeds, so that the backward pass can pull) of layer l+1 rides on the two partition launches of
// layer l; only a context that keeps one for the bottom layer pays two launches of its own, after
// the layer loop.
//
// Why one partition pass serves both frontiers: the rows of a level are ordered by split, so the
// slot stream in (row, slot) order is the concatenation of the splits' slot streams, and the ids an
// owner t receives, `for s: bucket[s -> t]`, are the per-split first occurrences owned by t in
// exactly that global order.  The first occurrence of a vertex among the received ids of its owner
// is therefore its first occurrence in the whole slot stream (which is always a per-split first
// occurrence too): a second table keyed by the vertex alone, filled by the sampler with the
// global slot positions, tells it without a pass over the received ids.
// A dependent HBM access costs about a microsecond, and these kernels are chains of them, so every
// element remembers the table entry it landed in (no second probe sequence) and the count passes
// leave their classification behind for the scatter passes.
#include <algorithm>
#include <mutex>

#include "gsplit_internal.h"

namespace {

constexpr int PART_BS = 256;     // threads of a partition workgroup
constexpr int PART_NK = 25;     // classes of a partition pass: 8 senders + 8 owners + 1 edge counter + 8 owners (new local)
constexpr int PART_MAX_NB = 1024;
constexpr unsigned long long EMPTY_ENTRY = ~0ull;
constexpr int CLAIM_FIRST_MAX = 1 << 18;     // destinations + slots up to which inserts claim before they read

// ------------------------------------------------------------------------------------------
// small device helpers
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

__device__ __forceinline__ uint64_t lanemask_lt() {
    return (1ull << lane_id()) - 1ull;
}

// which split a row of a split-concatenated array belongs to (off has S+1 entries)
__device__ __forceinline__ int split_of(const int32_t *off, int S, int i) {
    int s = 0;
    for (int k = 1; k < S; ++k) s += (off[k] <= i) ? 1 : 0;
    return s;
}

__device__ __forceinline__ int table_bits(int n_inputs) {
    // capacity = 2^bits >= 2 * n_inputs, at least 1024 entries
    int want = n_inputs < 512 ? 1024 : 2 * n_inputs;
    return 32 - __clz(want - 1);
}

__device__ __forceinline__ uint32_t table_slot(uint32_t key, int bits) {
    return (key * 0x9E3779B1u) >> (32 - bits);
}

// Open-addressing table with 64-bit entries (key << 32 | position).  Inserting a key keeps the
// smallest position that carried it: claim an empty entry with one compare-and-swap, otherwise
// (same key) lower it with a 64-bit atomic min; the entry is read first and the atomic skipped
// when it cannot change anything, which keeps hub vertices from serialising on one address.
// Returns the entry index (-1 and the error flag if the table is full, which sizing excludes).
// *behind (if given) is set when the key was already there with a smaller position.
// claim_first: try the compare-and-swap without reading first.  One access instead of two when the
// entry is free, which is what a small layer's path through this function consists of; only where
// few elements share a key, since every attempt on a taken entry is then an atomic on it.
__device__ __forceinline__ int table_insert(const GsTable &t, int bits, uint32_t key, uint32_t p,
                                            int32_t *err, bool *behind = nullptr, bool claim_first = false) {
    if (t.pos) {        // direct table: the key is its own entry index (bits carries the layer's stamp)
        const unsigned long long mine = ((unsigned long long)(uint32_t)bits << 32) | p;
        const unsigned long long old = atomicMin(&t.pos[key], mine);
        if (behind && (uint32_t)(old >> 32) == (uint32_t)bits && (uint32_t)old < p) *behind = true;
        return (int)key;
    }
    const uint32_t mask = (1u << bits) - 1u;
    const unsigned long long mine = ((unsigned long long)key << 32) | p;
    uint32_t h = table_slot(key, bits);
    for (uint32_t probe = 0; probe <= mask; ++probe) {
        unsigned long long cur;
        if (claim_first) {
            cur = atomicCAS(&t.slot[h], EMPTY_ENTRY, mine);
            if (cur == EMPTY_ENTRY) return (int)h;
        } else {
            cur = __hip_atomic_load(&t.slot[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (cur == EMPTY_ENTRY) {
                cur = atomicCAS(&t.slot[h], EMPTY_ENTRY, mine);
                if (cur == EMPTY_ENTRY) return (int)h;
            }
        }
        if ((uint32_t)(cur >> 32) == key) {
            if (mine < cur) atomicMin(&t.slot[h], mine);
            else if (behind) *behind = true;
            return (int)h;
        }
        h = (h + 1) & mask;
    }
    *err = 1;
    return -1;
}

// smallest position an entry has seen (the entry's key is known to be the caller's)
__device__ __forceinline__ uint32_t table_pos(const GsTable &t, int h) {
    return t.pos ? (uint32_t)t.pos[h] : (uint32_t)t.slot[h];
}

// The hashed table of a context with several splits holds (vertex, split) keys only, hashed by the
// vertex: the keys of a vertex start at the same line of 8 entries (64 bytes; a vertex has at most
// 8 keys) and lie there side by side, filled from the front, running over into the next line when
// one is full.  So the first occurrence of the vertex in the whole stream (the smallest position
// among its keys) is read off the line the slot's own entry is in, and there is no second table
// keyed by the vertex, with its own insert and its own access to the memory per slot.
// (Lines of 16 entries, the 128 bytes one access to the memory moves anyway, measured slower: what
// a lane asks of a line costs by the request, and half the line is half the requests.)
constexpr int LINE_ENTRIES = 8;
constexpr int LINE_LOG = 3;
__device__ __forceinline__ uint32_t table_line(uint32_t vertex, int bits) {
    return ((vertex * 0x9E3779B1u) >> (32 - (bits - LINE_LOG))) << LINE_LOG;
}

// Insert into that table.  The line is read once, with plain loads: what such a read shows of a taken
// entry is true for good (an entry keeps its key, its position only falls), and an entry it shows
// empty is taken with a compare-and-swap, which answers with the truth.  The probe starts at the first
// entry that is the key's or empty, and from there is the linear probe of table_insert.
// claim_first (small layers): no read at all, a compare-and-swap on one entry after the other from
// the front of the line.
__device__ __forceinline__ int table_insert_line(const GsTable &t, int bits, uint32_t vertex, uint32_t S, uint32_t split,
                                                 uint32_t p, int32_t *err, bool *behind, bool claim_first) {
    const uint32_t key = vertex * S + split;
    const uint32_t mask = (1u << bits) - 1u;
    const unsigned long long mine = ((unsigned long long)key << 32) | p;
    uint32_t h = table_line(vertex, bits);
    for (uint32_t probe = 0; probe <= mask; probe += LINE_ENTRIES) {
        int j0 = 0;
        unsigned long long at0 = EMPTY_ENTRY;
        if (!claim_first) {
            const ulonglong2 *line = reinterpret_cast<const ulonglong2 *>(t.slot + h);
            ulonglong2 q[LINE_ENTRIES / 2];
#pragma unroll
            for (int i = 0; i < LINE_ENTRIES / 2; ++i) q[i] = line[i];
            j0 = LINE_ENTRIES;
#pragma unroll
            for (int j = LINE_ENTRIES - 1; j >= 0; --j) {
                const unsigned long long e = (j & 1) ? q[j >> 1].y : q[j >> 1].x;
                if (e == EMPTY_ENTRY || (uint32_t)(e >> 32) == key) { j0 = j; at0 = e; }
            }
        }
        for (int j = j0; j < LINE_ENTRIES; ++j) {
            unsigned long long cur = (claim_first || j == j0) ? at0
                                         : __hip_atomic_load(&t.slot[h + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (cur == EMPTY_ENTRY) {
                cur = atomicCAS(&t.slot[h + j], EMPTY_ENTRY, mine);
                if (cur == EMPTY_ENTRY) return (int)(h + j);
            }
            if ((uint32_t)(cur >> 32) == key) {
                if (mine < cur) atomicMin(&t.slot[h + j], mine);
                else if (behind) *behind = true;
                return (int)(h + j);
            }
        }
        h = (h + LINE_ENTRIES) & mask;
    }
    *err = 1;
    return -1;
}

// smallest position among the keys of a vertex in that table (at most `start`): its lines are read
// until one shows an empty entry
__device__ __forceinline__ uint32_t table_line_first(const GsTable &t, int bits, uint32_t vertex, uint32_t S, uint32_t start) {
    const uint32_t mask = (1u << bits) - 1u;
    const uint32_t base = vertex * S;
    uint32_t h = table_line(vertex, bits), best = start;
    for (uint32_t probe = 0; probe <= mask; probe += LINE_ENTRIES) {
        const ulonglong2 *line = reinterpret_cast<const ulonglong2 *>(t.slot + h);
        ulonglong2 q[LINE_ENTRIES / 2];
#pragma unroll
        for (int i = 0; i < LINE_ENTRIES / 2; ++i) q[i] = line[i];
        bool open = false;
#pragma unroll
        for (int j = 0; j < LINE_ENTRIES; ++j) {
            const unsigned long long e = (j & 1) ? q[j >> 1].y : q[j >> 1].x;
            if (e == EMPTY_ENTRY) open = true;
            else if ((uint32_t)(e >> 32) - base < S) best = min(best, (uint32_t)e);
        }
        if (open) break;
        h = (h + LINE_ENTRIES) & mask;
    }
    return best;
}

// Stamp of the direct tables for sampling layer `layer` of the batch a context is working on: falls
// with every batch and, inside a batch, from the top layer down (8 = GSPLIT_MAX_LAYERS per batch).
__device__ __forceinline__ uint32_t table_stamp(const GsLevelMeta *meta_level0, uint32_t layer) {
    return 0xFFFFFFF0u - (meta_level0->batches * 8u + (7u - layer));
}

// ------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): counter-based generator, 10 rounds.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint2 k) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c.x), lo0 = 0xD2511F53u * c.x;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c.z), lo1 = 0xCD9E8D57u * c.z;
        c = make_uint4(hi1 ^ c.y ^ k.x, lo1, hi0 ^ c.w ^ k.y, lo0);
        k.x += 0x9E3779B9u;
        k.y += 0xBB67AE85u;
    }
    return c;
}

// ------------------------------------------------------------------------------------------
// sample_layer: G lanes cooperate on one frontier vertex (G = 16, 32 or 64 >= fanout).
// degree <= fanout: copy the row in CSR order.  Otherwise Floyd's selection: lane q draws
// t_q in [0, d-fan+q] from its own Philox word; the sequential "already chosen -> take j"
// rule is resolved with fan-1 rounds of broadcast + ballot inside the lane group.
// The random word of draw q is word (q mod 4) of Philox(counter = (v, iter lo, iter hi,
// layer * 65536 + q / 4), key = (seed lo, seed hi)): a function of the global vertex id only.
// Every destination vertex (position i) and every sampled slot (position n1 + slot index) is
// also entered into the mixed-frontier table under the key (vertex, split of the row) and into the
// local-frontier table under the key vertex; the entry indices are kept in ent_mixed / ent_local
// (destinations first, then slots; -1 for padding slots, -2 - index for a slot that found its
// (vertex, split) key already there with a smaller position).
// ------------------------------------------------------------------------------------------
// Arguments of one mini-batch of a launch.  Every sampling kernel serves up to GS_MAXB independent
// mini-batches (contexts over the same graph) at once, blockIdx.y = batch: the kernels of a small
// layer are chains of dependent accesses that leave the chip idle, and the chains of several batches
// overlap (sampling does not depend on the weights, so the batches of the next steps are known).
constexpr int GS_MAXB = GSPLIT_MAX_MULTI;

struct SampleArgs {
    const int32_t *front; GsLevelMeta *meta_lo; const GsLevelMeta *meta_up;
    GsTable tab, tab_local;
    int32_t *ent_mixed, *ent_local, *nbr, *cnt; int64_t *epos;
    uint64_t iter; const uint64_t *seed_iter;
};
struct SampleArgsSet { SampleArgs b[GS_MAXB]; };

template <int G, typename IndPtrT>
__global__ __launch_bounds__(256) void k_sample_layer(const IndPtrT *__restrict__ indptr,
                                                      const int32_t *__restrict__ indices,
                                                      SampleArgsSet set, int S,
                                                      int fan, uint32_t layer, uint64_t seed) {
    const SampleArgs &a = set.b[blockIdx.y];
    const int32_t *__restrict__ front = a.front;
    GsLevelMeta *meta_lo = a.meta_lo;
    const GsLevelMeta *__restrict__ meta_up = a.meta_up;
    const GsTable tab = a.tab, tab_local = a.tab_local;
    // direct tables with several splits: the (vertex, split) entries of a vertex are neighbours in
    // memory, the partition reads them together, and there is no table keyed by the vertex alone
    const bool no_local = !tab_local.pos && !tab_local.slot;
    const bool lines = no_local && !tab.pos;     // hashed, several splits: the keys of a vertex share lines
    int32_t *__restrict__ ent_mixed = a.ent_mixed;
    int32_t *__restrict__ ent_local = a.ent_local;
    int32_t *__restrict__ nbr = a.nbr;
    int32_t *__restrict__ cnt = a.cnt;
    int64_t *__restrict__ epos = a.epos;
    uint64_t iter = a.iter;
    if (a.seed_iter) {      // seed and iteration counter kept in device memory (replayed graphs)
        seed = a.seed_iter[0];
        iter = a.seed_iter[1];
    }
    const int n1 = meta_up->front_off[S];
    const int bits = tab.pos ? (int)table_stamp(meta_lo - layer, layer) : table_bits(n1 * (1 + fan));
    const bool claim_first = n1 * (1 + fan) <= CLAIM_FIRST_MAX;
    const int groups_per_block = PART_BS / G;
    const int q = threadIdx.x % G;
    const int sub = lane_id() / G;
    const uint64_t gmask = (G == 64) ? ~0ull : ((1ull << (G & 63)) - 1ull);
    const int stride = gridDim.x * groups_per_block;
    // every lane of a wave runs the same number of iterations (ballots/shuffles need that)
    const int first = blockIdx.x * groups_per_block + (threadIdx.x / 64) * (64 / G);
    for (int base = first; base < n1; base += stride) {
        const int row = base + sub;
        const bool active = row < n1;
        int32_t v = 0;
        int64_t beg = 0;
        uint32_t d = 0;
        if (active) {
            v = front[row];
            beg = (int64_t)indptr[v];
            d = (uint32_t)((int64_t)indptr[v + 1] - beg);
        }
        int32_t val = -1;
        const bool floyd = active && d > (uint32_t)fan;
        uint32_t chosen = 0, t = 0, j = 0;
        if (floyd && q < fan) {
            uint4 ctr = make_uint4((uint32_t)v, (uint32_t)iter, (uint32_t)(iter >> 32),
                                   (layer << 16) | ((uint32_t)q >> 2));
            uint4 r = philox4x32_10(ctr, make_uint2((uint32_t)seed, (uint32_t)(seed >> 32)));
            uint32_t w = (q & 3) == 0 ? r.x : (q & 3) == 1 ? r.y : (q & 3) == 2 ? r.z : r.w;
            j = d - (uint32_t)fan + (uint32_t)q;
            t = __umulhi(w, j + 1u);
            chosen = t;
        }
        // does any group of this wave need the sequential resolution?
        if (__ballot(floyd) != 0ull) {
            for (int s = 1; s < fan; ++s) {
                const uint32_t ts = __shfl(t, s, G);
                const bool hit = floyd && q < s && chosen == ts;
                const uint64_t any = (__ballot(hit) >> (sub * G)) & gmask;
                if (floyd && q == s && any != 0ull) chosen = j;
            }
        }
        // What a lane enters into the two tables: its sampled neighbour (lanes q < fan) with the
        // slot's global position, or, in the first spare lane of the group, the destination vertex
        // itself with its row (destinations hold the smallest positions).  All of them go through
        // the same insert instructions, so the destination's inserts cost the wave no extra round
        // trips; only a group without a spare lane (fan == G) has lane 0 do them first.
        const bool spare = fan < G;
        int32_t key_v = -1;
        uint32_t pos_v = 0;
        int64_t out = -1;
        const uint32_t sp = active ? (uint32_t)split_of(meta_up->front_off, S, row) : 0u;
        if (active && q < fan) {
            int64_t pos = -1;
            if (floyd) pos = beg + (int64_t)chosen;
            else if ((uint32_t)q < d) pos = beg + q;
            // (the graph is read once, at random: a load that leaves the caches to what is used again)
            if (pos >= 0) val = __builtin_nontemporal_load(&indices[pos]);
            const int64_t g = (int64_t)row * fan + q;
            nbr[g] = val;
            if (epos) epos[g] = pos;
            if (q == 0) {
                cnt[row] = d < (uint32_t)fan ? (int32_t)d : fan;
                if (!spare) {
                    const int hm = lines ? table_insert_line(tab, bits, (uint32_t)v, (uint32_t)S, sp, (uint32_t)row,
                                                             &meta_lo->error, nullptr, false)
                                         : table_insert(tab, bits, (uint32_t)v * (uint32_t)S + sp, (uint32_t)row,
                                                        &meta_lo->error);
                    ent_mixed[row] = hm;
                    ent_local[row] = (S == 1 || no_local) ? hm : table_insert(tab_local, bits, (uint32_t)v, (uint32_t)row,
                                                                              &meta_lo->error);
                }
            }
            key_v = val;
            pos_v = (uint32_t)(n1 + g);
            out = n1 + g;
        } else if (active && spare && q == fan) {
            key_v = v;
            pos_v = (uint32_t)row;
            out = row;
        }
        if (out >= 0) {
            int hm = -1, hl = -1;
            bool behind = false;
            if (key_v >= 0) {
                // a slot that finds its (vertex, split) key with a smaller position is not the first
                // occurrence in its split, let alone in the whole stream: nothing will ask for its
                // entry in the vertex table, so it does not make one
                // (with a single split the two keys are the same key, the two tables the same table,
                // and a vertex has the same row in the mixed and in the next local frontier)
                hm = lines ? table_insert_line(tab, bits, (uint32_t)key_v, (uint32_t)S, sp, pos_v, &meta_lo->error, &behind, claim_first)
                           : table_insert(tab, bits, (uint32_t)key_v * (uint32_t)S + sp, pos_v, &meta_lo->error, &behind,
                                          claim_first);
                if (S == 1 || no_local) hl = hm;
                else if (!behind)
                    hl = table_insert(tab_local, bits, (uint32_t)key_v, pos_v, &meta_lo->error, nullptr, claim_first);
            }
            // a slot known not to be the first of its key says so in its entry index (-2 - index):
            // the partition then classifies it without looking the entry up again
            ent_mixed[out] = (behind && out >= n1) ? -2 - hm : hm;
            ent_local[out] = hl;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Stable multi-class partition in two launches over `nb` chunks: count per chunk, then scatter.
// Every scatter workgroup first turns the chunk histograms into its own bases (the sums over all
// chunks and over the chunks before it), so no launch sits between the two passes.
// A functor F describes the elements:
//   n()                          number of elements (read from device memory)
//   used(k)                      whether class k can occur at all (uniform; the others are skipped)
//   classify(g)                  count pass: bit k set <=> element g counts in class k (k < F::NK);
//                                may leave the mask behind for the scatter pass
//   cached(g)                    scatter pass: the same mask
//   upper_offset(s)              split offset s of the level above (fetched by 9 threads up front)
//   key_bases(totals, bases, o, up)  where each class starts, and the offsets `o` that follow from
//                                the totals; pure, run by one thread of every scatter workgroup
//   publish(o)                   writes those offsets to the batch's device bookkeeping (one thread
//                                of the whole launch; later launches read them there, this launch
//                                takes them from `o`)
//   emit(g, mask, rk, o)         rk[k] = bases[k] + number of class-k elements before g
//   n_extra(o), extra(g, o)      independent element-wise work appended to the scatter pass
//   n_side(), side(g, n)         independent work appended to the count pass: called by whole
//                                workgroups, 256 consecutive g at a time (g >= n in the last one)
// Elements keep their order inside every class (wave ballots + running chunk counters).
// ------------------------------------------------------------------------------------------
struct PartOffs {
    int a[GS_MAXS + 1];     // first offset array of the pass (front_off of the targets, or mixed_off)
    int b[GS_MAXS + 1];     // recv_off
    int c[GS_MAXS + 1];     // front_off of the level below
    int total;              // class-16 total (edges)
};

__device__ __forceinline__ int part_chunk(int n, int nb) {
    int c = (n + nb - 1) / nb;
    return ((c + PART_BS - 1) / PART_BS) * PART_BS;
}

// one functor and one histogram per mini-batch of the launch (blockIdx.y = batch)
template <class F>
struct PartSet { F f[GS_MAXB]; int32_t *hist[GS_MAXB]; };

// hist is class-major: hist[k * gridDim.x + chunk]
template <class F>
__global__ __launch_bounds__(PART_BS) void k_part_count(PartSet<F> set) {
    const F &f = set.f[blockIdx.y];
    int32_t *__restrict__ hist = set.hist[blockIdx.y];
    __shared__ int s_cnt[PART_NK];
    if (threadIdx.x < PART_NK) s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const int n = f.n();
    const int chunk = part_chunk(n, gridDim.x);
    const int64_t beg64 = (int64_t)blockIdx.x * chunk;
    if (beg64 < n) {
        const int beg = (int)beg64;
        const int end = (n - beg < chunk) ? n : beg + chunk;
        int local[F::NK];
#pragma unroll
        for (int k = 0; k < F::NK; ++k) local[k] = 0;
        for (int g = beg + threadIdx.x; g < end; g += PART_BS) {
            const unsigned m = f.classify(g);
#pragma unroll
            for (int k = 0; k < F::NK; ++k) local[k] += (m >> k) & 1u;
        }
#pragma unroll
        for (int k = 0; k < F::NK; ++k) {
            if (!f.used(k)) continue;               // uniform: classes of splits the context does not have
            int v = local[k];
            for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
            if (lane_id() == 0 && v) atomicAdd(&s_cnt[k], v);
        }
    }
    __syncthreads();
    if (threadIdx.x < F::NK) hist[threadIdx.x * gridDim.x + blockIdx.x] = s_cnt[threadIdx.x];
    // every thread of the workgroup makes every call (side may synchronise the workgroup).  The
    // side work is dealt from the last workgroup backwards: in a small layer the first workgroups
    // hold all the elements and the rest are idle, so the two run side by side.
    const int64_t ns = f.n_side();
    for (int64_t base = (int64_t)(gridDim.x - 1 - blockIdx.x) * PART_BS; base < ns; base += (int64_t)gridDim.x * PART_BS)
        f.side(base + threadIdx.x, ns);
}

// gridDim.x = 256 * PER chunks
template <class F, int PER>
__global__ __launch_bounds__(PART_BS) void k_part_scatter(PartSet<F> set) {
    const F &f = set.f[blockIdx.y];
    const int32_t *__restrict__ hist = set.hist[blockIdx.y];
    __shared__ int s_tot[PART_NK], s_pre[PART_NK], s_base[PART_NK];
    __shared__ int s_run[PART_NK];
    __shared__ int s_wcnt[PART_BS / 64][PART_NK];
    __shared__ PartOffs s_o;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    // classes are dealt to the four waves; a wave reads a class's histogram row 64 chunks at a time
    // (all loads issued before any sum) and reduces both sums with one shuffle tree
    __shared__ int s_up[GS_MAXS + 1];
    if (threadIdx.x <= GS_MAXS) s_up[threadIdx.x] = f.upper_offset(threadIdx.x);
    // the class mask of this thread's first element does not depend on the histograms: it is
    // fetched now and travels while they are read and summed
    const int n = f.n();
    const int chunk = part_chunk(n, gridDim.x);
    const int64_t beg64 = (int64_t)blockIdx.x * chunk;
    unsigned m_first = 0u;
    if (beg64 < n) {
        const int end0 = (n - (int)beg64 < chunk) ? n : (int)beg64 + chunk;
        if ((int)beg64 + (int)threadIdx.x < end0) m_first = f.cached((int)beg64 + threadIdx.x);
    }
    {
        constexpr int CPW = (F::NK + PART_BS / 64 - 1) / (PART_BS / 64);     // classes per wave
        constexpr int LPC = PER * 4;                                          // 64-chunk loads per class
        int v[CPW][LPC];
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const int k = wave + c * (PART_BS / 64);
#pragma unroll
            for (int j = 0; j < LPC; ++j)
                v[c][j] = k < F::NK ? hist[k * (int)gridDim.x + j * 64 + lane] : 0;
        }
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const int k = wave + c * (PART_BS / 64);
            int tot = 0, pre = 0;
#pragma unroll
            for (int j = 0; j < LPC; ++j) {
                tot += v[c][j];
                pre += (j * 64 + lane < (int)blockIdx.x) ? v[c][j] : 0;
            }
            for (int o = 32; o > 0; o >>= 1) { tot += __shfl_down(tot, o); pre += __shfl_down(pre, o); }
            if (lane == 0 && k < F::NK) { s_tot[k] = tot; s_pre[k] = pre; }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        f.key_bases(s_tot, s_base, s_o, s_up);
        if (blockIdx.x == 0) f.publish(s_o);
    }
    __syncthreads();
    if (threadIdx.x < F::NK) s_run[threadIdx.x] = s_base[threadIdx.x] + s_pre[threadIdx.x];
    __syncthreads();
    const PartOffs &o = s_o;
    if (beg64 < n) {
        const int beg = (int)beg64;
        const int end = (n - beg < chunk) ? n : beg + chunk;
        for (int tile = beg; tile < end; tile += PART_BS) {
            const int g = tile + threadIdx.x;
            const bool in = g < end;
            const unsigned m = tile == beg ? m_first : in ? f.cached(g) : 0u;
            int rk[F::NK];
#pragma unroll
            for (int k = 0; k < F::NK; ++k) {
                rk[k] = 0;
                if (!f.used(k)) continue;           // uniform: classes of splits the context does not have
                const uint64_t bal = __ballot((m >> k) & 1u);
                rk[k] = __popcll(bal & lanemask_lt());
                if (lane == 0) s_wcnt[wave][k] = __popcll(bal);
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < F::NK; ++k) {
                if (!f.used(k)) continue;
                int pre = s_run[k];
                for (int w = 0; w < PART_BS / 64; ++w) pre += (w < wave) ? s_wcnt[w][k] : 0;
                rk[k] += pre;
            }
            if (in) f.emit(g, m, rk, o);
            __syncthreads();
            if (threadIdx.x < F::NK && f.used(threadIdx.x)) {
                int add = 0;
                for (int w = 0; w < PART_BS / 64; ++w) add += s_wcnt[w][threadIdx.x];
                s_run[threadIdx.x] += add;
            }
            __syncthreads();
        }
    }
    // (dealt from the last workgroup backwards, like the count pass's side work)
    const int64_t nx = f.n_extra(o);
    for (int64_t g = (int64_t)(gridDim.x - 1 - blockIdx.x) * PART_BS + threadIdx.x; g < nx;
         g += (int64_t)gridDim.x * PART_BS)
        f.extra(g, o);
}

// ---- local_front[L] = targets separated by owner, order kept ---------------------------------
struct PartTargets {
    static constexpr int NK = GS_MAXS;
    const int32_t *targets; int n_targets; const uint8_t *pmap; int S; uint32_t n_vertices;
    int32_t *front; int32_t *perm; GsLevelMeta *meta; GsTable tab_mixed; int fan_top;
    GsLevelMeta *meta_all; int n_levels; GsTable tab_local;
    __device__ int n() const { return n_targets; }
    __device__ bool used(int k) const { return k < S; }
    // an id outside the graph is replaced by vertex 0 and reported through the error flag (by the
    // scatter pass only: the count pass is where the flags of the previous batch are cleared)
    __device__ int32_t target(int g) const {
        const uint32_t id = (uint32_t)targets[g];
        if (id < n_vertices) return (int32_t)id;
        meta->error = 3;
        return 0;
    }
    __device__ unsigned classify(int g) const {
        const uint32_t id = (uint32_t)targets[g];
        return 1u << (pmap[id < n_vertices ? id : 0u] & (GS_MAXS - 1));
    }
    __device__ unsigned cached(int g) const { return classify(g); }
    __device__ int upper_offset(int) const { return 0; }
    __device__ void key_bases(const int *tot, int *bases, PartOffs &o, const int *) const {     // o.a = front_off
        int acc = 0;
        for (int k = 0; k < GS_MAXS; ++k) {
            bases[k] = acc;
            o.a[k] = acc;
            acc += (k < S) ? tot[k] : 0;
        }
        o.a[S] = acc;
    }
    __device__ void publish(const PartOffs &o) const {
        for (int k = 0; k <= S; ++k) meta->front_off[k] = o.a[k];
    }
    __device__ void emit(int g, unsigned m, const int *rk, const PartOffs &) const {
        const int k = __ffs(m) - 1;
        front[rk[k]] = target(g);
        perm[rk[k]] = g;
    }
    // (the tables are clean when a batch starts: the last kernel of the previous batch cleared the
    // part a top layer of max_targets targets can use, gsplit_create all of them)
    __device__ int64_t n_extra(const PartOffs &) const { return 0; }
    __device__ void extra(int64_t, const PartOffs &) const {}
    // the count pass is the first kernel of a batch: it clears the error flags of every level
    __device__ int64_t n_side() const { return n_levels; }
    __device__ void side(int64_t x, int64_t ns) const {
        if (x < ns) meta_all[x].error = 0;
        if (x == 0) meta_all[0].batches += 1;
    }
};

// A batch of at most 1024 targets takes the whole step in one workgroup, one target per thread:
// the two launches of the general partition are chains of a few dependent accesses each, and a
// launch by itself costs about as much as this kernel's work.
constexpr int TARGETS_SMALL = 1024;

struct TargetsSet { PartTargets f[GS_MAXB]; };

__global__ __launch_bounds__(TARGETS_SMALL) void k_targets_small(TargetsSet set) {
    const PartTargets &f = set.f[blockIdx.x];
    __shared__ int s_cnt[TARGETS_SMALL / 64][GS_MAXS];
    __shared__ int s_tot[GS_MAXS], s_base[GS_MAXS];
    __shared__ PartOffs s_o;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    if (tid < f.n_levels) f.meta_all[tid].error = 0;
    if (tid == 0) f.meta_all[0].batches += 1;
    __syncthreads();                                   // the flags are cleared before target() may set one
    const bool in = tid < f.n_targets;
    int32_t id = 0;
    int k = -1;
    if (in) {
        id = f.target(tid);
        k = f.pmap[id] & (GS_MAXS - 1);
    }
    int rank = 0;
#pragma unroll
    for (int c = 0; c < GS_MAXS; ++c) {
        const uint64_t bal = __ballot(k == c);
        if (k == c) rank = __popcll(bal & lanemask_lt());
        if (lane == 0) s_cnt[wave][c] = __popcll(bal);
    }
    __syncthreads();
    if (tid < GS_MAXS) {
        int acc = 0;
        for (int w = 0; w < TARGETS_SMALL / 64; ++w) { const int x = s_cnt[w][tid]; s_cnt[w][tid] = acc; acc += x; }
        s_tot[tid] = acc;
    }
    __syncthreads();
    if (tid == 0) {
        f.key_bases(s_tot, s_base, s_o, nullptr);
        f.publish(s_o);
    }
    __syncthreads();
    if (in) {
        const int r = s_base[k] + s_cnt[wave][k] + rank;
        f.front[r] = id;
        f.perm[r] = tid;
    }
    const int64_t nx = f.n_extra(s_o);
    for (int64_t x = tid; x < nx; x += TARGETS_SMALL) f.extra(x, s_o);
}

// The scatter side of the shuffle index of the sampling layer above (layer l+1) is finished while
// layer l is partitioned: its rows are this layer's destination vertices, and its counters are
// complete once the shuffle-index kernel of layer l+1 has run.  The count pass hands every row a
// segment of rev_list (segments need not be in row order: one atomic per workgroup of 256 rows
// on the cursor, a single address), the scatter pass lists, for every source row, the destination
// rows it feeds (slot q of destination i is a sampled edge when q < cnt[i]).
struct RevUp {
    int on;
    const int32_t *rev_cnt; int32_t *rev_ptr; int32_t *rev_fill; int32_t *rev_list; int32_t *rev_eid;
    const int32_t *cnt; const int32_t *blk_indptr; const int32_t *self_row; const int32_t *edge_row;
    int fan; int32_t *cursor; const GsLevelMeta *meta_up2; int32_t *rev_long; int32_t *n_long;
    __device__ void alloc(int64_t x, int64_t n_rows, int S) const {
        __shared__ int s_wave[PART_BS / 64];
        __shared__ int s_base;
        const int lane = lane_id(), wave = threadIdx.x >> 6;
        const int c = x < n_rows ? rev_cnt[x] : 0;
        int inc = c;
        for (int o = 1; o < 64; o <<= 1) {
            const int below = __shfl_up(inc, o);
            if (lane >= o) inc += below;
        }
        if (lane == 63) s_wave[wave] = inc;
        __syncthreads();
        if (threadIdx.x == 0) {
            int tot = 0;
            for (int w = 0; w < PART_BS / 64; ++w) { const int t = s_wave[w]; s_wave[w] = tot; tot += t; }
            s_base = tot > 0 ? atomicAdd(cursor, tot) : 0;
        }
        __syncthreads();
        if (x < n_rows) {
            rev_ptr[x] = s_base + s_wave[wave] + inc - c;
            rev_fill[x] = 0;
            if (c > GS_REV_LONG) rev_long[atomicAdd(n_long, 1)] = (int32_t)x;      // (rare: one atomic per such row)
        }
        __syncthreads();
    }
    __device__ int64_t n_items(int S) const { return on ? (int64_t)meta_up2->front_off[S] * (1 + fan) : 0; }
    __device__ void fill(int64_t x, int S) const {
        const int n_dst = meta_up2->front_off[S];
        int u, code, eid = -1;
        if (x < n_dst) {
            u = self_row[x];
            code = 2 * (int)x;
        } else {
            const int64_t g = x - n_dst;
            const int i = (int)(g / fan), q = (int)(g - (int64_t)i * fan);
            if (q >= cnt[i]) return;
            eid = blk_indptr[i] + q;
            u = edge_row[eid];
            code = 2 * i + 1;
        }
        if (u < 0) return;
        const int p = atomicAdd(&rev_fill[u], 1);
        rev_list[rev_ptr[u] + p] = code;
        if (rev_eid) rev_eid[rev_ptr[u] + p] = eid;
    }
};

// ---- the partition of a sampling layer: mixed frontiers, block CSR offsets, owner buckets and
// next local frontiers in one pass over the slots.  A slot that is the first occurrence of its
// vertex inside its split s ("winner") gets
//   class s       -> its row in mixed_front_s (destination vertices occupy the rows before)
//   class 8 + t   -> its place in bucket[s -> t], t = f_G(vertex): partitioning the sender-ordered
//                    slot stream by owner yields, for each receiver t, bucket[0->t] | bucket[1->t]
//                    | ...: on one GPU the send buffers and the received concatenation are the
//                    same memory.
// Class 16 counts valid slots: its exclusive rank is the edge number (block CSR offsets).
// A slot that is the first occurrence of its vertex in the whole stream (and whose vertex is not a
// destination vertex, which the table decides: destinations hold the smallest positions) gets
//   class 17 + t  -> its row in local_front[l]_t (the owner's own destination vertices come first).
struct PartLayer {
    static constexpr int NK = PART_NK;
    GsTable tab_mixed, tab_local;
    const int32_t *front; const int32_t *nbr; const uint8_t *pmap;
    int32_t *ent_mixed; int32_t *ent_local; uint32_t *cls; int32_t *mixed_ent;
    int32_t *mixed; int32_t *blk_indptr; int32_t *recv; int32_t *front_lo; int32_t *rev_cnt;
    GsLevelMeta *meta_lo; const GsLevelMeta *meta_up; int S; int fan; int rev;
    RevUp up;
    int layer;
    int32_t *pos_pair; int32_t *mixed_pos;      // a wide layer's (null otherwise)
    __device__ int n1() const { return meta_up->front_off[S]; }
    __device__ int n() const { return n1() * fan; }
    // classes s and 8 + t and 17 + t exist for the splits the context has, class 16 always
    __device__ bool used(int k) const { return k < 8 ? k < S : k < 16 ? k - 8 < S : k == 16 || k - 17 < S; }
    // From here on an element's ent_mixed / ent_local no longer name table entries but the position
    // of the first occurrence of its key (what the entries hold): the rows are handed out by
    // position (tab.row is indexed by it), so the later passes read two small dense arrays instead
    // of following every element into the tables again.
    __device__ unsigned classify(int g) const {
        const int at = n1() + g;
        // what the branches below may need is fetched side by side, the owner byte beside the table
        // entries (read for a slot that turns out not to need it, too: the kernel is a chain of
        // dependent accesses, and every level taken out of the chain shortens it)
        const int h = ent_mixed[at];
        const int32_t id = nbr[g];                          // -1 in an empty slot
        const int hl = ent_local[at];
        const uint32_t idc = id >= 0 ? (uint32_t)id : 0u;
        // (with hashed tables, the form of the large layers, the owner is fetched for the winners alone:
        // such a layer runs at the rate of its random accesses, not of the chain)
        const bool owner_late = !tab_mixed.pos;
        unsigned t = owner_late ? 0u : pmap[idc] & (GS_MAXS - 1);
        const uint32_t pos = (uint32_t)at;
        unsigned m = 0u;
        if (!tab_local.pos && !tab_local.slot) {
            // one table of (vertex, split) keys.  Direct: the vertex's entries for the single splits lie
            // side by side; the slot's own one tells where its key first occurs, the smallest of those
            // that carry this layer's stamp where the vertex first occurs in the whole stream.  Hashed:
            // the slot's own entry, and for a winner the smallest position in the vertex's lines.
            if (h != -1) {
                const int s = split_of(meta_up->front_off, S, g / fan);
                uint32_t first = pos, lfirst = pos;
                if (tab_mixed.pos) {
                    const uint32_t stamp = table_stamp(meta_lo - layer, (uint32_t)layer);
                    const unsigned long long *e = tab_mixed.pos + (size_t)idc * (uint32_t)S;
                    // (all of the vertex's entries are asked for at once; an entry the context does not
                    // have reads as empty, whose upper half is no stamp)
                    unsigned long long v[GS_MAXS];
#pragma unroll
                    for (int ss = 0; ss < GS_MAXS; ++ss) v[ss] = ss < S ? e[ss] : EMPTY_ENTRY;
#pragma unroll
                    for (int ss = 0; ss < GS_MAXS; ++ss) {
                        if (ss == s) first = (uint32_t)v[ss];
                        if ((uint32_t)(v[ss] >> 32) == stamp) lfirst = min(lfirst, (uint32_t)v[ss]);
                    }
                } else {
                    first = (uint32_t)tab_mixed.slot[h >= 0 ? h : -2 - h];
                    if (h >= 0 && first == pos && hl >= 0)       // (one split: the vertex has this one key)
                        lfirst = S == 1 ? first : table_line_first(tab_mixed, table_bits(n1() * (1 + fan)), idc, (uint32_t)S, pos);
                }
                m = 1u << 16;
                ent_mixed[at] = (int32_t)first;
                if (h >= 0 && first == pos) {
                    if (owner_late) t = pmap[idc] & (GS_MAXS - 1);
                    m |= (1u << s) | (1u << (8 + t));
                    if (hl >= 0) {
                        ent_local[at] = (int32_t)lfirst;
                        if (lfirst == pos) m |= 1u << (17 + t);
                    }
                }
            }
            cls[g] = m;
            return m;
        }
        if (h < -1) {       // a valid slot the sampler saw behind another occurrence of its key (entry -2 - h): no winner
            m = 1u << 16;
            ent_mixed[at] = (int32_t)table_pos(tab_mixed, -2 - h);
        }
        if (h >= 0) {
            m = 1u << 16;
            const uint32_t first = table_pos(tab_mixed, h);
            ent_mixed[at] = (int32_t)first;
            if (first == pos) {
                const int s = split_of(meta_up->front_off, S, g / fan);
                if (owner_late) t = pmap[idc] & (GS_MAXS - 1);
                m |= (1u << s) | (1u << (8 + t));
                if (hl >= 0) {
                    const uint32_t lfirst = table_pos(tab_local, hl);
                    ent_local[at] = (int32_t)lfirst;
                    if (lfirst == pos) m |= 1u << (17 + t);
                }
            }
        }
        cls[g] = m;
        return m;
    }
    __device__ unsigned cached(int g) const { return cls[g]; }
    __device__ int upper_offset(int s) const { return meta_up->front_off[s]; }
    // o.a = mixed_off, o.b = recv_off, o.c = front_off of the level below
    __device__ void key_bases(const int *tot, int *bases, PartOffs &o, const int *up) const {
        int acc = 0, racc = 0, lacc = 0;
        for (int s = 0; s < GS_MAXS; ++s) {
            const int n_dst = (s < S) ? up[s + 1] - up[s] : 0;
            o.a[s] = acc; o.b[s] = racc; o.c[s] = lacc;
            bases[s] = acc + n_dst;
            bases[8 + s] = racc;
            bases[17 + s] = lacc + n_dst;
            acc += n_dst + ((s < S) ? tot[s] : 0);
            racc += (s < S) ? tot[8 + s] : 0;
            lacc += n_dst + ((s < S) ? tot[17 + s] : 0);
        }
        o.a[S] = acc;
        o.b[S] = racc;
        o.c[S] = lacc;
        bases[16] = 0;
        o.total = tot[16];
    }
    __device__ void publish(const PartOffs &o) const {
        for (int s = 0; s <= S; ++s) {
            meta_lo->mixed_off[s] = o.a[s]; meta_lo->recv_off[s] = o.b[s]; meta_lo->front_off[s] = o.c[s];
        }
        meta_lo->nnz = o.total;
        blk_indptr[n1()] = o.total;
    }
    __device__ void emit(int g, unsigned m, const int *rk, const PartOffs &o) const {
        const int i = g / fan, q = g - i * fan;
        if (q == 0) {
            blk_indptr[i] = rk[16];
            // the first row of a sender marks where its buckets start at every receiver
            // (senders are consecutive in the slot stream); sizes follow by subtraction on the host
            const int s = split_of(meta_up->front_off, S, i);
            if (i == meta_up->front_off[s])
                for (int ss = s; ss >= 0 && meta_up->front_off[ss] == i; --ss)
                    for (int t = 0; t < S; ++t) meta_lo->bucket_start[ss * GS_MAXS + t] = rk[8 + t];
        }
        const unsigned sm = m & 0xFFu;
        if (!sm) return;
        const int s = __ffs(sm) - 1;
        const int t = __ffs((m >> 8) & 0xFFu) - 1;
        const int32_t id = nbr[g];
        const int at = n1() + g;               // a winner: the first occurrence of its (vertex, split) key
        mixed[rk[s]] = id;
        if (pos_pair) { pos_pair[2 * (size_t)at] = rk[s] - o.a[s]; mixed_pos[rk[s]] = at; }
        else tab_mixed.row[at] = rk[s] - o.a[s];
        mixed_ent[rk[s]] = ent_local[at];      // where the vertex first occurs in the whole stream (-1: no entry)
        recv[rk[8 + t]] = id;
        if ((m >> 17) & 0xFFu) {               // that place is this one
            front_lo[rk[17 + t]] = id;
            tab_local.row[at] = rk[17 + t];
        }
    }
    // scatter pass extras: destination vertices are rows 0 .. n_dst-1 of their split's mixed
    // frontier and of their owner's next local frontier; then (layers that have one) the counters
    // of this layer's reverse index are zeroed; then the reverse index of the layer above is filled
    __device__ int64_t n_extra(const PartOffs &o) const { return n1() + (rev ? o.c[S] : 0) + up.n_items(S); }
    __device__ void extra(int64_t x, const PartOffs &o) const {
        const int64_t own = n1() + (rev ? o.c[S] : 0);
        if (x >= own) {
            up.fill(x - own, S);
            return;
        }
        if (x >= n1()) {
            rev_cnt[x - n1()] = 0;
            if (x == n1()) { meta_lo->rev_cursor = 0; meta_lo->n_long = 0; }
            return;
        }
        const int i = (int)x;
        const int s = split_of(meta_up->front_off, S, i);
        const int loc = i - meta_up->front_off[s];
        const int32_t id = front[i];
        const int hl = ent_local[i];
        const int j = o.a[s] + loc, rowp = o.c[s] + loc;
        // a destination vertex holds the smallest position of both of its keys: position i
        mixed[j] = id;
        if (pos_pair) { pos_pair[2 * (size_t)i] = loc; mixed_pos[j] = i; }
        else tab_mixed.row[i] = loc;
        mixed_ent[j] = hl >= 0 ? i : -1;
        front_lo[rowp] = id;
        tab_local.row[i] = rowp;
    }
    // count pass side work: segments of the reverse index of the layer above
    __device__ int64_t n_side() const { return up.on ? n1() : 0; }
    __device__ void side(int64_t x, int64_t ns) const { up.alloc(x, ns, S); }
};

// shuffle index of every mixed-frontier row, the same lookup composed with edges[l] for the
// on-GPU forward/backward (rows of local_cat[l] per destination vertex and per edge), and edges[l]
// itself relabelled to rows of the owning split's mixed frontier; + reset of both tables for the
// next sampling layer
struct ShuffleArgs {
    GsTable tab_local, tab_mixed;
    const int32_t *ent_mixed, *ent_local, *mixed_ent, *blk_indptr;
    int32_t *blk_src, *src_row, *self_row, *edge_row, *rev_cnt;
    const GsLevelMeta *meta_lo, *meta_up;
    int32_t *pos_pair; const int32_t *mixed_pos;        // a wide layer's (null otherwise)
};
struct ShuffleArgsSet { ShuffleArgs b[GS_MAXB]; };

__global__ __launch_bounds__(256) void k_shuffle_index(ShuffleArgsSet set, int S, int fan, int fan_next, int64_t top_cap) {
    const ShuffleArgs &a = set.b[blockIdx.y];
    const GsTable tab_local = a.tab_local, tab_mixed = a.tab_mixed;
    const int32_t *__restrict__ ent_mixed = a.ent_mixed;
    const int32_t *__restrict__ ent_local = a.ent_local;
    const int32_t *__restrict__ mixed_ent = a.mixed_ent;
    const int32_t *__restrict__ blk_indptr = a.blk_indptr;
    int32_t *__restrict__ blk_src = a.blk_src;
    int32_t *__restrict__ src_row = a.src_row;
    int32_t *__restrict__ self_row = a.self_row;
    int32_t *__restrict__ edge_row = a.edge_row;
    int32_t *__restrict__ rev_cnt = a.rev_cnt;
    const GsLevelMeta *__restrict__ meta_lo = a.meta_lo;
    const GsLevelMeta *__restrict__ meta_up = a.meta_up;
    const int n1 = meta_up->front_off[S];
    const int64_t n_mixed = meta_lo->mixed_off[S];
    // A wide layer leaves the slots to k_shuffle_edges: here every mixed-frontier row also notes its row
    // of local_cat at the position where its key first occurs, beside the row the scatter pass left there.
    const int64_t n_slots = a.pos_pair ? 0 : (int64_t)n1 * fan;
    const int64_t total = n_mixed + n1 + n_slots;
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < total;
         x += (int64_t)gridDim.x * blockDim.x) {
        if (x < n_mixed) {
            const int p = mixed_ent[x];
            const int r = p >= 0 ? tab_local.row[p] : -1;
            src_row[x] = r;
            if (a.pos_pair) a.pos_pair[2 * (size_t)a.mixed_pos[x] + 1] = r;
        } else if (x < n_mixed + n1) {
            const int i = (int)(x - n_mixed);
            const int h = ent_local[i];
            const int r = h >= 0 ? tab_local.row[i] : -1;
            self_row[i] = r;
            if (rev_cnt && r >= 0) atomicAdd(&rev_cnt[r], 1);

        } else {
            const int64_t g = x - n_mixed - n1;
            const int first = ent_mixed[n1 + g];     // where the slot's key first occurs (left by the count pass)
            if (first < 0) continue;
            const int i = (int)(g / fan), q = (int)(g - (int64_t)i * fan);
            const int s = split_of(meta_up->front_off, S, i);
            const int mrow = tab_mixed.row[first];
            const int pl = mixed_ent[meta_lo->mixed_off[s] + mrow];
            const int r = pl >= 0 ? tab_local.row[pl] : -1;
            blk_src[blk_indptr[i] + q] = mrow;          // edges[l] as rows of the split's mixed frontier
            edge_row[blk_indptr[i] + q] = r;
            if (rev_cnt && r >= 0) atomicAdd(&rev_cnt[r], 1);

        }
    }
    // layers above the bottom one: both tables are cleared for the next sampling layer (this kernel
    // only reads their row arrays, through the entry indices the elements remembered)
    // the bottom layer: cleared for the top layer of the next batch instead (top_cap entries cover
    // max_targets targets), so that the batch's first kernel, a single workgroup for a small batch,
    // does not have to
    if (!tab_mixed.pos && (fan_next > 0 || top_cap > 0)) {
        const int64_t nr = fan_next > 0 ? 1ll << table_bits(meta_lo->front_off[S] * (1 + fan_next)) : top_cap;
        const int64_t both = tab_local.slot ? 2 * nr : nr;       // (several splits: there is one table)
        for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < both;
             x += (int64_t)gridDim.x * blockDim.x) {
            if (x < nr) tab_mixed.slot[x] = EMPTY_ENTRY;
            else tab_local.slot[x - nr] = EMPTY_ENTRY;
        }
    }
}

// The slots of a wide layer, after k_shuffle_index.  In one launch a slot is three dependent random
// accesses (the mixed-frontier row kept where its key first occurs -> that row's vertex entry -> its
// row of local_cat), and a wide layer runs at the rate at which the memory completes such accesses;
// once every mixed-frontier row has left its row of local_cat at that same position, a slot is one
// access of 8 bytes.
__global__ __launch_bounds__(256) void k_shuffle_edges(ShuffleArgsSet set, int S, int fan) {
    const ShuffleArgs &a = set.b[blockIdx.y];
    const int32_t *__restrict__ ent_mixed = a.ent_mixed;
    const int32_t *__restrict__ blk_indptr = a.blk_indptr;
    const int2 *__restrict__ pair = reinterpret_cast<const int2 *>(a.pos_pair);
    int32_t *__restrict__ blk_src = a.blk_src;
    int32_t *__restrict__ edge_row = a.edge_row;
    int32_t *__restrict__ rev_cnt = a.rev_cnt;
    const int n1 = a.meta_up->front_off[S];
    const int64_t n_slots = (int64_t)n1 * fan;
    for (int64_t g = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; g < n_slots;
         g += (int64_t)gridDim.x * blockDim.x) {
        const int first = ent_mixed[n1 + g];
        if (first < 0) continue;
        const int i = (int)(g / fan), q = (int)(g - (int64_t)i * fan);
        const int2 v = pair[first];
        const int e = blk_indptr[i] + q;
        blk_src[e] = v.x;
        edge_row[e] = v.y;
        if (rev_cnt && v.y >= 0) atomicAdd(&rev_cnt[v.y], 1);
    }
}

// reverse index as two launches of its own (blockIdx.y = layer - first): used for the bottom layer,
// which has no partition below it; same steps as RevUp::alloc / RevUp::fill
struct RevArgs {
    const int32_t *rev_cnt; int32_t *rev_ptr; int32_t *rev_fill; int32_t *rev_list; int32_t *rev_eid; int32_t *rev_long;
    const int32_t *cnt; const int32_t *blk_indptr; const int32_t *self_row; const int32_t *edge_row;
    GsLevelMeta *meta;          // the batch's level bookkeeping, [L + 1]
};
struct RevArgsSet { RevArgs b[GS_MAXB]; };

// step 2: give every row of local_cat[l] a segment of rev_list (segments need not be in row order:
// one atomic per workgroup of 1024 rows hands out space; the cursor is a single address, and an
// atomic on it from every wave of a million-row level took longer than the rest of the kernel)
__global__ __launch_bounds__(1024) void k_rev_alloc(RevArgsSet set, int l, int S) {
    __shared__ int s_wave[16];
    __shared__ int s_base;
    const RevArgs &a = set.b[blockIdx.y];
    GsLevelMeta *meta_lo = a.meta + l;
    const int32_t *__restrict__ rev_cnt = a.rev_cnt;
    int32_t *__restrict__ rev_ptr = a.rev_ptr;
    int32_t *__restrict__ rev_fill = a.rev_fill;
    const int n_lo = meta_lo->front_off[S];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int stride = gridDim.x * blockDim.x;
    const int rounds = (n_lo + stride - 1) / stride;
    for (int it = 0; it < rounds; ++it) {
        const int u = it * stride + blockIdx.x * blockDim.x + threadIdx.x;
        const int c = u < n_lo ? rev_cnt[u] : 0;
        int inc = c;
        for (int o = 1; o < 64; o <<= 1) {
            int up = __shfl_up(inc, o);
            if (lane >= o) inc += up;
        }
        if (lane == 63) s_wave[wave] = inc;
        __syncthreads();
        if (threadIdx.x == 0) {
            int tot = 0;
            for (int w = 0; w < 16; ++w) { const int x = s_wave[w]; s_wave[w] = tot; tot += x; }
            s_base = tot > 0 ? atomicAdd(&meta_lo->rev_cursor, tot) : 0;
        }
        __syncthreads();
        if (u < n_lo) {
            rev_ptr[u] = s_base + s_wave[wave] + inc - c;
            rev_fill[u] = 0;
            if (c > GS_REV_LONG) a.rev_long[atomicAdd(&meta_lo->n_long, 1)] = u;
        }
        __syncthreads();
    }
}

// step 3: list, for every source row, the destination rows it feeds (slot q of destination i is a
// sampled edge when q < cnt[i])
__global__ __launch_bounds__(256) void k_rev_fill(RevArgsSet set, int l, int fan, int S) {
    const RevArgs &a = set.b[blockIdx.y];
    const int32_t *__restrict__ cnt = a.cnt;
    const int32_t *__restrict__ blk_indptr = a.blk_indptr;
    const int32_t *__restrict__ self_row = a.self_row;
    const int32_t *__restrict__ edge_row = a.edge_row;
    const int32_t *__restrict__ rev_ptr = a.rev_ptr;
    int32_t *__restrict__ rev_fill = a.rev_fill;
    int32_t *__restrict__ rev_list = a.rev_list;
    int32_t *__restrict__ rev_eid = a.rev_eid;
    const int n1 = a.meta[l + 1].front_off[S];
    const int64_t total = (int64_t)n1 * (1 + fan);
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < total;
         x += (int64_t)gridDim.x * blockDim.x) {
        int u, code, eid = -1;
        if (x < n1) {
            u = self_row[x];
            code = 2 * (int)x;
        } else {
            const int64_t g = x - n1;
            const int i = (int)(g / fan), q = (int)(g - (int64_t)i * fan);
            if (q >= cnt[i]) continue;
            eid = blk_indptr[i] + q;
            u = edge_row[eid];
            code = 2 * i + 1;
        }
        if (u < 0) continue;
        const int p = atomicAdd(&rev_fill[u], 1);
        rev_list[rev_ptr[u] + p] = code;
        if (rev_eid) rev_eid[rev_ptr[u] + p] = eid;
    }
}

int part_blocks(int64_t upper_items) {
    return upper_items <= (1 << 18) ? 256 : upper_items <= (1 << 20) ? 512 : PART_MAX_NB;
}

// kernel arguments are limited to 4 KiB
static_assert(sizeof(PartSet<PartLayer>) <= 4096 && sizeof(PartSet<PartTargets>) <= 4096 && sizeof(TargetsSet) <= 4096 &&
              sizeof(SampleArgsSet) <= 3072 && sizeof(ShuffleArgsSet) <= 3072 && sizeof(RevArgsSet) <= 3072,
              "argument block of a multi-batch launch too large");

template <class F>
void run_partition(gsplit_ctx *const *ctxs, int nbat, const PartSet<F> &set, int64_t upper_items, hipStream_t st,
                   const char *name, int layer) {
    gsplit_ctx *ctx = ctxs[0];
    const int nb = part_blocks(upper_items);
    const std::string nm(name);
    {
        GsTimeScope ts(ctx, (nm + "_count").c_str(), layer, st);
        hipLaunchKernelGGL(k_part_count<F>, dim3(nb, nbat), dim3(PART_BS), 0, st, set);
    }
    GsTimeScope ts(ctx, (nm + "_scatter").c_str(), layer, st);
    if (nb == 256)
        hipLaunchKernelGGL((k_part_scatter<F, 1>), dim3(nb, nbat), dim3(PART_BS), 0, st, set);
    else if (nb == 512)
        hipLaunchKernelGGL((k_part_scatter<F, 2>), dim3(nb, nbat), dim3(PART_BS), 0, st, set);
    else
        hipLaunchKernelGGL((k_part_scatter<F, 4>), dim3(nb, nbat), dim3(PART_BS), 0, st, set);
}

// grid of a grid-stride kernel over upper_items elements; with several batches in the launch the
// cap on resident workgroups is shared between them
int grid_for(const gsplit_ctx *ctx, int64_t upper_items, int nbat = 1) {
    int64_t want = gs_ceil_div(upper_items, 256);
    int64_t cap = std::max<int64_t>(1, (int64_t)ctx->n_cu * ctx->sampler_blocks_per_cu / nbat);
    if (want < 1) want = 1;
    return (int)(want < cap ? want : cap);
}

template <typename IndPtrT>
void launch_sample(gsplit_ctx *const *ctxs, int nbat, int l, uint64_t seed, const uint64_t *iters,
                   const uint64_t *d_seed_iter, hipStream_t st) {
    gsplit_ctx *ctx = ctxs[0];
    const int fan = ctx->fan[l];
    const int64_t ub = ctx->ub_front[l + 1];
    const IndPtrT *ip = (const IndPtrT *)ctx->graph.d_indptr;
    SampleArgsSet set{};
    for (int b = 0; b < nbat; ++b) {
        gsplit_ctx *c = ctxs[b];
        GsLayerBuf &B = c->layer[l];
        set.b[b] = SampleArgs{c->front[l + 1], c->d_meta + l, c->d_meta + (l + 1), c->tab_mixed, c->tab_local,
                              c->ent_mixed, c->ent_local, B.nbr, B.cnt, B.epos, iters[b], d_seed_iter};
    }
    GsTimeScope ts(ctx, "sample_layer", l, st);
    if (fan <= 16) {
        hipLaunchKernelGGL((k_sample_layer<16, IndPtrT>), dim3(grid_for(ctx, ub * 16, nbat), nbat), dim3(256), 0, st,
                           ip, ctx->graph.d_indices, set, ctx->S, fan, (uint32_t)l, seed);
    } else if (fan <= 32) {
        hipLaunchKernelGGL((k_sample_layer<32, IndPtrT>), dim3(grid_for(ctx, ub * 32, nbat), nbat), dim3(256), 0, st,
                           ip, ctx->graph.d_indices, set, ctx->S, fan, (uint32_t)l, seed);
    } else {
        hipLaunchKernelGGL((k_sample_layer<64, IndPtrT>), dim3(grid_for(ctx, ub * 64, nbat), nbat), dim3(256), 0, st,
                           ip, ctx->graph.d_indices, set, ctx->S, fan, (uint32_t)l, seed);
    }
}

// Algorithm 1 for nbat mini-batches at once, one context each (same graph, same configuration)
int sample_split(gsplit_ctx *const *ctxs, int nbat, const int32_t *const *d_targets, const int64_t *n_targets,
                 uint64_t seed, const uint64_t *iters, const uint64_t *d_seed_iter, void *stream) {
    gsplit_ctx *ctx = ctxs[0];
    for (int b = 0; b < nbat; ++b) {
        if (n_targets[b] < 0 || (n_targets[b] > 0 && !d_targets[b]))
            return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_sample_split: bad targets");
        if (n_targets[b] > ctxs[b]->max_targets)
            return gs_fail(ctx, GSPLIT_ECAPACITY, "gsplit_sample_split: n_targets exceeds max_targets");
    }
    hipStream_t st = (hipStream_t)stream;
    const int S = ctx->S, L = ctx->L;
    // Under stream capture the calls of a step become nodes of a graph: no event is recorded for the
    // host-side queries (they synchronise the device instead) and no timing events are taken.
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) != hipSuccess) {
        (void)hipGetLastError();
        cap = hipStreamCaptureStatusNone;
    }
    bool all_small = true;
    for (int b = 0; b < nbat; ++b) {
        gsplit_ctx *c = ctxs[b];
        c->captured = cap == hipStreamCaptureStatusActive;
        c->batch_id += 1;
        c->n_targets = n_targets[b];
        c->h_meta_valid = false;
        c->sage.fwd_done = false;
        c->last_stream = st;
        all_small = all_small && n_targets[b] <= TARGETS_SMALL;
    }

    int64_t top_cap = 1024;                             // = 1 << table_bits(max_targets * (1 + fan_top))
    while (top_cap < 2 * ctx->max_targets * (1 + ctx->fan[L - 1])) top_cap <<= 1;
    {
        auto targets_of = [&](int b) {
            gsplit_ctx *c = ctxs[b];
            return PartTargets{d_targets[b], (int)n_targets[b], c->graph.d_pmap, S, (uint32_t)c->graph.n_vertices,
                               c->front[L], c->target_perm, c->d_meta + L, c->tab_mixed, c->fan[L - 1],
                               c->d_meta, L + 1, c->tab_local};
        };
        if (all_small) {
            TargetsSet set{};
            for (int b = 0; b < nbat; ++b) set.f[b] = targets_of(b);
            GsTimeScope ts(ctx, "targets", -1, st);
            hipLaunchKernelGGL(k_targets_small, dim3(nbat), dim3(TARGETS_SMALL), 0, st, set);
        } else {
            PartSet<PartTargets> set{};
            for (int b = 0; b < nbat; ++b) { set.f[b] = targets_of(b); set.hist[b] = ctxs[b]->part_hist; }
            run_partition(ctxs, nbat, set, ctx->ub_front[L], st, "targets", -1);
        }
    }

    for (int l = L - 1; l >= 0; --l) {
        const int fan = ctx->fan[l];
        const int64_t ub1 = ctx->ub_front[l + 1];

        if (ctx->graph.indptr_is_64) launch_sample<int64_t>(ctxs, nbat, l, seed, iters, d_seed_iter, st);
        else launch_sample<int32_t>(ctxs, nbat, l, seed, iters, d_seed_iter, st);

        PartSet<PartLayer> pset{};
        ShuffleArgsSet sset{};
        bool wide = ub1 * fan >= ctx->wide_slots;
        for (int b = 0; b < nbat; ++b) wide = wide && ctxs[b]->pos_pair && ctxs[b]->mixed_pos;
        for (int b = 0; b < nbat; ++b) {
            gsplit_ctx *c = ctxs[b];
            GsLayerBuf &B = c->layer[l];
            GsLevelMeta *ml = c->d_meta + l;
            const GsLevelMeta *mu = c->d_meta + (l + 1);
            PartLayer pa{c->tab_mixed, c->tab_local, c->front[l + 1], B.nbr, c->graph.d_pmap,
                         c->ent_mixed, c->ent_local, c->cls, c->mixed_ent,
                         B.mixed, B.blk_indptr, B.recv, c->front[l], B.rev_cnt,
                         ml, mu, S, fan, l >= c->rev_from ? 1 : 0, RevUp{}, l,
                         wide ? c->pos_pair : nullptr, wide ? c->mixed_pos : nullptr};
            if (l + 1 < L && l + 1 >= c->rev_from) {
                const GsLayerBuf &U = c->layer[l + 1];
                pa.up = RevUp{1, U.rev_cnt, U.rev_ptr, U.rev_fill, U.rev_list, U.rev_eid, U.cnt, U.blk_indptr,
                              U.self_row, U.edge_row, c->fan[l + 1], &c->d_meta[l + 1].rev_cursor, c->d_meta + (l + 2),
                              U.rev_long, &c->d_meta[l + 1].n_long};
            }
            pset.f[b] = pa;
            pset.hist[b] = c->part_hist;
            sset.b[b] = ShuffleArgs{c->tab_local, c->tab_mixed, c->ent_mixed, c->ent_local, c->mixed_ent, B.blk_indptr,
                                    B.blk_src, B.src_row, B.self_row, B.edge_row, l >= c->rev_from ? B.rev_cnt : nullptr,
                                    ml, mu, wide ? c->pos_pair : nullptr, wide ? c->mixed_pos : nullptr};
        }
        run_partition(ctxs, nbat, pset, ub1 * fan, st, "mixed_buckets", l);
        {
            GsTimeScope ts(ctx, "shuffle_index", l, st);
            hipLaunchKernelGGL(k_shuffle_index, dim3(grid_for(ctx, ub1 * (2 + 2 * fan), nbat), nbat), dim3(256), 0, st,
                               sset, S, fan, l > 0 ? ctx->fan[l - 1] : 0, l == 0 ? top_cap : 0);
        }
        if (wide) {
            GsTimeScope ts(ctx, "shuffle_edges", l, st);
            hipLaunchKernelGGL(k_shuffle_edges, dim3(grid_for(ctx, ub1 * fan, nbat), nbat), dim3(256), 0, st, sset, S, fan);
        }
    }
    // the bottom layer's reverse index (contexts that keep one) has no partition below it to ride on
    if (ctx->rev_from == 0) {
        RevArgsSet ra{};
        for (int b = 0; b < nbat; ++b) {
            const GsLayerBuf &B = ctxs[b]->layer[0];
            ra.b[b] = RevArgs{B.rev_cnt, B.rev_ptr, B.rev_fill, B.rev_list, B.rev_eid, B.rev_long, B.cnt, B.blk_indptr,
                              B.self_row, B.edge_row, ctxs[b]->d_meta};
        }
        const int64_t rows = std::max<int64_t>(1, ctx->ub_front[0]);
        const int64_t items = std::max<int64_t>(1, ctx->ub_front[1] * (1 + ctx->fan[0]));
        {
            GsTimeScope ts(ctx, "rev_alloc", -1, st);
            hipLaunchKernelGGL(k_rev_alloc, dim3((unsigned)std::max<int64_t>(1, std::min<int64_t>(
                                   (int64_t)ctx->n_cu * 2, gs_ceil_div(rows, 1024))), nbat), dim3(1024), 0, st, ra, 0, S);
        }
        GsTimeScope ts(ctx, "rev_fill", -1, st);
        hipLaunchKernelGGL(k_rev_fill, dim3(grid_for(ctx, items, nbat), nbat), dim3(256), 0, st, ra, 0, ctx->fan[0], S);
    }
    GS_HIP(ctx, hipGetLastError());
    for (int b = 0; b < nbat; ++b)
        if (!ctxs[b]->captured && ctxs[b]->sample_done) GS_HIP(ctx, hipEventRecord(ctxs[b]->sample_done, st));
    return GSPLIT_OK;
}

// ------------------------------------------------------------------------------------------
// The same step without any allocation: everything a context would own (tables, per-element entry
// indices, class masks, histograms, level bookkeeping) lives in one static device array, carved up
// per call.  Each GPU holds its own copy of the array at its own address, taken once per device.
// ------------------------------------------------------------------------------------------
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)GSPLIT_NOALLOC_SCRATCH_MIB << 20;
constexpr int NOALLOC_MAX_DEVICES = 64;

static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

struct NoAllocDevice { unsigned char *ptr = nullptr; int n_cu = 0; };
NoAllocDevice g_noalloc[NOALLOC_MAX_DEVICES];
std::mutex g_noalloc_mutex;

// device address of this GPU's copy of the array (and its compute-unit count), taken on the first
// call with that device current
int noalloc_device(NoAllocDevice **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= NOALLOC_MAX_DEVICES)
        return gs_fail(nullptr, GSPLIT_EHIP, "gsplit_sample_split_noalloc: no current HIP device");
    std::lock_guard<std::mutex> lock(g_noalloc_mutex);
    NoAllocDevice &d = g_noalloc[dev];
    if (!d.ptr) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return gs_fail(nullptr, GSPLIT_EHIP, std::string("gsplit_sample_split_noalloc: hipGetSymbolAddress: ") +
                                                     hipGetErrorString(e));
        int n_cu = 0;
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) n_cu = 256;
        d.n_cu = n_cu;
        d.ptr = (unsigned char *)p;
    }
    *out = &d;
    return GSPLIT_OK;
}

// every table entry of the part a call can use starts empty, the level bookkeeping at zero (a fill
// kernel, not a memset: the call may be recorded into a graph)
__global__ __launch_bounds__(256) void k_noalloc_reset(GsTable a, GsTable b, int64_t n_entries, int32_t *meta_words,
                                                       int n_meta_words) {
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < n_entries; x += (int64_t)gridDim.x * blockDim.x) {
        a.slot[x] = EMPTY_ENTRY;
        if (b.slot && b.slot != a.slot) b.slot[x] = EMPTY_ENTRY;
    }
    if (blockIdx.x == 0)
        for (int x = threadIdx.x; x < n_meta_words; x += blockDim.x) meta_words[x] = 0;
}

// split offsets of every level and layer, from the internal bookkeeping to the caller's arrays
__global__ void k_noalloc_export(const GsLevelMeta *__restrict__ meta, int L, int S, int32_t *local_off,
                                 int32_t *mixed_off, int32_t *recv_off) {
    const int per = S + 1;
    for (int x = threadIdx.x; x < (L + 1) * per; x += blockDim.x) local_off[x] = meta[x / per].front_off[x % per];
    for (int x = threadIdx.x; x < L * per; x += blockDim.x) {
        mixed_off[x] = meta[x / per].mixed_off[x % per];
        recv_off[x] = meta[x / per].recv_off[x % per];
    }
}

}  // namespace

extern "C" int gsplit_sample_split_noalloc(const gsplit_graph *g, const gsplit_config *c, const int32_t *d_targets,
                                           int64_t n_targets, uint64_t seed, uint64_t iter,
                                           const gsplit_batch_out *out, void *stream) {
    const char *who = "gsplit_sample_split_noalloc: ";
    if (!g || !c || !out) return gs_fail(nullptr, GSPLIT_EINVAL, std::string(who) + "NULL argument");
    if (g->n_vertices <= 0 || g->n_vertices >= (1ll << 31) || g->n_edges < 0 || !g->d_indptr ||
        (g->n_edges > 0 && !g->d_indices) || !g->d_pmap || g->n_splits < 1 || g->n_splits > GSPLIT_MAX_SPLITS ||
        (unsigned long long)g->n_vertices * (unsigned long long)g->n_splits >= 0xFFFFFFFFull)
        return gs_fail(nullptr, GSPLIT_EINVAL, std::string(who) + "bad graph");
    if (c->n_layers < 1 || c->n_layers > GSPLIT_MAX_LAYERS || !c->fanouts || c->max_targets < 1 ||
        c->max_targets > g->n_vertices)
        return gs_fail(nullptr, GSPLIT_EINVAL, std::string(who) + "bad config");
    if (c->keep_edge_ids || c->gat_index)
        return gs_fail(nullptr, GSPLIT_EINVAL, std::string(who) + "keep_edge_ids and gat_index need a context");
    for (int l = 0; l < c->n_layers; ++l)
        if (c->fanouts[l] < 1 || c->fanouts[l] > GSPLIT_MAX_FANOUT)
            return gs_fail(nullptr, GSPLIT_EINVAL, std::string(who) + "fanout out of range");
    if (n_targets < 0 || (n_targets > 0 && !d_targets)) return gs_fail(nullptr, GSPLIT_EINVAL, std::string(who) + "bad targets");
    if (n_targets > c->max_targets) return gs_fail(nullptr, GSPLIT_ECAPACITY, std::string(who) + "n_targets exceeds max_targets");
    const int L = c->n_layers, S = g->n_splits;
    if (!out->d_local_off || !out->d_mixed_off || !out->d_recv_off)
        return gs_fail(nullptr, GSPLIT_EINVAL, std::string(who) + "NULL output");
    for (int l = 0; l <= L; ++l)
        if (!out->d_local_cat[l]) return gs_fail(nullptr, GSPLIT_EINVAL, std::string(who) + "NULL output");
    for (int l = 0; l < L; ++l)
        if (!out->d_nbr[l] || !out->d_cnt[l] || !out->d_mixed_cat[l] || !out->d_blk_indptr[l] || !out->d_blk_src[l] ||
            !out->d_shuffle_src_row[l] || !out->d_recv_cat[l])
            return gs_fail(nullptr, GSPLIT_EINVAL, std::string(who) + "NULL output");

    // a context on the host stack whose buffers are the caller's outputs and pieces of the static array
    gsplit_ctx ctx;
    ctx.graph = *g;
    ctx.L = L; ctx.S = S;
    ctx.max_targets = c->max_targets;
    ctx.sampler_blocks_per_cu = c->sampler_blocks_per_cu > 0 ? std::min(c->sampler_blocks_per_cu, 8) : 8;
    ctx.rev_from = L;                     // no scatter side: it serves the training passes of a context
    for (int l = 0; l < L; ++l) ctx.fan[l] = c->fanouts[l];
    ctx.ub_front[L] = c->max_targets;
    int64_t tab_cap = 1024, max_items = 1024;
    for (int l = L - 1; l >= 0; --l) {
        const int64_t grown = ctx.ub_front[l + 1] * (1 + ctx.fan[l]);
        max_items = std::max(max_items, grown);
        ctx.ub_front[l] = std::min<int64_t>(g->n_vertices, grown);
        while (tab_cap < 2 * grown) tab_cap <<= 1;
        if (grown >= (1ll << 29)) { max_items = 1ll << 40; break; }
    }
    ctx.tab_cap = tab_cap;
    size_t need = 0;
    auto carve = [&](size_t bytes) { const size_t at = need; need += (bytes + 255) & ~(size_t)255; return at; };
    const size_t o_meta = carve(sizeof(GsLevelMeta) * (L + 1));
    const size_t o_mslot = carve(sizeof(unsigned long long) * tab_cap), o_mrow = carve(sizeof(int32_t) * max_items);
    const size_t o_lrow = carve(sizeof(int32_t) * max_items);
    const size_t o_em = carve(sizeof(int32_t) * max_items), o_el = carve(sizeof(int32_t) * max_items);
    const size_t o_me = carve(sizeof(int32_t) * max_items), o_cls = carve(sizeof(uint32_t) * max_items);
    const size_t o_self = carve(sizeof(int32_t) * max_items), o_edge = carve(sizeof(int32_t) * max_items);
    const size_t o_hist = carve(sizeof(int32_t) * PART_MAX_NB * PART_NK);
    const size_t o_perm = carve(sizeof(int32_t) * ctx.ub_front[L]);
    if (max_items >= (1ll << 29) || need > NOALLOC_SCRATCH_BYTES)
        return gs_fail(nullptr, GSPLIT_ECAPACITY,
                       std::string(who) + "max_targets and fanouts need " + std::to_string(need >> 10) +
                           " KiB of working memory, the static array holds " +
                           std::to_string(NOALLOC_SCRATCH_BYTES >> 10) + " KiB; use a context (gsplit_create)");
    NoAllocDevice *dev = nullptr;
    int rc = noalloc_device(&dev);
    if (rc != GSPLIT_OK) return rc;
    unsigned char *base = dev->ptr;       // this GPU's copy of the array (never the array's name on the host)
    ctx.n_cu = dev->n_cu;
    ctx.d_meta = (GsLevelMeta *)(base + o_meta);
    ctx.tab_mixed = GsTable{(unsigned long long *)(base + o_mslot), (int32_t *)(base + o_mrow), nullptr};
    // (the table of (vertex, split) keys serves as both)
    ctx.tab_local = GsTable{nullptr, (int32_t *)(base + o_lrow), nullptr};
    ctx.ent_mixed = (int32_t *)(base + o_em); ctx.ent_local = (int32_t *)(base + o_el);
    ctx.mixed_ent = (int32_t *)(base + o_me); ctx.cls = (uint32_t *)(base + o_cls);
    ctx.part_hist = (int32_t *)(base + o_hist);
    ctx.target_perm = (int32_t *)(base + o_perm);
    for (int l = 0; l <= L; ++l) ctx.front[l] = out->d_local_cat[l];
    for (int l = 0; l < L; ++l) {
        GsLayerBuf &B = ctx.layer[l];
        B.nbr = out->d_nbr[l]; B.cnt = out->d_cnt[l]; B.mixed = out->d_mixed_cat[l]; B.blk_indptr = out->d_blk_indptr[l];
        B.blk_src = out->d_blk_src[l]; B.recv = out->d_recv_cat[l]; B.src_row = out->d_shuffle_src_row[l];
        // the shuffle index composed with edges[l] is a by-product nobody reads here: one region for all layers
        B.self_row = (int32_t *)(base + o_self); B.edge_row = (int32_t *)(base + o_edge);
    }
    hipStream_t st = (hipStream_t)stream;
    // the array keeps what the last call left: clear the table entries this call can touch and the
    // level bookkeeping before the first kernel reads them
    hipLaunchKernelGGL(k_noalloc_reset, dim3((unsigned)std::min<int64_t>(1024, gs_ceil_div(tab_cap, 256))), dim3(256), 0, st,
                       ctx.tab_mixed, ctx.tab_local, tab_cap, (int32_t *)ctx.d_meta,
                       (int)(sizeof(GsLevelMeta) * (L + 1) / sizeof(int32_t)));
    gsplit_ctx *one = &ctx;
    rc = sample_split(&one, 1, &d_targets, &n_targets, seed, &iter, nullptr, stream);
    if (rc != GSPLIT_OK) return gs_fail(nullptr, rc, std::string(who) + ctx.err);
    hipLaunchKernelGGL(k_noalloc_export, dim3(1), dim3(64), 0, st, ctx.d_meta, L, S, out->d_local_off, out->d_mixed_off,
                       out->d_recv_off);
    if (hipGetLastError() != hipSuccess) return gs_fail(nullptr, GSPLIT_EHIP, std::string(who) + "kernel launch failed");
    return GSPLIT_OK;
}

extern "C" int gsplit_sample_split(gsplit_ctx *ctx, const int32_t *d_targets, int64_t n_targets,
                                   uint64_t seed, uint64_t iter, void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    return sample_split(&ctx, 1, &d_targets, &n_targets, seed, &iter, nullptr, stream);
}

extern "C" int gsplit_sample_split_multi(gsplit_ctx *const *ctxs, int32_t n_batches, const int32_t *const *d_targets,
                                         const int64_t *n_targets, uint64_t seed, const uint64_t *iters, void *stream) {
    if (!ctxs || n_batches < 1 || !ctxs[0]) return GSPLIT_EINVAL;
    gsplit_ctx *first = ctxs[0];
    if (n_batches > GSPLIT_MAX_MULTI)
        return gs_fail(first, GSPLIT_ECAPACITY, "gsplit_sample_split_multi: more than GSPLIT_MAX_MULTI batches");
    if (!d_targets || !n_targets || !iters) return gs_fail(first, GSPLIT_EINVAL, "gsplit_sample_split_multi: NULL argument");
    for (int b = 0; b < n_batches; ++b) {
        const gsplit_ctx *c = ctxs[b];
        if (!c) return gs_fail(first, GSPLIT_EINVAL, "gsplit_sample_split_multi: NULL context");
        for (int a = 0; a < b; ++a)
            if (ctxs[a] == c) return gs_fail(first, GSPLIT_EINVAL, "gsplit_sample_split_multi: a context is listed twice");
        bool same = c->L == first->L && c->S == first->S && c->max_targets == first->max_targets &&
                    c->keep_edge_ids == first->keep_edge_ids && c->gat_index == first->gat_index &&
                    c->sampler_blocks_per_cu == first->sampler_blocks_per_cu && c->direct_tables == first->direct_tables &&
                    c->graph.d_indptr == first->graph.d_indptr && c->graph.d_indices == first->graph.d_indices &&
                    c->graph.d_pmap == first->graph.d_pmap && c->graph.n_vertices == first->graph.n_vertices &&
                    c->graph.indptr_is_64 == first->graph.indptr_is_64;
        for (int l = 0; same && l < first->L; ++l) same = c->fan[l] == first->fan[l];
        if (!same)
            return gs_fail(first, GSPLIT_EINVAL, "gsplit_sample_split_multi: the contexts differ in graph or configuration");
    }
    return sample_split(ctxs, n_batches, d_targets, n_targets, seed, iters, nullptr, stream);
}

extern "C" int gsplit_sample_split_dev(gsplit_ctx *ctx, const int32_t *d_targets, int64_t n_targets,
                                       const uint64_t *d_seed_iter, void *stream) {
    if (!ctx) return GSPLIT_EINVAL;
    if (!d_seed_iter) return gs_fail(ctx, GSPLIT_EINVAL, "gsplit_sample_split_dev: NULL seed / iteration buffer");
    const uint64_t zero = 0;
    return sample_split(&ctx, 1, &d_targets, &n_targets, 0, &zero, d_seed_iter, stream);
}
