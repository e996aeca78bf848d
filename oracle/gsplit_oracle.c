/*
 * CPU ORACLE -- test infrastructure only.
 *
 * A plain, slow, single-threaded restatement of one split-parallel mini-batch iteration as the
 * GSplit paper defines it (section 3 "Training pipeline" running example, section 4 online
 * splitting through the global partition function f_G, section 5 Algorithm 1 `sp_sample` and
 * Algorithm 2 `sp_forward`, plus the backward description that follows Algorithm 2).
 *
 * Only tests, the smoke check and the benchmark's cpu-baseline leg may call this.  It shares no
 * code, header, table or constant generator with the HIP library: its Philox, its Floyd
 * selection, its dedup and its aggregation are written here, on their own, from the published
 * definitions.  Every function takes flat host arrays and does exactly one step of the paper's
 * pipeline, in the paper's order, without blocking, fusion or reordering.
 *
 * Pins (see tests/): Philox against the known-answer vectors published with the generator;
 * Floyd against exhaustive enumeration of its random choices; the sampler against brute-force
 * k-hop expansion; split/dedup/relabel against set invariants and the paper's worked example;
 * aggregation against a dense-matrix product.  Nothing here is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",   */
/* SC'11).  Counter-based: out = bijection_key(counter).  Ten rounds; each round multiplies     */
/* words 0 and 2 by fixed odd constants, swaps the halves around, and xors in the key; the key  */
/* is bumped by the Weyl constants between rounds.                                              */
/* ------------------------------------------------------------------------------------------ */
void gso_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The draw-th 32-bit random word that vertex v consumes when it is expanded at sampling layer
 * `layer` of iteration `iter` under `seed`.  Keyed on the GLOBAL vertex id (never on a position
 * in a frontier), so that a vertex draws the same neighbours whichever split expands it: this is
 * what makes a split mini-batch identical to the unsplit one (section 3: splits partition one
 * mini-batch).
 *   key     = (seed low word, seed high word)
 *   counter = (v, iter low word, iter high word, layer * 65536 + draw / 4);  word = draw mod 4
 */
uint32_t gso_philox_word(uint64_t seed, uint64_t iter, uint32_t layer, uint32_t v, uint32_t draw)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t ctr[4] = { v, (uint32_t)iter, (uint32_t)(iter >> 32), (layer << 16) | (draw >> 2) };
    uint32_t out[4];
    gso_philox4x32_10(ctr, key, out);
    return out[draw & 3u];
}

/* ------------------------------------------------------------------------------------------ */
/* Floyd's algorithm for a uniform k-subset of {0..d-1} (Bentley & Floyd, CACM 1987):           */
/*   for j = d-k .. d-1:  t = uniform in [0, j];  insert t if new, else insert j.               */
/* Step i (0-based) uses random word words[i]; the word is mapped to [0, j] by the multiply-     */
/* high rule t = floor(word * (j+1) / 2^32).  chosen[i] is the position inserted at step i       */
/* (so the output order is insertion order).  Requires 0 < k < d.                                */
/* ------------------------------------------------------------------------------------------ */
void gso_floyd_select(int64_t d, int32_t k, const uint32_t *words, int64_t *chosen)
{
    for (int32_t i = 0; i < k; ++i) {
        int64_t j = d - k + i;
        int64_t t = (int64_t)(((uint64_t)words[i] * (uint64_t)(j + 1)) >> 32);
        int seen = 0;
        for (int32_t q = 0; q < i; ++q)
            if (chosen[q] == t) seen = 1;
        chosen[i] = seen ? j : t;
    }
}

/* ------------------------------------------------------------------------------------------ */
/* sample_layer (Algorithm 1, first line of the loop body; "standard neighborhood sampling" of  */
/* section 6.1).  For every vertex of a local frontier take min(deg, fan) distinct neighbours,   */
/* uniformly without replacement: all of them in CSR order when deg <= fan, otherwise the CSR    */
/* positions picked by Floyd's algorithm, in insertion order.  Output is slot-padded:            */
/* nbr[i*fan + q] for q < cnt[i] (remaining slots are set to -1).  epos (may be NULL) receives    */
/* the CSR position of the edge behind every slot (-1 for padding): the edge identity that the   */
/* pre-sampling stage of section 4 counts.                                                       */
/* ------------------------------------------------------------------------------------------ */
void gso_sample_layer(const int64_t *indptr, const int32_t *indices,
                      const int32_t *frontier, int64_t n_front, int32_t fan, uint32_t layer,
                      uint64_t seed, uint64_t iter, int32_t *nbr, int32_t *cnt, int64_t *epos)
{
    uint32_t *words = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(fan > 0 ? fan : 1));
    int64_t *chosen = (int64_t *)malloc(sizeof(int64_t) * (size_t)(fan > 0 ? fan : 1));
    for (int64_t i = 0; i < n_front; ++i) {
        int32_t v = frontier[i];
        int64_t beg = indptr[v], d = indptr[v + 1] - indptr[v];
        int32_t *row = nbr + i * fan;
        int64_t *prow = epos ? epos + i * fan : NULL;
        for (int32_t q = 0; q < fan; ++q) row[q] = -1;
        if (prow) for (int32_t q = 0; q < fan; ++q) prow[q] = -1;
        if (d <= fan) {
            for (int64_t q = 0; q < d; ++q) row[q] = indices[beg + q];
            if (prow) for (int64_t q = 0; q < d; ++q) prow[q] = beg + q;
            cnt[i] = (int32_t)d;
        } else {
            for (int32_t q = 0; q < fan; ++q)
                words[q] = gso_philox_word(seed, iter, layer, (uint32_t)v, (uint32_t)q);
            gso_floyd_select(d, fan, words, chosen);
            for (int32_t q = 0; q < fan; ++q) row[q] = indices[beg + chosen[q]];
            if (prow) for (int32_t q = 0; q < fan; ++q) prow[q] = beg + chosen[q];
            cnt[i] = fan;
        }
    }
    free(words);
    free(chosen);
}

/* The sampled id stream of one split: its slots in (frontier position, slot) order, padding
 * skipped.  Returns the stream length. */
int64_t gso_slot_stream(const int32_t *nbr, const int32_t *cnt, int64_t n_front, int32_t fan,
                        int32_t *sigma)
{
    int64_t m = 0;
    for (int64_t i = 0; i < n_front; ++i)
        for (int32_t q = 0; q < cnt[i]; ++q) sigma[m++] = nbr[i * fan + q];
    return m;
}

/* ------------------------------------------------------------------------------------------ */
/* Online splitting (section 4): every sampled vertex is mapped to its split independently and   */
/* in constant time by looking up the offline global partition function f_G (the partition map). */
/* The ids that go to split t form bucket t: the stable subsequence of the stream with owner t   */
/* (the contiguous send buffers of the sampling shuffle, section 3 / section 6.3).               */
/* bucket_off has n_splits+1 entries; bucketed has n entries, bucket t = [off[t], off[t+1]).     */
/* ------------------------------------------------------------------------------------------ */
void gso_split_buckets(const int32_t *sigma, int64_t n, const uint8_t *pmap, int32_t n_splits,
                       int32_t *bucketed, int64_t *bucket_off)
{
    for (int32_t t = 0; t <= n_splits; ++t) bucket_off[t] = 0;
    for (int64_t j = 0; j < n; ++j) bucket_off[pmap[sigma[j]] + 1] += 1;
    for (int32_t t = 0; t < n_splits; ++t) bucket_off[t + 1] += bucket_off[t];
    int64_t *cursor = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_splits);
    for (int32_t t = 0; t < n_splits; ++t) cursor[t] = bucket_off[t];
    for (int64_t j = 0; j < n; ++j) bucketed[cursor[pmap[sigma[j]]]++] = sigma[j];
    free(cursor);
}

/* ------------------------------------------------------------------------------------------ */
/* First-occurrence dedup: uniq = the distinct values of seq in order of first appearance.       */
/* `where` is caller scratch of n_vertices entries, all -1 on entry and on return; while the     */
/* call runs where[v] is v's index in uniq.  Returns |uniq|.  If local_of is not NULL,            */
/* local_of[j] receives the index in uniq of seq[j] (the relabelling of the sequence).            */
/* ------------------------------------------------------------------------------------------ */
int64_t gso_unique_first(const int32_t *seq, int64_t n, int32_t *where, int32_t *uniq,
                         int32_t *local_of)
{
    int64_t m = 0;
    for (int64_t j = 0; j < n; ++j) {
        int32_t v = seq[j];
        if (where[v] < 0) { where[v] = (int32_t)m; uniq[m++] = v; }
        if (local_of) local_of[j] = where[v];
    }
    for (int64_t q = 0; q < m; ++q) where[uniq[q]] = -1;
    return m;
}

/* Positions of `ids` inside the duplicate-free list `list` (-1 where absent).  Same scratch
 * convention as above. */
void gso_positions_in(const int32_t *list, int64_t n_list, const int32_t *ids, int64_t n_ids,
                      int32_t *where, int32_t *pos)
{
    for (int64_t q = 0; q < n_list; ++q) where[list[q]] = (int32_t)q;
    for (int64_t j = 0; j < n_ids; ++j) pos[j] = where[ids[j]];
    for (int64_t q = 0; q < n_list; ++q) where[list[q]] = -1;
}

/* ------------------------------------------------------------------------------------------ */
/* Loading (section 3): rows of the feature table for the layer-0 local frontier.  Row-major,    */
/* row_bytes bytes per row, a plain copy.                                                        */
/* ------------------------------------------------------------------------------------------ */
void gso_gather_rows(const uint8_t *table, int64_t row_stride_bytes, int64_t row_bytes,
                     const int32_t *ids, int64_t n, uint8_t *out)
{
    for (int64_t j = 0; j < n; ++j)
        memcpy(out + j * row_bytes, table + (int64_t)ids[j] * row_stride_bytes, (size_t)row_bytes);
}

/* ------------------------------------------------------------------------------------------ */
/* GraphSAGE mean aggregation over one block (Hamilton et al., mean aggregator):                 */
/*   M[i,:] = (1/cnt_i) * sum over the entries e of block row i of H[src[e], :],  0 if cnt_i = 0  */
/* fp64 throughout.  blk_indptr has n_dst+1 entries, src are local row numbers of H.             */
/* ------------------------------------------------------------------------------------------ */
void gso_mean_aggregate(int64_t n_dst, int64_t dim, const int64_t *blk_indptr, const int32_t *blk_src,
                        const double *H, double *M)
{
    for (int64_t i = 0; i < n_dst; ++i) {
        double *m = M + i * dim;
        for (int64_t c = 0; c < dim; ++c) m[c] = 0.0;
        int64_t cnt = blk_indptr[i + 1] - blk_indptr[i];
        for (int64_t e = blk_indptr[i]; e < blk_indptr[i + 1]; ++e) {
            const double *h = H + (int64_t)blk_src[e] * dim;
            for (int64_t c = 0; c < dim; ++c) m[c] += h[c];
        }
        if (cnt > 0)
            for (int64_t c = 0; c < dim; ++c) m[c] /= (double)cnt;
    }
}

/* Its adjoint: dH[src[e], :] += dM[i, :] / cnt_i for every entry e of row i (dH accumulates). */
void gso_mean_aggregate_adjoint(int64_t n_dst, int64_t dim, const int64_t *blk_indptr,
                                const int32_t *blk_src, const double *dM, double *dH)
{
    for (int64_t i = 0; i < n_dst; ++i) {
        int64_t cnt = blk_indptr[i + 1] - blk_indptr[i];
        const double *g = dM + i * dim;
        for (int64_t e = blk_indptr[i]; e < blk_indptr[i + 1]; ++e) {
            double *h = dH + (int64_t)blk_src[e] * dim;
            for (int64_t c = 0; c < dim; ++c) h[c] += g[c] / (double)cnt;
        }
    }
}

/* Row gather / scatter-add through an index (the training shuffle of Algorithm 2 and its
 * reverse in the backward pass), fp64 rows. */
void gso_rows_take(const double *src, int64_t dim, const int32_t *rows, int64_t n, double *out)
{
    for (int64_t j = 0; j < n; ++j)
        memcpy(out + j * dim, src + (int64_t)rows[j] * dim, sizeof(double) * (size_t)dim);
}

void gso_rows_add_into(double *dst, int64_t dim, const int32_t *rows, int64_t n, const double *src)
{
    for (int64_t j = 0; j < n; ++j) {
        double *d = dst + (int64_t)rows[j] * dim;
        const double *s = src + j * dim;
        for (int64_t c = 0; c < dim; ++c) d[c] += s[c];
    }
}
