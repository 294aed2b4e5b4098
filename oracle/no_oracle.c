/*
 * CPU oracle for the sample / gather / aggregate hot path of sample-based GNN training
 * (Algorithm 1; Eq. 1; Section 4.1.2 for hot-vertex selection).
 *
 * THIS IS TEST INFRASTRUCTURE. It is a plain, slow, single-threaded statement of what the
 * path computes, used only to check the GPU library and to serve as a timed CPU baseline.
 * It shares no code with the GPU library and must never be called from the product path.
 *
 * Integer parts (random sampling, relabelling, transposition, hot-vertex counting) are
 * fully specified algorithms and are bit-exact targets. Floating point is fp64 throughout.
 *
 * Readings where the paper is silent (see each function):
 *   - graph = CSR over in-neighbours (Eq. 1 aggregates over N_in(v));
 *   - sampling is uniform, without replacement, over the edge positions of a row, and takes
 *     the whole row in stored order when deg <= fanout (Section 2.2: a fixed number of neighbours per
 *     vertex, chosen uniformly);
 *   - the random source is Philox4x32-10 (Salmon et al., SC'11), counter-based so that a
 *     sample is a pure function of (stream, domain, hop, vertex, slot).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ Philox4x32-10 */

static void mul32(uint32_t a, uint32_t b, uint32_t* hi, uint32_t* lo) {
    uint64_t p = (uint64_t)a * (uint64_t)b;
    *hi = (uint32_t)(p >> 32);
    *lo = (uint32_t)p;
}

/* Ten rounds of the Philox 4x32 bijection; key schedule adds the Weyl constants each round. */
void ora_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint32_t hi0, lo0, hi1, lo1;
        mul32(0xD2511F53u, c0, &hi0, &lo0);
        mul32(0xCD9E8D57u, c2, &hi1, &lo1);
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* 64 random bits for (stream, domain, hop, vertex, slot):
 * counter = (v_lo, v_hi, slot, domain<<8 | hop), key = (stream_lo, stream_hi). */
uint64_t ora_random64(uint64_t stream, uint32_t domain, uint32_t hop, uint64_t v, uint32_t slot) {
    uint32_t ctr[4] = { (uint32_t)v, (uint32_t)(v >> 32), slot, (domain << 8) | hop };
    uint32_t key[2] = { (uint32_t)stream, (uint32_t)(stream >> 32) };
    uint32_t out[4];
    ora_philox4x32_10(ctr, key, out);
    return ((uint64_t)out[1] << 32) | (uint64_t)out[0];
}

/* floor(x * n / 2^64): maps 64 random bits to [0, n) */
uint64_t ora_mulhi64(uint64_t x, uint64_t n) {
    return (uint64_t)(((unsigned __int128)x * (unsigned __int128)n) >> 64);
}

/* ------------------------------------------------------------------ row sampling */

/* Partial Fisher-Yates shuffle of the virtual array a[i] = i (0 <= i < d), first k steps,
 * given the swap partners r[j] in [j, d). Step j swaps a[j] with a[r[j]]; out[j] is the value
 * that lands in position j. Only displaced entries are stored (a sparse map). */
void ora_fisher_yates_prefix(int64_t d, int32_t k, const int64_t* r, int64_t* out) {
    int64_t* pos = (int64_t*)malloc(sizeof(int64_t) * (size_t)(2 * k + 1));
    int64_t* val = (int64_t*)malloc(sizeof(int64_t) * (size_t)(2 * k + 1));
    int n_map = 0;
    (void)d;
    for (int32_t j = 0; j < k; ++j) {
        int64_t rj = r[j];
        int64_t aj = j, ar = rj;
        int ir = -1;
        for (int m = 0; m < n_map; ++m) {
            if (pos[m] == j) aj = val[m];
            if (pos[m] == rj) { ar = val[m]; ir = m; }
        }
        out[j] = ar;                 /* a[j] <- old a[r] */
        if (ir >= 0) val[ir] = aj;   /* a[r] <- old a[j] */
        else { pos[n_map] = rj; val[n_map] = aj; ++n_map; }
    }
    free(pos); free(val);
}

/* Positions (in [0, d)) of the sampled entries of one CSR row, in slot order.
 * Returns the count min(d, k). */
int32_t ora_sample_row(uint64_t stream, uint32_t domain, uint32_t hop, uint64_t v,
                       int64_t d, int32_t k, int64_t* out) {
    if (d <= (int64_t)k) {
        for (int64_t i = 0; i < d; ++i) out[i] = i;
        return (int32_t)d;
    }
    int64_t* r = (int64_t*)malloc(sizeof(int64_t) * (size_t)k);
    for (int32_t j = 0; j < k; ++j)
        r[j] = (int64_t)j + (int64_t)ora_mulhi64(ora_random64(stream, domain, hop, v, (uint32_t)j),
                                                  (uint64_t)(d - j));
    ora_fisher_yates_prefix(d, k, r, out);
    free(r);
    return k;
}

/* ------------------------------------------------------------------ CSR */

static int cmp_i32(const void* a, const void* b) {
    int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

/* In-neighbour CSR: edge (src -> dst) puts src into row dst. Rows ascending by src,
 * duplicates kept. rowptr has V+1 int64 entries; col has E int32 entries. */
void ora_build_csr(const int32_t* src, const int32_t* dst, int64_t n_edges, int64_t n_vertices,
                   int64_t* rowptr, int32_t* col) {
    memset(rowptr, 0, sizeof(int64_t) * (size_t)(n_vertices + 1));
    for (int64_t e = 0; e < n_edges; ++e) rowptr[dst[e] + 1] += 1;
    for (int64_t v = 0; v < n_vertices; ++v) rowptr[v + 1] += rowptr[v];
    int64_t* cursor = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n_vertices > 0 ? n_vertices : 1));
    memcpy(cursor, rowptr, sizeof(int64_t) * (size_t)n_vertices);
    for (int64_t e = 0; e < n_edges; ++e) col[cursor[dst[e]]++] = src[e];
    for (int64_t v = 0; v < n_vertices; ++v)
        qsort(col + rowptr[v], (size_t)(rowptr[v + 1] - rowptr[v]), sizeof(int32_t), cmp_i32);
    free(cursor);
}

/* ------------------------------------------------------------------ one sampled hop */

/* Samples fanout k for every destination (Algorithm 1, the sample() call of one hop) and
 * relabels the result into a bipartite block.
 *   in : dst_global[n_dst] (unique ids), CSR, scratch map[V] filled with -1 (restored on exit)
 *   out: indptr[n_dst+1], nbr_global[nnz], indices[nnz], src_global[<= n_dst + nnz]
 * src_global starts with dst_global; every further id is appended at its first occurrence
 * while scanning the sampled edges in (row, slot) order. Returns n_src. */
int64_t ora_sample_hop(const int64_t* rowptr, const int32_t* col,
                       const int32_t* dst_global, int64_t n_dst, int32_t k,
                       uint64_t stream, uint32_t domain, uint32_t hop,
                       int32_t* map,
                       int32_t* indptr, int32_t* nbr_global, int32_t* indices, int32_t* src_global) {
    int64_t* pos = (int64_t*)malloc(sizeof(int64_t) * (size_t)(k > 0 ? k : 1));
    int64_t n_src = 0;
    for (int64_t i = 0; i < n_dst; ++i) { map[dst_global[i]] = (int32_t)i; src_global[n_src++] = dst_global[i]; }
    int64_t nnz = 0;
    indptr[0] = 0;
    for (int64_t i = 0; i < n_dst; ++i) {
        int32_t v = dst_global[i];
        int64_t begin = rowptr[v], d = rowptr[v + 1] - rowptr[v];
        int32_t c = ora_sample_row(stream, domain, hop, (uint64_t)v, d, k, pos);
        for (int32_t j = 0; j < c; ++j) {
            int32_t u = col[begin + pos[j]];
            if (map[u] < 0) { map[u] = (int32_t)n_src; src_global[n_src++] = u; }
            nbr_global[nnz] = u;
            indices[nnz] = map[u];
            ++nnz;
        }
        indptr[i + 1] = (int32_t)nnz;
    }
    for (int64_t i = 0; i < n_src; ++i) map[src_global[i]] = -1;
    free(pos);
    return n_src;
}

/* Transpose of a block: for each local source u the (dst, edge id) pairs with indices[e] == u,
 * in ascending edge id. */
void ora_block_csc(const int32_t* indptr, const int32_t* indices, int64_t n_dst, int64_t n_src,
                   int32_t* csc_indptr, int32_t* csc_dst, int32_t* csc_eid) {
    int64_t nnz = indptr[n_dst];
    memset(csc_indptr, 0, sizeof(int32_t) * (size_t)(n_src + 1));
    for (int64_t e = 0; e < nnz; ++e) csc_indptr[indices[e] + 1] += 1;
    for (int64_t u = 0; u < n_src; ++u) csc_indptr[u + 1] += csc_indptr[u];
    int32_t* cursor = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_src > 0 ? n_src : 1));
    memcpy(cursor, csc_indptr, sizeof(int32_t) * (size_t)n_src);
    for (int64_t v = 0; v < n_dst; ++v)
        for (int32_t e = indptr[v]; e < indptr[v + 1]; ++e) {
            int32_t p = cursor[indices[e]]++;
            csc_dst[p] = (int32_t)v;
            csc_eid[p] = e;
        }
    free(cursor);
}

/* ------------------------------------------------------------------ hot-vertex counting */

/* Pre-sampling hotness (Section 4.1.2): the training vertices, in the order given, are cut
 * into batches of `batch`; every batch is sampled for hops 0 .. n_layers-2 (domain 1,
 * stream = seed + epoch*n_batches + b) and freq[v] is incremented once for every vertex of
 * the input set of the bottom hop (the vertices whose layer-1 embedding could be reused).
 * freq[V] must be zero on entry. */
void ora_presample_counts(const int64_t* rowptr, const int32_t* col, int64_t n_vertices,
                          const int32_t* train_ids, int64_t n_train, int32_t batch,
                          const int32_t* fanouts, int32_t n_layers, int32_t epochs,
                          uint64_t seed, int64_t* freq) {
    int64_t nb = (n_train + batch - 1) / batch;
    /* buffer sizes: the no-de-duplication bound of each hop, vertex sets capped at V */
    int64_t cap = batch, cap_e = 1, n_dst_bound = batch;
    for (int32_t h = 0; h + 1 < n_layers; ++h) {
        int64_t e_bound = n_dst_bound * fanouts[h];
        int64_t s_bound = n_dst_bound + e_bound;
        if (s_bound > n_vertices) s_bound = n_vertices;
        if (e_bound > cap_e) cap_e = e_bound;
        if (s_bound > cap) cap = s_bound;
        n_dst_bound = s_bound;
    }
    int32_t* map = (int32_t*)malloc(sizeof(int32_t) * (size_t)n_vertices);
    memset(map, 0xFF, sizeof(int32_t) * (size_t)n_vertices);
    int32_t* cur = (int32_t*)malloc(sizeof(int32_t) * (size_t)(cap + 1));
    int32_t* nxt = (int32_t*)malloc(sizeof(int32_t) * (size_t)(cap + 1));
    int32_t* indptr = (int32_t*)malloc(sizeof(int32_t) * (size_t)(cap + 2));
    int32_t* nbr = (int32_t*)malloc(sizeof(int32_t) * (size_t)cap_e);
    int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)cap_e);
    for (int32_t p = 0; p < epochs; ++p)
        for (int64_t b = 0; b < nb; ++b) {
            int64_t lo = b * batch, hi = lo + batch < n_train ? lo + batch : n_train;
            int64_t n = hi - lo;
            memcpy(cur, train_ids + lo, sizeof(int32_t) * (size_t)n);
            uint64_t stream = seed + (uint64_t)p * (uint64_t)nb + (uint64_t)b;
            for (int32_t h = 0; h + 1 < n_layers; ++h) {
                int64_t n_src = ora_sample_hop(rowptr, col, cur, n, fanouts[h], stream, 1u, (uint32_t)h,
                                               map, indptr, nbr, idx, nxt);
                int32_t* t = cur; cur = nxt; nxt = t;
                n = n_src;
            }
            for (int64_t i = 0; i < n; ++i) freq[cur[i]] += 1;
        }
    free(map); free(cur); free(nxt); free(indptr); free(nbr); free(idx);
}

/* ------------------------------------------------------------------ gather and mean */

/* Feature collection (Algorithm 1, the gather step): out[i,:] = table[ids[i],:], byte copy. */
void ora_gather_rows(const void* table, int64_t row_bytes, const int32_t* ids, int64_t n_ids, void* out) {
    for (int64_t i = 0; i < n_ids; ++i)
        memcpy((char*)out + i * row_bytes, (const char*)table + (int64_t)ids[i] * row_bytes, (size_t)row_bytes);
}

/* AGGREGATE = average (Eq. 1) over the sampled in-neighbours of each destination:
 * mean[v,:] = (1/len(row v)) * sum_{e in row v} x[indices[e],:]; an empty row gives zeros. */
void ora_mean_aggregate(const double* x, int64_t dim, const int32_t* indptr, const int32_t* indices,
                        int64_t n_dst, double* mean) {
    for (int64_t v = 0; v < n_dst; ++v) {
        double* m = mean + v * dim;
        for (int64_t f = 0; f < dim; ++f) m[f] = 0.0;
        int32_t b = indptr[v], e = indptr[v + 1];
        for (int32_t p = b; p < e; ++p) {
            const double* row = x + (int64_t)indices[p] * dim;
            for (int64_t f = 0; f < dim; ++f) m[f] += row[f];
        }
        if (e > b) { double inv = (double)(e - b); for (int64_t f = 0; f < dim; ++f) m[f] /= inv; }
    }
}

/* Adjoint of the mean: grad_x[u,:] += sum over edges e with indices[e] == u of
 * grad_mean[dst(e),:] / len(row dst(e)). grad_x[n_src, dim] must be initialised by the caller. */
void ora_mean_aggregate_adjoint(const double* grad_mean, int64_t dim, const int32_t* indptr,
                                const int32_t* indices, int64_t n_dst, double* grad_x) {
    for (int64_t v = 0; v < n_dst; ++v) {
        int32_t b = indptr[v], e = indptr[v + 1];
        if (e == b) continue;
        double inv = 1.0 / (double)(e - b);
        const double* g = grad_mean + v * dim;
        for (int32_t p = b; p < e; ++p) {
            double* row = grad_x + (int64_t)indices[p] * dim;
            for (int64_t f = 0; f < dim; ++f) row[f] += g[f] * inv;
        }
    }
}
