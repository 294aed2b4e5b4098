// no_sample_blocks: reverse multi-hop fanout sampling over the in-neighbour CSR (the sample()
// loop of Algorithm 1), de-duplication / relabelling of each frontier, the block transpose used
// by the backward pass, and the hot-vertex lookup that removes reusable vertices from the bottom
// hop (Section 4.1.2, Stage 1 of Section 4.2).
//
// Sampling: a sub-wave group of G lanes (G = 8/16/32/64 >= fanout) serves one destination; lane j
// draws slot j with Philox4x32-10 keyed by (stream; vertex, slot, domain, hop) and the group
// resolves the partial Fisher-Yates swap chain with cross-lane shuffles. The result is a pure
// function of the key, independent of launch shape.
#include "primitives.hpp"
#include "handles.hpp"

namespace no {

// ---------------------------------------------------------------------------- Philox4x32-10

__device__ __forceinline__ uint64_t philox_random64(uint32_t k0, uint32_t k1, uint32_t c0, uint32_t c1, uint32_t c2,
                                                    uint32_t c3) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return ((uint64_t)c1 << 32) | (uint64_t)c0;
}

template <typename RowT>
struct DegreeLoader {       // min(deg(dst[i]), k)
    const RowT* rowptr;
    const int32_t* dst;
    int32_t k;
    __device__ __forceinline__ int32_t operator()(int64_t i) const {
        int32_t v = dst[i];
        int64_t d = (int64_t)rowptr[v + 1] - (int64_t)rowptr[v];
        return d < (int64_t)k ? (int32_t)d : k;
    }
};

struct FirstSeenLoader {    // 1 iff edge e is the first occurrence of a vertex that is not a destination
    const int32_t* map;
    const int32_t* nbr;
    const int32_t* d_n_dst;
    __device__ __forceinline__ int32_t operator()(int64_t e) const { return map[nbr[e]] == *d_n_dst + (int32_t)e; }
};

struct ComputeLoader {      // 1 iff V^1 row i cannot be served from the cache at `step`
    const int32_t* v1;
    const int32_t* slot_of_vertex;
    const int32_t* version;
    int64_t step;
    int32_t staleness;
    __device__ __forceinline__ bool hit(int64_t i, int32_t* slot_out) const {
        int32_t s = slot_of_vertex[v1[i]];
        *slot_out = s;
        if (s < 0) return false;
        int32_t ver = version[s];
        return ver >= 0 && step - (int64_t)ver <= (int64_t)staleness;
    }
    __device__ __forceinline__ int32_t operator()(int64_t i) const { int32_t s; return hit(i, &s) ? 0 : 1; }
};

// ---------------------------------------------------------------------------- kernels

__global__ void hop_begin_kernel(const int32_t* dst, const int32_t* d_n_dst, int32_t cap, int32_t* map,
                                 int32_t* count_out) {
    int32_t n = *d_n_dst;
    if (n > cap) n = cap;
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) *count_out = n;
    if (i < n) map[dst[i]] = i;
}

template <int G, typename RowT>
__global__ void __launch_bounds__(256) sample_rows_kernel(const RowT* __restrict__ rowptr, const int32_t* __restrict__ col,
                                                          const int32_t* __restrict__ dst, const int32_t* d_n_dst,
                                                          int32_t k, uint32_t key0, uint32_t key1, uint32_t c3,
                                                          const int32_t* __restrict__ indptr, int32_t* __restrict__ nbr,
                                                          int32_t* __restrict__ edge_row, int32_t* map) {
    const int32_t n_dst = *d_n_dst;
    const int32_t i = (int32_t)(blockIdx.x * (256 / G) + threadIdx.x / G);
    const int32_t j = (int32_t)(threadIdx.x % G);
    const bool row_ok = i < n_dst;
    int32_t v = 0;
    int64_t begin = 0, d = 0;
    int32_t out0 = 0;
    if (row_ok) {
        v = dst[i];
        begin = (int64_t)rowptr[v];
        d = (int64_t)rowptr[v + 1] - begin;
        out0 = indptr[i];
    }
    int64_t pos = j;
    const bool take_all = d <= (int64_t)k;
    // The swap partner of slot j: r_j = j + floor(x * (d - j) / 2^64) in [j, d).
    int64_t r = -1 - (int64_t)j;          // distinct negative sentinels for idle lanes
    if (row_ok && !take_all && j < k) {
        uint64_t x = philox_random64(key0, key1, (uint32_t)v, 0u, (uint32_t)j, c3);
        r = (int64_t)j + (int64_t)__umul64hi(x, (uint64_t)(d - j));
    }
    // Whole groups with nothing to shuffle still take part in the cross-lane reads below.
    if (__ballot(row_ok && !take_all) != 0ull) {
        // a = latest earlier step that displaced position j; b = latest earlier step that hit r_j
        int32_t a = -1, b = -1;
        for (int32_t t = 0; t < k; ++t) {
            int64_t rt = __shfl(r, t, G);
            if (t < j) {
                if (rt == (int64_t)j) a = t;
                if (rt == r) b = t;
            }
        }
        // w_j = content of position j just before step j: j itself unless displaced, else w_a.
        int64_t w = j;
        bool done = a < 0;
        while (true) {
            int64_t wa = __shfl(w, a < 0 ? 0 : a, G);
            int da = __shfl((int)done, a < 0 ? 0 : a, G);
            if (!done && da) { w = wa; done = true; }
            if (__ballot(!done) == 0ull) break;
        }
        int64_t wb = __shfl(w, b < 0 ? 0 : b, G);
        if (!take_all) pos = b < 0 ? r : wb;
    }
    int32_t cnt = d < (int64_t)k ? (int32_t)d : k;
    if (row_ok && j < cnt) {
        int32_t u = col[begin + pos];
        int32_t e = out0 + j;
        nbr[e] = u;
        edge_row[e] = i;
        atomicMin(&map[u], n_dst + e);   // integer min: order independent
    }
}

__global__ void relabel_kernel(const int32_t* __restrict__ dst, const int32_t* d_n_dst, const int32_t* d_nnz,
                               const int32_t* __restrict__ nbr, const int32_t* __restrict__ map,
                               const int32_t* __restrict__ rank, int32_t* __restrict__ indices,
                               int32_t* __restrict__ src_global, int32_t* d_n_src, int32_t* csc_cnt, int32_t* iota) {
    const int32_t n_dst = *d_n_dst, nnz = *d_nnz;
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t == 0) *d_n_src = n_dst + rank[nnz];
    if (t < n_dst) { src_global[t] = dst[t]; return; }
    t -= n_dst;
    if (t >= nnz) return;
    int32_t e = (int32_t)t;
    int32_t u = nbr[e];
    int32_t m = map[u];
    int32_t local;
    if (m < n_dst) local = m;
    else {
        local = n_dst + rank[m - n_dst];
        if (m == n_dst + e) src_global[local] = u;
    }
    indices[e] = local;
    if (csc_cnt) { atomicAdd(&csc_cnt[local], 1); iota[e] = e; }
}

__global__ void csc_rows_kernel(const int32_t* d_nnz, const int32_t* __restrict__ csc_eid,
                                const int32_t* __restrict__ edge_row, int32_t* __restrict__ csc_dst) {
    int32_t p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p < *d_nnz) csc_dst[p] = edge_row[csc_eid[p]];
}

__global__ void hop_end_kernel(const int32_t* src_global, const int32_t* d_n_src, int32_t* map) {
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < *d_n_src) map[src_global[i]] = EMPTY;
}

__global__ void partition_v1_kernel(ComputeLoader ld, const int32_t* d_n_v1, const int32_t* __restrict__ rank,
                                    int32_t* compute_list, int32_t* compute_pos, int32_t* hit_pos, int32_t* hit_slot,
                                    int32_t* d_n_hit) {
    const int32_t n = *d_n_v1;
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) *d_n_hit = n - rank[n];
    if (i >= n) return;
    int32_t slot;
    if (ld.hit(i, &slot)) {
        int32_t p = i - rank[i];
        hit_pos[p] = i;
        hit_slot[p] = slot;
    } else {
        int32_t p = rank[i];
        compute_pos[p] = i;
        compute_list[p] = ld.v1[i];
    }
}

__global__ void set_count_kernel(int32_t* p, int32_t v) { *p = v; }

// ---------------------------------------------------------------------------- host side

template <typename RowT>
static int32_t sample_hop(const RowT* rowptr, const int32_t* col, no_blocks_s* b, int32_t h, const int32_t* d_dst,
                          const int32_t* d_n_dst_in, uint32_t key0, uint32_t key1, uint32_t domain, hipStream_t st) {
    HopBuffers& H = b->hop[h];
    int32_t* cnt = b->counts.p + 4 * h;              // n_dst, n_src, nnz
    int32_t* scratch_total = b->counts.p + 4 * b->n_layers + 2;
    const int32_t k = H.fanout;
    const int T = 256;
    H.d_dst = d_dst;
    H.d_n_dst = cnt;
    hipLaunchKernelGGL(hop_begin_kernel, dim3((unsigned)ceil_div(H.n_dst_cap, T)), dim3(T), 0, st, d_dst, d_n_dst_in,
                       H.n_dst_cap, b->map.p, cnt);
    NO_CHECK((exclusive_scan<DegreeLoader<RowT>, int32_t>(DegreeLoader<RowT>{rowptr, d_dst, k}, cnt, H.n_dst_cap,
                                                           H.indptr.p, cnt + 2, b->ws.p, st)));
    const uint32_t c3 = (domain << 8) | (uint32_t)h;
#define NO_LAUNCH_SAMPLE(G)                                                                                        \
    hipLaunchKernelGGL((sample_rows_kernel<G, RowT>), dim3((unsigned)ceil_div(H.n_dst_cap, 256 / G)), dim3(256), 0, st, \
                       rowptr, col, d_dst, cnt, k, key0, key1, c3, H.indptr.p, H.nbr_global.p, H.edge_row.p, b->map.p)
    if (k <= 8) NO_LAUNCH_SAMPLE(8);
    else if (k <= 16) NO_LAUNCH_SAMPLE(16);
    else if (k <= 32) NO_LAUNCH_SAMPLE(32);
    else NO_LAUNCH_SAMPLE(64);
#undef NO_LAUNCH_SAMPLE
    NO_CHECK((exclusive_scan<FirstSeenLoader, int32_t>(FirstSeenLoader{b->map.p, H.nbr_global.p, cnt}, cnt + 2, H.nnz_cap,
                                                        b->rank.p, scratch_total, b->ws.p, st)));
    int32_t* csc_cnt = H.has_csc ? H.csc_cnt.p : nullptr;
    if (H.has_csc) NO_CHECK(fill_i32(csc_cnt, 0, H.n_src_cap, st));
    hipLaunchKernelGGL(relabel_kernel, dim3((unsigned)ceil_div((int64_t)H.n_dst_cap + H.nnz_cap, T)), dim3(T), 0, st, d_dst,
                       cnt, cnt + 2, H.nbr_global.p, b->map.p, b->rank.p, H.indices.p, H.src_global.p, cnt + 1, csc_cnt,
                       H.csc_dst.p);
    if (H.has_csc) {
        NO_CHECK(exclusive_scan_i32(csc_cnt, cnt + 1, H.n_src_cap, H.csc_indptr.p, nullptr, b->ws.p, st));
        int bits = ilog2_ceil((uint64_t)H.n_src_cap);
        if (bits < 1) bits = 1;
        NO_CHECK(radix_sort_pairs((const uint32_t*)H.indices.p, (const uint32_t*)H.csc_dst.p, (uint32_t*)H.csc_keys.p,
                                  (uint32_t*)H.csc_eid.p, (uint32_t*)b->tmp_a.p, (uint32_t*)b->tmp_b.p, cnt + 2,
                                  H.nnz_cap, bits, b->ws.p, st));
        hipLaunchKernelGGL(csc_rows_kernel, dim3((unsigned)ceil_div(H.nnz_cap, T)), dim3(T), 0, st, cnt + 2, H.csc_eid.p,
                           H.edge_row.p, H.csc_dst.p);
    }
    hipLaunchKernelGGL(hop_end_kernel, dim3((unsigned)ceil_div(H.n_src_cap, T)), dim3(T), 0, st, H.src_global.p, cnt + 1,
                       b->map.p);
    return launch_status("sample_hop");
}

int32_t sample_blocks_impl(no_graph_s* g, const int32_t* d_seeds, int32_t n_seeds, uint64_t stream_key, uint32_t domain,
                           int32_t n_hops, no_cache_s* cache, int64_t step, no_blocks_s* b, hipStream_t st) {
    const int32_t L = b->n_layers;
    int32_t* extra = b->counts.p + 4 * L;     // n_compute, n_hit, scratch
    NO_HIP_CHECK(hipMemcpyAsync(b->seeds.p, d_seeds, (size_t)n_seeds * 4, hipMemcpyDeviceToDevice, st));
    hipLaunchKernelGGL(set_count_kernel, dim3(1), dim3(1), 0, st, extra + 3, n_seeds);
    const uint32_t key0 = (uint32_t)stream_key, key1 = (uint32_t)(stream_key >> 32);
    const int32_t* d_dst = b->seeds.p;
    const int32_t* d_n = extra + 3;
    const bool use_cache = cache != nullptr && L >= 2 && n_hops == L && cache->n_hot > 0;
    b->last_used_cache = false;
    for (int32_t h = 0; h < n_hops; ++h) {
        if (h == L - 1 && use_cache) {
            // split V^1 (= sources of hop L-2) into reusable rows and rows to compute
            HopBuffers& P = b->hop[h - 1];
            ComputeLoader ld{d_dst, cache->slot_of_vertex.p, cache->version.p, step, cache->staleness};
            NO_CHECK((exclusive_scan<ComputeLoader, int32_t>(ld, d_n, P.n_src_cap, b->rank.p, extra + 0, b->ws.p, st)));
            hipLaunchKernelGGL(partition_v1_kernel, dim3((unsigned)ceil_div(P.n_src_cap, 256)), dim3(256), 0, st, ld, d_n,
                               b->rank.p, b->compute_list.p, b->compute_pos.p, b->hit_pos.p, b->hit_slot.p, extra + 1);
            d_dst = b->compute_list.p;
            d_n = extra + 0;
            b->last_used_cache = true;
        }
        if (g->rowptr_bits == 64)
            NO_CHECK(sample_hop<int64_t>(g->rowptr64.p, g->col.p, b, h, d_dst, d_n, key0, key1, domain, st));
        else
            NO_CHECK(sample_hop<int32_t>(g->rowptr32.p, g->col.p, b, h, d_dst, d_n, key0, key1, domain, st));
        d_dst = b->hop[h].src_global.p;
        d_n = b->counts.p + 4 * h + 1;
    }
    if (!b->last_used_cache) {
        hipLaunchKernelGGL(set_count_kernel, dim3(1), dim3(1), 0, st, extra + 1, 0);
    }
    return launch_status("sample_blocks");
}

int32_t blocks_create_impl(no_graph_s* g, int32_t n_seeds_cap, const int32_t* fanouts, int32_t n_layers,
                           bool build_csc, no_blocks_s** out) {
    *out = nullptr;
    no_blocks_s* b = new no_blocks_s();
    struct Guard { no_blocks_s* b; ~Guard() { if (b) { b->release(); delete b; } } } guard{b};
    b->n_layers = n_layers;
    b->n_seeds_cap = n_seeds_cap;
    b->n_vertices = g->n_vertices;
    b->build_csc = build_csc;
    int64_t dst_cap = n_seeds_cap;
    int64_t max_rank = 1, max_sort = 1, max_scan = 1;
    for (int32_t h = 0; h < n_layers; ++h) {
        HopBuffers& H = b->hop[h];
        int64_t nnz_cap = dst_cap * fanouts[h];
        int64_t src_cap = dst_cap + nnz_cap;
        if (src_cap > g->n_vertices) src_cap = g->n_vertices;
        NO_REQUIRE(nnz_cap + dst_cap < (1ll << 31) - 1, NO_ERR_OVERFLOW, "blocks: hop %d capacity exceeds int32", h);
        H.fanout = fanouts[h];
        H.n_dst_cap = (int32_t)dst_cap;
        H.nnz_cap = (int32_t)nnz_cap;
        H.n_src_cap = (int32_t)src_cap;
        H.has_csc = build_csc && h < n_layers - 1;
        NO_CHECK(H.src_global.alloc((size_t)src_cap));
        NO_CHECK(H.indptr.alloc((size_t)dst_cap + 1));
        NO_CHECK(H.nbr_global.alloc((size_t)nnz_cap));
        NO_CHECK(H.indices.alloc((size_t)nnz_cap));
        NO_CHECK(H.edge_row.alloc((size_t)nnz_cap));
        if (H.has_csc) {
            NO_CHECK(H.csc_indptr.alloc((size_t)src_cap + 1));
            NO_CHECK(H.csc_cnt.alloc((size_t)src_cap + 1));
            NO_CHECK(H.csc_dst.alloc((size_t)nnz_cap));
            NO_CHECK(H.csc_eid.alloc((size_t)nnz_cap));
            NO_CHECK(H.csc_keys.alloc((size_t)nnz_cap));
            if (nnz_cap > max_sort) max_sort = nnz_cap;
        }
        if (nnz_cap > max_rank) max_rank = nnz_cap;
        if (src_cap > max_rank) max_rank = src_cap;
        if (dst_cap > max_rank) max_rank = dst_cap;
        dst_cap = src_cap;
    }
    max_scan = max_rank;
    NO_CHECK(b->counts.alloc((size_t)4 * n_layers + 8));
    NO_HIP_CHECK(hipMemset(b->counts.p, 0, ((size_t)4 * n_layers + 8) * 4));
    NO_CHECK(b->seeds.alloc((size_t)n_seeds_cap));
    NO_CHECK(b->map.alloc((size_t)g->n_vertices));
    NO_CHECK(fill_i32(b->map.p, EMPTY, g->n_vertices, nullptr));
    NO_CHECK(b->rank.alloc((size_t)max_rank + 2));
    NO_CHECK(b->tmp_a.alloc((size_t)max_sort));
    NO_CHECK(b->tmp_b.alloc((size_t)max_sort));
    size_t ws = scan_ws_bytes(max_scan + 1);
    size_t rs = radix_ws_bytes(max_sort);
    NO_CHECK(b->ws.alloc(ws > rs ? ws : rs));
    if (n_layers >= 2) {
        size_t v1_cap = (size_t)b->hop[n_layers - 2].n_src_cap;
        NO_CHECK(b->compute_list.alloc(v1_cap));
        NO_CHECK(b->compute_pos.alloc(v1_cap));
        NO_CHECK(b->hit_pos.alloc(v1_cap));
        NO_CHECK(b->hit_slot.alloc(v1_cap));
    }
    NO_HIP_CHECK(hipDeviceSynchronize());
    guard.b = nullptr;
    *out = b;
    return NO_OK;
}

void fill_block_view(const no_blocks_s* b, int32_t h, no_block_view* v) {
    const HopBuffers& H = b->hop[h];
    const int32_t* cnt = b->counts.p + 4 * h;
    const int32_t* extra = b->counts.p + 4 * b->n_layers;
    v->n_dst_cap = H.n_dst_cap;
    v->n_src_cap = H.n_src_cap;
    v->nnz_cap = H.nnz_cap;
    v->d_n_dst = cnt;
    v->d_n_src = cnt + 1;
    v->d_nnz = cnt + 2;
    v->d_dst_global = H.d_dst ? H.d_dst : (h == 0 ? b->seeds.p : b->hop[h - 1].src_global.p);
    v->d_src_global = H.src_global.p;
    v->d_indptr = H.indptr.p;
    v->d_nbr_global = H.nbr_global.p;
    v->d_indices = H.indices.p;
    v->d_csc_indptr = H.has_csc ? H.csc_indptr.p : nullptr;
    v->d_csc_dst = H.has_csc ? H.csc_dst.p : nullptr;
    v->d_csc_eid = H.has_csc ? H.csc_eid.p : nullptr;
    const bool bottom_cached = (h == b->n_layers - 1) && b->last_used_cache;
    v->d_compute_pos = bottom_cached ? b->compute_pos.p : nullptr;
    v->d_hit_pos = bottom_cached ? b->hit_pos.p : nullptr;
    v->d_hit_slot = bottom_cached ? b->hit_slot.p : nullptr;
    v->d_n_compute = bottom_cached ? extra + 0 : nullptr;
    v->d_n_hit = bottom_cached ? extra + 1 : nullptr;
}

}  // namespace no

using namespace no;

static int32_t check_fanouts(const int32_t* f, int32_t n_layers, const char* who) {
    NO_REQUIRE(f != nullptr, NO_ERR_INVALID_ARG, "%s: fanouts is NULL", who);
    NO_REQUIRE(n_layers >= 1 && n_layers <= NO_MAX_LAYERS, NO_ERR_INVALID_ARG, "%s: n_layers must be in [1, %d]", who,
               NO_MAX_LAYERS);
    for (int32_t h = 0; h < n_layers; ++h)
        NO_REQUIRE(f[h] >= 1 && f[h] <= NO_MAX_FANOUT, NO_ERR_INVALID_ARG, "%s: fanout[%d] must be in [1, %d]", who, h,
                   NO_MAX_FANOUT);
    return NO_OK;
}

extern "C" int32_t no_blocks_create(no_graph_t g, int32_t n_seeds_cap, const int32_t* h_fanouts, int32_t n_layers,
                                    no_blocks_t* out) {
    clear_error();
    NO_REQUIRE(out != nullptr, NO_ERR_INVALID_ARG, "no_blocks_create: out is NULL");
    *out = nullptr;
    NO_REQUIRE(g != nullptr, NO_ERR_INVALID_ARG, "no_blocks_create: graph is NULL");
    NO_REQUIRE(n_seeds_cap >= 1, NO_ERR_INVALID_ARG, "no_blocks_create: n_seeds_cap must be positive");
    NO_REQUIRE(n_seeds_cap <= g->n_vertices, NO_ERR_INVALID_ARG, "no_blocks_create: more seeds than vertices");
    NO_CHECK(check_fanouts(h_fanouts, n_layers, "no_blocks_create"));
    return blocks_create_impl(g, n_seeds_cap, h_fanouts, n_layers, true, out);
}

extern "C" int32_t no_sample_blocks(no_graph_t g, const int32_t* d_seeds, int32_t n_seeds, uint64_t seed, int64_t step,
                                    no_cache_t cache, no_blocks_t blocks, void* stream) {
    clear_error();
    NO_REQUIRE(g && blocks && d_seeds, NO_ERR_INVALID_ARG, "no_sample_blocks: NULL argument");
    NO_REQUIRE(n_seeds >= 1, NO_ERR_INVALID_ARG, "no_sample_blocks: n_seeds must be positive");
    NO_REQUIRE(n_seeds <= blocks->n_seeds_cap, NO_ERR_CAPACITY, "no_sample_blocks: %d seeds exceed the capacity %d",
               n_seeds, blocks->n_seeds_cap);
    NO_REQUIRE(blocks->n_vertices == g->n_vertices, NO_ERR_INVALID_ARG, "no_sample_blocks: blocks belong to another graph");
    NO_REQUIRE(step >= 0, NO_ERR_INVALID_ARG, "no_sample_blocks: step must be >= 0");
    NO_REQUIRE(!cache || cache->n_vertices == g->n_vertices, NO_ERR_INVALID_ARG,
               "no_sample_blocks: cache belongs to another graph");
    return sample_blocks_impl(g, d_seeds, n_seeds, seed + (uint64_t)step, 0u, blocks->n_layers, cache, step, blocks,
                              (hipStream_t)stream);
}

extern "C" int32_t no_blocks_view(no_blocks_t blocks, int32_t hop, no_block_view* out) {
    clear_error();
    NO_REQUIRE(blocks && out, NO_ERR_INVALID_ARG, "no_blocks_view: NULL argument");
    NO_REQUIRE(hop >= 0 && hop < blocks->n_layers, NO_ERR_INVALID_ARG, "no_blocks_view: hop out of range");
    fill_block_view(blocks, hop, out);
    return NO_OK;
}

extern "C" int32_t no_blocks_sizes(no_blocks_t blocks, void* stream, int32_t* h_sizes) {
    clear_error();
    NO_REQUIRE(blocks && h_sizes, NO_ERR_INVALID_ARG, "no_blocks_sizes: NULL argument");
    const int32_t L = blocks->n_layers;
    int32_t tmp[4 * NO_MAX_LAYERS + 8];
    NO_HIP_CHECK(hipMemcpyAsync(tmp, blocks->counts.p, ((size_t)4 * L + 8) * 4, hipMemcpyDeviceToHost, (hipStream_t)stream));
    NO_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
    for (int32_t h = 0; h < L; ++h) {
        h_sizes[4 * h + 0] = tmp[4 * h + 0];
        h_sizes[4 * h + 1] = tmp[4 * h + 1];
        h_sizes[4 * h + 2] = tmp[4 * h + 2];
        h_sizes[4 * h + 3] = (h == L - 1 && blocks->last_used_cache) ? tmp[4 * L + 1] : 0;
    }
    return NO_OK;
}

extern "C" int32_t no_blocks_destroy(no_blocks_t blocks) {
    clear_error();
    if (!blocks) return NO_OK;
    blocks->release();
    delete blocks;
    return NO_OK;
}
