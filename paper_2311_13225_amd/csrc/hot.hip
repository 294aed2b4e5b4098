// no_select_hot and the embedding cache (Section 4.1.2): hotness = how often a vertex lands in
// V^1 (the set whose layer-1 embedding could be reused) while pre-sampling the training batches;
// the hot set is the top floor(fraction * V) by (count descending, id ascending).
#include <mutex>
#include <unordered_set>
#include "primitives.hpp"
#include "handles.hpp"

#include <math.h>

namespace no {

// n_vertices > 0: the ids come straight from the caller; one outside [0, V) is not counted and raises *bad_flag
__global__ void count_members_kernel(const int32_t* ids, const int32_t* d_n, int32_t n_fixed, int32_t* freq,
                                     int32_t n_vertices, int32_t* bad_flag) {
    int32_t n = d_n ? *d_n : n_fixed;
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t v = ids[i];
    if (n_vertices > 0 && (uint32_t)v >= (uint32_t)n_vertices) { *bad_flag = 1; return; }
    atomicAdd(&freq[v], 1);       // integer count: order independent
}

__global__ void hot_keys_kernel(const int32_t* freq, int64_t n, uint32_t max_count, uint32_t* keys, uint32_t* ids) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) { keys[i] = max_count - (uint32_t)freq[i]; ids[i] = (uint32_t)i; }
}

__global__ void hot_slots_kernel(const uint32_t* order, int64_t n_hot, int32_t* hot_ids, int32_t* slot_of_vertex) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_hot) { int32_t v = (int32_t)order[i]; hot_ids[i] = v; slot_of_vertex[v] = (int32_t)i; }
}

}  // namespace no

using namespace no;

namespace no {
static std::mutex g_cache_mutex;
static std::unordered_set<no_cache_s*> g_live_caches;
static uint64_t g_next_cache_uid = 1;
void cache_register(no_cache_s* c) { std::lock_guard<std::mutex> l(g_cache_mutex); c->uid = g_next_cache_uid++; g_live_caches.insert(c); }
void cache_unregister(no_cache_s* c) { std::lock_guard<std::mutex> l(g_cache_mutex); g_live_caches.erase(c); }
bool cache_is_live(no_cache_s* c) { std::lock_guard<std::mutex> l(g_cache_mutex); return g_live_caches.count(c) != 0; }
}  // namespace no

extern "C" int32_t no_select_hot(no_graph_t g, const int32_t* d_train_ids, int64_t n_train, int32_t batch,
                                 const int32_t* h_fanouts, int32_t n_layers, int32_t presample_epochs,
                                 double hot_fraction, int32_t staleness, int32_t emb_dim, uint64_t seed, void* stream,
                                 no_cache_t* out) {
    clear_error();
    NO_REQUIRE(out != nullptr, NO_ERR_INVALID_ARG, "no_select_hot: out is NULL");
    *out = nullptr;
    NO_REQUIRE(g && d_train_ids && h_fanouts, NO_ERR_INVALID_ARG, "no_select_hot: NULL argument");
    NO_REQUIRE(n_train >= 1 && batch >= 1, NO_ERR_INVALID_ARG, "no_select_hot: n_train and batch must be positive");
    NO_REQUIRE(n_layers >= 1 && n_layers <= NO_MAX_LAYERS, NO_ERR_INVALID_ARG, "no_select_hot: bad n_layers");
    for (int32_t h = 0; h < n_layers; ++h)
        NO_REQUIRE(h_fanouts[h] >= 1 && h_fanouts[h] <= NO_MAX_FANOUT, NO_ERR_INVALID_ARG, "no_select_hot: bad fanout[%d]", h);
    NO_REQUIRE(presample_epochs >= 1, NO_ERR_INVALID_ARG, "no_select_hot: presample_epochs must be >= 1");
    NO_REQUIRE(hot_fraction >= 0.0 && hot_fraction <= 1.0, NO_ERR_INVALID_ARG, "no_select_hot: hot_fraction outside [0,1]");
    NO_REQUIRE(staleness >= 0, NO_ERR_INVALID_ARG, "no_select_hot: staleness must be >= 0");
    NO_REQUIRE(emb_dim >= 1, NO_ERR_INVALID_ARG, "no_select_hot: emb_dim must be positive");
    NO_REQUIRE(batch <= g->n_vertices, NO_ERR_INVALID_ARG, "no_select_hot: batch larger than the graph");
    hipStream_t st = (hipStream_t)stream;
    const int64_t V = g->n_vertices;
    const int64_t nb = ceil_div(n_train, batch);
    const int64_t max_count = (int64_t)presample_epochs * nb;
    NO_REQUIRE(max_count < (1ll << 31), NO_ERR_OVERFLOW, "no_select_hot: too many pre-sampling batches");

    no_cache_s* c = new no_cache_s();
    struct Guard { no_cache_s* c; ~Guard() { if (c) { c->release(); delete c; } } } guard{c};
    c->n_vertices = V;
    c->staleness = staleness;
    c->emb_dim = emb_dim;
    c->n_hot = (int64_t)floor(hot_fraction * (double)V);
    NO_CHECK(c->freq.alloc((size_t)V));
    NO_CHECK(c->slot_of_vertex.alloc((size_t)V));
    NO_CHECK(c->hot_ids.alloc((size_t)c->n_hot));
    NO_CHECK(c->version.alloc((size_t)c->n_hot));
    NO_CHECK(c->emb.alloc((size_t)c->n_hot * emb_dim));
    NO_CHECK(fill_i32(c->freq.p, 0, V, st));
    NO_CHECK(fill_i32(c->slot_of_vertex.p, -1, V, st));
    NO_CHECK(fill_i32(c->version.p, -1, c->n_hot, st));
    NO_CHECK(fill_i32((int32_t*)c->emb.p, 0, c->n_hot * emb_dim, st));

    // pre-sampling: hops 0 .. L-2 of every batch, Philox domain 1
    no_blocks_s* b = nullptr;
    if (n_layers >= 2) NO_CHECK(blocks_create_impl(g, batch, h_fanouts, n_layers - 1, false, &b));
    struct BGuard { no_blocks_s* b; ~BGuard() { if (b) { b->release(); delete b; } } } bguard{b};
    DevBuf<int32_t> bad_flag;          // single-layer models: an id outside [0, V) among the train ids
    struct FGuard { DevBuf<int32_t>* f; ~FGuard() { f->release(); } } fguard{&bad_flag};
    NO_CHECK(bad_flag.alloc(1));
    NO_CHECK(fill_i32(bad_flag.p, 0, 1, st));
    for (int32_t p = 0; p < presample_epochs; ++p)
        for (int64_t bi = 0; bi < nb; ++bi) {
            const int64_t lo = bi * batch;
            const int32_t n = (int32_t)((lo + batch <= n_train) ? batch : (n_train - lo));
            if (n_layers >= 2) {
                NO_CHECK(sample_blocks_impl(g, d_train_ids + lo, n, seed + (uint64_t)p * (uint64_t)nb + (uint64_t)bi, 1u,
                                            n_layers - 1, nullptr, 0, b, st));
                const HopBuffers& H = b->hop[n_layers - 2];
                hipLaunchKernelGGL(count_members_kernel, dim3((unsigned)ceil_div(H.n_src_cap, 256)), dim3(256), 0, st,
                                   (const int32_t*)H.src_global.p, (const int32_t*)(b->counts.p + 4 * (n_layers - 2) + 1), 0,
                                   c->freq.p, 0, (int32_t*)nullptr);
            } else {
                hipLaunchKernelGGL(count_members_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, st,
                                   d_train_ids + lo, (const int32_t*)nullptr, n, c->freq.p, (int32_t)V, bad_flag.p);
            }
        }
    NO_CHECK(launch_status("presample"));

    // rank: stable sort of ids by (max_count - freq) keeps ascending id among equal counts
    if (c->n_hot > 0) {
        DevBuf<uint32_t> k_in, v_in, k_out, v_out, k_tmp, v_tmp;
        DevBuf<char> ws;
        struct Tmp { DevBuf<uint32_t>* u[6]; DevBuf<char>* w; ~Tmp() { for (auto p : u) p->release(); w->release(); } }
            tmp{{&k_in, &v_in, &k_out, &v_out, &k_tmp, &v_tmp}, &ws};
        NO_CHECK(k_in.alloc((size_t)V)); NO_CHECK(v_in.alloc((size_t)V));
        NO_CHECK(k_out.alloc((size_t)V)); NO_CHECK(v_out.alloc((size_t)V));
        NO_CHECK(k_tmp.alloc((size_t)V)); NO_CHECK(v_tmp.alloc((size_t)V));
        NO_CHECK(ws.alloc(radix_ws_bytes(V)));
        int64_t blocks = ceil_div(V, 256 * 4);
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(hot_keys_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const int32_t*)c->freq.p, V,
                           (uint32_t)max_count, k_in.p, v_in.p);
        int bits = ilog2_ceil((uint64_t)max_count + 1);
        if (bits < 1) bits = 1;
        NO_CHECK(radix_sort_pairs(k_in.p, v_in.p, k_out.p, v_out.p, k_tmp.p, v_tmp.p, nullptr, V, bits, ws.p, st));
        hipLaunchKernelGGL(hot_slots_kernel, dim3((unsigned)ceil_div(c->n_hot, 256)), dim3(256), 0, st,
                           (const uint32_t*)v_out.p, c->n_hot, c->hot_ids.p, c->slot_of_vertex.p);
        NO_CHECK(launch_status("hot ranking"));
        NO_HIP_CHECK(hipStreamSynchronize(st));
    }
    NO_HIP_CHECK(hipStreamSynchronize(st));
    {
        // the private blocks start with zeroed flag words, so anything in them was raised by one of the batches above
        int32_t flags[4] = {0, 0, 0, 0};
        if (b) NO_HIP_CHECK(hipMemcpy(flags, b->counts.p + 4 * (n_layers - 1) + 5, 2 * sizeof(int32_t), hipMemcpyDeviceToHost));
        NO_HIP_CHECK(hipMemcpy(flags + 2, bad_flag.p, sizeof(int32_t), hipMemcpyDeviceToHost));
        NO_REQUIRE(flags[1] == 0, NO_ERR_TIMEOUT, "no_select_hot: a scan gave up waiting for an earlier tile");
        NO_REQUIRE(flags[0] == 0 && flags[2] == 0, NO_ERR_OUT_OF_RANGE, "no_select_hot: a train id lies outside [0, V)");
    }
    guard.c = nullptr;
    no::cache_register(c);
    *out = c;
    return NO_OK;
}

extern "C" int32_t no_cache_view(no_cache_t c, int64_t* n_hot, int32_t* staleness, int32_t* emb_dim,
                                 const int32_t** d_hot_ids, const int32_t** d_slot_of_vertex, int32_t** d_version,
                                 float** d_emb, const int32_t** d_freq) {
    clear_error();
    NO_REQUIRE(c != nullptr, NO_ERR_INVALID_ARG, "no_cache_view: cache is NULL");
    if (n_hot) *n_hot = c->n_hot;
    if (staleness) *staleness = c->staleness;
    if (emb_dim) *emb_dim = c->emb_dim;
    if (d_hot_ids) *d_hot_ids = c->hot_ids.p;
    if (d_slot_of_vertex) *d_slot_of_vertex = c->slot_of_vertex.p;
    if (d_version) *d_version = c->version.p;
    if (d_emb) *d_emb = c->emb.p;
    if (d_freq) *d_freq = c->freq.p;
    return NO_OK;
}

extern "C" int32_t no_cache_set_staleness(no_cache_t c, int32_t staleness) {
    clear_error();
    NO_REQUIRE(c != nullptr, NO_ERR_INVALID_ARG, "no_cache_set_staleness: cache is NULL");
    NO_REQUIRE(staleness >= 0, NO_ERR_INVALID_ARG, "no_cache_set_staleness: staleness must be >= 0");
    c->staleness = staleness;
    ++c->generation;
    return NO_OK;
}

extern "C" int32_t no_cache_set_layer_form(no_cache_t c, no_arch form) {
    clear_error();
    NO_REQUIRE(c != nullptr, NO_ERR_INVALID_ARG, "no_cache_set_layer_form: cache is NULL");
    NO_REQUIRE(form == NO_ARCH_GCN || form == NO_ARCH_GCN_SUM || form == NO_ARCH_GCN_SYM, NO_ERR_INVALID_ARG,
               "no_cache_set_layer_form: not a GCN-style form");
    NO_REQUIRE(!(c->refresh && c->refresh->pending), NO_ERR_INVALID_ARG, "no_cache_set_layer_form: a refresh is pending");
    c->gcn_form = form;
    return NO_OK;
}

extern "C" int32_t no_cache_invalidate(no_cache_t c, void* stream) {
    clear_error();
    NO_REQUIRE(c != nullptr, NO_ERR_INVALID_ARG, "no_cache_invalidate: cache is NULL");
    ++c->generation;
    ++c->contents;
    return fill_i32(c->version.p, -1, c->n_hot, (hipStream_t)stream);
}

extern "C" int32_t no_cache_destroy(no_cache_t c) {
    clear_error();
    if (!c) return NO_OK;
    no::cache_unregister(c);
    c->release();
    delete c;
    return NO_OK;
}
