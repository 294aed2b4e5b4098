// no_train_step: the loop body of Algorithm 1 on one stream with no host synchronisation:
// sample -> gather -> forward -> loss -> backward -> SGD, with hot-vertex embedding reuse
// (Section 4.1.2): layer-1 rows of reusable hot vertices come from the cache, take no gradient,
// and every computed hot vertex refreshes its slot with version = step.
#include "handles.hpp"
#include "layers.hpp"

#include <condition_variable>
#include <functional>
#include <mutex>
#include <string>
#include <thread>
#include <utility>

namespace no {
// A helper thread that enqueues the preparation of the next batch (about as many launches as the step itself) while
// the calling thread enqueues the step: enqueueing, not the GPU, bounds a step once the kernels are short. One job at a
// time; the job may wait once for a signal from the caller (the point in the caller's stream its second half depends
// on has been recorded). The caller always joins before it returns, so no call overlaps another.
struct AheadWorker {
    std::thread th;
    std::mutex mu;
    std::condition_variable cv;
    std::function<int32_t()> job;
    bool has_job = false, busy = false, stop = false;
    int signal = 0;               // 0: not yet; 1: go on; 2: the caller gave up (skip the second half)
    int32_t status = NO_OK;
    std::string msg;
    int device = 0;
    void start(int dev) {
        device = dev;
        th = std::thread([this] {
            (void)hipSetDevice(device);
            std::unique_lock<std::mutex> l(mu);
            for (;;) {
                cv.wait(l, [this] { return has_job || stop; });
                if (stop) return;
                has_job = false;
                std::function<int32_t()> f = std::move(job);
                l.unlock();
                const int32_t s = f();
                std::string m = s == NO_OK ? std::string() : std::string(no_last_error());
                l.lock();
                status = s;
                msg = std::move(m);
                busy = false;
                cv.notify_all();
            }
        });
    }
    void submit(std::function<int32_t()> f) {
        std::lock_guard<std::mutex> l(mu);
        job = std::move(f);
        has_job = busy = true;
        signal = 0;
        cv.notify_all();
    }
    void send(int value) {
        std::lock_guard<std::mutex> l(mu);
        if (signal == 0) signal = value;
        cv.notify_all();
    }
    int wait_signal() {
        std::unique_lock<std::mutex> l(mu);
        cv.wait(l, [this] { return signal != 0; });
        return signal;
    }
    int32_t join() {          // the job's status; its message becomes the calling thread's
        std::unique_lock<std::mutex> l(mu);
        cv.wait(l, [this] { return !busy; });
        const int32_t s = status;
        status = NO_OK;
        if (s != NO_OK) set_error("%s", msg.c_str());
        return s;
    }
    void shutdown() {
        if (!th.joinable()) return;
        { std::lock_guard<std::mutex> l(mu); stop = true; if (signal == 0) signal = 2; cv.notify_all(); }
        th.join();
    }
};
}  // namespace no

struct no_model_s {
    int32_t n_layers = 0;
    int32_t dims[NO_MAX_LAYERS + 1] = {0};
    int32_t fanouts[NO_MAX_LAYERS] = {0};
    int32_t n_seeds_cap = 0;
    no_dtype feat_dtype = NO_F32;
    int64_t n_vertices = 0;
    no_blocks_s* blocks = nullptr;
    no::DevBuf<float> params, grads;                 // per layer: w_self, w_neigh, bias
    size_t off_w_self[NO_MAX_LAYERS], off_w_neigh[NO_MAX_LAYERS], off_bias[NO_MAX_LAYERS];
    size_t n_params = 0;
    no::DevBuf<char> x0;                             // gathered rows of the bottom hop's destinations [n_dst_cap, F]
    // bf16 tables with GraphSAGE-mean layers: layer 1's products take bf16 operands; its two matrices as bf16 copies
    // [2][d_1][Kpad] in the product's layout, rewritten by every step's update (and from the parameters when the
    // caller may have changed them: weights_dirty)
    no::DevBuf<uint16_t> wt1;
    int32_t wt1_kpad = 0;
    hipEvent_t ev_dw_join = nullptr;
    bool weights_dirty = true;
    no::DevBuf<float> mean[NO_MAX_LAYERS];           // layer l (index l-1): [n_dst_cap, d_{l-1}]
    no::DevBuf<float> h[NO_MAX_LAYERS];              // layer l output [rows, d_l]; h[0] holds all of V^1
    no::DevBuf<float> gh[NO_MAX_LAYERS];             // gradient w.r.t. h[l-1]
    no::DevBuf<char> ws;                             // one region per layer (a layer writes the next one's gz while its own is in use)
    size_t ws_bytes = 0;
    size_t ws_off[NO_MAX_LAYERS] = {0};
    no::DevBuf<float> row_loss;
    no::DevBuf<no_step_stats> stats;
    bool last_used_cache = false;
    int32_t arch = NO_ARCH_SAGE_MEAN;
    // sampling ahead (Section 4.2, Stage 1): a second set of blocks and destination rows filled on a stream of its
    // own while the current batch trains; created by the first call that asks for it
    no_blocks_s* blocks_alt = nullptr;
    no::DevBuf<char> x0_alt;
    no::DevBuf<float> mean_alt;          // layer-1 aggregate of the batch prepared ahead
    no::DevBuf<float> h0_alt;            // H^1 of that batch (its reused rows arrive with the aggregate)
    hipStream_t sample_stream = nullptr;
    no::AheadWorker* worker = nullptr;   // enqueues the next batch's preparation beside the calling thread
    hipEvent_t ev_can_sample = nullptr, ev_sampled = nullptr, ev_l1_done = nullptr;
    bool ahead_valid = false;
    bool ahead_aggregated = false;       // mean_alt (and the reused rows of H^1) were written for the batch prepared ahead
    int64_t ahead_step = -1;
    uint64_t ahead_seed = 0;
    const int32_t* ahead_seeds = nullptr;
    int32_t ahead_n = 0;
    no_cache_s* ahead_cache = nullptr;
    uint64_t ahead_cache_uid = 0, ahead_cache_generation = 0;
    const void* ahead_features = nullptr;
    no::StageProfiler prof;
    void release() {
        if (prof.created) { for (auto& e : prof.ev) (void)hipEventDestroy(e); prof.created = false; }
        if (ev_dw_join) { (void)hipEventDestroy(ev_dw_join); ev_dw_join = nullptr; }
        if (worker) { worker->shutdown(); delete worker; worker = nullptr; }
        // a batch prepared ahead and never trained on: its split's stamps leave the cache with the model
        if (ahead_valid && blocks_alt && sample_stream) (void)no::blocks_unstamp(blocks_alt, sample_stream);
        ahead_valid = false;
        if (sample_stream) { (void)hipStreamSynchronize(sample_stream); (void)hipStreamDestroy(sample_stream); sample_stream = nullptr; }
        if (ev_can_sample) { (void)hipEventDestroy(ev_can_sample); ev_can_sample = nullptr; }
        if (ev_sampled) { (void)hipEventDestroy(ev_sampled); ev_sampled = nullptr; }
        if (ev_l1_done) { (void)hipEventDestroy(ev_l1_done); ev_l1_done = nullptr; }
        mean_alt.release();
        h0_alt.release();
        if (blocks_alt) { blocks_alt->release(); delete blocks_alt; blocks_alt = nullptr; }
        x0_alt.release(); wt1.release();
        if (blocks) { blocks->release(); delete blocks; blocks = nullptr; }
        params.release(); grads.release(); x0.release();
        for (auto& b : mean) b.release();
        for (auto& b : h) b.release();
        for (auto& b : gh) b.release();
        ws.release(); row_loss.release(); stats.release();
    }
};

namespace no {

// One wavefront per seed: numerically stable softmax cross-entropy and its gradient, scaled by 1/n.
__global__ void __launch_bounds__(256) softmax_xent_kernel(const float* __restrict__ logits, const int32_t* __restrict__ labels,
                                                           const int32_t* __restrict__ seeds, int32_t n, int32_t n_classes,
                                                           float* __restrict__ grad, float* __restrict__ row_loss,
                                                           int32_t* bad_label_flag, int32_t flag_value) {
    const int lane = (int)(threadIdx.x & 63);
    const int row = (int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (row >= n) return;
    const float* z = logits + (int64_t)row * n_classes;
    float mx = -INFINITY;
    for (int c = lane; c < n_classes; c += 64) mx = fmaxf(mx, z[c]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    float s = 0.f;
    for (int c = lane; c < n_classes; c += 64) s += expf(z[c] - mx);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    const int y = labels[seeds[row]];
    if ((uint32_t)y >= (uint32_t)n_classes) {
        // a label outside [0, C): the seed adds nothing to the loss or the gradient, and the step is flagged
        for (int c = lane; c < n_classes; c += 64) grad[(int64_t)row * n_classes + c] = 0.f;
        if (lane == 0) { row_loss[row] = 0.f; *bad_label_flag = flag_value; }
        return;
    }
    const float inv = 1.f / s, inv_n = 1.f / (float)n;
    for (int c = lane; c < n_classes; c += 64) {
        float p = expf(z[c] - mx) * inv;
        grad[(int64_t)row * n_classes + c] = (p - (c == y ? 1.f : 0.f)) * inv_n;
    }
    if (lane == 0) row_loss[row] = -(z[y] - mx - logf(s));
}

static inline unsigned wave_rows_blocks(int64_t rows) { int64_t b = ceil_div(rows, 4); return (unsigned)(b < 1 ? 1 : b); }

}  // namespace no

using namespace no;

extern "C" int32_t no_model_create(no_graph_t g, int32_t n_layers, const int32_t* h_dims, int32_t n_seeds_cap,
                                   const int32_t* h_fanouts, no_dtype feat_dtype, no_model_t* out) {
    clear_error();
    NO_REQUIRE(out != nullptr, NO_ERR_INVALID_ARG, "no_model_create: out is NULL");
    *out = nullptr;
    NO_REQUIRE(g && h_dims && h_fanouts, NO_ERR_INVALID_ARG, "no_model_create: NULL argument");
    NO_REQUIRE(n_layers >= 1 && n_layers <= NO_MAX_LAYERS, NO_ERR_INVALID_ARG, "no_model_create: bad n_layers");
    NO_REQUIRE(n_seeds_cap >= 1 && n_seeds_cap <= g->n_vertices, NO_ERR_INVALID_ARG, "no_model_create: bad n_seeds_cap");
    NO_REQUIRE(feat_dtype == NO_F32 || feat_dtype == NO_BF16, NO_ERR_INVALID_ARG, "no_model_create: unknown dtype");
    for (int32_t l = 0; l <= n_layers; ++l)
        NO_REQUIRE(h_dims[l] >= 1 && h_dims[l] <= 65536, NO_ERR_INVALID_ARG, "no_model_create: bad dims[%d]", l);
    for (int32_t h = 0; h < n_layers; ++h)
        NO_REQUIRE(h_fanouts[h] >= 1 && h_fanouts[h] <= NO_MAX_FANOUT, NO_ERR_INVALID_ARG, "no_model_create: bad fanout[%d]", h);
    no_model_s* m = new no_model_s();
    struct Guard { no_model_s* m; ~Guard() { if (m) { m->release(); delete m; } } } guard{m};
    m->n_layers = n_layers;
    m->n_seeds_cap = n_seeds_cap;
    m->feat_dtype = feat_dtype;
    m->n_vertices = g->n_vertices;
    for (int32_t l = 0; l <= n_layers; ++l) m->dims[l] = h_dims[l];
    for (int32_t h = 0; h < n_layers; ++h) m->fanouts[h] = h_fanouts[h];
    NO_CHECK(blocks_create_impl(g, n_seeds_cap, h_fanouts, n_layers, true, &m->blocks));
    size_t off = 0;
    for (int32_t l = 0; l < n_layers; ++l) {
        const size_t wsz = (size_t)m->dims[l] * m->dims[l + 1];
        m->off_w_self[l] = off;  off += (wsz + 63) & ~(size_t)63;
        m->off_w_neigh[l] = off; off += (wsz + 63) & ~(size_t)63;
        m->off_bias[l] = off;    off += ((size_t)m->dims[l + 1] + 63) & ~(size_t)63;
    }
    m->n_params = off;
    NO_CHECK(m->params.alloc(off));
    NO_CHECK(m->grads.alloc(off));
    NO_HIP_CHECK(hipMemset(m->params.p, 0, off * 4));
    NO_HIP_CHECK(hipMemset(m->grads.p, 0, off * 4));
    const int32_t L = n_layers;
    const HopBuffers& bottom = m->blocks->hop[L - 1];
    const size_t es = feat_dtype == NO_F32 ? 4 : 2;
    NO_CHECK(m->x0.alloc((size_t)bottom.n_dst_cap * m->dims[0] * es));
    if (feat_dtype == NO_BF16) {
        m->wt1_kpad = bf16_kpad(m->dims[0]);
        NO_CHECK(m->wt1.alloc((size_t)2 * m->dims[1] * m->wt1_kpad));
        NO_HIP_CHECK(hipEventCreateWithFlags(&m->ev_dw_join, NO_SYNC_EVENT_FLAGS));
    }
    size_t ws_bytes = 0;
    for (int32_t l = 1; l <= L; ++l) {
        const HopBuffers& H = m->blocks->hop[L - l];
        NO_CHECK(m->mean[l - 1].alloc((size_t)H.n_dst_cap * m->dims[l - 1]));
        NO_CHECK(m->h[l - 1].alloc((size_t)H.n_dst_cap * m->dims[l]));
        NO_CHECK(m->gh[l - 1].alloc((size_t)H.n_dst_cap * m->dims[l]));
        m->ws_off[l - 1] = ws_bytes;
        ws_bytes += carve_workspace(nullptr, H.n_dst_cap, m->dims[l - 1], m->dims[l]).bytes;
    }
    m->ws_bytes = ws_bytes;
    NO_CHECK(m->ws.alloc(ws_bytes));
    NO_CHECK(m->row_loss.alloc((size_t)n_seeds_cap));
    NO_CHECK(m->stats.alloc(2));        // the record, and behind it the two words of the weight-drift query
    NO_HIP_CHECK(hipMemset(m->stats.p, 0, sizeof(no_step_stats)));
    NO_HIP_CHECK(hipDeviceSynchronize());
    guard.m = nullptr;
    *out = m;
    return NO_OK;
}

static int32_t check_layer_index(no_model_t m, int32_t layer, const char* who) {
    NO_REQUIRE(m != nullptr, NO_ERR_INVALID_ARG, "%s: model is NULL", who);
    NO_REQUIRE(layer >= 1 && layer <= m->n_layers, NO_ERR_INVALID_ARG, "%s: layer must be in [1, %d]", who, m->n_layers);
    return NO_OK;
}

extern "C" int32_t no_model_params(no_model_t m, int32_t layer, float** d_w_self, float** d_w_neigh, float** d_bias) {
    clear_error();
    NO_CHECK(check_layer_index(m, layer, "no_model_params"));
    m->weights_dirty = true;      // the caller may write through these pointers: layer 1's bf16 copies are made again
    if (d_w_self) *d_w_self = m->params.p + m->off_w_self[layer - 1];
    if (d_w_neigh) *d_w_neigh = m->params.p + m->off_w_neigh[layer - 1];
    if (d_bias) *d_bias = m->params.p + m->off_bias[layer - 1];
    return NO_OK;
}

extern "C" int32_t no_model_set_arch(no_model_t m, no_arch arch) {
    clear_error();
    NO_REQUIRE(m != nullptr, NO_ERR_INVALID_ARG, "no_model_set_arch: model is NULL");
    NO_REQUIRE(arch == NO_ARCH_SAGE_MEAN || arch_is_gcn(arch), NO_ERR_INVALID_ARG, "no_model_set_arch: unknown layer form");
    m->arch = arch;
    // the symmetric normalisation needs the number of edges that leave each source, in the bottom hop too
    m->blocks->count_sources = arch == NO_ARCH_GCN_SYM;
    if (m->blocks_alt) m->blocks_alt->count_sources = arch == NO_ARCH_GCN_SYM;
    return NO_OK;
}

extern "C" int32_t no_model_grads(no_model_t m, int32_t layer, float** d_gw_self, float** d_gw_neigh, float** d_gbias) {
    clear_error();
    NO_CHECK(check_layer_index(m, layer, "no_model_grads"));
    if (d_gw_self) *d_gw_self = m->grads.p + m->off_w_self[layer - 1];
    if (d_gw_neigh) *d_gw_neigh = m->grads.p + m->off_w_neigh[layer - 1];
    if (d_gbias) *d_gbias = m->grads.p + m->off_bias[layer - 1];
    return NO_OK;
}

extern "C" int32_t no_model_activations(no_model_t m, int32_t layer, const float** d_h, const float** d_mean) {
    clear_error();
    NO_CHECK(check_layer_index(m, layer, "no_model_activations"));
    if (d_h) *d_h = m->h[layer - 1].p;
    if (d_mean) *d_mean = m->mean[layer - 1].p;
    return NO_OK;
}

extern "C" int32_t no_model_blocks(no_model_t m, no_blocks_t* blocks) {
    clear_error();
    NO_REQUIRE(m && blocks, NO_ERR_INVALID_ARG, "no_model_blocks: NULL argument");
    *blocks = m->blocks;
    return NO_OK;
}

extern "C" int32_t no_model_gathered(no_model_t m, const void** d_x0) {
    clear_error();
    NO_REQUIRE(m && d_x0, NO_ERR_INVALID_ARG, "no_model_gathered: NULL argument");
    *d_x0 = m->x0.p;
    return NO_OK;
}

static int32_t ensure_lookahead(no_model_s* m, no_graph_s* g) {
    if (m->blocks_alt) return NO_OK;
    NO_CHECK(blocks_create_impl(g, m->n_seeds_cap, m->fanouts, m->n_layers, true, &m->blocks_alt));
    m->blocks_alt->count_sources = m->arch == NO_ARCH_GCN_SYM;
    NO_CHECK(m->x0_alt.alloc(m->x0.n));
    NO_CHECK(m->mean_alt.alloc(m->mean[0].n));
    NO_CHECK(m->h0_alt.alloc(m->h[0].n));
    NO_HIP_CHECK(hipStreamCreateWithFlags(&m->sample_stream, hipStreamNonBlocking));
    NO_HIP_CHECK(hipEventCreateWithFlags(&m->ev_can_sample, NO_SYNC_EVENT_FLAGS));
    NO_HIP_CHECK(hipEventCreateWithFlags(&m->ev_sampled, NO_SYNC_EVENT_FLAGS));
    NO_HIP_CHECK(hipEventCreateWithFlags(&m->ev_l1_done, NO_SYNC_EVENT_FLAGS));
    int dev = 0;
    NO_HIP_CHECK(hipGetDevice(&dev));
    m->worker = new AheadWorker();
    m->worker->start(dev);
    return NO_OK;
}

static int32_t train_step_impl(no_model_t m, no_graph_t g, const void* d_features, const int32_t* d_labels,
                               const int32_t* d_seeds, int32_t n_seeds, const int32_t* d_next_seeds, int32_t n_next_seeds,
                               int32_t commit_refresh_before_next, no_cache_t cache, int64_t step, uint64_t seed,
                               float lr, no_step_stats* d_stats, no_step_stats* h_stats, void* stream) {
    clear_error();
    NO_REQUIRE(m && g && d_features && d_labels && d_seeds, NO_ERR_INVALID_ARG, "no_train_step: NULL argument");
    NO_REQUIRE(n_seeds >= 1, NO_ERR_INVALID_ARG, "no_train_step: n_seeds must be positive");
    NO_REQUIRE(n_seeds <= m->n_seeds_cap, NO_ERR_CAPACITY, "no_train_step: %d seeds exceed the capacity %d", n_seeds,
               m->n_seeds_cap);
    NO_REQUIRE(m->n_vertices == g->n_vertices, NO_ERR_INVALID_ARG, "no_train_step: model was created for another graph");
    NO_REQUIRE(step >= 0 && step < (1ll << 31), NO_ERR_INVALID_ARG, "no_train_step: step out of range");
    const int32_t L = m->n_layers;
    if (cache) {
        NO_REQUIRE(cache->n_vertices == g->n_vertices, NO_ERR_INVALID_ARG, "no_train_step: cache belongs to another graph");
        NO_REQUIRE(L < 2 || cache->emb_dim == m->dims[1], NO_ERR_INVALID_ARG,
                   "no_train_step: cache rows have %d columns, layer 1 has %d", cache->emb_dim, m->dims[1]);
    }
    hipStream_t st = (hipStream_t)stream;
    if (d_next_seeds) {
        NO_REQUIRE(n_next_seeds >= 1 && n_next_seeds <= m->n_seeds_cap, NO_ERR_CAPACITY,
                   "no_train_step_ahead: %d next seeds outside [1, %d]", n_next_seeds, m->n_seeds_cap);
        NO_REQUIRE(step + 1 < (1ll << 31), NO_ERR_INVALID_ARG, "no_train_step_ahead: step out of range");
        NO_CHECK(ensure_lookahead(m, g));
    }
    // a batch sampled ahead by the previous call is used if it is exactly this one; anything else is dropped
    // (a cache is the same cache only with the same identity and an unchanged generation: a refresh commit, an
    //  invalidate or a new bound since the split make the prepared batch another batch than a step would sample now)
    const bool presampled = m->ahead_valid && m->ahead_step == step && m->ahead_seed == seed && m->ahead_seeds == d_seeds &&
                            m->ahead_n == n_seeds && m->ahead_cache == cache && m->ahead_features == d_features &&
                            (!cache || (cache->uid == m->ahead_cache_uid && cache->generation == m->ahead_cache_generation));
    bool aggregated = false;
    if (m->ahead_valid) {
        // (ev_sampled is recorded after everything the sampling stream did for that batch, the aggregation included)
        NO_HIP_CHECK(hipStreamWaitEvent(st, m->ev_sampled, 0));
        if (presampled) {
            std::swap(m->blocks, m->blocks_alt);
            std::swap(m->x0.p, m->x0_alt.p);
            if (m->ahead_aggregated) {
                std::swap(m->mean[0].p, m->mean_alt.p);
                std::swap(m->h[0].p, m->h0_alt.p);
                aggregated = true;
            }
        } else {
            NO_CHECK(blocks_join(m->blocks_alt, st));
            NO_CHECK(blocks_unstamp(m->blocks_alt, st));      // the batch prepared ahead is not the one asked for
        }
        m->ahead_valid = false;
        m->ahead_aggregated = false;
    }
    no_blocks_s* B = m->blocks;
    no_step_stats* stats = d_stats ? d_stats : m->stats.p;

    StageProfiler& prof = m->prof;
    prof.st = st;
    prof.n = 0;

    // Sample. Only the destination rows of the bottom hop are gathered densely (the self path of layer 1 and
    // its weight gradient read them); that copy runs on the blocks' side stream next to the layer-1 aggregation,
    // which reads the neighbour rows from the feature table itself through the sampled global ids, so those
    // rows are never written and re-read.
    const int32_t es = m->feat_dtype == NO_F32 ? 4 : 2;
    const int32_t row_bytes = m->dims[0] * es;
    SideGather sg;
    sg.table = arch_is_gcn(m->arch) ? nullptr : d_features;    // GCN-style layers read every row inside the aggregation
    sg.row_bytes = row_bytes;
    sg.out = m->x0.p;
    sg.needed_by_forward = false;    // the forward product reads the destinations' table rows itself (fp32 and bf16)
    // bf16 table: layer 1's products take bf16 operands (features as stored; mean, weights, output gradient rounded)
    const bool bf16_products = m->feat_dtype == NO_BF16 && m->arch == NO_ARCH_SAGE_MEAN;
    uint16_t* wt_self = m->wt1.p;
    uint16_t* wt_neigh = m->wt1.p ? m->wt1.p + (size_t)m->dims[1] * m->wt1_kpad : nullptr;
    if (bf16_products && m->weights_dirty) {
        NO_CHECK(weights_to_bf16_t(m->params.p + m->off_w_self[0], m->dims[0], m->dims[1], m->wt1_kpad, wt_self, st));
        NO_CHECK(weights_to_bf16_t(m->params.p + m->off_w_neigh[0], m->dims[0], m->dims[1], m->wt1_kpad, wt_neigh, st));
        m->weights_dirty = false;
    }
    hipEvent_t sev0 = nullptr, sev1 = nullptr;
    if (!presampled) prof.kernel_pair(NO_STAGE_SAMPLE_ROWS_BOTTOM, &sev0, &sev1);
    prof.begin(NO_STAGE_SAMPLE);
    if (!presampled) B->scan_two_pass = false;
    if (!presampled) {
        B->time_ev0 = sev0; B->time_ev1 = sev1; B->time_hop = sev0 ? L - 1 : -1;
        NO_CHECK(sample_blocks_impl(g, d_seeds, n_seeds, seed + (uint64_t)step, 0u, L, cache, step, B, st, false, &sg, true));
        // measurement passes count the side stream's share of the sampling (local indices, transposes, map wipe) too
        if (prof.enabled) NO_CHECK(blocks_join(B, st));
    }
    prof.end();
    const bool used_cache = B->last_used_cache;
    m->last_used_cache = used_cache;
    const int32_t* extra = B->counts.p + 4 * L;
    const HopBuffers& bottom = B->hop[L - 1];
    (void)bottom;

    // The next batch is prepared on the sampling stream in two parts. Part one: sampling and the dense copy of its
    // destination rows. Its split into reused and computed rows reads the cache's versions only, and those are
    // stamped by the splits themselves (this step's split stamped the slots this step recomputes), so part one
    // depends on no kernel of this step and starts with it. Only a bulk refresh due at the boundary between the two
    // steps holds it back: that is committed after this step's layer 1, and the next batch is split against the new
    // rows. Part two, after this step's layer 1: the batch's layer-1 aggregation (mean aggregator, two or more
    // layers), which depends on no weight, into a second aggregate buffer; with it the batch's reused rows are copied
    // from the cache (they may be rows this step's layer 1 has just refreshed) into a second H^1, so this step's
    // buffers stay as the step leaves them. Both run beside this step's matrix-bound kernels.
    // (The transposes, the local indices of the upper hops and the dense copy go to that batch's own side stream: they
    // are needed by its backward pass and upper layers only, and would otherwise sit between its sampling and its
    // aggregation on the sampling stream, which is the longer of the two chains.)
    auto launch_sampling_ahead = [=]() -> int32_t {
        NO_HIP_CHECK(hipStreamWaitEvent(m->sample_stream, m->ev_can_sample, 0));
        SideGather sg2 = sg;
        sg2.out = m->x0_alt.p;
        m->blocks_alt->scan_two_pass = true;      // this sampling shares the chip with the step's products
        NO_CHECK(sample_blocks_impl(g, d_next_seeds, n_next_seeds, seed + (uint64_t)(step + 1), 0u, L, cache, step + 1,
                                    m->blocks_alt, m->sample_stream, false, &sg2, true));
        NO_HIP_CHECK(hipEventRecord(m->ev_sampled, m->sample_stream));
        m->ahead_valid = true;
        m->ahead_step = step + 1;
        m->ahead_seed = seed;
        m->ahead_seeds = d_next_seeds;
        m->ahead_n = n_next_seeds;
        m->ahead_cache = cache;
        m->ahead_cache_uid = cache ? cache->uid : 0;
        m->ahead_cache_generation = cache ? cache->generation : 0;
        m->ahead_features = d_features;
        return NO_OK;
    };
    // (ev_l1_done is recorded on the step's stream, by the calling thread, after layer 1's launch)
    auto launch_aggregate_ahead = [=]() -> int32_t {
        if (L < 2 || m->arch != NO_ARCH_SAGE_MEAN) return NO_OK;
        no_blocks_s* NB = m->blocks_alt;
        no_block_view nv;
        fill_block_view(NB, L - 1, &nv);
        RowCopyJob next_hits{};
        const bool next_cache = NB->last_used_cache;
        if (next_cache) {
            NO_HIP_CHECK(hipStreamWaitEvent(m->sample_stream, m->ev_l1_done, 0));
            next_hits.src = cache->emb.p; next_hits.src_rows = NB->hit_slot.p; next_hits.dst_rows = NB->hit_pos.p;
            next_hits.d_n = NB->counts.p + 4 * L + 1; next_hits.n_cap = nv.n_dst_cap; next_hits.dst = m->h0_alt.p;
            next_hits.dim = m->dims[1];
        }
        const PaddedSlots next_slots{NB->hop[L - 1].nbr_pad.p, NB->hop[L - 1].fanout};
        NO_CHECK(mean_aggregate(d_features, m->feat_dtype, m->dims[0], nv.d_indptr, nv.d_nbr_global, nv.d_n_dst, nv.n_dst_cap,
                                m->mean_alt.p, m->sample_stream, AGG_NEIGH_MEAN, nullptr, next_cache ? &next_hits : nullptr,
                                nullptr, nullptr, nullptr, &next_slots));
        NO_HIP_CHECK(hipEventRecord(m->ev_sampled, m->sample_stream));
        m->ahead_aggregated = true;
        return NO_OK;
    };
    // Part one starts with the step unless a refresh commit is due at the boundary. Then a helper thread enqueues both
    // parts (it waits for the caller's signal between them) while this thread enqueues the step itself; otherwise
    // both parts are enqueued here, after layer 1.
    const bool lookahead_early = d_next_seeds && !(commit_refresh_before_next && cache);
    const bool next_uses_cache = cache != nullptr && L >= 2 && cache->n_hot > 0;
    struct WorkerScope {      // whatever way this call ends, the helper is told and waited for
        AheadWorker* w = nullptr;
        ~WorkerScope() { if (w) { w->send(2); (void)w->join(); } }
    } scope;
    if (lookahead_early) {
        NO_HIP_CHECK(hipEventRecord(m->ev_can_sample, st));
        m->ahead_valid = false;
        scope.w = m->worker;
        m->worker->submit([=]() -> int32_t {
            NO_CHECK(launch_sampling_ahead());
            if (m->worker->wait_signal() != 1) return NO_OK;      // (the batch is sampled; it just has no aggregate yet)
            return launch_aggregate_ahead();
        });
    }

    // forward
    no_block_view view[NO_MAX_LAYERS];
    for (int32_t h = 0; h < L; ++h) fill_block_view(B, h, &view[h]);
    for (int32_t l = 1; l <= L; ++l) {
        const no_block_view& blk = view[L - l];
        const int32_t d_in = m->dims[l - 1], d_out = m->dims[l];
        const void* x = l == 1 ? (const void*)m->x0.p : (const void*)m->h[l - 2].p;
        const no_dtype dt = l == 1 ? m->feat_dtype : NO_F32;
        float* h_out = m->h[l - 1].p;
        Layer1Reuse reuse;
        if (l == 1 && used_cache) {
            // H^1 holds all of V^1: the computed rows are scattered to their positions by the product's epilogue,
            // which also refreshes the cache slot of a recomputed hot vertex (rows made by the step's pre-update
            // weights, version = step); the reused rows are copied from the cache beside the aggregation
            reuse.compute_pos = B->compute_pos.p;
            reuse.refresh_slot = B->refresh_slot.p;
            reuse.emb = cache->emb.p; reuse.version = nullptr /* stamped by the split */; reuse.step = (int32_t)step;
            reuse.hits.src = cache->emb.p; reuse.hits.src_rows = B->hit_slot.p; reuse.hits.dst_rows = B->hit_pos.p;
            reuse.hits.d_n = extra + 1; reuse.hits.n_cap = blk.n_dst_cap; reuse.hits.dst = m->h[0].p; reuse.hits.dim = d_out;
        }
        LayerWorkspace w = carve_workspace(m->ws.p + m->ws_off[l - 1], blk.n_dst_cap, d_in, d_out);
        // symmetric normalisation: the column sums of the block's adjacency are the per-source edge counts of the hop
        // (written with the local indices on the blocks' side stream); the fused layer-1 aggregate reads global ids,
        // so it also takes the local index of every entry
        SourceWeights sw;
        if (m->arch == NO_ARCH_GCN_SYM) {
            sw.cnt = B->hop[L - l].csc_cnt.p;
            if (l == 1) { sw.local = B->hop[L - 1].indices.p; NO_HIP_CHECK(hipStreamWaitEvent(st, B->ev_indices_done, 0)); }
        }
        if (l == 2) prof.begin(NO_STAGE_FWD_UPPER);
        // layers above the bottom one aggregate through local indices; without the cache split those are written
        // on the blocks' side stream
        if (l == 2 && B->upper_indices_deferred) NO_HIP_CHECK(hipStreamWaitEvent(st, B->ev_indices_done, 0));
        if (l == 1) {
            // fused gather + aggregate: rows of the table addressed by the sampled neighbours' global ids; the
            // dense product then waits for the destination rows copied on the side stream
            no_block_view fused = blk;
            fused.d_indices = blk.d_nbr_global;
            const PaddedSlots slots{B->hop[L - 1].nbr_pad.p, B->hop[L - 1].fanout};
            Bf16Products bfp;
            if (bf16_products) {
                bfp.x_table = (const uint16_t*)d_features; bfp.ldx = d_in; bfp.x_rows = blk.d_src_global;
                bfp.wt_self = wt_self; bfp.wt_neigh = wt_neigh; bfp.Kpad = m->wt1_kpad;
            }
            NO_CHECK(sage_forward(fused, x, dt, d_in, m->params.p + m->off_w_self[0], m->params.p + m->off_w_neigh[0],
                                  m->params.p + m->off_bias[0], d_out, l < L ? 1 : 0, m->mean[0].p, h_out, w, st, &prof,
                                  NO_STAGE_AGG_L1, NO_STAGE_GEMM_FWD_L1, d_features,
                                  arch_is_gcn(m->arch) ? nullptr : B->ev_gather_done, m->arch,
                                  (l == 1 && used_cache) ? &reuse : nullptr, aggregated, &sw, &slots,
                                  bf16_products ? &bfp : nullptr));
        } else
        NO_CHECK(sage_forward(blk, x, dt, d_in, m->params.p + m->off_w_self[l - 1], m->params.p + m->off_w_neigh[l - 1],
                              m->params.p + m->off_bias[l - 1], d_out, l < L ? 1 : 0, m->mean[l - 1].p, h_out, w, st,
                              l == 1 ? &prof : nullptr, NO_STAGE_AGG_L1, NO_STAGE_GEMM_FWD_L1, nullptr, nullptr, m->arch,
                              nullptr, false, &sw));
        if (l == L && L >= 2) prof.end();
        if (l == 1 && d_next_seeds) {
            if (next_uses_cache && L >= 2 && m->arch == NO_ARCH_SAGE_MEAN) NO_HIP_CHECK(hipEventRecord(m->ev_l1_done, st));
            if (lookahead_early) {
                m->worker->send(1);
            } else {
                if (commit_refresh_before_next && cache) NO_CHECK(refresh_commit_impl(cache, st));
                NO_HIP_CHECK(hipEventRecord(m->ev_can_sample, st));
                NO_CHECK(launch_sampling_ahead());
                NO_CHECK(launch_aggregate_ahead());
            }
        }
    }

    // loss on the seeds
    const int32_t C = m->dims[L];
    prof.begin(NO_STAGE_LOSS);
    hipLaunchKernelGGL(softmax_xent_kernel, dim3(wave_rows_blocks(n_seeds)), dim3(256), 0, st, (const float*)m->h[L - 1].p,
                       d_labels, (const int32_t*)B->seeds.p, n_seeds, C, m->gh[L - 1].p, m->row_loss.p,
                       B->counts.p + 4 * L + 7, B->call_id);
    prof.end();
    // (mean loss and block sizes are written by an extra block of the step's last kernel, the layer-1 reduction)
    StatsJob stats_job;
    stats_job.row_loss = m->row_loss.p; stats_job.n = n_seeds;
    stats_job.counts = B->counts.p; stats_job.n_layers = L; stats_job.used_cache = used_cache ? 1 : 0;
    stats_job.call_id = B->call_id;
    stats_job.feat_row_bytes = row_bytes;
    stats_job.emb_row_bytes = (L >= 2 && used_cache) ? m->dims[1] * 4 : 0;
    stats_job.stats = stats;

    // backward (first joins the side stream: the transposes are needed from here on)
    NO_CHECK(blocks_join(B, st));
    // The weight gradients of the layers above the bottom one (and their SGD step) are nobody's input within the step:
    // their products and reductions are carried by the bottom layer's two launches, which end the step, instead of
    // adding two launches per layer to the chain of dependent kernels.
    GradJobs pending;
    if (bf16_products) {
        // the bottom layer's products are of another kind (bf16 operands) and cannot carry the upper layers' fp32 ones in
        // their launch: those run on the blocks' side stream (joined above, idle from here on), launched once layer 2
        // has handed over its job, beside layer 2's input gradient and the bottom layer's products
        pending.side = B->side;
        pending.fork = B->ev_fork[0];
        pending.join = m->ev_dw_join;
    }
    for (int32_t l = L; l >= 1; --l) {
        const no_block_view& blk = view[L - l];
        const int32_t d_in = m->dims[l - 1], d_out = m->dims[l];
        const void* x = l == 1 ? (const void*)m->x0.p : (const void*)m->h[l - 2].p;
        const no_dtype dt = l == 1 ? m->feat_dtype : NO_F32;
        const float* h_l = m->h[l - 1].p;
        const float* gh_l = m->gh[l - 1].p;
        if (l == L && L >= 2) prof.begin(NO_STAGE_BWD_UPPER);
        if (l == 1 && L >= 2) prof.end();
        const int32_t* grad_rows = nullptr;
        if (l == 1 && used_cache) {
            // reused rows take no gradient: the layer reads only the rows of the computed vertices (its gz arrives
            // compacted from the layer above)
            grad_rows = B->compute_pos.p;
        }
        // the input gradient of layer l >= 2 is written as the gz of layer l-1: masked by that layer's ReLU and,
        // with reuse, compacted to the computed rows (so layer l-1 launches no masking pass)
        BelowLayer below;
        const float* gz_in = nullptr;
        if (l >= 2) {
            const no_block_view& blk_below = view[L - l + 1];
            below.h = m->h[l - 2].p;
            below.out_rows = (l == 2 && used_cache) ? B->compute_inv.p : nullptr;
            below.gz_out = carve_workspace(m->ws.p + m->ws_off[l - 2], blk_below.n_dst_cap, m->dims[l - 2], m->dims[l - 1]).gz;
        }
        if (l < L) gz_in = carve_workspace(m->ws.p + m->ws_off[l - 1], blk.n_dst_cap, d_in, d_out).gz;
        LayerWorkspace w = carve_workspace(m->ws.p + m->ws_off[l - 1], blk.n_dst_cap, d_in, d_out);
        SourceWeights sw;
        if (m->arch == NO_ARCH_GCN_SYM) sw.cnt = B->hop[L - l].csc_cnt.p;
        Bf16Products bfp;
        if (bf16_products && l == 1) {
            bfp.x_dense = (const uint16_t*)m->x0.p;
            bfp.wt_self = wt_self; bfp.wt_neigh = wt_neigh; bfp.Kpad = m->wt1_kpad;
        }
        const bool launch_beside = pending.side && l == 2;
        if (launch_beside) NO_HIP_CHECK(hipEventRecord(pending.fork, st));      // (every deferred job's inputs are ready here)
        NO_CHECK(sage_backward(blk, x, dt, d_in, m->mean[l - 1].p, h_l, gh_l, m->params.p + m->off_w_self[l - 1],
                               m->params.p + m->off_w_neigh[l - 1], d_out, l < L ? 1 : 0,
                               m->grads.p + m->off_w_self[l - 1], m->grads.p + m->off_w_neigh[l - 1],
                               m->grads.p + m->off_bias[l - 1], l > 1 ? m->gh[l - 2].p : nullptr, w, st,
                               l == 1 ? &prof : nullptr, NO_STAGE_BWD_L1_PREP, NO_STAGE_GEMM_DW_L1, NO_STAGE_BWD_L1_REDUCE,
                               -1, grad_rows, lr, m->params.p + m->off_w_self[l - 1], m->params.p + m->off_w_neigh[l - 1],
                               m->params.p + m->off_bias[l - 1], m->arch, l == 1 ? &stats_job : nullptr, gz_in,
                               l >= 2 ? &below : nullptr, &pending, l >= 2, &sw, (bf16_products && l == 1) ? &bfp : nullptr));
        if (launch_beside && pending.n > 0) {
            NO_HIP_CHECK(hipStreamWaitEvent(pending.side, pending.fork, 0));
            NO_CHECK(gemm_tn_partials(pending.tn, pending.n, pending.side, nullptr, nullptr));
            NO_HIP_CHECK(hipEventRecord(pending.join, pending.side));
            pending.launched_beside = true;
        }
    }

    // (the SGD step ran inside each layer's gradient reduction, after every kernel that read the weights;
    //  the cache was refreshed during the forward pass with rows made by the pre-update weights)
    if (scope.w) {      // the helper's enqueues are part of this call
        AheadWorker* wk = scope.w;
        scope.w = nullptr;
        NO_CHECK(wk->join());
    }
    NO_CHECK(launch_status("train_step"));
    if (prof.enabled) {
        NO_HIP_CHECK(hipStreamSynchronize(st));
        for (int i = 0; i < prof.n; ++i) {
            float ms = 0.f;
            NO_HIP_CHECK(hipEventElapsedTime(&ms, prof.ev[2 * i], prof.ev[2 * i + 1]));
            prof.total_ms[prof.stage_of[i]] += (double)ms;
        }
        prof.steps += 1;
    }
    if (h_stats) {
        NO_HIP_CHECK(hipMemcpyAsync(h_stats, stats, sizeof(no_step_stats), hipMemcpyDeviceToHost, st));
        NO_HIP_CHECK(hipStreamSynchronize(st));
        NO_REQUIRE(!h_stats->scan_timeout, NO_ERR_TIMEOUT,
                   "no_train_step: a scan of the sampling gave up waiting for an earlier tile; the step's results are invalid");
    }
    return NO_OK;
}

extern "C" int32_t no_train_step(no_model_t m, no_graph_t g, const void* d_features, const int32_t* d_labels,
                                 const int32_t* d_seeds, int32_t n_seeds, no_cache_t cache, int64_t step, uint64_t seed,
                                 float lr, no_step_stats* d_stats, no_step_stats* h_stats, void* stream) {
    return train_step_impl(m, g, d_features, d_labels, d_seeds, n_seeds, nullptr, 0, 0, cache, step, seed, lr, d_stats, h_stats,
                           stream);
}

extern "C" int32_t no_train_step_ahead(no_model_t m, no_graph_t g, const void* d_features, const int32_t* d_labels,
                                       const int32_t* d_seeds, int32_t n_seeds, const int32_t* d_next_seeds,
                                       int32_t n_next_seeds, int32_t commit_refresh_before_next, no_cache_t cache,
                                       int64_t step, uint64_t seed, float lr, no_step_stats* d_stats,
                                       no_step_stats* h_stats, void* stream) {
    return train_step_impl(m, g, d_features, d_labels, d_seeds, n_seeds, d_next_seeds, n_next_seeds,
                           commit_refresh_before_next, cache, step, seed, lr, d_stats, h_stats, stream);
}

namespace no {
// out[0] = max(out[0], scale * max_i |a[i] - (b ? b[i] : 0)|) on the bit pattern (values are >= 0, so the unsigned
// integer order is the float order and the integer max is order independent)
__global__ void __launch_bounds__(256) max_abs_diff_kernel(const float* __restrict__ a, const float* __restrict__ b, int64_t n,
                                                           float scale, uint32_t* out_bits) {
    float m = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        m = fmaxf(m, fabsf(a[i] - (b ? b[i] : 0.f)));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    if ((threadIdx.x & 63) == 0) atomicMax(out_bits, __float_as_uint(m * scale));
}
}  // namespace no

extern "C" int32_t no_model_weight_drift(no_model_t m, no_cache_t cache, float lr, float* h_max_update, float* h_drift,
                                         void* stream) {
    clear_error();
    NO_REQUIRE(m && h_max_update && h_drift, NO_ERR_INVALID_ARG, "no_model_weight_drift: NULL argument");
    NO_REQUIRE(lr >= 0.f, NO_ERR_INVALID_ARG, "no_model_weight_drift: lr must be >= 0");
    hipStream_t st = (hipStream_t)stream;
    const int32_t d_in = m->dims[0], d_out = m->dims[1];
    const size_t wsz = (size_t)d_in * d_out;
    const bool gcn = arch_is_gcn(m->arch);
    uint32_t* bits = (uint32_t*)(m->stats.p + 1);           // two words behind the statistics record
    NO_CHECK(fill_i32((int32_t*)bits, 0, 2, st));
    auto launch = [&](const float* a, const float* b, size_t n, float scale, uint32_t* out) {
        int64_t blocks = ceil_div((int64_t)n, 256 * 8);
        if (blocks > 256) blocks = 256;
        if (blocks < 1) blocks = 1;
        hipLaunchKernelGGL(max_abs_diff_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a, b, (int64_t)n, scale, out);
    };
    // the largest change of a layer-1 parameter in the last update: lr * max |gradient|
    launch(m->grads.p + m->off_w_self[0], nullptr, wsz, lr, bits);
    if (!gcn) launch(m->grads.p + m->off_w_neigh[0], nullptr, wsz, lr, bits);
    launch(m->grads.p + m->off_bias[0], nullptr, (size_t)d_out, lr, bits);
    // the drift of the layer-1 parameters away from the ones the rows now in the cache were refreshed with
    const RefreshState* r = cache ? cache->refresh : nullptr;
    const bool have = r && r->have_cur && r->feat_dim == d_in && cache->emb_dim == d_out && arch_is_gcn(r->snap_arch) == gcn;
    if (have) {
        const float* s_self = r->snap_cur.p;
        const float* s_neigh = s_self + wsz;
        const float* s_bias = s_neigh + wsz;
        launch(m->params.p + m->off_w_self[0], s_self, wsz, 1.f, bits + 1);
        if (!gcn) launch(m->params.p + m->off_w_neigh[0], s_neigh, wsz, 1.f, bits + 1);
        launch(m->params.p + m->off_bias[0], s_bias, (size_t)d_out, 1.f, bits + 1);
    }
    NO_CHECK(launch_status("weight drift"));
    float host[2];
    NO_HIP_CHECK(hipMemcpyAsync(host, bits, 8, hipMemcpyDeviceToHost, st));
    NO_HIP_CHECK(hipStreamSynchronize(st));
    *h_max_update = host[0];
    *h_drift = have ? host[1] : -1.f;
    return NO_OK;
}

extern "C" int32_t no_model_destroy(no_model_t m) {
    clear_error();
    if (!m) return NO_OK;
    m->release();
    delete m;
    return NO_OK;
}

extern "C" int32_t no_model_profile(no_model_t m, int32_t enable) {
    clear_error();
    NO_REQUIRE(m != nullptr, NO_ERR_INVALID_ARG, "no_model_profile: model is NULL");
    StageProfiler& p = m->prof;
    if (enable && !p.created) {
        for (auto& e : p.ev) NO_HIP_CHECK(hipEventCreate(&e));
        p.created = true;
    }
    if (enable) {
        for (auto& t : p.total_ms) t = 0.0;
        p.steps = 0;
    }
    p.enabled = enable != 0;
    return NO_OK;
}

extern "C" int32_t no_model_stage_ms(no_model_t m, double* h_total_ms, int32_t* h_steps) {
    clear_error();
    NO_REQUIRE(m && h_total_ms && h_steps, NO_ERR_INVALID_ARG, "no_model_stage_ms: NULL argument");
    for (int s = 0; s < NO_STAGE_COUNT; ++s) h_total_ms[s] = m->prof.total_ms[s];
    *h_steps = m->prof.steps;
    return NO_OK;
}

extern "C" const char* no_stage_name(int32_t stage) {
    static const char* names[NO_STAGE_COUNT] = {"sample", "gather", "agg_l1", "gemm_fwd_l1", "fwd_upper", "loss",
                                                "bwd_upper", "bwd_l1_prep", "gemm_dw_l1", "bwd_l1_reduce", "update",
                                                "sample_rows_bottom"};
    return (stage >= 0 && stage < NO_STAGE_COUNT) ? names[stage] : "?";
}
