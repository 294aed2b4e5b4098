// no_refresh_hot_begin / no_refresh_hot_commit: bulk refresh of the hot embeddings per super-batch
// (Section 4.2: Stage 2 and "Bounded Staleness"). While one super-batch of n steps trains, the layer-1
// embedding of EVERY hot vertex is recomputed for the next one: a one-hop sample at the bottom fanout
// (Philox domain 2, stream seed + version), the fused gather + mean aggregate and the dense update with a
// snapshot of the layer-1 parameters taken in stream order. The paper gives this work to the CPU; here it
// runs on a second stream of the same GPU, next to the training steps, into a second copy of the cache
// that becomes current at the super-batch boundary. A row made from parameter version k*n then serves
// steps (k+1)*n ... (k+2)*n - 1: version gap at most 2n - 1.
#include "primitives.hpp"
#include "handles.hpp"
#include "layers.hpp"

#include <utility>

using namespace no;

static int32_t refresh_create(no_cache_s* c, no_graph_s* g, no_dtype dt, int32_t feat_dim, int32_t fanout) {
    RefreshState* r = new RefreshState();
    struct Guard { RefreshState* r; ~Guard() { if (r) { r->release(); delete r; } } } guard{r};
    r->fanout = fanout;
    r->feat_dim = feat_dim;
    r->dt = dt;
    NO_CHECK(blocks_create_impl(g, (int32_t)c->n_hot, &fanout, 1, false, &r->blocks));
    NO_CHECK(r->emb_pending.alloc((size_t)c->n_hot * c->emb_dim));
    NO_CHECK(r->version_pending.alloc((size_t)c->n_hot));
    r->snap_n = (size_t)2 * feat_dim * c->emb_dim + c->emb_dim;
    NO_CHECK(r->snap.alloc(r->snap_n));
    NO_CHECK(r->snap_cur.alloc(r->snap_n));
    NO_CHECK(r->mean.alloc((size_t)c->n_hot * feat_dim));
    if (dt == NO_BF16) {
        NO_CHECK(r->x0.alloc((size_t)c->n_hot * feat_dim * 2));
        NO_CHECK(r->x_f32.alloc((size_t)c->n_hot * feat_dim));
    }
    NO_HIP_CHECK(hipStreamCreateWithFlags(&r->stream, hipStreamNonBlocking));
    NO_HIP_CHECK(hipEventCreateWithFlags(&r->ev_snap, NO_SYNC_EVENT_FLAGS));
    NO_HIP_CHECK(hipEventCreateWithFlags(&r->ev_done, NO_SYNC_EVENT_FLAGS));
    c->refresh = r;
    guard.r = nullptr;
    return NO_OK;
}

extern "C" int32_t no_refresh_hot_begin(no_cache_t c, no_graph_t g, const void* d_features, no_dtype dt, int32_t feat_dim,
                                        const float* d_w_self, const float* d_w_neigh, const float* d_bias, int32_t fanout,
                                        int64_t version, uint64_t seed, void* stream) {
    clear_error();
    NO_REQUIRE(c && g && d_features && d_w_self && d_bias, NO_ERR_INVALID_ARG, "no_refresh_hot_begin: NULL argument");
    const int32_t arch = d_w_neigh ? NO_ARCH_SAGE_MEAN : c->gcn_form;       // one matrix: the GCN-style layer
    NO_REQUIRE(dt == NO_F32 || dt == NO_BF16, NO_ERR_INVALID_ARG, "no_refresh_hot_begin: unknown dtype");
    NO_REQUIRE(feat_dim >= 1, NO_ERR_INVALID_ARG, "no_refresh_hot_begin: feat_dim must be positive");
    NO_REQUIRE(fanout >= 1 && fanout <= NO_MAX_FANOUT, NO_ERR_INVALID_ARG, "no_refresh_hot_begin: bad fanout");
    NO_REQUIRE(version >= 0 && version < (1ll << 31), NO_ERR_INVALID_ARG, "no_refresh_hot_begin: version out of range");
    NO_REQUIRE(c->n_vertices == g->n_vertices, NO_ERR_INVALID_ARG, "no_refresh_hot_begin: cache belongs to another graph");
    if (c->n_hot == 0) return NO_OK;
    NO_REQUIRE(c->n_hot * ((int64_t)fanout + 1) < (1ll << 31) - 1, NO_ERR_OVERFLOW,
               "no_refresh_hot_begin: %lld hot vertices x fanout %d exceed int32", (long long)c->n_hot, fanout);
    if (!c->refresh) NO_CHECK(refresh_create(c, g, dt, feat_dim, fanout));
    RefreshState* r = c->refresh;
    NO_REQUIRE(r->fanout == fanout && r->feat_dim == feat_dim && r->dt == dt, NO_ERR_INVALID_ARG,
               "no_refresh_hot_begin: the refresh buffers were created for fanout %d, %d features", r->fanout, r->feat_dim);
    NO_REQUIRE(!r->pending, NO_ERR_INVALID_ARG, "no_refresh_hot_begin: a refresh is pending; commit it first");
    hipStream_t st = (hipStream_t)stream;
    const int32_t d_out = c->emb_dim;
    const int32_t n_hot = (int32_t)c->n_hot;

    // snapshot of the layer-1 parameters in the caller's stream order; everything else on the refresh stream
    float* w_self = r->snap.p;
    float* w_neigh = w_self + (size_t)feat_dim * d_out;
    float* bias = w_neigh + (size_t)feat_dim * d_out;
    NO_HIP_CHECK(hipMemcpyAsync(w_self, d_w_self, (size_t)feat_dim * d_out * 4, hipMemcpyDeviceToDevice, st));
    if (d_w_neigh)
        NO_HIP_CHECK(hipMemcpyAsync(w_neigh, d_w_neigh, (size_t)feat_dim * d_out * 4, hipMemcpyDeviceToDevice, st));
    NO_HIP_CHECK(hipMemcpyAsync(bias, d_bias, (size_t)d_out * 4, hipMemcpyDeviceToDevice, st));
    NO_HIP_CHECK(hipEventRecord(r->ev_snap, st));
    NO_HIP_CHECK(hipStreamWaitEvent(r->stream, r->ev_snap, 0));

    r->snap_arch = arch;
    const bool bf16 = dt == NO_BF16 && arch == NO_ARCH_SAGE_MEAN;    // only the separate self path needs the rows' own copy
    SideGather sg;
    sg.table = d_features;
    sg.row_bytes = feat_dim * (dt == NO_BF16 ? 2 : 4);
    sg.out = r->x0.p;
    sg.needed_by_forward = true;
    r->blocks->count_sources = arch == NO_ARCH_GCN_SYM;
    NO_CHECK(sample_blocks_impl(g, c->hot_ids.p, n_hot, seed + (uint64_t)version, 2u, 1, nullptr, 0, r->blocks, r->stream, true,
                                bf16 ? &sg : nullptr));
    no_block_view view;
    fill_block_view(r->blocks, 0, &view);
    view.d_indices = view.d_nbr_global;        // aggregate straight from the table through the global ids
    LayerWorkspace w;
    w.x_dst_f32 = bf16 ? r->x_f32.p : nullptr;
    const PaddedSlots slots{r->blocks->hop[0].nbr_pad.p, r->blocks->hop[0].fanout};
    SourceWeights sw;
    if (arch == NO_ARCH_GCN_SYM) { sw.cnt = r->blocks->hop[0].csc_cnt.p; sw.local = r->blocks->hop[0].indices.p; }
    NO_CHECK(sage_forward(view, bf16 ? (const void*)r->x0.p : d_features, dt, feat_dim, w_self, w_neigh, bias, d_out, 1,
                          r->mean.p, r->emb_pending.p, w, r->stream, nullptr, -1, -1, d_features,
                          bf16 ? r->blocks->ev_gather_done : nullptr, arch, nullptr, false, &sw, &slots));
    NO_CHECK(fill_i32(r->version_pending.p, (int32_t)version, n_hot, r->stream));
    NO_HIP_CHECK(hipEventRecord(r->ev_done, r->stream));
    r->pending = true;
    return NO_OK;
}

namespace no {
int32_t refresh_commit_impl(no_cache_s* c, hipStream_t st) {
    if (c->n_hot == 0) return NO_OK;
    RefreshState* r = c->refresh;
    NO_REQUIRE(r && r->pending, NO_ERR_INVALID_ARG, "no_refresh_hot_commit: no refresh is pending");
    NO_HIP_CHECK(hipStreamWaitEvent(st, r->ev_done, 0));
    // work queued on `st` so far holds the old pointers; work queued from here on sees the new rows
    std::swap(c->emb.p, r->emb_pending.p);
    std::swap(c->version.p, r->version_pending.p);
    std::swap(r->snap.p, r->snap_cur.p);
    r->have_cur = true;
    r->pending = false;
    ++c->generation;      // a batch split against the previous rows is no longer the batch a step would sample now
    ++c->contents;
    return NO_OK;
}
}  // namespace no

extern "C" int32_t no_refresh_hot_commit(no_cache_t c, void* stream) {
    clear_error();
    NO_REQUIRE(c != nullptr, NO_ERR_INVALID_ARG, "no_refresh_hot_commit: cache is NULL");
    return refresh_commit_impl(c, (hipStream_t)stream);
}
