// Definitions of the opaque handles of the C ABI.
#pragma once
#include "common.hpp"

struct no_graph_s {
    int64_t n_vertices = 0, n_edges = 0;
    int32_t rowptr_bits = 64;
    no::DevBuf<int32_t> rowptr32;
    no::DevBuf<int64_t> rowptr64;
    no::DevBuf<int32_t> col;
    void release() { rowptr32.release(); rowptr64.release(); col.release(); }
};

namespace no {

// Per-hop device arrays of a sampled block. Scalars live in `counts` of the owning handle.
struct HopBuffers {
    int32_t fanout = 0;
    int32_t n_dst_cap = 0, n_src_cap = 0, nnz_cap = 0;
    bool has_csc = false;
    const int32_t* d_dst = nullptr;     // alias: seeds copy, previous hop's src_global, or compute list
    const int32_t* d_n_dst = nullptr;   // alias into counts
    DevBuf<int32_t> src_global, indptr, nbr_pad, nbr_global, indices, edge_row;
    DevBuf<int32_t> csc_indptr, csc_cnt, csc_cur, csc_dst, csc_eid;
    void release() {
        src_global.release(); indptr.release(); nbr_pad.release(); nbr_global.release(); indices.release();
        edge_row.release(); csc_indptr.release(); csc_cnt.release(); csc_cur.release(); csc_dst.release();
        csc_eid.release();
    }
};

}  // namespace no

struct no_blocks_s {
    int32_t n_layers = 0;
    int32_t n_seeds_cap = 0;
    int64_t n_vertices = 0;
    bool build_csc = true;             // transpose hops 0..L-2 (select_hot's private blocks skip it)
    bool count_sources = false;        // count the edges that leave each source in every hop, the bottom one too
                                       // (column sums of the symmetric normalisation)
    no::HopBuffers hop[NO_MAX_LAYERS];
    // counts[4*h + {0,1,2}] = n_dst, n_src, nnz of hop h; counts[4*L + {0,1,4}] = n_compute, n_hit, n_refresh;
    // counts[4*L + {5,6,7}] = flag words (bad seed id, a scan's bounded wait expired, bad label): a kernel that meets
    // the condition stores the id of the sampling call it works for, so a word counts only while it equals call_id
    // and never has to be cleared
    no::DevBuf<int32_t> counts;
    int32_t call_id = 0;               // id of the last sampling call into these blocks (1, 2, ...; never 0)
    no::DevBuf<int32_t> seeds;          // copy of the seed ids (hop 0 destinations)
    no::DevBuf<int32_t> map;            // vertex -> local id, EMPTY between calls, [V]
    no::DevBuf<int32_t> tmp_a;          // unordered transpose fill [max nnz_cap with a transpose]
    no::DevBuf<char> ws;                // tile sums of the scans
    // bottom hop with a cache
    no::DevBuf<int32_t> compute_list, compute_pos, hit_pos, hit_slot, probe_slot, probe_ver;
    no::DevBuf<int32_t> refresh_slot;        // [n_compute]: cache slot a computed row refreshes (its vertex is hot), else -1
    no::DevBuf<int32_t> refresh_old;         // [n_compute]: the version that slot held before the split stamped it
    no_cache_s* stamped_cache = nullptr;     // the cache whose versions the last split stamped (NULL: none)
    uint64_t stamped_uid = 0;                // ... its identity and the state of its contents when they were stamped
    uint64_t stamped_contents = 0;
    bool scan_two_pass = false;              // the edge compaction of the next sampling call: two launches instead of one
    no::DevBuf<int32_t> compute_inv;         // [|V^1|]: index in the compute list of position i of V^1, -1 if served from the cache
    bool last_used_cache = false;
    // The transposes and the final wipe of the id map do not feed the forward pass: they run on a side
    // stream (same priority) and are joined where their results are first needed.
    hipStream_t side = nullptr;
    hipEvent_t ev_fork[NO_MAX_LAYERS] = {nullptr};
    hipEvent_t ev_side_done = nullptr;
    hipEvent_t ev_gather_done = nullptr;
    hipEvent_t ev_indices_done = nullptr;    // side stream: local indices of every hop written
    bool upper_indices_deferred = false;     // the last call left the upper hops' indices to the side stream
    bool side_pending = false;
    no::DevBuf<char> ws_side;
    // measurement only: a pair of events for the next call's sampling kernel of hop time_hop (taken by that call)
    hipEvent_t time_ev0 = nullptr, time_ev1 = nullptr;
    int32_t time_hop = -1;
    void release() {
        if (side) { (void)hipStreamSynchronize(side); (void)hipStreamDestroy(side); side = nullptr; }
        for (auto& e : ev_fork) if (e) { (void)hipEventDestroy(e); e = nullptr; }
        if (ev_side_done) { (void)hipEventDestroy(ev_side_done); ev_side_done = nullptr; }
        if (ev_gather_done) { (void)hipEventDestroy(ev_gather_done); ev_gather_done = nullptr; }
        if (ev_indices_done) { (void)hipEventDestroy(ev_indices_done); ev_indices_done = nullptr; }
        ws_side.release();
        for (auto& h : hop) h.release();
        counts.release(); seeds.release(); map.release(); tmp_a.release(); ws.release(); compute_list.release(); compute_pos.release(); hit_pos.release(); hit_slot.release();
        probe_slot.release(); probe_ver.release(); compute_inv.release(); refresh_slot.release(); refresh_old.release();
    }
};

// Buffers of the bulk refresh (Section 4.2, Stage 2), created by the first no_refresh_hot_begin.
struct RefreshState {
    no_blocks_s* blocks = nullptr;         // one hop over all hot vertices
    int32_t fanout = 0, feat_dim = 0;
    no_dtype dt = NO_F32;
    no::DevBuf<float> emb_pending;         // [n_hot, emb_dim]: swapped with the cache's rows at the commit
    no::DevBuf<int32_t> version_pending;   // [n_hot]
    no::DevBuf<float> snap;                // parameter snapshot of the pending refresh: w_self, w_neigh, bias
    no::DevBuf<float> snap_cur;            // the snapshot the committed rows were made with (swapped at the commit)
    bool have_cur = false;                 // a refresh has been committed
    size_t snap_n = 0;                     // floats in a snapshot
    int32_t snap_arch = 0;
    no::DevBuf<float> mean;                // [n_hot, feat_dim]
    no::DevBuf<char> x0;                   // bf16 tables only: the hot vertices' own rows
    no::DevBuf<float> x_f32;               // bf16 tables only: the same rows in fp32
    hipStream_t stream = nullptr;          // default priority, non-blocking
    hipEvent_t ev_snap = nullptr, ev_done = nullptr;
    bool pending = false;
    void release() {
        if (stream) { (void)hipStreamSynchronize(stream); (void)hipStreamDestroy(stream); stream = nullptr; }
        if (ev_snap) { (void)hipEventDestroy(ev_snap); ev_snap = nullptr; }
        if (ev_done) { (void)hipEventDestroy(ev_done); ev_done = nullptr; }
        if (blocks) { blocks->release(); delete blocks; blocks = nullptr; }
        emb_pending.release(); version_pending.release(); snap.release(); snap_cur.release(); mean.release(); x0.release(); x_f32.release();
        pending = false;
    }
};

struct no_cache_s {
    int64_t n_vertices = 0;
    int64_t n_hot = 0;
    int32_t staleness = 0;
    int32_t emb_dim = 0;
    no::DevBuf<int32_t> hot_ids, slot_of_vertex, version, freq;
    no::DevBuf<float> emb;
    // identity and change counters: a batch split ahead of time is only valid against the cache as it stood
    uint64_t uid = 0;                  // unique per cache ever created (an address may be reused after a destroy)
    uint64_t generation = 0;           // bumped by a refresh commit, an invalidate and a change of the bound
    uint64_t contents = 0;             // bumped by a refresh commit and an invalidate (all versions replaced)
    int32_t gcn_form = NO_ARCH_GCN;    // the GCN-style form a one-matrix bulk refresh computes
    RefreshState* refresh = nullptr;
    void release() {
        if (refresh) { refresh->release(); delete refresh; refresh = nullptr; }
        hot_ids.release(); slot_of_vertex.release(); version.release(); freq.release(); emb.release();
    }
};

namespace no {
// Internal entry used by no_sample_blocks and no_select_hot.
// With join == false the caller must call blocks_join(b, st) before anything on `st` reads a transpose
// or starts another sampling call on the same blocks.
// Optional job run first on the side stream: dense copy of the last hop's destination feature rows
// (out[i,:] = table[dst[i],:]); the caller waits on b->ev_gather_done before reading `out`.
struct SideGather { const void* table = nullptr; int32_t row_bytes = 0; void* out = nullptr; bool needed_by_forward = true; };
int32_t sample_blocks_impl(no_graph_s* g, const int32_t* d_seeds, int32_t n_seeds, uint64_t stream_key,
                           uint32_t domain, int32_t n_hops, no_cache_s* cache, int64_t step, no_blocks_s* b,
                           hipStream_t st, bool join = true, const SideGather* gather = nullptr,
                           bool stamp_refresh = false);
int32_t blocks_join(no_blocks_s* b, hipStream_t st);
// stamp_refresh: the split writes `step` into the version of every cache slot the batch will recompute (training
// calls; the row follows with the layer-1 product). blocks_unstamp takes the stamps back for a batch that is dropped.
int32_t blocks_unstamp(no_blocks_s* b, hipStream_t st);
// Test aid (no_debug_scan_wait): spin limit of the single-pass scans' bounded waits, and whether tile 0 withholds its word.
struct ScanWaitDebug { int32_t spin_limit; int32_t withhold_first_tile; };
ScanWaitDebug scan_wait_debug();
// Caches handed out and not yet destroyed: a dropped batch's stamps are only taken back from a cache that still exists.
void cache_register(no_cache_s* c);
void cache_unregister(no_cache_s* c);
bool cache_is_live(no_cache_s* c);
// The pending bulk refresh becomes the cache contents once `st` has waited for it (no_refresh_hot_commit).
int32_t refresh_commit_impl(no_cache_s* c, hipStream_t st);
int32_t blocks_create_impl(no_graph_s* g, int32_t n_seeds_cap, const int32_t* fanouts, int32_t n_layers,
                           bool build_csc, no_blocks_s** out);
void fill_block_view(const no_blocks_s* b, int32_t hop, no_block_view* v);

// Layer pieces used by no_sage_layer_* and no_train_step (sage.hip / gemm.hip).
struct GemmOperand { const float* p; int64_t ld; };
}  // namespace no
