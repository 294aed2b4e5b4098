// Internal interfaces between the layer kernels (sage.hip, gather.hip) and the step driver.
#pragma once
#include "common.hpp"
#include "gemm.hpp"

namespace no {

// Event-pair timer for the stages of a step; a disabled profiler costs one branch per mark.
struct StageProfiler {
    static constexpr int MAX_MARKS = 96;
    bool enabled = false;
    bool created = false;
    hipStream_t st = nullptr;
    hipEvent_t ev[2 * MAX_MARKS];
    int stage_of[MAX_MARKS];
    int n = 0;
    double total_ms[NO_STAGE_COUNT] = {0};
    int32_t steps = 0;
    void begin(int stage) {
        if (!enabled || n >= MAX_MARKS) return;
        stage_of[n] = stage;
        (void)hipEventRecord(ev[2 * n], st);
    }
    void end() {
        if (!enabled || n >= MAX_MARKS) return;
        (void)hipEventRecord(ev[2 * n + 1], st);
        ++n;
    }
    // a stage that is one kernel: the pair is handed to the launch and takes the kernel's own start and end
    void kernel_pair(int stage, hipEvent_t* a, hipEvent_t* b) {
        *a = *b = nullptr;
        if (!enabled || n >= MAX_MARKS) return;
        stage_of[n] = stage;
        *a = ev[2 * n];
        *b = ev[2 * n + 1];
        ++n;
    }
};

struct LayerWorkspace {
    float* gz = nullptr;             // [n_dst_cap, d_out] masked output gradient
    float* gmean = nullptr;          // [n_dst_cap, d_in]  gradient of the mean, pre-divided by the row length
    float* x_dst_f32 = nullptr;      // [n_dst_cap, d_in]  fp32 copy of bf16 destination rows
    float* partials = nullptr;       // [2, splits, d_in + 1, d_out]
    int32_t splits = 1;
    size_t bytes = 0;
};

// Row copies carried by extra blocks of an aggregation launch: dst[dst_rows[i], :] = src[src_rows[i], :] for i < *d_n.
struct RowCopyJob {
    const float* src = nullptr; const int32_t* src_rows = nullptr; const int32_t* dst_rows = nullptr;
    const int32_t* d_n = nullptr; int32_t n_cap = 0; float* dst = nullptr; int32_t dim = 0;
    uint32_t first_block = 0;             // set by the launcher
};

// How segment_rows_kernel combines a destination's row (forward aggregate, Eq. 1).
enum { AGG_NEIGH_MEAN = 0,   // average of the sampled row (GraphSAGE-mean; the self path is a separate product)
       AGG_SELF_MEAN = 1,    // over N_in(v) U {v}: average
       AGG_SELF_SUM = 2,     //                     sum
       AGG_SELF_SYM = 3 };   //                     symmetric normalisation (per-source weights)

inline bool arch_is_gcn(int32_t arch) { return arch == NO_ARCH_GCN || arch == NO_ARCH_GCN_SUM || arch == NO_ARCH_GCN_SYM; }

// Where the number of block edges that leave each source comes from (symmetric normalisation): counts per local
// source, or the row pointers of the block's transpose (is_ptr); `local` maps entry p of the aggregated index array
// to its local source when that array holds other ids (the fused layer-1 aggregate reads global ids).
struct SourceWeights {
    const int32_t* cnt = nullptr; int32_t is_ptr = 0; const int32_t* local = nullptr;
};

// The sampler's fixed-stride slot array of a hop (row r: entries [r*k, r*k + k), global ids in slot order, -1 from the
// first unused slot on, first occurrences possibly marked as -2 - id): lets the fused layer-1 aggregate skip the row
// pointers and the compacted index array.
struct PaddedSlots { const int32_t* pad = nullptr; int32_t k = 0; };

// A layer fed by a bf16 feature table whose products take bf16 operands on the matrix cores (fp32 accumulation): the
// destinations' rows come straight from the table in the forward pass (row m = table row x_rows[m]) and from the dense
// bf16 copy in the backward pass; the two weight matrices are kept as bf16 copies in the product's layout.
struct Bf16Products {
    const uint16_t* x_table = nullptr; int64_t ldx = 0; const int32_t* x_rows = nullptr;
    const uint16_t* x_dense = nullptr;
    uint16_t* wt_self = nullptr; uint16_t* wt_neigh = nullptr; int32_t Kpad = 0;
};

// Layer 1 with reuse (Section 4.1.2): where the computed rows go, which of them refresh the cache, and the reused
// rows to copy in from the cache.
struct Layer1Reuse {
    const int32_t* compute_pos = nullptr;     // row m of the layer's output -> row of H^1
    const int32_t* refresh_slot = nullptr;    // >= 0: the row is also stored in that cache slot, stamped `step`
    float* emb = nullptr; int32_t* version = nullptr; int32_t step = 0;
    RowCopyJob hits;                          // H^1[hit_pos[i]] = emb[hit_slot[i]]
};

// What the layer below needs from a layer's input gradient: masked by its ReLU decision (its output h, one row per
// source row of this layer) and, when only some rows take a gradient, compacted to them (out_rows[u] = row of gz_out
// for source row u, -1 = none; NULL = same row). With this the input gradient goes straight to gz_out.
struct BelowLayer { const float* h = nullptr; const int32_t* out_rows = nullptr; float* gz_out = nullptr; };

int32_t layer_splits(int32_t n_dst_cap, int32_t d_in, int32_t d_out);
LayerWorkspace carve_workspace(void* ws, int32_t n_dst_cap, int32_t d_in, int32_t d_out);

// agg_mode other than AGG_NEIGH_MEAN: the destination's own row (row r of x_src, or row self_idx[r]) joins the
// aggregate (Eq. 1 over N_in(v) U {v})
int32_t mean_aggregate(const void* x_src, no_dtype dt, int32_t dim, const int32_t* indptr, const int32_t* indices,
                       const int32_t* d_n_dst, int32_t n_dst_cap, float* mean, hipStream_t st,
                       int32_t agg_mode = AGG_NEIGH_MEAN, const int32_t* self_idx = nullptr, const RowCopyJob* copy = nullptr,
                       hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr, const SourceWeights* weights = nullptr,
                       const PaddedSlots* padded = nullptr);
int32_t transpose_aggregate(const float* gmean_scaled, int32_t dim, const int32_t* csc_indptr, const int32_t* csc_dst,
                            const int32_t* d_n_src, int32_t n_src_cap, const int32_t* d_n_dst, float* grad_x,
                            hipStream_t st, const float* mask_h = nullptr, const int32_t* out_rows = nullptr,
                            float* masked_out = nullptr, const SourceWeights* weights = nullptr);
int32_t sage_forward(const no_block_view& blk, const void* x_src, no_dtype dt, int32_t d_in, const float* w_self,
                     const float* w_neigh, const float* bias, int32_t d_out, int32_t relu, float* mean, float* h,
                     const LayerWorkspace& w, hipStream_t st, StageProfiler* prof = nullptr, int agg_stage = -1,
                     int gemm_stage = -1, const void* agg_table = nullptr, hipEvent_t wait_before_gemm = nullptr,
                     int32_t arch = NO_ARCH_SAGE_MEAN, const Layer1Reuse* reuse = nullptr, bool aggregate_done = false,
                     const SourceWeights* weights = nullptr, const PaddedSlots* padded = nullptr,
                     const Bf16Products* bf = nullptr);
int32_t sage_backward(const no_block_view& blk, const void* x_src, no_dtype dt, int32_t d_in, const float* mean,
                      const float* h, const float* grad_h, const float* w_self, const float* w_neigh, int32_t d_out,
                      int32_t relu, float* gw_self, float* gw_neigh, float* gbias, float* grad_x_src,
                      const LayerWorkspace& w, hipStream_t st, StageProfiler* prof = nullptr, int prep_stage = -1,
                      int dw_stage = -1, int reduce_stage = -1, int dx_stage = -1,
                      const int32_t* grad_rows = nullptr, float lr = 0.f, float* w_self_rw = nullptr,
                      float* w_neigh_rw = nullptr, float* bias_rw = nullptr, int32_t arch = NO_ARCH_SAGE_MEAN,
                      const StatsJob* stats_job = nullptr, const float* gz_in = nullptr,
                      const BelowLayer* below = nullptr, GradJobs* pending = nullptr, bool defer = false,
                      const SourceWeights* weights = nullptr, const Bf16Products* bf = nullptr);
int32_t gather_rows(const void* d_table, int32_t row_bytes, int64_t table_stride, const int32_t* d_ids,
                    const int32_t* d_n, int32_t n_cap, void* d_out, int64_t out_stride, hipStream_t st);

}  // namespace no
