/*
 * neutronorch.h - C ABI of the MI355X (gfx950) hot path of one sample-based GNN training
 * step with hot-vertex embedding reuse: sample -> gather -> train (Algorithm 1), with a
 * staleness-bounded cache of hot vertices' layer-1 embeddings (Section 4.1.2).
 *
 * Conventions
 *   - Every function returns a status: NO_OK (0) or a negative NO_ERR_* code; on failure
 *     no_last_error() gives a thread-local message and no output is written unless stated.
 *   - Pointers named d_* are DEVICE addresses, h_* are HOST addresses. Buffers passed in are
 *     owned by the caller and are never freed or reallocated by the library. Opaque handles
 *     are owned by the library and released with the matching *_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream). All work is
 *     enqueued on it; calls return without synchronising unless a host out-parameter is
 *     documented to need it. Data-dependent sizes live in device scalars; kernels are
 *     launched at capacity bounds and exit early.
 *   - Handles are not thread-safe. Same inputs => bit-identical outputs (no float atomics).
 *   - Vertex ids are int32. Edge (src -> dst) makes src an in-neighbour of dst (Eq. 1).
 *   - Matrices are row-major; weights are [d_in, d_out].
 */
#ifndef NEUTRONORCH_H_
#define NEUTRONORCH_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    NO_OK = 0,
    NO_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, bad enum, S < 0, fraction outside [0,1] */
    NO_ERR_OUT_OF_RANGE = -2,  /* a vertex id outside [0, V) (only where a host-side check is possible) */
    NO_ERR_CAPACITY = -3,      /* a handle or workspace is too small for the request */
    NO_ERR_OVERFLOW = -4,      /* 32-bit row pointers requested but E >= 2^31, or V >= 2^31 */
    NO_ERR_HIP = -5,           /* a HIP runtime call failed; see no_last_error() */
    NO_ERR_UNSUPPORTED = -6,
    NO_ERR_TIMEOUT = -7        /* a kernel's bounded wait on another workgroup expired; the outputs of that call are invalid */
};

typedef enum { NO_F32 = 0, NO_BF16 = 1 } no_dtype;
/* Layer form: GraphSAGE-mean (separate self path, two matrices) or GCN-style (Eq. 1 as printed: the aggregate runs
 * over N_in(v) U {v}; Eq. 2 with one matrix). The GCN-style aggregate a_v = r_v (s_v x_v + sum over the sampled row of
 * s_u x_u) comes in the forms Eq. 1 and Table 1 name:
 *   NO_ARCH_GCN      average:  r_v = 1 / (len(row v) + 1), s = 1
 *   NO_ARCH_GCN_SUM  sum:      r = s = 1
 *   NO_ARCH_GCN_SYM  symmetric normalisation of the block's adjacency with self loops, D_r^-1/2 (A + I) D_c^-1/2:
 *                    r_v = (len(row v) + 1)^-1/2, s_u = c_u^-1/2 with c_u = number of the block's edges that leave
 *                    source u, plus one if u is a destination (row and column sums of A + I). */
typedef enum { NO_ARCH_SAGE_MEAN = 0, NO_ARCH_GCN = 1, NO_ARCH_GCN_SUM = 2, NO_ARCH_GCN_SYM = 3 } no_arch;

enum { NO_MAX_LAYERS = 8, NO_MAX_FANOUT = 64 };

typedef struct no_graph_s* no_graph_t;    /* in-neighbour CSR, device resident            */
typedef struct no_blocks_s* no_blocks_t;  /* L sampled blocks, capacity sized             */
typedef struct no_cache_s* no_cache_t;    /* hot set + embedding cache + version record   */
typedef struct no_model_s* no_model_t;    /* weights, activations and gradient workspace  */

/* Last error message of the calling thread ("" if none). Never NULL. */
const char* no_last_error(void);

/* ------------------------------------------------------------------------------------------
 * Graph (input G(V,E) of Algorithm 1; N_in(v) of Eq. 1)
 * ---------------------------------------------------------------------------------------- */

enum {
    NO_CSR_INPUT_ON_DEVICE = 1u,   /* src / dst are device pointers */
    NO_CSR_IDS_64 = 2u,            /* src / dst are int64 arrays (the ids themselves must still lie in [0, V), V < 2^31) */
    NO_CSR_SYMMETRISE = 4u,        /* every edge (s -> d) is also taken as (d -> s): 2 * n_edges edges */
    NO_CSR_DEDUP = 8u              /* of several equal edges (s -> d) one is kept (after symmetrising); needs < 2^31 edges */
};

/* Builds the in-neighbour CSR of a directed multigraph: row v lists every src with an edge
 * (src -> v), ascending by src; self-loops are kept, and so are duplicates unless NO_CSR_DEDUP is given.
 *   src, dst     int32[n_edges] (int64[n_edges] with NO_CSR_IDS_64); host pointers, or device pointers with
 *                NO_CSR_INPUT_ON_DEVICE.
 *   rowptr_bits  32 or 64: width of the row-pointer array (32 needs fewer than 2^31 edges after symmetrising).
 * Errors: NO_ERR_OUT_OF_RANGE for an endpoint outside [0, V), NO_ERR_OVERFLOW / NO_ERR_UNSUPPORTED for sizes beyond
 * the limits above (at most 2^32 - 2 edges), NO_ERR_INVALID_ARG for unknown flags.
 * Synchronises the stream before returning (it validates ids and sizes scratch). */
int32_t no_build_csr(const void* src, const void* dst, int64_t n_edges, int64_t n_vertices,
                     int32_t rowptr_bits, uint32_t flags, void* stream, no_graph_t* out);

/* Device pointers into the graph: d_rowptr is int32[V+1] or int64[V+1] by *rowptr_bits. */
int32_t no_graph_view(no_graph_t g, int64_t* n_vertices, int64_t* n_edges, int32_t* rowptr_bits,
                      const void** d_rowptr, const int32_t** d_col);
int32_t no_graph_destroy(no_graph_t g);

/* ------------------------------------------------------------------------------------------
 * Sampled blocks (the sample() loop of Algorithm 1, lines 4-7)
 * ---------------------------------------------------------------------------------------- */

/* One hop as a bipartite block. Rows are destinations; the first n_dst sources are the
 * destinations themselves, further sources follow in order of first occurrence over the
 * sampled edges in (row, slot) order. All pointers are device addresses inside the handle. */
typedef struct no_block_view {
    int32_t n_dst_cap, n_src_cap, nnz_cap;
    const int32_t* d_n_dst;       /* device scalars */
    const int32_t* d_n_src;
    const int32_t* d_nnz;
    const int32_t* d_dst_global;  /* [n_dst]  */
    const int32_t* d_src_global;  /* [n_src]  */
    const int32_t* d_indptr;      /* [n_dst+1] */
    const int32_t* d_nbr_global;  /* [nnz] sampled neighbour ids, row-major, slot order */
    const int32_t* d_indices;     /* [nnz] local source index of each sampled edge */
    const int32_t* d_csc_indptr;  /* [n_src+1] transpose; NULL when not built (bottom hop) */
    const int32_t* d_csc_dst;     /* [nnz] destination row of each transposed entry */
    const int32_t* d_csc_eid;     /* [nnz] edge id, ascending inside a column */
    /* bottom hop only, when sampled with a cache (else NULL): split of V^1 */
    const int32_t* d_compute_pos; /* [n_compute] positions in V^1 of this block's destinations */
    const int32_t* d_hit_pos;     /* [n_hit] positions in V^1 served from the cache */
    const int32_t* d_hit_slot;    /* [n_hit] their cache slots */
    const int32_t* d_n_compute;
    const int32_t* d_n_hit;
} no_block_view;

/* Allocates blocks for up to n_seeds_cap seeds and the given fanouts (hop order counted from
 * the seeds: fanouts[0] applies to the seed batch, the last entry to the bottom hop).
 * Capacities are the no-de-duplication bounds, vertex sets capped at V. The transpose of hop
 * h is built for h < n_layers-1 (the bottom layer back-propagates nothing to its inputs). */
int32_t no_blocks_create(no_graph_t g, int32_t n_seeds_cap, const int32_t* h_fanouts, int32_t n_layers,
                         no_blocks_t* out);

/* Samples n_layers hops from d_seeds[n_seeds] (unique ids). Hop h gives every destination v
 * min(deg(v), fanouts[h]) distinct entries of its CSR row, uniformly without replacement, as a
 * pure function of (seed + step, domain 0, h, v, slot) through Philox4x32-10; the whole row in
 * stored order when deg <= fanout. The destinations of hop h+1 are the sources of hop h. Seed ids outside
 * [0, V) are read as vertex 0 and flagged (no_step_stats.bad_seed, status of no_blocks_sizes); the blocks are then
 * meaningless but every access stays inside the library's and the graph's arrays.
 * With cache != NULL (and n_layers >= 2) the destinations of the bottom hop are only those
 * vertices of V^1 that cannot be served from the cache at `step` (not hot, empty slot, or
 * step - version > S). Asynchronous. */
int32_t no_sample_blocks(no_graph_t g, const int32_t* d_seeds, int32_t n_seeds, uint64_t seed, int64_t step,
                         no_cache_t cache, no_blocks_t blocks, void* stream);

int32_t no_blocks_view(no_blocks_t blocks, int32_t hop, no_block_view* out);
/* Copies (n_dst, n_src, nnz, n_hit) of every hop to h_sizes[4*n_layers] (n_hit is 0 except at
 * the bottom hop with a cache). Synchronises the stream. The sizes are written in every case; the status is
 * NO_ERR_TIMEOUT if a scan of the last sampling call into these blocks gave up its bounded wait (the blocks are then
 * invalid), else NO_ERR_OUT_OF_RANGE if that call met a seed id outside [0, V). */
int32_t no_blocks_sizes(no_blocks_t blocks, void* stream, int32_t* h_sizes);
int32_t no_blocks_destroy(no_blocks_t blocks);

/* ------------------------------------------------------------------------------------------
 * Hot set and embedding cache (Section 4.1.2; version record of Section 4.2)
 * ---------------------------------------------------------------------------------------- */

/* Pre-sampling hotness: the train ids, in the given order, are cut into batches of `batch`;
 * for presample_epochs epochs every batch is sampled for hops 0..n_layers-2 (Philox domain 1,
 * stream seed + epoch*n_batches + b) and each vertex of the resulting V^1 counts once. The hot
 * set is the floor(hot_fraction * V) most frequent vertices, ties by ascending id; slot = rank.
 * Creates an empty cache [n_hot, emb_dim] fp32 (versions -1). Synchronises the stream. A train id outside [0, V)
 * gives NO_ERR_OUT_OF_RANGE (it is never followed), an expired scan wait NO_ERR_TIMEOUT; no cache is returned then. */
int32_t no_select_hot(no_graph_t g, const int32_t* d_train_ids, int64_t n_train, int32_t batch,
                      const int32_t* h_fanouts, int32_t n_layers, int32_t presample_epochs,
                      double hot_fraction, int32_t staleness, int32_t emb_dim, uint64_t seed,
                      void* stream, no_cache_t* out);

/* d_hot_ids int32[n_hot] (hotness order), d_slot_of_vertex int32[V] (-1 = cold),
 * d_version int32[n_hot] (step whose weights produced the row; -1 = empty), d_emb fp32[n_hot, emb_dim],
 * d_freq int32[V] pre-sampling counts. Any out pointer may be NULL. */
int32_t no_cache_view(no_cache_t c, int64_t* n_hot, int32_t* staleness, int32_t* emb_dim,
                      const int32_t** d_hot_ids, const int32_t** d_slot_of_vertex,
                      int32_t** d_version, float** d_emb, const int32_t** d_freq);
int32_t no_cache_set_staleness(no_cache_t c, int32_t staleness);
/* Which GCN-style form no_refresh_hot_begin computes when it is given one matrix (default NO_ARCH_GCN, the average). */
int32_t no_cache_set_layer_form(no_cache_t c, no_arch form);
int32_t no_cache_invalidate(no_cache_t c, void* stream);   /* all versions = -1 */
int32_t no_cache_destroy(no_cache_t c);

/* Bulk refresh of the hot embeddings for the next super-batch (Section 4.2: Stage 2, "Embedding computation
 * for hot vertices", and "Bounded Staleness"). The paper lets the CPU do this while the GPU trains the n
 * batches of the current super-batch; here it runs on a stream of its own on the same GPU.
 *
 * no_refresh_hot_begin: for every hot vertex v (slot order): min(deg(v), fanout) in-neighbours drawn like a
 * bottom-hop destination (Philox stream seed + version, domain 2, hop 0), their mean, and
 * relu(W_self^T x_v + W_neigh^T mean + b) (Eq. 1 / Eq. 2), into a PENDING copy of the cache stamped
 * `version` (the parameter version = number of updates the given weights have seen). d_features is the
 * [V, feat_dim] table (fp32 or bf16 bits), d_w_self / d_w_neigh [feat_dim, emb_dim] and d_bias [emb_dim]
 * fp32 device arrays: they are copied in `stream` order before the call returns to the host, so later updates
 * of them on `stream` do not race with the refresh; the table must stay unchanged until the commit. All other
 * work runs on the cache's own stream (default priority) after that copy. The first call allocates the
 * refresh buffers (a one-hop block over n_hot destinations, the mean rows, the pending rows) and fixes
 * (dt, feat_dim, fanout) for later calls. Errors: NO_ERR_INVALID_ARG (NULL, bad sizes, another refresh still
 * pending, parameters differing from the first call), NO_ERR_OVERFLOW (n_hot * (fanout + 1) >= 2^31),
 * NO_ERR_HIP. A cache without hot vertices makes both calls no-ops. d_w_neigh == NULL selects the GCN-style
 * layer (one matrix d_w_self, aggregate over N_in(v) U {v} in the form set by no_cache_set_layer_form).
 *
 * no_refresh_hot_commit: `stream` waits for the pending refresh, then the pending rows and versions
 * become the cache's contents (the two copies are swapped: pointers returned by no_cache_view before the
 * commit now name the other copy). Rows written by a step's own refresh-on-miss since the begin are
 * replaced as well. Work already queued on `stream` keeps reading the previous copy. With the commit at
 * every n-th step, begin right after it, and staleness bound 2n - 1, every hot vertex is served from the
 * cache from the second super-batch on and the largest version gap is 2n - 1. */
int32_t no_refresh_hot_begin(no_cache_t c, no_graph_t g, const void* d_features, no_dtype dt, int32_t feat_dim,
                             const float* d_w_self, const float* d_w_neigh, const float* d_bias, int32_t fanout,
                             int64_t version, uint64_t seed, void* stream);
int32_t no_refresh_hot_commit(no_cache_t c, void* stream);

/* ------------------------------------------------------------------------------------------
 * Gather (feature collection, Algorithm 1 line 9)
 * ---------------------------------------------------------------------------------------- */

/* d_out[i, 0:dim] = d_table[d_ids[i], 0:dim] for i < n, a bit copy of `dim` elements of dt.
 * n = *d_n_ids when d_n_ids != NULL (must be <= n_ids_cap), else n_ids_cap. Strides in bytes,
 * multiples of the element size. Ids must lie in [0, n_rows) (not checked). */
int32_t no_gather_features(const void* d_table, no_dtype dt, int64_t n_rows, int32_t dim,
                           int64_t table_stride_bytes, const int32_t* d_ids, const int32_t* d_n_ids,
                           int32_t n_ids_cap, void* d_out, int64_t out_stride_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * GraphSAGE-mean layer (Eq. 1 with AGGREGATE = average, Eq. 2 with a dense UPDATE)
 * ---------------------------------------------------------------------------------------- */

size_t no_sage_layer_ws_bytes(int32_t n_dst_cap, int32_t n_src_cap, int32_t d_in, int32_t d_out);

/* Forward: d_mean[v,:] = average of d_x_src[indices[e],:] over row v (zeros for an empty row);
 * d_h = act(d_x_src[0:n_dst] * W_self + d_mean * W_neigh + bias), act = ReLU if relu else identity.
 * d_x_src [n_src, d_in] of dt_x (bf16 is upcast; accumulation is fp32), d_mean [n_dst_cap, d_in]
 * and d_h [n_dst_cap, d_out] fp32, dense. Uses d_indptr/d_indices/d_n_dst of the view. */
int32_t no_sage_layer_fwd(const no_block_view* blk, const void* d_x_src, no_dtype dt_x, int32_t d_in,
                          const float* d_w_self, const float* d_w_neigh, const float* d_bias,
                          int32_t d_out, int32_t relu, float* d_mean, float* d_h,
                          void* d_ws, size_t ws_bytes, void* stream);

/* Backward: gz = d_grad_h * [d_h > 0] (or d_grad_h when relu == 0);
 * d_gw_self = x_dst^T gz, d_gw_neigh = mean^T gz, d_gbias = column sums of gz (all overwritten);
 * if d_grad_x_src != NULL (not the bottom layer; needs the transpose in the view):
 *   d_grad_x_src[u,:] = [u < n_dst] gz[u,:] W_self^T + sum over transposed entries (v,e) of u of
 *   (gz[v,:] W_neigh^T) / len(row v), rows u < n_src, fp32 [n_src_cap, d_in].
 * Reductions run in a fixed order (no float atomics). */
int32_t no_sage_layer_bwd(const no_block_view* blk, const void* d_x_src, no_dtype dt_x, int32_t d_in,
                          const float* d_mean, const float* d_h, const float* d_grad_h,
                          const float* d_w_self, const float* d_w_neigh, int32_t d_out, int32_t relu,
                          float* d_gw_self, float* d_gw_neigh, float* d_gbias, float* d_grad_x_src,
                          void* d_ws, size_t ws_bytes, void* stream);

/* no_sage_layer_bwd for callers that can neither allocate device memory nor hand over a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels and results, with the
 * workspace in a static device array of NO_LAYER_STATIC_WS_BYTES that the library's code object carries (each GPU the
 * library runs on holds its copy until the process ends). The call allocates nothing and frees nothing. It returns
 * NO_ERR_CAPACITY, before any launch, when no_sage_layer_ws_bytes(n_dst_cap, n_src_cap, d_in, d_out) exceeds
 * NO_LAYER_STATIC_WS_BYTES. All calls on one GPU share that GPU's array and nothing in it survives a call: two calls
 * that overlap in time on one GPU (different streams, or different threads) race; calls in stream order do not. */
#define NO_LAYER_STATIC_WS_BYTES ((size_t)64 << 20)
int32_t no_sage_layer_bwd_static(const no_block_view* blk, const void* d_x_src, no_dtype dt_x, int32_t d_in,
                                 const float* d_mean, const float* d_h, const float* d_grad_h,
                                 const float* d_w_self, const float* d_w_neigh, int32_t d_out, int32_t relu,
                                 float* d_gw_self, float* d_gw_neigh, float* d_gbias, float* d_grad_x_src,
                                 void* stream);

/* GCN-style layer (Eq. 1 as printed, AGGREGATE over N_in(v) U {v}; Eq. 2 with one matrix); `form` is one of
 * NO_ARCH_GCN (average), NO_ARCH_GCN_SUM, NO_ARCH_GCN_SYM (Table 1's symmetric normalisation), see no_arch.
 * Forward: d_agg[v,:] = r_v (s_v d_x_src[v,:] + sum of s_u d_x_src[u,:] over the entries u = indices[e] of row v)
 * (destination v is source row v); d_h = act(d_agg * W + bias). Shapes, dtypes, workspace and errors as
 * no_sage_layer_fwd. Backward: gz as above; d_gw = agg^T gz, d_gbias = column sums of gz; if d_grad_x_src != NULL:
 * with ga[v,:] = r_v (gz[v,:] W^T): d_grad_x_src[u,:] = s_u ([u < n_dst] ga[u,:] + sum of ga[v,:] over the transposed
 * entries (v,e) of u). NO_ARCH_GCN_SYM reads the column sums from the view's transpose (d_csc_indptr must be set:
 * NO_ERR_INVALID_ARG otherwise), in the forward pass and for the input gradient. The workspace size is
 * no_sage_layer_ws_bytes. */
int32_t no_gcn_layer_fwd(const no_block_view* blk, no_arch form, const void* d_x_src, no_dtype dt_x, int32_t d_in,
                         const float* d_w, const float* d_bias, int32_t d_out, int32_t relu, float* d_agg,
                         float* d_h, void* d_ws, size_t ws_bytes, void* stream);
int32_t no_gcn_layer_bwd(const no_block_view* blk, no_arch form, int32_t d_in, const float* d_agg, const float* d_h,
                         const float* d_grad_h, const float* d_w, int32_t d_out, int32_t relu, float* d_gw,
                         float* d_gbias, float* d_grad_x_src, void* d_ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Whole step (loop body of Algorithm 1 with plain SGD, plus hot-embedding reuse)
 * ---------------------------------------------------------------------------------------- */

typedef struct no_step_stats {
    float loss;
    int32_t n_dst[NO_MAX_LAYERS], n_src[NO_MAX_LAYERS], nnz[NO_MAX_LAYERS];  /* per hop */
    int32_t n_hit;        /* rows of V^1 served from the cache */
    int32_t n_refresh;    /* computed rows written back to the cache */
    int32_t n_v1;         /* |V^1| */
    int32_t bad_seed;     /* 1 if a seed id of this step lay outside [0, V) (it was read as vertex 0) */
    int32_t n_miss_hot;   /* hot vertices of V^1 that could not be served (empty or too old a row) and were computed */
    int32_t n_cold;       /* vertices of V^1 outside the hot set: n_v1 = n_hit + n_miss_hot + n_cold */
    int32_t scan_timeout; /* 1 if a scan of this step's sampling gave up its bounded wait: the step's results are invalid */
    int32_t bad_label;    /* 1 if a seed's label lay outside [0, C) (that seed then adds nothing to loss and gradient) */
    int64_t bytes_gathered_features;    /* feature rows the step collected: n_src of the bottom hop x row bytes */
    int64_t bytes_gathered_embeddings;  /* cached layer-1 rows it pulled instead: n_hit x hidden x 4 */
} no_step_stats;

/* dims = [F, hidden.., C] (n_layers+1 entries). Weights live inside the handle; the caller
 * fills them through no_model_params before the first step. */
int32_t no_model_create(no_graph_t g, int32_t n_layers, const int32_t* h_dims, int32_t n_seeds_cap,
                        const int32_t* h_fanouts, no_dtype feat_dtype, no_model_t* out);
int32_t no_model_params(no_model_t m, int32_t layer /*1-based*/, float** d_w_self, float** d_w_neigh,
                        float** d_bias);
/* Selects the layer form of every layer (default NO_ARCH_SAGE_MEAN); call before the first step. With a GCN-style
 * form (NO_ARCH_GCN, NO_ARCH_GCN_SUM, NO_ARCH_GCN_SYM) layer l computes h = act(W^T a + b) with the aggregate a of
 * that form over N_in(v) U {v} (Eq. 1; Eq. 2): W is the layer's w_self array, w_neigh and its gradient are unused,
 * the `mean` activation holds a, and no_model_gathered is not filled (the aggregation reads the table itself). */
int32_t no_model_set_arch(no_model_t m, no_arch arch);
/* Gradients of the last step, device pointers (same shapes as the parameters). */
int32_t no_model_grads(no_model_t m, int32_t layer, float** d_gw_self, float** d_gw_neigh, float** d_gbias);
/* Activations of the last step: d_h fp32 [rows, dims[layer]] (layer 1 with a cache: all of V^1),
 * d_mean fp32 [n_dst, dims[layer-1]]. */
int32_t no_model_activations(no_model_t m, int32_t layer, const float** d_h, const float** d_mean);
int32_t no_model_blocks(no_model_t m, no_blocks_t* blocks);   /* blocks of the last step (owned by m) */
/* Gathered feature rows of the last step: the rows of the bottom hop's destinations [n_dst, F] (the
 * neighbour rows are read from the table by the fused layer-1 aggregation and are not materialised). */
int32_t no_model_gathered(no_model_t m, const void** d_x0);

/* One training step at parameter version `step` (= number of updates already applied):
 * sample (with hot skipping if cache != NULL), gather the bottom hop's feature rows (destination rows
 * densely, neighbour rows inside the layer-1 aggregation), forward
 * (layer-1 rows of reusable hot vertices come from the cache), mean softmax cross-entropy on the
 * seeds, backward (reused rows take no gradient), W <- W - lr * grad for every tensor; every computed
 * hot vertex's layer-1 row (made by the pre-update weights) is stored in the cache with version = step.
 * Precision: fp32 throughout, except that GraphSAGE-mean layer 1 on a bf16 feature table takes the operands of its
 * products in bf16 with fp32 accumulation (the features as stored; the fp32 mean, the weights and the output gradient
 * rounded to nearest-even on their way into the forward and weight-gradient products; the bias gradient, the mean itself,
 * the layers above, the loss and the update stay fp32). The standalone layer entry points and the bulk refresh upcast
 * bf16 rows and multiply in fp32.
 * d_stats (device, may be NULL) receives the statistics; if h_stats != NULL the stream is
 * synchronised and the statistics are copied to the host, and the call returns NO_ERR_TIMEOUT if they say that a
 * scan's wait expired (h_stats is filled all the same). */
int32_t no_train_step(no_model_t m, no_graph_t g, const void* d_features, const int32_t* d_labels,
                      const int32_t* d_seeds, int32_t n_seeds, no_cache_t cache, int64_t step,
                      uint64_t seed, float lr, no_step_stats* d_stats, no_step_stats* h_stats, void* stream);

/* no_train_step for batch `step`, plus preparing the next batch ahead (Section 4.2, Stage 1: sampling runs ahead of
 * training so that the two do not wait for each other). Results of the step are those of no_train_step. In
 * addition, if d_next_seeds != NULL, batch step + 1 (d_next_seeds[n_next_seeds], same seed) is prepared on the
 * model's own sampling stream (default priority) beside this step: it is sampled into a second set of blocks from
 * the step's start, and after this step's layer 1 its layer-1 aggregation runs into a second buffer (mean
 * aggregator with two or more layers), together with the copy of its reused rows out of the cache. The next call
 * uses that batch if it asks for exactly it (step + 1, the same d_next_seeds pointer and count, seed, cache and
 * d_features); otherwise it is dropped and the batch is sampled again. d_next_seeds and d_features must stay valid
 * and unchanged until then.
 * Cache versions: the split of a batch into reused and computed vertices writes the batch's step into the version
 * of every slot the batch will recompute (the row follows when its layer 1 runs), so while a batch is prepared
 * ahead those entries of no_cache_view already read step + 1; a dropped batch's entries are restored by the call
 * that drops it. A bulk-refresh commit, an invalidate or a change of the bound between the two calls also drops the
 * prepared batch (it was split against the cache as it stood; nothing is restored where all versions were replaced),
 * and the batch is sampled again.
 * commit_refresh_before_next != 0: a pending bulk refresh (no_refresh_hot_begin) is committed after this step's
 * last use of the cache and before the next batch is sampled (which then starts after this step's layer 1); use it
 * on the last step of a super-batch instead of calling no_refresh_hot_commit between the two steps. The first
 * call with d_next_seeds != NULL allocates the second set of blocks (as much memory as no_blocks_create for the
 * same capacities) plus second copies of the destination rows, the layer-1 aggregate and H^1, and starts a helper
 * thread owned by the model: it enqueues the next batch's preparation on the model's own streams while the calling
 * thread enqueues the step (half of a step's launches each), and the call joins it before it returns, so nothing of a
 * call is still being enqueued afterwards; no_model_destroy ends the thread. Errors as no_train_step (an error of the
 * helper's launches is reported by this call), and NO_ERR_CAPACITY for n_next_seeds outside [1, capacity]. */
int32_t no_train_step_ahead(no_model_t m, no_graph_t g, const void* d_features, const int32_t* d_labels,
                            const int32_t* d_seeds, int32_t n_seeds, const int32_t* d_next_seeds, int32_t n_next_seeds,
                            int32_t commit_refresh_before_next, no_cache_t cache, int64_t step, uint64_t seed,
                            float lr, no_step_stats* d_stats, no_step_stats* h_stats, void* stream);
/* Weight-drift monitor (convergence analysis, Section 4.3: the tolerated drift of the parameters behind stale
 * embeddings is epsilon = (largest change of a weight in one update) x 2n for super-batches of n steps).
 * *h_max_update = lr * max |g| over the layer-1 gradients of the last step (the largest change that step made to a
 * layer-1 parameter; lr is the rate that step used); *h_drift = max |W - W~| between the layer-1 parameters now and
 * the snapshot behind the rows installed by the last no_refresh_hot_commit of `cache`, or -1 when there is no such
 * snapshot (cache NULL, nothing committed yet, or made for another layer shape). The caller keeps the running
 * maximum of the first value and compares the second with epsilon. Synchronises `stream`; meant for super-batch
 * boundaries, not for the inside of a step. */
int32_t no_model_weight_drift(no_model_t m, no_cache_t cache, float lr, float* h_max_update, float* h_drift,
                              void* stream);
int32_t no_model_destroy(no_model_t m);

/* Per-stage timing of no_train_step with HIP events on the step's own stream. While enabled,
 * every step records an event pair around each stage and synchronises the stream at its end to
 * accumulate the elapsed times (so it is for measurement passes, not for throughput runs).
 * Stages that are a single kernel launch: NO_STAGE_GATHER, NO_STAGE_AGG_L1, NO_STAGE_GEMM_FWD_L1,
 * NO_STAGE_GEMM_DW_L1, NO_STAGE_SAMPLE_ROWS_BOTTOM. While enabled, the step's stream also waits for the blocks' side
 * stream (local indices, transposes, id-map wipe) before the end of NO_STAGE_SAMPLE, so that stage is all of the
 * sampling work of the step. */
enum {
    NO_STAGE_SAMPLE = 0,      /* all hops: sampling, relabel, hot lookup, and (joined) local indices + transposes */
    NO_STAGE_GATHER = 1,      /* feature rows of the bottom hop's sources */
    NO_STAGE_AGG_L1 = 2,      /* layer-1 mean aggregation kernel */
    NO_STAGE_GEMM_FWD_L1 = 3, /* layer-1 dense update kernel */
    NO_STAGE_FWD_UPPER = 4,   /* cache row assembly and refresh + layers 2..L forward */
    NO_STAGE_LOSS = 5,
    NO_STAGE_BWD_UPPER = 6,   /* layers L..2 backward */
    NO_STAGE_BWD_L1_PREP = 7, /* gradient row selection, ReLU mask */
    NO_STAGE_GEMM_DW_L1 = 8,  /* layer-1 weight-gradient kernel (split partial products) */
    NO_STAGE_BWD_L1_REDUCE = 9,
    NO_STAGE_UPDATE = 10,     /* unused: the SGD step is fused into the gradient reductions */
    NO_STAGE_SAMPLE_ROWS_BOTTOM = 11, /* the bottom hop's sampling kernel alone (a part of NO_STAGE_SAMPLE) */
    NO_STAGE_COUNT = 12
};
int32_t no_model_profile(no_model_t m, int32_t enable);   /* enabling resets the accumulators */
/* Test aid for the error path of the single-pass scans (edge compaction and V^1 split in one launch): their blocks
 * wait, for at most spin_limit polls, on the status word of an earlier tile. spin_limit > 0 replaces the limit
 * (default 2^20; 0 restores it); withhold_first_tile != 0 makes tile 0 keep its word back, so that with two or more
 * tiles the wait of tile 1 is certain to expire. Every kernel still runs to its end; the call's results are wrong and
 * flagged (no_step_stats.scan_timeout, NO_ERR_TIMEOUT). Process-wide; for callers that test that path only. */
int32_t no_debug_scan_wait(int32_t spin_limit, int32_t withhold_first_tile);
/* h_total_ms[NO_STAGE_COUNT]: summed milliseconds per stage; *h_steps: steps accumulated. */
int32_t no_model_stage_ms(no_model_t m, double* h_total_ms, int32_t* h_steps);
const char* no_stage_name(int32_t stage);

#ifdef __cplusplus
}
#endif
#endif /* NEUTRONORCH_H_ */
