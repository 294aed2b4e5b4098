// fp32 matrix products for the dense UPDATE of Eq. 2 and its gradients, on the gfx950 matrix
// cores (v_mfma_f32_32x32x2_f32). Two shapes:
//   NN: C[M,N] = sum_p A_p[M,K_p] * B_p[K_p,N] (+ bias, ReLU, optional 1/len row scale); M is a
//       device scalar (rows past it are skipped); B may be given transposed; the rows of A_p may be
//       picked out of a larger table by an index (gather fused into the operand load).
//   TN: P[s][K',N] = A[rows of split s]^T * G[rows of split s]; the reduction length is a device
//       scalar; splits are summed in a fixed order afterwards (no float atomics).
#pragma once
#include "common.hpp"

namespace no {

struct GemmNNArgs {
    const float* A[2]; int64_t lda[2]; int a_align[2];
    const int32_t* a_rows[2];             // per problem: row m of the operand is row a_rows[m] of A (NULL: row m)
    const float* B[2]; int64_t ldb[2]; int b_align[2];
    int32_t K[2];
    float* C[2]; int64_t ldc[2];
    const int32_t* row_scale_indptr[2];   // per problem: multiply row m by 1/(indptr[m+1]-indptr[m]+row_scale_plus) (0 if that is 0)
    int32_t row_scale_plus;               // 1 when the row itself counts in the average (Eq. 1 over N_in(v) U {v})
    int32_t row_scale_rsqrt;              // 1: the factor is that count to the power -1/2 (symmetric normalisation)
    int32_t n_problems;                   // 1 or 2
    int32_t accumulate;                   // 1: both products are summed into C[0]; 0: independent problems (grid.z)
    const int32_t* d_M; int32_t M_cap; int32_t N;
    const float* bias; int32_t relu;
    // Scattered output of C[0] (layer 1 with reuse, Section 4.1.2): row m goes to row c_rows[m] (NULL: m); a row with
    // c_keep_rows[m] >= 0 is also stored as row c_keep_rows[m] of c_keep (same leading dimension) and
    // c_keep_stamp[that row] = stamp: the cache refresh of a recomputed hot vertex.
    const int32_t* c_rows;
    float* c_keep; const int32_t* c_keep_rows; int32_t* c_keep_stamp; int32_t stamp;
};

struct GemmTNArgs {
    const float* A[2]; int64_t lda[2]; int a_align[2];   // [R, Kp] row-major; two problems share G
    const float* G; int64_t ldg; int g_align;            // [R, N]
    float* P;                                            // partials [2][splits][Kp+1][N]; row Kp of product 0 = column sums of G
    int32_t Kp, N;
    const int32_t* d_R; int32_t R_cap; int32_t splits;   // splits: the most row slices (the partials' layout is sized for it)
    int32_t n_problems = 2;                              // 1: only A[0]
    int32_t rows_per_split = 0;                          // > 0: only ceil(R / rows_per_split) slices are used when that is fewer
};

// The number of row slices a split product over R rows really uses: the capacity-sized bound `splits`, cut down so that a
// slice keeps about rows_per_split rows (a function of R alone, so the summation order is the same in every run).
__host__ __device__ inline int32_t tn_used_splits(int32_t R, int32_t splits, int32_t rows_per_split) {
    if (rows_per_split <= 0) return splits;
    int32_t s = (R + rows_per_split - 1) / rows_per_split;
    if (s < 1) s = 1;
    return s < splits ? s : splits;
}

// Products with bf16 operands (a layer fed by a bf16 feature table): see gemm_bf16.hip.
struct GemmBf16NNArgs {
    const uint16_t* X; int64_t ldx; const int32_t* x_rows;   // first operand: bf16 rows; row m is row x_rows[m] of X (NULL: m)
    const float* Mn; int64_t ldm;                            // second operand: fp32 rows, rounded to bf16 on load
    const uint16_t* Wt[2]; int32_t Kpad;                     // the two weight matrices as bf16 [N][Kpad] (weights_to_bf16_t)
    int32_t K, N;
    float* C; int64_t ldc;
    const int32_t* d_M; int32_t M_cap;
    const float* bias; int32_t relu;
    const int32_t* c_rows; float* c_keep; const int32_t* c_keep_rows;   // as in GemmNNArgs
};
struct GemmBf16TNArgs {
    const uint16_t* X; int64_t ldx;                          // [R, Kp] bf16 (product 0)
    const float* Mn; int64_t ldm;                            // [R, Kp] fp32, rounded on load (product 1)
    const float* G; int64_t ldg;                             // [R, N] fp32, rounded on load
    float* P; int32_t Kp, N;                                 // partials in the layout of GemmTNArgs
    const int32_t* d_R; int32_t R_cap; int32_t splits; int32_t rows_per_split;
};
inline int32_t bf16_kpad(int32_t K) { return (K + 15) / 16 * 16; }
int32_t weights_to_bf16_t(const float* w, int32_t K, int32_t N, int32_t Kpad, uint16_t* out, hipStream_t st);
int32_t gemm_bf16_nn(const GemmBf16NNArgs& a, hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
int32_t gemm_bf16_tn_partials(const GemmBf16TNArgs& a, hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);

// Statistics of a training step, written by one extra block of the last gradient reduction of the step (they are
// nobody's input, so they do not get a launch of their own on the step's dependency chain): mean of the per-seed
// losses in a fixed order and the block sizes.
struct StatsJob {
    const float* row_loss = nullptr; int32_t n = 0;
    const int32_t* counts = nullptr; int32_t n_layers = 0; int32_t used_cache = 0;
    int32_t call_id = 0;                  // a flag word of `counts` is raised iff it holds this value
    int32_t feat_row_bytes = 0, emb_row_bytes = 0;
    no_step_stats* stats = nullptr;       // NULL: no job
};

// The reduction that follows a split product: sums the partials in split order into the three gradients; with
// lr != 0 also applies W <- W - lr * g.
struct ReduceArgs {
    const float* P; int32_t splits, Kp, N;
    float* g_self; float* g_neigh; float* g_bias;
    float lr; float* w_self; float* w_neigh; float* w_bias;
    int32_t n_problems;                                  // 2, or 1: only g_self and g_bias
    const int32_t* d_R = nullptr; int32_t R_cap = 0; int32_t rows_per_split = 0;   // as in the product: the slices it used
    // bf16 copies of the two matrices ([N][Kpad], weights_to_bf16_t's layout), rewritten with the updated values (or NULL)
    uint16_t* wt_self = nullptr; uint16_t* wt_neigh = nullptr; int32_t Kpad = 0;
};

// Weight-gradient work of several layers carried by one product launch and one reduction launch: the gradients of an
// upper layer are nobody's input within the step, so they need not sit on the step's chain of dependent launches
// between that layer's input gradient and the layer below. Job 0's blocks are dealt out first.
struct GradJobs {
    GemmTNArgs tn[NO_MAX_LAYERS]; ReduceArgs red[NO_MAX_LAYERS];
    int32_t n = 0;
    // side != NULL: where the bottom layer's products are of another kind (bf16 operands) and cannot carry the deferred
    // fp32 ones in their launch, those are launched together on this otherwise idle stream as soon as the last of them
    // has its inputs (behind `fork`, recorded before layer 2's own backward kernels; the reduction waits for `join`), so
    // they run beside layer 2's input gradient and the bottom layer's products. One fork: launching each job as soon as
    // its own layer had made its inputs measured no faster (every fork is an event on the backward chain).
    hipStream_t side = nullptr; hipEvent_t fork = nullptr; hipEvent_t join = nullptr;
    bool launched_beside = false;
};

// ev0 / ev1 (optional): events that take the product kernel's own start and end times
int32_t gemm_nn(const GemmNNArgs& a, bool b_transposed, hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
int32_t gemm_tn_partials(const GemmTNArgs* jobs, int32_t n_jobs, hipStream_t st, hipEvent_t ev0 = nullptr,
                         hipEvent_t ev1 = nullptr);
int32_t reduce_grads(const ReduceArgs* jobs, int32_t n_jobs, hipStream_t st, const StatsJob* stats_job = nullptr);

inline int ptr_align(const void* p, int64_t ld) {
    if ((((uintptr_t)p) & 15) == 0 && (ld & 3) == 0) return 4;
    if ((((uintptr_t)p) & 7) == 0 && (ld & 1) == 0) return 2;
    return 1;
}

}  // namespace no
