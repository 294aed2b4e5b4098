// no_sage_layer_fwd / no_sage_layer_bwd: one GraphSAGE-mean layer over a sampled block.
// Forward: mean over each destination's sampled row (Eq. 1, AGGREGATE = average), then the dense
// UPDATE of Eq. 2 on the matrix cores. Backward: the matching weight gradients and, for layers
// above the bottom one, the input gradient through the transposed block (segment sums in a fixed
// order, no float atomics). The bottom layer needs only the saved mean and the new embedding.
#include "layers.hpp"

#include <stdlib.h>
#include <mutex>

namespace no {

// ------------------------------------------------------------------------ row segment reduce

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

template <typename T, int VEC> struct RowVec;
template <> struct RowVec<float, 4> {
    static __device__ __forceinline__ void add(float (&acc)[4], const float* p) {
        float4 v = *reinterpret_cast<const float4*>(p);
        acc[0] += v.x; acc[1] += v.y; acc[2] += v.z; acc[3] += v.w;
    }
};
template <> struct RowVec<float, 2> {
    static __device__ __forceinline__ void add(float (&acc)[2], const float* p) {
        float2 v = *reinterpret_cast<const float2*>(p);
        acc[0] += v.x; acc[1] += v.y;
    }
};
template <> struct RowVec<float, 1> {
    static __device__ __forceinline__ void add(float (&acc)[1], const float* p) { acc[0] += p[0]; }
};
template <> struct RowVec<uint16_t, 8> {
    static __device__ __forceinline__ void add(float (&acc)[8], const uint16_t* p) {
        uint4 v = *reinterpret_cast<const uint4*>(p);
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] += __uint_as_float(w[i] << 16);
            acc[2 * i + 1] += __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};
template <> struct RowVec<uint16_t, 2> {
    static __device__ __forceinline__ void add(float (&acc)[2], const uint16_t* p) {
        uint32_t w = *reinterpret_cast<const uint32_t*>(p);
        acc[0] += __uint_as_float(w << 16);
        acc[1] += __uint_as_float(w & 0xffff0000u);
    }
};
template <> struct RowVec<uint16_t, 1> {
    static __device__ __forceinline__ void add(float (&acc)[1], const uint16_t* p) { acc[0] += bf16_to_f32(p[0]); }
};

// Per-source weights of the symmetric normalisation (Table 1: the adjacency matrix after symmetric normalisation, here
// of the sampled block with self loops): s_u = (c_u + [u < n_self])^-1/2, c_u = number of the block's edges that leave u.
__device__ __forceinline__ float source_weight(const SourceWeights& sw, int32_t u, int32_t n_self) {
    const int32_t c = (sw.is_ptr ? sw.cnt[u + 1] - sw.cnt[u] : sw.cnt[u]) + (u < n_self ? 1 : 0);
    return c > 0 ? 1.f / sqrtf((float)c) : 0.f;
}

// A vector unit as it comes from memory, and its accumulation in fp32 (the two halves of RowVec::add, for kernels that
// keep many units in flight in their memory form: 4 registers per bf16 unit of 8 instead of 8)
template <typename T, int VEC> struct RawUnit;
template <> struct RawUnit<float, 4> { using type = float4; };
template <> struct RawUnit<float, 2> { using type = float2; };
template <> struct RawUnit<float, 1> { using type = float; };
template <> struct RawUnit<uint16_t, 8> { using type = uint4; };
template <> struct RawUnit<uint16_t, 2> { using type = uint32_t; };
template <> struct RawUnit<uint16_t, 1> { using type = uint16_t; };
__device__ __forceinline__ void accum_unit(float (&acc)[4], const float4& v) { acc[0] += v.x; acc[1] += v.y; acc[2] += v.z; acc[3] += v.w; }
__device__ __forceinline__ void accum_unit(float (&acc)[2], const float2& v) { acc[0] += v.x; acc[1] += v.y; }
__device__ __forceinline__ void accum_unit(float (&acc)[1], const float& v) { acc[0] += v; }
__device__ __forceinline__ void accum_unit(float (&acc)[8], const uint4& v) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        acc[2 * i] += __uint_as_float(w[i] << 16);
        acc[2 * i + 1] += __uint_as_float(w[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void accum_unit(float (&acc)[2], const uint32_t& w) {
    acc[0] += __uint_as_float(w << 16);
    acc[1] += __uint_as_float(w & 0xffff0000u);
}
__device__ __forceinline__ void accum_unit(float (&acc)[1], const uint16_t& b) { acc[0] += bf16_to_f32(b); }

// out[row, :] = init + scale * sum_{p in [seg[row], seg[row+1])} w_p * src[idx[p], :]
//   MEAN: init = 0 and, by agg_mode: AGG_NEIGH_MEAN scale = 1/len (0 for an empty segment): forward aggregate of the
//         GraphSAGE-mean layer. The other modes add the row's own source row first (Eq. 1 over N_in(v) U {v}):
//         AGG_SELF_MEAN scale = 1/(len + 1); AGG_SELF_SUM scale = 1; AGG_SELF_SYM scale = (len + 1)^-1/2 and every term
//         (the self row included) is weighed by its source's s_u (WEIGHTED).
//   else: scale = 1, w = 1, init = out[row,:] for row < *d_n_init, else 0 (backward through the transpose); WEIGHTED: the
//         result is multiplied by s_row (the adjoint of the forward weights, row = source).
// A group of G = 2^g_log2 lanes owns one work item = (row, chunk of G vector units); a lane owns one
// vector unit of it. Rows wider than 64 units are split into several items handled by different
// wavefronts, so a wide row keeps many short independent load chains in flight instead of one long one;
// the items of a row are consecutive, which keeps the reads of a source row next to each other in time.
// Up to eight source rows are loaded before the first add; the adds stay in segment order.
template <typename T, int VEC, bool MEAN, bool WEIGHTED>
__global__ void __launch_bounds__(256) segment_rows_kernel(RowCopyJob job, const T* __restrict__ src, int64_t ld_src,
                                                           const int32_t* __restrict__ seg, const int32_t* __restrict__ idx,
                                                           const int32_t* d_n_rows, int32_t n_rows_cap,
                                                           const int32_t* d_n_init, float* __restrict__ out, int64_t ld_out,
                                                           int32_t units, int32_t g_log2, int32_t n_chunks,
                                                           const int32_t* __restrict__ self_idx, int32_t agg_mode,
                                                           const float* __restrict__ mask_h, const int32_t* __restrict__ out_rows,
                                                           float* __restrict__ masked_out, SourceWeights sw) {
    if (job.dst && blockIdx.x >= job.first_block) {
        // extra blocks of the launch: dst[dst_rows[i], :] = src[src_rows[i], :], one wavefront per row (rows that are
        // ready before this kernel's own output is, e.g. the cached layer-1 rows of the reused vertices)
        const int32_t nj = *job.d_n;
        const int64_t w0 = (((int64_t)(blockIdx.x - job.first_block)) * blockDim.x + threadIdx.x) >> 6;
        const int64_t nw = ((int64_t)(gridDim.x - job.first_block) * blockDim.x) >> 6;
        const int ln = (int)(threadIdx.x & 63);
        for (int64_t i = w0; i < nj; i += nw) {
            const float* s_ = job.src + (int64_t)job.src_rows[i] * job.dim;
            float* d_ = job.dst + (int64_t)job.dst_rows[i] * job.dim;
            for (int c = ln; c < job.dim; c += 64) d_[c] = s_[c];
        }
        return;
    }
    int32_t n = *d_n_rows;
    if (n > n_rows_cap) n = n_rows_cap;
    const int32_t n_init = (!MEAN && d_n_init) ? *d_n_init : 0;
    const int32_t lane = (int32_t)(threadIdx.x & 63);
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)(job.dst ? job.first_block : gridDim.x) * blockDim.x) >> 6;
    const int32_t items_per_pass = 64 >> g_log2;
    const int32_t sub = lane >> g_log2, u0 = lane & ((1 << g_log2) - 1);
    const int64_t n_items = (int64_t)n * n_chunks;
    const bool with_self = MEAN && agg_mode != AGG_NEIGH_MEAN;
    for (int64_t item = wave * items_per_pass + sub; item < n_items; item += n_waves * items_per_pass) {
        const int64_t row = item / n_chunks;
        const int32_t u = (int32_t)(item - row * n_chunks) * (1 << g_log2) + u0;
        if (u >= units) continue;
        const int32_t b = seg[row], e = seg[row + 1];
        float scale = MEAN ? (e > b ? 1.f / (float)(e - b) : 0.f) : 1.f;
        const T* col = src + (int64_t)u * VEC;
        float acc[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc[c] = 0.f;
        if (with_self) {
            // Eq. 1 over N_in(v) U {v}: the destination's own row (row `row` of src, or self_idx[row]) joins the aggregate
            RowVec<T, VEC>::add(acc, col + (int64_t)(self_idx ? self_idx[row] : (int32_t)row) * ld_src);
            if (WEIGHTED) {
                const float ws = source_weight(sw, (int32_t)row, n);
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] *= ws;
            }
            scale = agg_mode == AGG_SELF_MEAN ? 1.f / (float)(e - b + 1)
                  : agg_mode == AGG_SELF_SUM  ? 1.f : 1.f / sqrtf((float)(e - b + 1));
        }
        float* o = out + row * ld_out + (int64_t)u * VEC;
        if (!MEAN && row < n_init) {
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc[c] = o[c];
        }
        int32_t p = b;
        if (!MEAN && g_log2 == 6 && (units & 63) == 0) {      // (every lane of the wavefront is at work on this row)
            // Backward through the transpose, one wavefront per source row: a popular source has hundreds of entries, and
            // eight rows per round trip (each behind a round trip for its indices) would make that one row the kernel's
            // critical path. The wavefront reads 64 indices with one load and keeps 16 rows in flight; segments shorter
            // than 16 (nearly all of them) fall through to the rounds of 8, 4 and 1-3 below.
            for (; p + 16 <= e;) {
                const int32_t n = min(64, e - p);
                const int32_t mine = lane < n ? idx[p + lane] : 0;
                int32_t t = 0;
                for (; t + 16 <= n; t += 16) {
                    float a[16][VEC];
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const int32_t ix = __shfl(mine, t + j, 64);
#pragma unroll
                        for (int c = 0; c < VEC; ++c) a[j][c] = 0.f;
                        RowVec<T, VEC>::add(a[j], col + (int64_t)ix * ld_src);
                    }
#pragma unroll
                    for (int j = 0; j < 16; ++j)
#pragma unroll
                        for (int c = 0; c < VEC; ++c) acc[c] += a[j][c];
                }
                p += t;
            }
        }
        for (; p + 8 <= e; p += 8) {
            int32_t ix[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) ix[j] = idx[p + j];
            float wt[8];
            if (MEAN && WEIGHTED) {
#pragma unroll
                for (int j = 0; j < 8; ++j) wt[j] = source_weight(sw, sw.local ? sw.local[p + j] : ix[j], n);
            }
            float a[8][VEC];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) a[j][c] = 0.f;
                RowVec<T, VEC>::add(a[j], col + (int64_t)ix[j] * ld_src);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] += (MEAN && WEIGHTED) ? wt[j] * a[j][c] : a[j][c];
        }
        if (p + 4 <= e) {
            int32_t ix[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) ix[j] = idx[p + j];
            float wt[4];
            if (MEAN && WEIGHTED) {
#pragma unroll
                for (int j = 0; j < 4; ++j) wt[j] = source_weight(sw, sw.local ? sw.local[p + j] : ix[j], n);
            }
            float a[4][VEC];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) a[j][c] = 0.f;
                RowVec<T, VEC>::add(a[j], col + (int64_t)ix[j] * ld_src);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] += (MEAN && WEIGHTED) ? wt[j] * a[j][c] : a[j][c];
            p += 4;
        }
        if (p < e) {        // one to three rows left
            const int32_t i0 = idx[p], i1 = p + 1 < e ? idx[p + 1] : i0, i2 = p + 2 < e ? idx[p + 2] : i0;
            float w0 = 1.f, w1 = 1.f, w2 = 1.f;
            if (MEAN && WEIGHTED) {
                w0 = source_weight(sw, sw.local ? sw.local[p] : i0, n);
                w1 = p + 1 < e ? source_weight(sw, sw.local ? sw.local[p + 1] : i1, n) : 0.f;
                w2 = p + 2 < e ? source_weight(sw, sw.local ? sw.local[p + 2] : i2, n) : 0.f;
            }
            float a[3][VEC];
#pragma unroll
            for (int j = 0; j < 3; ++j)
#pragma unroll
                for (int c = 0; c < VEC; ++c) a[j][c] = 0.f;
            RowVec<T, VEC>::add(a[0], col + (int64_t)i0 * ld_src);
            if (p + 1 < e) RowVec<T, VEC>::add(a[1], col + (int64_t)i1 * ld_src);
            if (p + 2 < e) RowVec<T, VEC>::add(a[2], col + (int64_t)i2 * ld_src);
#pragma unroll
            for (int c = 0; c < VEC; ++c)
                acc[c] = (MEAN && WEIGHTED) ? ((acc[c] + w0 * a[0][c]) + w1 * a[1][c]) + w2 * a[2][c]
                                            : ((acc[c] + a[0][c]) + a[1][c]) + a[2][c];
        }
        if (!MEAN && WEIGHTED) {
            const float ws = source_weight(sw, (int32_t)row, n_init);
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc[c] *= ws;
        }
        if (!MEAN && masked_out) {
            // the consumer is the layer below: apply its ReLU decision (its output h, row `row`) and place the row
            // where that layer's gradient rows live (out_rows[row], -1 = the row takes no gradient)
            const int64_t r = out_rows ? (int64_t)out_rows[row] : row;
            if (r >= 0) {
                const float* hm = mask_h + row * ld_out + (int64_t)u * VEC;
                float* mo = masked_out + r * ld_out + (int64_t)u * VEC;
#pragma unroll
                for (int c = 0; c < VEC; ++c) mo[c] = hm[c] > 0.f ? acc[c] : 0.f;
            }
            continue;
        }
#pragma unroll
        for (int c = 0; c < VEC; ++c) o[c] = acc[c] * scale;
    }
}

template <typename T, int VEC, bool MEAN>
static void launch_segment(const T* src, int64_t ld_src, const int32_t* seg, const int32_t* idx, const int32_t* d_n,
                           int32_t n_cap, const int32_t* d_n_init, float* out, int64_t ld_out, int32_t dim, hipStream_t st,
                           const int32_t* self_idx = nullptr, int32_t agg_mode = AGG_NEIGH_MEAN, const float* mask_h = nullptr,
                           const int32_t* out_rows = nullptr, float* masked_out = nullptr, const RowCopyJob* copy = nullptr,
                           hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr, const SourceWeights* weights = nullptr) {
    const int32_t units = dim / VEC;
    int g_log2 = 0;
    while ((1 << g_log2) < units && g_log2 < 6) ++g_log2;
    const int32_t n_chunks = (int32_t)ceil_div(units, 1 << g_log2);
    int64_t waves = ceil_div((int64_t)n_cap * n_chunks, 64 >> g_log2);
    int64_t blocks = ceil_div(waves, 4);
    if (blocks > 256 * 64) blocks = 256 * 64;
    if (blocks < 1) blocks = 1;
    RowCopyJob job = copy ? *copy : RowCopyJob{};
    int64_t copy_blocks = 0;
    if (job.dst) {
        job.first_block = (uint32_t)blocks;
        copy_blocks = ceil_div(job.n_cap, 4);
        if (copy_blocks > 1024) copy_blocks = 1024;
        if (copy_blocks < 1) copy_blocks = 1;
    }
    const SourceWeights sw = weights ? *weights : SourceWeights{};
    if (sw.cnt)
        NO_LAUNCH_TIMED((segment_rows_kernel<T, VEC, MEAN, true>), dim3((unsigned)(blocks + copy_blocks)), dim3(256), st, ev0, ev1, job, src, ld_src, seg, idx, d_n,
                        n_cap, d_n_init, out, ld_out, units, g_log2, n_chunks, self_idx, agg_mode, mask_h, out_rows, masked_out, sw);
    else
        NO_LAUNCH_TIMED((segment_rows_kernel<T, VEC, MEAN, false>), dim3((unsigned)(blocks + copy_blocks)), dim3(256), st, ev0, ev1, job, src, ld_src, seg, idx, d_n,
                        n_cap, d_n_init, out, ld_out, units, g_log2, n_chunks, self_idx, agg_mode, mask_h, out_rows, masked_out, sw);
}

// The layer-1 aggregate straight from the sampler's fixed-stride slot array: row r's sampled neighbours are the
// entries pad[r*k .. r*k + k) in slot order (the order of the compacted row), -1 from the first unused slot on, and a
// first occurrence may carry the relabelling's mark (-2 - id in place of id). Reading the slots needs neither the row
// pointers nor the compacted index array, so a work item's chain of dependent memory round trips is "row count -> slots
// -> rows -> store" instead of "row count -> row pointers -> indices -> rows -> store": the kernel is bound by that chain
// (every wave handles one or two items), not by bytes in flight. NS (8 or 16) slots and their rows are in flight at a time. Same sums in the same order as segment_rows_kernel<MEAN>.
// agg_mode as there (no per-source weights here).
template <typename T, int VEC, int NS>
__global__ void __launch_bounds__(256) padded_rows_kernel(RowCopyJob job, const T* __restrict__ src, int64_t ld_src,
                                                          const int32_t* __restrict__ pad, int32_t k,
                                                          const int32_t* d_n_rows, int32_t n_rows_cap,
                                                          float* __restrict__ out, int64_t ld_out, int32_t units,
                                                          int32_t g_log2, int32_t n_chunks,
                                                          const int32_t* __restrict__ self_idx, int32_t agg_mode) {
    if (job.dst && blockIdx.x >= job.first_block) {
        const int32_t nj = *job.d_n;
        const int64_t w0 = (((int64_t)(blockIdx.x - job.first_block)) * blockDim.x + threadIdx.x) >> 6;
        const int64_t nw = ((int64_t)(gridDim.x - job.first_block) * blockDim.x) >> 6;
        const int ln = (int)(threadIdx.x & 63);
        for (int64_t i = w0; i < nj; i += nw) {
            const float* s_ = job.src + (int64_t)job.src_rows[i] * job.dim;
            float* d_ = job.dst + (int64_t)job.dst_rows[i] * job.dim;
            for (int c = ln; c < job.dim; c += 64) d_[c] = s_[c];
        }
        return;
    }
    using Raw = typename RawUnit<T, VEC>::type;
    int32_t n = *d_n_rows;
    if (n > n_rows_cap) n = n_rows_cap;
    const int32_t lane = (int32_t)(threadIdx.x & 63);
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)(job.dst ? job.first_block : gridDim.x) * blockDim.x) >> 6;
    const int32_t items_per_pass = 64 >> g_log2;
    const int32_t sub = lane >> g_log2, u0 = lane & ((1 << g_log2) - 1);
    const int64_t n_items = (int64_t)n * n_chunks;
    const bool with_self = agg_mode != AGG_NEIGH_MEAN;
    for (int64_t item = wave * items_per_pass + sub; item < n_items; item += n_waves * items_per_pass) {
        const int64_t row = item / n_chunks;
        const int32_t u = (int32_t)(item - row * n_chunks) * (1 << g_log2) + u0;
        if (u >= units) continue;
        const int32_t* slots = pad + row * k;
        int32_t e[NS];
#pragma unroll
        for (int j = 0; j < NS; ++j) e[j] = j < k ? slots[j] : -1;
        int32_t self_row = (int32_t)row;
        if (with_self && self_idx) self_row = self_idx[row];
        const T* col = src + (int64_t)u * VEC;
        float acc[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc[c] = 0.f;
        if (with_self) RowVec<T, VEC>::add(acc, col + (int64_t)self_row * ld_src);
        int32_t len = 0;
        for (int32_t j0 = 0;;) {
            Raw raw[NS];
#pragma unroll
            for (int j = 0; j < NS; ++j)
                if (e[j] != -1) raw[j] = *reinterpret_cast<const Raw*>(col + (int64_t)(e[j] <= -2 ? -2 - e[j] : e[j]) * ld_src);
#pragma unroll
            for (int j = 0; j < NS; ++j)
                if (e[j] != -1) {
                    accum_unit(acc, raw[j]);
                    ++len;
                }
            j0 += NS;
            if (j0 >= k || e[NS - 1] == -1) break;          // unused slots are at the end of a row
#pragma unroll
            for (int j = 0; j < NS; ++j) e[j] = j0 + j < k ? slots[j0 + j] : -1;
        }
        const float scale = agg_mode == AGG_NEIGH_MEAN ? (len > 0 ? 1.f / (float)len : 0.f)
                          : agg_mode == AGG_SELF_MEAN  ? 1.f / (float)(len + 1) : 1.f;
        float* o = out + row * ld_out + (int64_t)u * VEC;
#pragma unroll
        for (int c = 0; c < VEC; ++c) o[c] = acc[c] * scale;
    }
}

template <typename T, int VEC>
static void launch_padded(const T* src, int64_t ld_src, const int32_t* pad, int32_t k, const int32_t* d_n, int32_t n_cap,
                          float* out, int64_t ld_out, int32_t dim, hipStream_t st, const int32_t* self_idx, int32_t agg_mode,
                          const RowCopyJob* copy, hipEvent_t ev0, hipEvent_t ev1) {
    const int32_t units = dim / VEC;
    int g_log2 = 0;
    while ((1 << g_log2) < units && g_log2 < 6) ++g_log2;
    const int32_t n_chunks = (int32_t)ceil_div(units, 1 << g_log2);
    int64_t waves = ceil_div((int64_t)n_cap * n_chunks, 64 >> g_log2);
    int64_t blocks = ceil_div(waves, 4);
    if (blocks > 256 * 64) blocks = 256 * 64;
    if (blocks < 1) blocks = 1;
    RowCopyJob job = copy ? *copy : RowCopyJob{};
    int64_t copy_blocks = 0;
    if (job.dst) {
        job.first_block = (uint32_t)blocks;
        copy_blocks = ceil_div(job.n_cap, 4);
        if (copy_blocks > 1024) copy_blocks = 1024;
        if (copy_blocks < 1) copy_blocks = 1;
    }
    if (k <= 8)
        NO_LAUNCH_TIMED((padded_rows_kernel<T, VEC, 8>), dim3((unsigned)(blocks + copy_blocks)), dim3(256), st, ev0, ev1, job, src,
                        ld_src, pad, k, d_n, n_cap, out, ld_out, units, g_log2, n_chunks, self_idx, agg_mode);
    else
        NO_LAUNCH_TIMED((padded_rows_kernel<T, VEC, 16>), dim3((unsigned)(blocks + copy_blocks)), dim3(256), st, ev0, ev1, job, src,
                        ld_src, pad, k, d_n, n_cap, out, ld_out, units, g_log2, n_chunks, self_idx, agg_mode);
}

int32_t mean_aggregate(const void* x_src, no_dtype dt, int32_t dim, const int32_t* indptr, const int32_t* indices,
                       const int32_t* d_n_dst, int32_t n_dst_cap, float* mean, hipStream_t st, int32_t agg_mode,
                       const int32_t* self_idx, const RowCopyJob* copy, hipEvent_t ev0, hipEvent_t ev1,
                       const SourceWeights* weights, const PaddedSlots* padded) {
    if (n_dst_cap <= 0) return NO_OK;
    if (padded && padded->pad && !(weights && weights->cnt)) {
        // the rows are addressed through the sampler's slot array (global ids): two memory round trips fewer per item
        const int32_t* pad = padded->pad;
        const int32_t k = padded->k;
#define NO_PAD_FWD(T, V, ptr) \
    launch_padded<T, V>(ptr, dim, pad, k, d_n_dst, n_dst_cap, mean, dim, dim, st, self_idx, agg_mode, copy, ev0, ev1)
        if (dt == NO_F32) {
            const float* x = (const float*)x_src;
            const bool a16 = (((uintptr_t)x | (uintptr_t)mean) & 15) == 0, a8 = (((uintptr_t)x | (uintptr_t)mean) & 7) == 0;
            if (dim % 4 == 0 && a16) NO_PAD_FWD(float, 4, x);
            else if (dim % 2 == 0 && a8) NO_PAD_FWD(float, 2, x);
            else NO_PAD_FWD(float, 1, x);
        } else {
            const uint16_t* x = (const uint16_t*)x_src;
            if (dim % 8 == 0 && ((uintptr_t)x & 15) == 0 && ((uintptr_t)mean & 15) == 0) NO_PAD_FWD(uint16_t, 8, x);
            else if (dim % 2 == 0 && ((uintptr_t)x & 3) == 0) NO_PAD_FWD(uint16_t, 2, x);
            else NO_PAD_FWD(uint16_t, 1, x);
        }
#undef NO_PAD_FWD
        return launch_status("mean_aggregate (slot array)");
    }
#define NO_SEG_FWD(T, V, ptr) \
    launch_segment<T, V, true>(ptr, dim, indptr, indices, d_n_dst, n_dst_cap, nullptr, mean, dim, dim, st, self_idx, agg_mode, \
                               nullptr, nullptr, nullptr, copy, ev0, ev1, weights)
    if (dt == NO_F32) {
        const float* x = (const float*)x_src;
        const bool a16 = (((uintptr_t)x | (uintptr_t)mean) & 15) == 0, a8 = (((uintptr_t)x | (uintptr_t)mean) & 7) == 0;
        if (dim % 4 == 0 && a16) NO_SEG_FWD(float, 4, x);
        else if (dim % 2 == 0 && a8) NO_SEG_FWD(float, 2, x);
        else NO_SEG_FWD(float, 1, x);
    } else {
        const uint16_t* x = (const uint16_t*)x_src;
        if (dim % 8 == 0 && ((uintptr_t)x & 15) == 0 && ((uintptr_t)mean & 15) == 0) NO_SEG_FWD(uint16_t, 8, x);
        else if (dim % 2 == 0 && ((uintptr_t)x & 3) == 0) NO_SEG_FWD(uint16_t, 2, x);
        else NO_SEG_FWD(uint16_t, 1, x);
    }
#undef NO_SEG_FWD
    return launch_status("mean_aggregate");
}

// grad_x[u,:] = s_u * ((u < n_dst ? grad_x[u,:] : 0) + sum over transposed entries of u of gmean_scaled[csc_dst[p],:]),
// s_u = 1 unless source weights are given
int32_t transpose_aggregate(const float* gmean_scaled, int32_t dim, const int32_t* csc_indptr, const int32_t* csc_dst,
                            const int32_t* d_n_src, int32_t n_src_cap, const int32_t* d_n_dst, float* grad_x,
                            hipStream_t st, const float* mask_h, const int32_t* out_rows, float* masked_out,
                            const SourceWeights* weights) {
    if (n_src_cap <= 0) return NO_OK;
    const uintptr_t al = (uintptr_t)gmean_scaled | (uintptr_t)grad_x | (uintptr_t)mask_h | (uintptr_t)masked_out;
    const bool a16 = (al & 15) == 0, a8 = (al & 7) == 0;
#define NO_SEG_BWD(V) \
    launch_segment<float, V, false>(gmean_scaled, dim, csc_indptr, csc_dst, d_n_src, n_src_cap, d_n_dst, grad_x, dim, dim, st, \
                                    nullptr, AGG_NEIGH_MEAN, mask_h, out_rows, masked_out, nullptr, nullptr, nullptr, weights)
    if (dim % 4 == 0 && a16) NO_SEG_BWD(4);
    else if (dim % 2 == 0 && a8) NO_SEG_BWD(2);
    else NO_SEG_BWD(1);
#undef NO_SEG_BWD
    return launch_status("transpose_aggregate");
}

// ------------------------------------------------------------------------ small elementwise kernels

// gz[r,:] = grad_h[rows ? rows[r] : r, :] masked by [h[r,:] > 0] when relu: selects the rows that take a gradient
// (the computed vertices when hot rows were reused) and applies the activation's derivative in one pass.
__global__ void mask_rows_kernel(const float* __restrict__ grad_h, const int32_t* __restrict__ rows,
                                 const float* __restrict__ h, const int32_t* d_n, int32_t n_cap, int32_t dim, int32_t relu,
                                 float* __restrict__ gz) {
    int32_t n = *d_n;
    if (n > n_cap) n = n_cap;
    const int64_t total = (int64_t)n * dim;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < total; i += stride) {
        const int64_t r = i / dim, c = i - r * dim;
        const float g = rows ? grad_h[(int64_t)rows[r] * dim + c] : grad_h[i];
        gz[i] = (!relu || h[i] > 0.f) ? g : 0.f;
    }
}

__global__ void bf16_rows_to_f32_kernel(const uint16_t* __restrict__ x, const int32_t* d_n, int32_t n_cap, int32_t dim,
                                        float* __restrict__ out) {
    int32_t n = *d_n;
    if (n > n_cap) n = n_cap;
    const int64_t total = (int64_t)n * dim;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < total; i += stride) out[i] = bf16_to_f32(x[i]);
}

static inline unsigned ew_blocks(int64_t total) {
    int64_t b = ceil_div(total, 256 * 4);
    if (b > 256 * 16) b = 256 * 16;
    if (b < 1) b = 1;
    return (unsigned)b;
}

static int32_t bf16_rows_to_f32(const uint16_t* x, const int32_t* d_n, int32_t n_cap, int32_t dim, float* out, hipStream_t st) {
    if (n_cap <= 0 || dim <= 0) return NO_OK;
    hipLaunchKernelGGL(bf16_rows_to_f32_kernel, dim3(ew_blocks((int64_t)n_cap * dim)), dim3(256), 0, st, x, d_n, n_cap, dim, out);
    return launch_status("bf16_rows_to_f32");
}

// ------------------------------------------------------------------------ workspace layout

// Number of row slices of the weight-gradient product: enough 64x64 output tiles x slices to give every
// compute unit several blocks, bounded so that a slice keeps at least 64 rows of the capacity.
int32_t layer_splits(int32_t n_dst_cap, int32_t d_in, int32_t d_out) {
    const int64_t tiles = 2 * ceil_div(d_in + 1, 64) * ceil_div(d_out, 64);
    const int64_t target = 1600;      // blocks of the split product (measured: flat from 960 to 1600, slower beyond)
    int64_t s = ceil_div(target, tiles);
    const int64_t by_rows = ceil_div(n_dst_cap, 64);
    if (s > by_rows) s = by_rows;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    return (int32_t)s;
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

LayerWorkspace carve_workspace(void* ws, int32_t n_dst_cap, int32_t d_in, int32_t d_out) {
    LayerWorkspace w;
    w.splits = layer_splits(n_dst_cap, d_in, d_out);
    size_t off = 0;
    char* base = (char*)ws;
    w.gz = (float*)(base + off);        off += align256((size_t)n_dst_cap * d_out * 4);
    w.gmean = (float*)(base + off);     off += align256((size_t)n_dst_cap * d_in * 4);
    w.x_dst_f32 = (float*)(base + off); off += align256((size_t)n_dst_cap * d_in * 4);
    w.partials = (float*)(base + off);  off += align256((size_t)2 * w.splits * (d_in + 1) * d_out * 4);
    w.bytes = off;
    return w;
}

// ------------------------------------------------------------------------ layer forward / backward

int32_t sage_forward(const no_block_view& blk, const void* x_src, no_dtype dt, int32_t d_in, const float* w_self,
                     const float* w_neigh, const float* bias, int32_t d_out, int32_t relu, float* mean, float* h,
                     const LayerWorkspace& w, hipStream_t st, StageProfiler* prof, int agg_stage, int gemm_stage,
                     const void* agg_table, hipEvent_t wait_before_gemm, int32_t arch, const Layer1Reuse* reuse,
                     bool aggregate_done, const SourceWeights* weights, const PaddedSlots* padded,
                     const Bf16Products* bf) {
    // aggregate_done: `mean` (and the reused rows of H^1) were already written by an earlier launch of the same
    // aggregation (a batch prepared ahead); only the product runs
    // reuse: the output rows are scattered into H^1, recomputed hot rows also refresh the cache, and the reused
    // rows are copied in from the cache by extra blocks of the aggregation launch (they do not depend on this layer)
    const RowCopyJob* hits = (reuse && reuse->hits.dst) ? &reuse->hits : nullptr;
    auto scatter = [&](GemmNNArgs& a) {
        if (!reuse) return;
        a.c_rows = reuse->compute_pos;
        a.c_keep = reuse->emb; a.c_keep_rows = reuse->refresh_slot; a.c_keep_stamp = reuse->version; a.stamp = reuse->step;      // version == NULL: stamped by the split already
    };
    if (arch_is_gcn(arch)) {
        // Eq. 1 over N_in(v) U {v} (the destination's own row joins the aggregate: average, sum, or symmetric
        // normalisation with per-source weights), Eq. 2 with one matrix
        hipEvent_t e0 = nullptr, e1 = nullptr;
        if (prof && agg_stage >= 0) prof->kernel_pair(agg_stage, &e0, &e1);
        const int32_t mode = arch == NO_ARCH_GCN_SUM ? AGG_SELF_SUM : arch == NO_ARCH_GCN_SYM ? AGG_SELF_SYM : AGG_SELF_MEAN;
        if (arch == NO_ARCH_GCN_SYM && !(weights && weights->cnt)) {
            set_error("GCN-style layer with symmetric normalisation: the block has no per-source edge counts");
            return NO_ERR_INVALID_ARG;
        }
        NO_CHECK(mean_aggregate(agg_table ? agg_table : x_src, dt, d_in, blk.d_indptr, blk.d_indices, blk.d_n_dst,
                                blk.n_dst_cap, mean, st, mode, agg_table ? blk.d_src_global : nullptr, hits, e0, e1,
                                arch == NO_ARCH_GCN_SYM ? weights : nullptr, agg_table ? padded : nullptr));
        GemmNNArgs a{};
        a.A[0] = mean; a.lda[0] = d_in; a.a_align[0] = ptr_align(mean, d_in);
        a.B[0] = w_self; a.ldb[0] = d_out; a.b_align[0] = ptr_align(w_self, d_out);
        a.K[0] = d_in;
        a.C[0] = h; a.ldc[0] = d_out;
        a.n_problems = 1; a.accumulate = 1;
        a.d_M = blk.d_n_dst; a.M_cap = blk.n_dst_cap; a.N = d_out;
        a.bias = bias; a.relu = relu;
        scatter(a);
        e0 = e1 = nullptr;
        if (prof && gemm_stage >= 0) prof->kernel_pair(gemm_stage, &e0, &e1);
        return gemm_nn(a, false, st, e0, e1);
    }
    // agg_table != NULL: the rows to average are rows of that table addressed by blk.d_indices (global ids),
    // while x_src holds only the destination rows (fused gather + aggregate of the bottom layer). An fp32
    // table also feeds the self product directly, row m = table row src_global[m], so the forward pass
    // does not wait for the dense copy of the destination rows at all.
    const bool direct_self = agg_table && dt == NO_F32 && blk.d_src_global;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (prof && agg_stage >= 0 && !aggregate_done) prof->kernel_pair(agg_stage, &e0, &e1);
    if (!aggregate_done)
        NO_CHECK(mean_aggregate(agg_table ? agg_table : x_src, dt, d_in, blk.d_indptr, blk.d_indices, blk.d_n_dst,
                                blk.n_dst_cap, mean, st, AGG_NEIGH_MEAN, nullptr, hits, e0, e1, nullptr,
                                agg_table ? padded : nullptr));
    if (bf) {
        // bf16 operands on the matrix cores: the destinations' rows straight from the table (bf16 as stored), the mean
        // rounded on load, the weights from their bf16 copies; nothing to wait for on another stream
        GemmBf16NNArgs a{};
        a.X = bf->x_table; a.ldx = bf->ldx; a.x_rows = bf->x_rows;
        a.Mn = mean; a.ldm = d_in;
        a.Wt[0] = bf->wt_self; a.Wt[1] = bf->wt_neigh; a.Kpad = bf->Kpad;
        a.K = d_in; a.N = d_out;
        a.C = h; a.ldc = d_out;
        a.d_M = blk.d_n_dst; a.M_cap = blk.n_dst_cap;
        a.bias = bias; a.relu = relu;
        if (reuse) { a.c_rows = reuse->compute_pos; a.c_keep = reuse->emb; a.c_keep_rows = reuse->refresh_slot; }
        e0 = e1 = nullptr;
        if (prof && gemm_stage >= 0) prof->kernel_pair(gemm_stage, &e0, &e1);
        return gemm_bf16_nn(a, st, e0, e1);
    }
    if (wait_before_gemm && !direct_self)
        NO_HIP_CHECK(hipStreamWaitEvent(st, wait_before_gemm, 0));   // x_src rows come from another stream
    const float* x_dst = direct_self ? (const float*)agg_table : (const float*)x_src;
    if (dt == NO_BF16) {
        NO_CHECK(bf16_rows_to_f32((const uint16_t*)x_src, blk.d_n_dst, blk.n_dst_cap, d_in, w.x_dst_f32, st));
        x_dst = w.x_dst_f32;
    }
    GemmNNArgs a{};
    a.A[0] = x_dst; a.lda[0] = d_in; a.a_align[0] = ptr_align(x_dst, d_in);
    a.a_rows[0] = direct_self ? blk.d_src_global : nullptr;
    a.A[1] = mean;  a.lda[1] = d_in; a.a_align[1] = ptr_align(mean, d_in);
    a.B[0] = w_self;  a.ldb[0] = d_out; a.b_align[0] = ptr_align(w_self, d_out);
    a.B[1] = w_neigh; a.ldb[1] = d_out; a.b_align[1] = ptr_align(w_neigh, d_out);
    a.K[0] = a.K[1] = d_in;
    a.C[0] = h; a.ldc[0] = d_out;
    a.n_problems = 2; a.accumulate = 1;
    a.d_M = blk.d_n_dst; a.M_cap = blk.n_dst_cap; a.N = d_out;
    a.bias = bias; a.relu = relu;
    scatter(a);
    e0 = e1 = nullptr;
    if (prof && gemm_stage >= 0) prof->kernel_pair(gemm_stage, &e0, &e1);
    return gemm_nn(a, false, st, e0, e1);
}

int32_t sage_backward(const no_block_view& blk, const void* x_src, no_dtype dt, int32_t d_in, const float* mean,
                      const float* h, const float* grad_h, const float* w_self, const float* w_neigh, int32_t d_out,
                      int32_t relu, float* gw_self, float* gw_neigh, float* gbias, float* grad_x_src,
                      const LayerWorkspace& w, hipStream_t st, StageProfiler* prof, int prep_stage, int dw_stage,
                      int reduce_stage, int dx_stage, const int32_t* grad_rows, float lr, float* w_self_rw,
                      float* w_neigh_rw, float* bias_rw, int32_t arch, const StatsJob* stats_job, const float* gz_in,
                      const BelowLayer* below, GradJobs* pending, bool defer, const SourceWeights* weights,
                      const Bf16Products* bf) {
    const bool gcn = arch_is_gcn(arch);
    if (arch == NO_ARCH_GCN_SYM && grad_x_src && !(weights && weights->cnt)) {
        set_error("GCN-style layer with symmetric normalisation: the block has no per-source edge counts");
        return NO_ERR_INVALID_ARG;
    }
    const int32_t n_cap = blk.n_dst_cap;
    if (prof && prep_stage >= 0) prof->begin(prep_stage);
    // gz_in: the layer above already applied this layer's ReLU decision and row selection while it wrote the gradient
    const float* gz = gz_in ? gz_in : grad_h;
    if (!gz_in && (relu || grad_rows)) {
        hipLaunchKernelGGL(mask_rows_kernel, dim3(ew_blocks((int64_t)n_cap * d_out)), dim3(256), 0, st, grad_h, grad_rows, h,
                           blk.d_n_dst, n_cap, d_out, relu, w.gz);
        gz = w.gz;
    }
    const float* x_dst = (const float*)x_src;
    if (dt == NO_BF16 && !gcn && !bf) {
        NO_CHECK(bf16_rows_to_f32((const uint16_t*)x_src, blk.d_n_dst, n_cap, d_in, w.x_dst_f32, st));
        x_dst = w.x_dst_f32;
    }
    if (prof && prep_stage >= 0) prof->end();
    if (grad_x_src) {
        // uses the pre-update weights, so it runs before the reduce that may apply the SGD step:
        // gz W_self^T -> rows [0, n_dst) of grad_x; (gz W_neigh^T) / len(row) -> gmean; then the transpose adds
        if (prof && dx_stage >= 0) prof->begin(dx_stage);
        GemmNNArgs a{};
        a.A[0] = a.A[1] = gz; a.lda[0] = a.lda[1] = d_out; a.a_align[0] = a.a_align[1] = ptr_align(gz, d_out);
        a.B[0] = w_self;  a.ldb[0] = d_out; a.b_align[0] = ptr_align(w_self, d_out);
        a.B[1] = w_neigh; a.ldb[1] = d_out; a.b_align[1] = ptr_align(w_neigh, d_out);
        a.K[0] = a.K[1] = d_out;
        a.C[0] = grad_x_src; a.ldc[0] = d_in;
        a.C[1] = w.gmean;    a.ldc[1] = d_in;
        a.row_scale_indptr[1] = blk.d_indptr;
        if (gcn) {
            // one matrix: gz W^T / (len + 1) is both the destination's own share (rows [0, n_dst) of grad_x) and
            // what the transpose spreads over the sampled sources
            // (sum: no factor; symmetric normalisation: (len + 1)^-1/2 here, the source's own factor after the transpose)
            a.B[1] = w_self; a.b_align[1] = a.b_align[0];
            a.row_scale_indptr[0] = blk.d_indptr;
            a.row_scale_plus = 1;
            a.row_scale_rsqrt = arch == NO_ARCH_GCN_SYM ? 1 : 0;
            if (arch == NO_ARCH_GCN_SUM) a.row_scale_indptr[0] = a.row_scale_indptr[1] = nullptr;
        }
        a.n_problems = 2; a.accumulate = 0;
        a.d_M = blk.d_n_dst; a.M_cap = n_cap; a.N = d_in;
        NO_CHECK(gemm_nn(a, true, st));
        NO_CHECK(transpose_aggregate(w.gmean, d_in, blk.d_csc_indptr, blk.d_csc_dst, blk.d_n_src, blk.n_src_cap,
                                     blk.d_n_dst, grad_x_src, st, below ? below->h : nullptr, below ? below->out_rows : nullptr,
                                     below ? below->gz_out : nullptr, arch == NO_ARCH_GCN_SYM ? weights : nullptr));
        if (prof && dx_stage >= 0) prof->end();
    }
    // weight gradients x_dst^T gz, mean^T gz and the bias gradient (column sums of gz, carried by a virtual
    // column of ones in the first product), split over rows and summed in split order
    GemmTNArgs t{};
    t.A[0] = x_dst; t.lda[0] = d_in; t.a_align[0] = ptr_align(x_dst, d_in);
    t.A[1] = mean;  t.lda[1] = d_in; t.a_align[1] = ptr_align(mean, d_in);
    if (gcn) { t.A[0] = mean; t.a_align[0] = t.a_align[1]; t.n_problems = 1; }
    t.G = gz; t.ldg = d_out; t.g_align = ptr_align(gz, d_out);
    t.P = w.partials; t.Kp = d_in; t.N = d_out;
    t.d_R = blk.d_n_dst; t.R_cap = n_cap; t.splits = w.splits;
    // Batches that fill a fraction of the capacity use fewer slices than the capacity-sized bound: a slice keeps at least
    // this many rows. Measured on a batch of 24 K rows (bound: 64 slices): the product takes the same time from 64 down
    // to 93 slices' worth of rows (256 per slice) and 10 % longer at 384 and above (too few blocks), while the reduction
    // after it reads fewer partial tiles.
    t.rows_per_split = 256;
    ReduceArgs r{w.partials, w.splits, d_in, d_out, gw_self, gw_neigh, gbias, lr, w_self_rw, w_neigh_rw, bias_rw, gcn ? 1 : 2};
    r.d_R = t.d_R; r.R_cap = t.R_cap; r.rows_per_split = t.rows_per_split;
    if (bf) { r.wt_self = bf->wt_self; r.wt_neigh = bf->wt_neigh; r.Kpad = bf->Kpad; }
    if (pending && defer) {
        // an upper layer inside a step: its product and reduction ride on the bottom layer's launches
        if (pending->n >= NO_MAX_LAYERS) { set_error("sage_backward: too many deferred layers"); return NO_ERR_CAPACITY; }
        pending->tn[pending->n] = t;
        pending->red[pending->n] = r;
        ++pending->n;
        return launch_status("sage_backward");
    }
    GemmTNArgs tj[NO_MAX_LAYERS];
    ReduceArgs rj[NO_MAX_LAYERS];
    int32_t n_jobs = 0, n_tn = 0;
    rj[n_jobs++] = r;
    if (!bf) tj[n_tn++] = t;
    for (int32_t i = 0; pending && i < pending->n && n_jobs < NO_MAX_LAYERS; ++i) { tj[n_tn++] = pending->tn[i]; rj[n_jobs++] = pending->red[i]; }
    const bool beside = pending && pending->launched_beside;      // the deferred products already run on the side stream
    if (beside) n_tn = bf ? 0 : 1;
    if (pending) { pending->n = 0; pending->launched_beside = false; }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (bf) {
        // this layer's two products take bf16 operands (their own launch); the deferred fp32 products of the layers
        // above go first
        if (n_tn > 0) {
            if (prof && prep_stage >= 0) prof->begin(prep_stage);
            NO_CHECK(gemm_tn_partials(tj, n_tn, st, nullptr, nullptr));
            if (prof && prep_stage >= 0) prof->end();
        }
        GemmBf16TNArgs b{};
        b.X = bf->x_dense; b.ldx = d_in; b.Mn = mean; b.ldm = d_in; b.G = gz; b.ldg = d_out;
        b.P = w.partials; b.Kp = d_in; b.N = d_out;
        b.d_R = t.d_R; b.R_cap = t.R_cap; b.splits = t.splits; b.rows_per_split = t.rows_per_split;
        if (prof && dw_stage >= 0) prof->kernel_pair(dw_stage, &e0, &e1);
        NO_CHECK(gemm_bf16_tn_partials(b, st, e0, e1));
    } else {
        if (prof && dw_stage >= 0) prof->kernel_pair(dw_stage, &e0, &e1);
        NO_CHECK(gemm_tn_partials(tj, n_tn, st, e0, e1));
    }
    if (beside) NO_HIP_CHECK(hipStreamWaitEvent(st, pending->join, 0));      // only the reduction needs the products beside
    if (prof && reduce_stage >= 0) prof->begin(reduce_stage);
    NO_CHECK(reduce_grads(rj, n_jobs, st, stats_job));
    if (prof && reduce_stage >= 0) prof->end();
    return launch_status("sage_backward");
}

}  // namespace no

using namespace no;

static int32_t check_layer_args(const no_block_view* blk, const void* x, no_dtype dt, int32_t d_in, int32_t d_out,
                                const char* who) {
    NO_REQUIRE(blk && x, NO_ERR_INVALID_ARG, "%s: NULL argument", who);
    NO_REQUIRE(dt == NO_F32 || dt == NO_BF16, NO_ERR_INVALID_ARG, "%s: unknown dtype", who);
    NO_REQUIRE(d_in >= 1 && d_out >= 1, NO_ERR_INVALID_ARG, "%s: dimensions must be positive", who);
    NO_REQUIRE(blk->n_dst_cap >= 1 && blk->n_src_cap >= blk->n_dst_cap, NO_ERR_INVALID_ARG, "%s: bad block capacities", who);
    NO_REQUIRE(blk->d_n_dst && blk->d_indptr && blk->d_indices, NO_ERR_INVALID_ARG, "%s: block view lacks CSR arrays", who);
    return NO_OK;
}

extern "C" size_t no_sage_layer_ws_bytes(int32_t n_dst_cap, int32_t n_src_cap, int32_t d_in, int32_t d_out) {
    (void)n_src_cap;
    if (n_dst_cap < 1 || d_in < 1 || d_out < 1) return 0;
    return carve_workspace(nullptr, n_dst_cap, d_in, d_out).bytes;
}

extern "C" int32_t no_sage_layer_fwd(const no_block_view* blk, const void* d_x_src, no_dtype dt_x, int32_t d_in,
                                     const float* d_w_self, const float* d_w_neigh, const float* d_bias, int32_t d_out,
                                     int32_t relu, float* d_mean, float* d_h, void* d_ws, size_t ws_bytes, void* stream) {
    clear_error();
    NO_CHECK(check_layer_args(blk, d_x_src, dt_x, d_in, d_out, "no_sage_layer_fwd"));
    NO_REQUIRE(d_w_self && d_w_neigh && d_bias && d_mean && d_h, NO_ERR_INVALID_ARG, "no_sage_layer_fwd: NULL argument");
    LayerWorkspace w = carve_workspace(d_ws, blk->n_dst_cap, d_in, d_out);
    NO_REQUIRE(d_ws != nullptr && ws_bytes >= w.bytes, NO_ERR_CAPACITY, "no_sage_layer_fwd: workspace too small (%zu < %zu)",
               ws_bytes, w.bytes);
    return sage_forward(*blk, d_x_src, dt_x, d_in, d_w_self, d_w_neigh, d_bias, d_out, relu, d_mean, d_h, w,
                        (hipStream_t)stream);
}

extern "C" int32_t no_sage_layer_bwd(const no_block_view* blk, const void* d_x_src, no_dtype dt_x, int32_t d_in,
                                     const float* d_mean, const float* d_h, const float* d_grad_h, const float* d_w_self,
                                     const float* d_w_neigh, int32_t d_out, int32_t relu, float* d_gw_self,
                                     float* d_gw_neigh, float* d_gbias, float* d_grad_x_src, void* d_ws, size_t ws_bytes,
                                     void* stream) {
    clear_error();
    NO_CHECK(check_layer_args(blk, d_x_src, dt_x, d_in, d_out, "no_sage_layer_bwd"));
    NO_REQUIRE(d_mean && d_h && d_grad_h && d_w_self && d_w_neigh && d_gw_self && d_gw_neigh && d_gbias, NO_ERR_INVALID_ARG,
               "no_sage_layer_bwd: NULL argument");
    NO_REQUIRE(!d_grad_x_src || (blk->d_csc_indptr && blk->d_csc_dst && blk->d_n_src), NO_ERR_INVALID_ARG,
               "no_sage_layer_bwd: input gradient requested but the block has no transpose");
    LayerWorkspace w = carve_workspace(d_ws, blk->n_dst_cap, d_in, d_out);
    NO_REQUIRE(d_ws != nullptr && ws_bytes >= w.bytes, NO_ERR_CAPACITY, "no_sage_layer_bwd: workspace too small (%zu < %zu)",
               ws_bytes, w.bytes);
    return sage_backward(*blk, d_x_src, dt_x, d_in, d_mean, d_h, d_grad_h, d_w_self, d_w_neigh, d_out, relu, d_gw_self,
                         d_gw_neigh, d_gbias, d_grad_x_src, w, (hipStream_t)stream);
}

// ------------------------------------------------------------------------ backward without any allocation
//
// The workspace of no_sage_layer_bwd (masked gradient, mean gradient, fp32 copy of bf16 rows, split partial products)
// held in a file-scope device array instead of a caller's buffer, for callers that cannot allocate or pass one.
constexpr size_t kStaticWsBytes = NO_LAYER_STATIC_WS_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];

namespace {
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {nullptr};

// The address of this device's copy of `scratch` (every GPU holds its own copy at its own address; the array's name
// is only a host-side handle for the lookup and is never passed to a kernel or a memory call).
static int32_t static_workspace(void** out) {
    int dev = -1;
    NO_HIP_CHECK(hipGetDevice(&dev));
    NO_REQUIRE(dev >= 0 && dev < kMaxDevices, NO_ERR_UNSUPPORTED, "static workspace: device index %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        NO_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        NO_REQUIRE(p != nullptr, NO_ERR_HIP, "static workspace: no device address for the scratch array");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return NO_OK;
}
}  // namespace

extern "C" int32_t no_sage_layer_bwd_static(const no_block_view* blk, const void* d_x_src, no_dtype dt_x, int32_t d_in,
                                            const float* d_mean, const float* d_h, const float* d_grad_h,
                                            const float* d_w_self, const float* d_w_neigh, int32_t d_out, int32_t relu,
                                            float* d_gw_self, float* d_gw_neigh, float* d_gbias, float* d_grad_x_src,
                                            void* stream) {
    clear_error();
    NO_CHECK(check_layer_args(blk, d_x_src, dt_x, d_in, d_out, "no_sage_layer_bwd_static"));
    NO_REQUIRE(d_mean && d_h && d_grad_h && d_w_self && d_w_neigh && d_gw_self && d_gw_neigh && d_gbias, NO_ERR_INVALID_ARG,
               "no_sage_layer_bwd_static: NULL argument");
    NO_REQUIRE(!d_grad_x_src || (blk->d_csc_indptr && blk->d_csc_dst && blk->d_n_src), NO_ERR_INVALID_ARG,
               "no_sage_layer_bwd_static: input gradient requested but the block has no transpose");
    const size_t need = carve_workspace(nullptr, blk->n_dst_cap, d_in, d_out).bytes;
    NO_REQUIRE(need <= kStaticWsBytes, NO_ERR_CAPACITY,
               "no_sage_layer_bwd_static: the layer needs %zu bytes of workspace, the static one holds %zu", need,
               kStaticWsBytes);
    void* ws = nullptr;
    NO_CHECK(static_workspace(&ws));
    // (every part of the workspace is written by this call's kernels before it is read: nothing has to start at zero)
    LayerWorkspace w = carve_workspace(ws, blk->n_dst_cap, d_in, d_out);
    return sage_backward(*blk, d_x_src, dt_x, d_in, d_mean, d_h, d_grad_h, d_w_self, d_w_neigh, d_out, relu, d_gw_self,
                         d_gw_neigh, d_gbias, d_grad_x_src, w, (hipStream_t)stream);
}

static int32_t check_gcn_form(const no_block_view* blk, no_arch form, SourceWeights* sw, const char* who) {
    NO_REQUIRE(form == NO_ARCH_GCN || form == NO_ARCH_GCN_SUM || form == NO_ARCH_GCN_SYM, NO_ERR_INVALID_ARG,
               "%s: form must be one of the GCN-style layer forms", who);
    *sw = SourceWeights{};
    if (form == NO_ARCH_GCN_SYM) {
        // the column sums of the block's adjacency are the lengths of the transpose's columns
        NO_REQUIRE(blk->d_csc_indptr != nullptr, NO_ERR_INVALID_ARG,
                   "%s: symmetric normalisation needs the block's transpose (its column lengths)", who);
        sw->cnt = blk->d_csc_indptr;
        sw->is_ptr = 1;
    }
    return NO_OK;
}

extern "C" int32_t no_gcn_layer_fwd(const no_block_view* blk, no_arch form, const void* d_x_src, no_dtype dt_x, int32_t d_in,
                                    const float* d_w, const float* d_bias, int32_t d_out, int32_t relu, float* d_agg,
                                    float* d_h, void* d_ws, size_t ws_bytes, void* stream) {
    clear_error();
    NO_CHECK(check_layer_args(blk, d_x_src, dt_x, d_in, d_out, "no_gcn_layer_fwd"));
    SourceWeights sw;
    NO_CHECK(check_gcn_form(blk, form, &sw, "no_gcn_layer_fwd"));
    NO_REQUIRE(d_w && d_bias && d_agg && d_h, NO_ERR_INVALID_ARG, "no_gcn_layer_fwd: NULL argument");
    LayerWorkspace w = carve_workspace(d_ws, blk->n_dst_cap, d_in, d_out);
    NO_REQUIRE(d_ws != nullptr && ws_bytes >= w.bytes, NO_ERR_CAPACITY, "no_gcn_layer_fwd: workspace too small (%zu < %zu)",
               ws_bytes, w.bytes);
    return sage_forward(*blk, d_x_src, dt_x, d_in, d_w, nullptr, d_bias, d_out, relu, d_agg, d_h, w, (hipStream_t)stream,
                        nullptr, -1, -1, nullptr, nullptr, form, nullptr, false, &sw);
}

extern "C" int32_t no_gcn_layer_bwd(const no_block_view* blk, no_arch form, int32_t d_in, const float* d_agg, const float* d_h,
                                    const float* d_grad_h, const float* d_w, int32_t d_out, int32_t relu, float* d_gw,
                                    float* d_gbias, float* d_grad_x_src, void* d_ws, size_t ws_bytes, void* stream) {
    clear_error();
    NO_CHECK(check_layer_args(blk, d_agg, NO_F32, d_in, d_out, "no_gcn_layer_bwd"));
    SourceWeights sw;
    NO_CHECK(check_gcn_form(blk, d_grad_x_src ? form : (form == NO_ARCH_GCN_SYM ? NO_ARCH_GCN : form), &sw, "no_gcn_layer_bwd"));
    NO_REQUIRE(d_h && d_grad_h && d_w && d_gw && d_gbias, NO_ERR_INVALID_ARG, "no_gcn_layer_bwd: NULL argument");
    NO_REQUIRE(!d_grad_x_src || (blk->d_csc_indptr && blk->d_csc_dst && blk->d_n_src), NO_ERR_INVALID_ARG,
               "no_gcn_layer_bwd: input gradient requested but the block has no transpose");
    LayerWorkspace w = carve_workspace(d_ws, blk->n_dst_cap, d_in, d_out);
    NO_REQUIRE(d_ws != nullptr && ws_bytes >= w.bytes, NO_ERR_CAPACITY, "no_gcn_layer_bwd: workspace too small (%zu < %zu)",
               ws_bytes, w.bytes);
    return sage_backward(*blk, d_agg, NO_F32, d_in, d_agg, d_h, d_grad_h, d_w, nullptr, d_out, relu, d_gw, nullptr, d_gbias,
                         d_grad_x_src, w, (hipStream_t)stream, nullptr, -1, -1, -1, -1, nullptr, 0.f, nullptr, nullptr, nullptr,
                         form, nullptr, nullptr, nullptr, nullptr, false, &sw);
}
