// no_build_csr: COO -> in-neighbour CSR on the device (input G(V,E) of Algorithm 1; rows are
// the N_in(v) of Eq. 1). Two stable radix sorts (by src, then by dst) give rows ascending by
// src with duplicates kept; the row pointers come from a degree histogram and a prefix sum.
#include "primitives.hpp"
#include "handles.hpp"

namespace no {

__global__ void csr_check_and_count_kernel(const int32_t* src, const int32_t* dst, int64_t n_edges, int64_t n_vertices,
                                           int32_t* degree, int32_t* bad) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n_edges; i += stride) {
        int32_t s = src[i], d = dst[i];
        if (s < 0 || s >= n_vertices || d < 0 || d >= n_vertices) { *bad = 1; continue; }
        atomicAdd(&degree[d], 1);     // integer count: order independent
    }
}

// 64-bit ids on input (NO_CSR_IDS_64): narrowed to the library's 32-bit ids; an id outside [0, V) raises *bad (and V < 2^31)
__global__ void narrow_ids_kernel(const int64_t* in, uint32_t* out, int64_t n, int64_t n_vertices, int32_t* bad) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int64_t v = in[i];
        if (v < 0 || v >= n_vertices) { *bad = 1; out[i] = 0u; } else out[i] = (uint32_t)v;
    }
}

// NO_CSR_DEDUP: entry i of the (dst, src)-sorted edge list is kept iff it differs from entry i - 1
__global__ void mark_first_of_run_kernel(const uint32_t* dst, const uint32_t* src, int64_t n, int32_t* keep) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) keep[i] = (i == 0 || dst[i] != dst[i - 1] || src[i] != src[i - 1]) ? 1 : 0;
}

__global__ void compact_edges_kernel(const uint32_t* dst, const uint32_t* src, const int32_t* keep, const int32_t* pos,
                                     int64_t n, int32_t* col_out, int32_t* degree) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride)
        if (keep[i]) {
            col_out[pos[i]] = (int32_t)src[i];
            atomicAdd(&degree[dst[i]], 1);     // integer count: order independent
        }
}

__global__ void narrow_rowptr_kernel(const int64_t* in, int32_t* out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) out[i] = (int32_t)in[i];
}

}  // namespace no

using namespace no;

extern "C" int32_t no_build_csr(const void* src, const void* dst, int64_t n_edges_in, int64_t n_vertices,
                                int32_t rowptr_bits, uint32_t flags, void* stream, no_graph_t* out) {
    clear_error();
    NO_REQUIRE(out != nullptr, NO_ERR_INVALID_ARG, "no_build_csr: out is NULL");
    *out = nullptr;
    NO_REQUIRE(n_vertices > 0 && n_edges_in >= 0, NO_ERR_INVALID_ARG, "no_build_csr: need n_vertices > 0, n_edges >= 0");
    NO_REQUIRE(n_edges_in == 0 || (src && dst), NO_ERR_INVALID_ARG, "no_build_csr: src/dst is NULL");
    NO_REQUIRE(rowptr_bits == 32 || rowptr_bits == 64, NO_ERR_INVALID_ARG, "no_build_csr: rowptr_bits must be 32 or 64");
    NO_REQUIRE((flags & ~(uint32_t)(NO_CSR_INPUT_ON_DEVICE | NO_CSR_IDS_64 | NO_CSR_SYMMETRISE | NO_CSR_DEDUP)) == 0,
               NO_ERR_INVALID_ARG, "no_build_csr: unknown flag");
    NO_REQUIRE(n_vertices < (1ll << 31), NO_ERR_OVERFLOW, "no_build_csr: vertex ids are int32 inside the library, V must be < 2^31");
    const bool symmetrise = (flags & NO_CSR_SYMMETRISE) != 0, dedup = (flags & NO_CSR_DEDUP) != 0, ids64 = (flags & NO_CSR_IDS_64) != 0;
    const int64_t n_edges = symmetrise ? 2 * n_edges_in : n_edges_in;       // before duplicates are dropped
    NO_REQUIRE(rowptr_bits == 64 || n_edges < (1ll << 31), NO_ERR_OVERFLOW,
               "no_build_csr: 32-bit row pointers need fewer than 2^31 edges");
    NO_REQUIRE(n_edges < (1ll << 32) - 1, NO_ERR_UNSUPPORTED, "no_build_csr: at most 2^32-2 edges");
    NO_REQUIRE(!dedup || n_edges < (1ll << 31), NO_ERR_UNSUPPORTED, "no_build_csr: NO_CSR_DEDUP takes fewer than 2^31 edges");
    hipStream_t st = (hipStream_t)stream;

    no_graph_s* g = new no_graph_s();
    g->n_vertices = n_vertices;
    g->n_edges = n_edges;
    g->rowptr_bits = rowptr_bits;
    struct Guard { no_graph_s* g; ~Guard() { if (g) { g->release(); delete g; } } } guard{g};

    const size_t ne = (size_t)n_edges, ne_in = (size_t)n_edges_in;
    DevBuf<uint32_t> a_k, a_v, b_k, b_v, c_k, c_v;
    DevBuf<int32_t> degree, bad;
    DevBuf<char> ws;
    DevBuf<int64_t> rowptr64, wide;
    struct Tmp { DevBuf<uint32_t>*u[6]; DevBuf<int32_t>* i[2]; DevBuf<char>* w; DevBuf<int64_t>* r[2];
                 ~Tmp() { for (auto p : u) p->release(); for (auto p : i) p->release(); w->release(); for (auto p : r) p->release(); } }
        tmp{{&a_k, &a_v, &b_k, &b_v, &c_k, &c_v}, {&degree, &bad}, &ws, {&rowptr64, &wide}};

    NO_CHECK(a_k.alloc(ne)); NO_CHECK(a_v.alloc(ne));
    NO_CHECK(b_k.alloc(ne)); NO_CHECK(b_v.alloc(ne));
    NO_CHECK(c_k.alloc(ne)); NO_CHECK(c_v.alloc(ne));
    NO_CHECK(degree.alloc((size_t)n_vertices)); NO_CHECK(bad.alloc(1));
    size_t ws_bytes = radix_ws_bytes(n_edges);
    size_t sb = scan_ws_bytes(n_vertices > n_edges ? n_vertices : n_edges);
    if (sb > ws_bytes) ws_bytes = sb;
    NO_CHECK(ws.alloc(ws_bytes));
    NO_CHECK(rowptr64.alloc((size_t)n_vertices + 1));
    NO_CHECK(g->col.alloc(ne));
    NO_CHECK(fill_i32(degree.p, 0, n_vertices, st));
    NO_CHECK(fill_i32(bad.p, 0, 1, st));

    // a_k = src, a_v = dst (32-bit ids)
    const hipMemcpyKind kind = (flags & NO_CSR_INPUT_ON_DEVICE) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    auto grid_for = [](int64_t n) { int64_t b = ceil_div(n, 256 * 4); if (b > 65536) b = 65536; if (b < 1) b = 1; return dim3((unsigned)b); };
    if (n_edges_in > 0) {
        if (ids64) {
            NO_CHECK(wide.alloc(ne_in));
            for (int which = 0; which < 2; ++which) {
                NO_HIP_CHECK(hipMemcpyAsync(wide.p, which == 0 ? src : dst, ne_in * 8, kind, st));
                hipLaunchKernelGGL(narrow_ids_kernel, grid_for(n_edges_in), dim3(256), 0, st, (const int64_t*)wide.p,
                                   which == 0 ? a_k.p : a_v.p, n_edges_in, n_vertices, bad.p);
            }
            NO_CHECK(launch_status("narrow_ids"));
        } else {
            NO_HIP_CHECK(hipMemcpyAsync(a_k.p, src, ne_in * 4, kind, st));
            NO_HIP_CHECK(hipMemcpyAsync(a_v.p, dst, ne_in * 4, kind, st));
        }
        if (symmetrise) {       // every edge once more the other way round
            NO_HIP_CHECK(hipMemcpyAsync(a_k.p + ne_in, a_v.p, ne_in * 4, hipMemcpyDeviceToDevice, st));
            NO_HIP_CHECK(hipMemcpyAsync(a_v.p + ne_in, a_k.p, ne_in * 4, hipMemcpyDeviceToDevice, st));
        }
    }
    if (n_edges > 0) {
        // range check of every endpoint; without NO_CSR_DEDUP this pass also takes the degree histogram
        hipLaunchKernelGGL(csr_check_and_count_kernel, grid_for(n_edges), dim3(256), 0, st, (const int32_t*)a_k.p,
                           (const int32_t*)a_v.p, n_edges, n_vertices, degree.p, bad.p);
        NO_CHECK(launch_status("csr_check_and_count"));
    }
    int32_t h_bad = 0;
    NO_HIP_CHECK(hipMemcpyAsync(&h_bad, bad.p, 4, hipMemcpyDeviceToHost, st));
    NO_HIP_CHECK(hipStreamSynchronize(st));
    NO_REQUIRE(h_bad == 0, NO_ERR_OUT_OF_RANGE, "no_build_csr: an edge endpoint lies outside [0, V)");

    if (n_edges > 0) {
        int bits = ilog2_ceil((uint64_t)n_vertices);
        if (bits < 1) bits = 1;
        // sort by src (key a_k, value a_v=dst) -> b; then by dst (key b_v, value b_k=src) -> (a_k = dst, col or c_v = src)
        NO_CHECK(radix_sort_pairs(a_k.p, a_v.p, b_k.p, b_v.p, c_k.p, c_v.p, nullptr, n_edges, bits, ws.p, st));
        if (!dedup) {
            NO_CHECK(radix_sort_pairs(b_v.p, b_k.p, a_k.p, (uint32_t*)g->col.p, c_k.p, c_v.p, nullptr, n_edges, bits, ws.p, st));
        } else {
            // sorted (dst, src) pairs in (a_k, a_v); keep the first of every run of equal pairs
            NO_CHECK(radix_sort_pairs(b_v.p, b_k.p, a_k.p, a_v.p, c_k.p, c_v.p, nullptr, n_edges, bits, ws.p, st));
            int32_t* keep = (int32_t*)b_k.p;           // (the first sort's outputs are free again)
            hipLaunchKernelGGL(mark_first_of_run_kernel, grid_for(n_edges), dim3(256), 0, st, (const uint32_t*)a_k.p,
                               (const uint32_t*)a_v.p, n_edges, keep);
            DevBuf<int32_t> pos_buf;
            struct PGuard { DevBuf<int32_t>* p; ~PGuard() { p->release(); } } pguard{&pos_buf};
            NO_CHECK(pos_buf.alloc(ne + 1));
            NO_CHECK(exclusive_scan_i32(keep, nullptr, n_edges, pos_buf.p, bad.p, ws.p, st));      // (total -> the spare word)
            NO_CHECK(fill_i32(degree.p, 0, n_vertices, st));
            hipLaunchKernelGGL(compact_edges_kernel, grid_for(n_edges), dim3(256), 0, st, (const uint32_t*)a_k.p,
                               (const uint32_t*)a_v.p, (const int32_t*)keep, (const int32_t*)pos_buf.p, n_edges, g->col.p, degree.p);
            NO_CHECK(launch_status("csr dedup"));
            int32_t kept = 0;
            NO_HIP_CHECK(hipMemcpyAsync(&kept, bad.p, 4, hipMemcpyDeviceToHost, st));
            NO_HIP_CHECK(hipStreamSynchronize(st));
            g->n_edges = kept;
        }
    }
    NO_CHECK(exclusive_scan_i32_to_i64(degree.p, n_vertices, rowptr64.p, ws.p, st));
    if (rowptr_bits == 64) {
        g->rowptr64 = rowptr64;          // hand the buffer over
        rowptr64.p = nullptr;
    } else {
        NO_CHECK(g->rowptr32.alloc((size_t)n_vertices + 1));
        hipLaunchKernelGGL(narrow_rowptr_kernel, dim3((unsigned)ceil_div(n_vertices + 1, 256)), dim3(256), 0, st,
                           (const int64_t*)rowptr64.p, g->rowptr32.p, n_vertices + 1);
        NO_CHECK(launch_status("narrow_rowptr"));
    }
    NO_HIP_CHECK(hipStreamSynchronize(st));
    guard.g = nullptr;
    *out = g;
    return NO_OK;
}

extern "C" int32_t no_graph_view(no_graph_t g, int64_t* n_vertices, int64_t* n_edges, int32_t* rowptr_bits,
                                 const void** d_rowptr, const int32_t** d_col) {
    clear_error();
    NO_REQUIRE(g != nullptr, NO_ERR_INVALID_ARG, "no_graph_view: graph is NULL");
    if (n_vertices) *n_vertices = g->n_vertices;
    if (n_edges) *n_edges = g->n_edges;
    if (rowptr_bits) *rowptr_bits = g->rowptr_bits;
    if (d_rowptr) *d_rowptr = g->rowptr_bits == 64 ? (const void*)g->rowptr64.p : (const void*)g->rowptr32.p;
    if (d_col) *d_col = g->col.p;
    return NO_OK;
}

extern "C" int32_t no_graph_destroy(no_graph_t g) {
    clear_error();
    if (!g) return NO_OK;
    g->release();
    delete g;
    return NO_OK;
}
