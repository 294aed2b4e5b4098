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

__global__ void narrow_rowptr_kernel(const int64_t* in, int32_t* out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) out[i] = (int32_t)in[i];
}

}  // namespace no

using namespace no;

extern "C" int32_t no_build_csr(const int32_t* src, const int32_t* dst, int64_t n_edges, int64_t n_vertices,
                                int32_t rowptr_bits, uint32_t flags, void* stream, no_graph_t* out) {
    clear_error();
    NO_REQUIRE(out != nullptr, NO_ERR_INVALID_ARG, "no_build_csr: out is NULL");
    *out = nullptr;
    NO_REQUIRE(n_vertices > 0 && n_edges >= 0, NO_ERR_INVALID_ARG, "no_build_csr: need n_vertices > 0, n_edges >= 0");
    NO_REQUIRE(n_edges == 0 || (src && dst), NO_ERR_INVALID_ARG, "no_build_csr: src/dst is NULL");
    NO_REQUIRE(rowptr_bits == 32 || rowptr_bits == 64, NO_ERR_INVALID_ARG, "no_build_csr: rowptr_bits must be 32 or 64");
    NO_REQUIRE(n_vertices < (1ll << 31), NO_ERR_OVERFLOW, "no_build_csr: vertex ids are int32, V must be < 2^31");
    NO_REQUIRE(rowptr_bits == 64 || n_edges < (1ll << 31), NO_ERR_OVERFLOW,
               "no_build_csr: 32-bit row pointers need fewer than 2^31 edges");
    NO_REQUIRE(n_edges < (1ll << 32) - 1, NO_ERR_UNSUPPORTED, "no_build_csr: at most 2^32-2 edges");
    hipStream_t st = (hipStream_t)stream;

    no_graph_s* g = new no_graph_s();
    g->n_vertices = n_vertices;
    g->n_edges = n_edges;
    g->rowptr_bits = rowptr_bits;
    struct Guard { no_graph_s* g; ~Guard() { if (g) { g->release(); delete g; } } } guard{g};

    const size_t ne = (size_t)n_edges;
    DevBuf<uint32_t> a_k, a_v, b_k, b_v, c_k, c_v;
    DevBuf<int32_t> degree, bad;
    DevBuf<char> ws;
    DevBuf<int64_t> rowptr64;
    struct Tmp { DevBuf<uint32_t>*u[6]; DevBuf<int32_t>* i[2]; DevBuf<char>* w; DevBuf<int64_t>* r;
                 ~Tmp() { for (auto p : u) p->release(); for (auto p : i) p->release(); w->release(); r->release(); } }
        tmp{{&a_k, &a_v, &b_k, &b_v, &c_k, &c_v}, {&degree, &bad}, &ws, &rowptr64};

    NO_CHECK(a_k.alloc(ne)); NO_CHECK(a_v.alloc(ne));
    NO_CHECK(b_k.alloc(ne)); NO_CHECK(b_v.alloc(ne));
    NO_CHECK(c_k.alloc(ne)); NO_CHECK(c_v.alloc(ne));
    NO_CHECK(degree.alloc((size_t)n_vertices)); NO_CHECK(bad.alloc(1));
    size_t ws_bytes = radix_ws_bytes(n_edges);
    size_t sb = scan_ws_bytes(n_vertices);
    if (sb > ws_bytes) ws_bytes = sb;
    NO_CHECK(ws.alloc(ws_bytes));
    NO_CHECK(rowptr64.alloc((size_t)n_vertices + 1));
    NO_CHECK(g->col.alloc(ne));

    // a_k = src, a_v = dst
    hipMemcpyKind kind = (flags & NO_CSR_INPUT_ON_DEVICE) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    if (n_edges > 0) {
        NO_HIP_CHECK(hipMemcpyAsync(a_k.p, src, ne * 4, kind, st));
        NO_HIP_CHECK(hipMemcpyAsync(a_v.p, dst, ne * 4, kind, st));
    }
    NO_CHECK(fill_i32(degree.p, 0, n_vertices, st));
    NO_CHECK(fill_i32(bad.p, 0, 1, st));
    if (n_edges > 0) {
        int64_t blocks = ceil_div(n_edges, 256 * 4);
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(csr_check_and_count_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const int32_t*)a_k.p,
                           (const int32_t*)a_v.p, n_edges, n_vertices, degree.p, bad.p);
        NO_CHECK(launch_status("csr_check_and_count"));
    }
    int32_t h_bad = 0;
    NO_HIP_CHECK(hipMemcpyAsync(&h_bad, bad.p, 4, hipMemcpyDeviceToHost, st));
    NO_HIP_CHECK(hipStreamSynchronize(st));
    NO_REQUIRE(h_bad == 0, NO_ERR_OUT_OF_RANGE, "no_build_csr: an edge endpoint lies outside [0, V)");

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
    if (n_edges > 0) {
        int bits = ilog2_ceil((uint64_t)n_vertices);
        if (bits < 1) bits = 1;
        // sort by src (key a_k, value a_v=dst) -> b; then by dst (key b_v, value b_k=src) -> (c_k, col)
        NO_CHECK(radix_sort_pairs(a_k.p, a_v.p, b_k.p, b_v.p, c_k.p, c_v.p, nullptr, n_edges, bits, ws.p, st));
        NO_CHECK(radix_sort_pairs(b_v.p, b_k.p, a_k.p, (uint32_t*)g->col.p, c_k.p, c_v.p, nullptr, n_edges, bits, ws.p, st));
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
