// no_gather_features: feature collection (Algorithm 1, line 9): copy the rows of the feature
// table named by an id list into a dense matrix. Pure data movement, HBM bound.
//
// A row is cut into vector units of W bytes (the widest of 16/8/4/2 that the row size, strides and
// base addresses allow). A group of G = min(64, pow2 >= units) lanes copies one row, so a wavefront
// reads 64/G rows at once with fully coalesced 64*W-byte requests; up to four lane-group widths of a
// row are kept in flight per group.
#include "common.hpp"

namespace no {

template <typename VecT, int ROWS, int UNR>
__global__ void __launch_bounds__(256) gather_rows_kernel(const char* __restrict__ table, int64_t table_stride,
                                                          const int32_t* __restrict__ ids, const int32_t* d_n,
                                                          int32_t n_cap, char* __restrict__ out, int64_t out_stride,
                                                          int32_t units, int32_t g_log2) {
    int32_t n = d_n ? *d_n : n_cap;
    if (n > n_cap) n = n_cap;
    const int32_t lane = (int32_t)(threadIdx.x & 63);
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int32_t rows_per_pass = 64 >> g_log2;
    const int32_t sub = lane >> g_log2;
    const int32_t u0 = lane & ((1 << g_log2) - 1);
    const int32_t g = 1 << g_log2;
    // The ids of a wavefront's next pass are requested before the rows of the current one, so that a pass costs one
    // memory round trip (rows) instead of two dependent ones (ids, then rows).
    static_assert(ROWS == 1, "one row per lane group and pass");
    const int64_t stride_rows = n_waves * rows_per_pass;
    int64_t r = wave * rows_per_pass + sub;
    int32_t id_cur = r < n ? ids[r] : -1;
    for (; r - sub < n; r += stride_rows) {
        const int64_t r_next = r + stride_rows;
        const int32_t id_next = r_next < n ? ids[r_next] : -1;
        const char* src = id_cur >= 0 ? table + (int64_t)id_cur * table_stride : nullptr;
        // UNR lane-group widths of the row are requested before the first store (a 2408-byte row in 8-byte units is
        // five widths: one round trip per pass instead of five)
        for (int32_t ub = u0; ub < units; ub += g * UNR) {
            VecT v[UNR];
#pragma unroll
            for (int j = 0; j < UNR; ++j) {
                const int32_t u = ub + j * g;
                if (src && u < units) v[j] = *reinterpret_cast<const VecT*>(src + (int64_t)u * sizeof(VecT));
            }
#pragma unroll
            for (int j = 0; j < UNR; ++j) {
                const int32_t u = ub + j * g;
                if (src && u < units) *reinterpret_cast<VecT*>(out + r * out_stride + (int64_t)u * sizeof(VecT)) = v[j];
            }
        }
        id_cur = id_next;
    }
}

template <typename VecT>
static void launch_gather(const char* table, int64_t ts, const int32_t* ids, const int32_t* d_n, int32_t n_cap, char* out,
                          int64_t os, int32_t row_bytes, hipStream_t st) {
    const int32_t units = row_bytes / (int32_t)sizeof(VecT);
    int g_log2 = 0;
    while ((1 << g_log2) < units && g_log2 < 6) ++g_log2;
    // One row per lane group and pass: with 2, 4 or 8 rows per group in flight the kernel measured slower on every row
    // size tried, with the ids repeated (rows served by the caches: 5-45 % slower) and with fresh ids and buffers every
    // launch (256-byte rows out of a 28 GB table: 15 -> 27 us; 2408-byte rows: 35 -> 37-50 us). A group then alternates
    // loads and stores at a finer grain, and the many short wavefronts keep reads and writes overlapped across the chip.
    // A plain contiguous copy of the same bytes takes 13 us and 29 us: the gather pays one more dependent round trip
    // (ids, then rows).
    constexpr int ROWS = 1;
    const int64_t rows_per_wave = (int64_t)(64 >> g_log2) * ROWS;
    int64_t waves = ceil_div(n_cap, rows_per_wave);
    int64_t blocks = ceil_div(waves, 4);
    // 8192 wavefronts fill the chip's wave slots once; each then walks its passes with the next ids already requested
    // (measured, 118 K rows of 256 bytes from fresh ids and buffers: 2048 blocks 14.7 us, 4096 15.5, 1024 17.7)
    const int64_t max_blocks = 256 * 8;
    if (blocks > max_blocks) blocks = max_blocks;
    if (blocks < 1) blocks = 1;
    const int32_t widths = (int32_t)ceil_div(units, 1 << g_log2);      // lane-group widths per row
#define NO_GATHER_LAUNCH(U)                                                                                                \
    hipLaunchKernelGGL((gather_rows_kernel<VecT, ROWS, U>), dim3((unsigned)blocks), dim3(256), 0, st, table, ts, ids, d_n, \
                       n_cap, out, os, units, g_log2)
    if (widths > 2) NO_GATHER_LAUNCH(4);
    else if (widths == 2) NO_GATHER_LAUNCH(2);
    else NO_GATHER_LAUNCH(1);
#undef NO_GATHER_LAUNCH
}

int32_t gather_rows(const void* d_table, int32_t row_bytes, int64_t table_stride, const int32_t* d_ids,
                    const int32_t* d_n, int32_t n_cap, void* d_out, int64_t out_stride, hipStream_t st) {
    if (n_cap <= 0 || row_bytes <= 0) return NO_OK;
    const uintptr_t mix = (uintptr_t)d_table | (uintptr_t)d_out | (uintptr_t)table_stride | (uintptr_t)out_stride |
                          (uintptr_t)row_bytes;
    const char* t = (const char*)d_table;
    char* o = (char*)d_out;
    if ((mix & 15) == 0) launch_gather<uint4>(t, table_stride, d_ids, d_n, n_cap, o, out_stride, row_bytes, st);
    else if ((mix & 7) == 0) launch_gather<uint2>(t, table_stride, d_ids, d_n, n_cap, o, out_stride, row_bytes, st);
    else if ((mix & 3) == 0) launch_gather<uint32_t>(t, table_stride, d_ids, d_n, n_cap, o, out_stride, row_bytes, st);
    else launch_gather<uint16_t>(t, table_stride, d_ids, d_n, n_cap, o, out_stride, row_bytes, st);
    return launch_status("gather_rows");
}

}  // namespace no

using namespace no;

extern "C" int32_t no_gather_features(const void* d_table, no_dtype dt, int64_t n_rows, int32_t dim,
                                      int64_t table_stride_bytes, const int32_t* d_ids, const int32_t* d_n_ids,
                                      int32_t n_ids_cap, void* d_out, int64_t out_stride_bytes, void* stream) {
    clear_error();
    NO_REQUIRE(d_table && d_ids && d_out, NO_ERR_INVALID_ARG, "no_gather_features: NULL argument");
    NO_REQUIRE(dt == NO_F32 || dt == NO_BF16, NO_ERR_INVALID_ARG, "no_gather_features: unknown dtype");
    NO_REQUIRE(n_rows >= 1 && dim >= 1 && n_ids_cap >= 0, NO_ERR_INVALID_ARG, "no_gather_features: bad sizes");
    const int32_t es = dt == NO_F32 ? 4 : 2;
    const int64_t row_bytes = (int64_t)dim * es;
    NO_REQUIRE(row_bytes < (1ll << 30), NO_ERR_INVALID_ARG, "no_gather_features: row too large");
    NO_REQUIRE(table_stride_bytes >= row_bytes && out_stride_bytes >= row_bytes, NO_ERR_INVALID_ARG,
               "no_gather_features: stride smaller than a row");
    NO_REQUIRE(table_stride_bytes % es == 0 && out_stride_bytes % es == 0, NO_ERR_INVALID_ARG,
               "no_gather_features: strides must be multiples of the element size");
    NO_REQUIRE(((uintptr_t)d_table % es) == 0 && ((uintptr_t)d_out % es) == 0, NO_ERR_INVALID_ARG,
               "no_gather_features: misaligned pointer");
    return gather_rows(d_table, (int32_t)row_bytes, table_stride_bytes, d_ids, d_n_ids, n_ids_cap, d_out, out_stride_bytes,
                       (hipStream_t)stream);
}
