// Error state, fills, the tile-offset stage of the prefix sum and a stable LSD radix sort of
// (key, value) pairs. The sort is what makes the block transpose, the CSR build and the hot-set
// ranking deterministic: equal keys keep their input order.
#include "primitives.hpp"

#include <string.h>

namespace no {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
void clear_error() { g_err[0] = 0; }

// ------------------------------------------------------------------------------------ fill

__global__ void fill_i32_kernel(int32_t* d, int32_t value, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) d[i] = value;
}

int32_t fill_i32(int32_t* d, int32_t value, int64_t n, hipStream_t st) {
    if (n <= 0) return NO_OK;
    int64_t blocks = ceil_div(n, 256 * 8);
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, d, value, n);
    return launch_status("fill_i32");
}

// ------------------------------------------------------------------------------------ scan

__global__ void __launch_bounds__(1024) scan_tile_offsets_kernel(const int32_t* d_n, int64_t cap, int64_t* tile_sums) {
    int64_t n = d_n ? (int64_t)*d_n : cap;
    if (n > cap) n = cap;
    int64_t tiles = (n + SCAN_TILE - 1) / SCAN_TILE;
    __shared__ int64_t smem[1024 / 64 + 1];
    int64_t carry = 0;
    for (int64_t base = 0; base < tiles; base += 1024) {
        int64_t i = base + threadIdx.x;
        int64_t v = i < tiles ? tile_sums[i] : 0;
        int64_t total;
        int64_t ex = block_exclusive_scan<int64_t, 1024>(v, &total, smem);
        if (i < tiles) tile_sums[i] = carry + ex;
        carry += total;
    }
}

size_t scan_ws_bytes(int64_t cap) { return scan_ws_bytes_impl(cap); }

int32_t exclusive_scan_i32(const int32_t* d_in, const int32_t* d_n, int64_t cap, int32_t* d_out, int32_t* d_total,
                           void* ws, hipStream_t st) {
    return exclusive_scan<ArrayLoader, int32_t>(ArrayLoader{d_in}, d_n, cap, d_out, d_total, ws, st);
}

int32_t exclusive_scan_i32_to_i64(const int32_t* d_in, int64_t n, int64_t* d_out, void* ws, hipStream_t st) {
    return exclusive_scan<ArrayLoader, int64_t>(ArrayLoader{d_in}, nullptr, n, d_out, nullptr, ws, st);
}

// ------------------------------------------------------------------------------------ radix sort

constexpr int RS_THREADS = 256;
constexpr int RS_WAVES = RS_THREADS / 64;
constexpr int RS_ITEMS = 16;                       // per lane
constexpr int RS_TILE = RS_THREADS * RS_ITEMS;     // 4096 keys per block; wave w owns keys [w*1024, (w+1)*1024)
constexpr int RS_RADIX = 256;

__device__ __forceinline__ int64_t rs_count(const int32_t* d_n, int64_t cap) {
    int64_t n = d_n ? (int64_t)*d_n : cap;
    return n > cap ? cap : n;
}

// hist[digit * n_tiles + tile] = number of keys of the tile with that digit (zeros past the end).
__global__ void __launch_bounds__(RS_THREADS) rs_hist_kernel(const uint32_t* keys, const int32_t* d_n, int64_t cap,
                                                             int shift, int64_t n_tiles, uint32_t* hist) {
    __shared__ uint32_t cnt[RS_RADIX];
    int64_t n = rs_count(d_n, cap);
    cnt[threadIdx.x] = 0;
    __syncthreads();
    int64_t base = (int64_t)blockIdx.x * RS_TILE;
    if (base < n) {
        for (int it = 0; it < RS_ITEMS; ++it) {
            int64_t i = base + (int64_t)it * RS_THREADS + threadIdx.x;
            if (i < n) atomicAdd(&cnt[(keys[i] >> shift) & (RS_RADIX - 1)], 1u);
        }
    }
    __syncthreads();
    hist[(int64_t)threadIdx.x * n_tiles + blockIdx.x] = cnt[threadIdx.x];
}

struct U32Loader {
    const uint32_t* p;
    __device__ __forceinline__ int32_t operator()(int64_t i) const { return (int32_t)p[i]; }
};

__global__ void __launch_bounds__(RS_THREADS) rs_scatter_kernel(const uint32_t* keys, const uint32_t* vals,
                                                                const int32_t* d_n, int64_t cap, int shift,
                                                                int64_t n_tiles, const uint32_t* offsets,
                                                                uint32_t* keys_out, uint32_t* vals_out) {
    int64_t n = rs_count(d_n, cap);
    int64_t base = (int64_t)blockIdx.x * RS_TILE;
    if (base >= n) return;
    __shared__ uint32_t cnt[RS_WAVES][RS_RADIX];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    for (int w = 0; w < RS_WAVES; ++w) cnt[w][threadIdx.x] = 0;
    __syncthreads();
    volatile uint32_t* my_cnt = cnt[wave];
    uint32_t key[RS_ITEMS];
    uint32_t rank[RS_ITEMS];
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    const int64_t wave_base = base + (int64_t)wave * (RS_ITEMS * 64);
#pragma unroll
    for (int it = 0; it < RS_ITEMS; ++it) {
        int64_t i = wave_base + (int64_t)it * 64 + lane;
        bool valid = i < n;
        uint32_t k = valid ? keys[i] : 0u;
        uint32_t d = (k >> shift) & (RS_RADIX - 1);
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            bool bit = (d >> b) & 1u;
            uint64_t m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        uint32_t before = (uint32_t)__popcll(peers & lt_mask);
        uint32_t group = (uint32_t)__popcll(peers);
        uint32_t prev = valid ? my_cnt[d] : 0u;
        key[it] = k;
        rank[it] = prev + before;
        __builtin_amdgcn_wave_barrier();
        if (valid && before == group - 1) my_cnt[d] = prev + group;   // last lane of the group publishes
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    {
        // thread d: turn per-wave counts into per-wave global bases for digit d
        uint32_t run = offsets[(int64_t)threadIdx.x * n_tiles + blockIdx.x];
        for (int w = 0; w < RS_WAVES; ++w) {
            uint32_t c = cnt[w][threadIdx.x];
            cnt[w][threadIdx.x] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < RS_ITEMS; ++it) {
        int64_t i = wave_base + (int64_t)it * 64 + lane;
        if (i < n) {
            uint32_t d = (key[it] >> shift) & (RS_RADIX - 1);
            uint32_t pos = cnt[wave][d] + rank[it];
            keys_out[pos] = key[it];
            vals_out[pos] = vals[i];
        }
    }
}

static inline int64_t rs_tiles(int64_t cap) { int64_t t = ceil_div(cap, RS_TILE); return t < 1 ? 1 : t; }

size_t radix_ws_bytes(int64_t cap) {
    int64_t m = rs_tiles(cap) * RS_RADIX;
    return (size_t)(2 * m + 2) * sizeof(uint32_t) + scan_ws_bytes_impl(m) + 64;
}

int32_t radix_sort_pairs(const uint32_t* keys_in, const uint32_t* vals_in, uint32_t* keys_out, uint32_t* vals_out,
                         uint32_t* keys_tmp, uint32_t* vals_tmp, const int32_t* d_n, int64_t cap, int bits, void* ws,
                         hipStream_t st) {
    if (cap <= 0) return NO_OK;
    if (cap >= (1ll << 32)) { set_error("radix sort: more than 2^32-1 items"); return NO_ERR_UNSUPPORTED; }
    int passes = (bits + 7) / 8;
    if (passes < 1) passes = 1;
    int64_t n_tiles = rs_tiles(cap);
    int64_t m = n_tiles * RS_RADIX;
    uint32_t* hist = (uint32_t*)ws;
    uint32_t* offs = hist + m;
    void* scan_ws = (void*)(((uintptr_t)(offs + m + 2) + 15) & ~(uintptr_t)15);
    const uint32_t* src_k = keys_in;
    const uint32_t* src_v = vals_in;
    for (int p = 0; p < passes; ++p) {
        bool to_out = ((passes - 1 - p) % 2) == 0;
        uint32_t* dst_k = to_out ? keys_out : keys_tmp;
        uint32_t* dst_v = to_out ? vals_out : vals_tmp;
        hipLaunchKernelGGL(rs_hist_kernel, dim3((unsigned)n_tiles), dim3(RS_THREADS), 0, st, src_k, d_n, cap, p * 8,
                           n_tiles, hist);
        NO_CHECK((exclusive_scan<U32Loader, uint32_t>(U32Loader{hist}, nullptr, m, offs, nullptr, scan_ws, st)));
        hipLaunchKernelGGL(rs_scatter_kernel, dim3((unsigned)n_tiles), dim3(RS_THREADS), 0, st, src_k, src_v, d_n, cap,
                           p * 8, n_tiles, offs, dst_k, dst_v);
        src_k = dst_k;
        src_v = dst_v;
    }
    return launch_status("radix_sort_pairs");
}

}  // namespace no

extern "C" const char* no_last_error(void) { return no::g_err; }
