// Device-wide primitives written for 64-lane wavefronts: reduce-then-scan prefix sums whose
// element count lives in device memory, and helpers for wave / block scans.
#pragma once
#include "common.hpp"

namespace no {

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 8;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_ITEMS;

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v) {
    const int lane = lane_id();
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        T u = __shfl_up(v, o, 64);
        if (lane >= o) v += u;
    }
    return v;
}

// Exclusive scan of one value per thread over a block of NT threads (NT multiple of 64, <= 1024).
// Returns the exclusive prefix; *block_total receives the block sum (same value in all threads).
template <typename T, int NT>
__device__ __forceinline__ T block_exclusive_scan(T v, T* block_total, T* smem /* NT/64 + 1 entries */) {
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    constexpr int NW = NT / 64;
    T incl = wave_inclusive_scan(v);
    if (lane == 63) smem[wave] = incl;
    __syncthreads();
    T wave_off = 0, total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        T s = smem[w];
        if (w < wave) wave_off += s;
        total += s;
    }
    __syncthreads();
    *block_total = total;
    return wave_off + incl - v;
}

// ---- reduce-then-scan over n = min(*d_n, cap) values produced by a loader functor -----------

template <typename Loader>
__global__ void __launch_bounds__(SCAN_THREADS) scan_tile_sums_kernel(Loader load, const int32_t* d_n, int64_t cap,
                                                                      int64_t* tile_sums) {
    int64_t n = d_n ? (int64_t)*d_n : cap;
    if (n > cap) n = cap;
    int64_t base = (int64_t)blockIdx.x * SCAN_TILE;
    if (base >= n) return;
    __shared__ int64_t smem[SCAN_THREADS / 64 + 1];
    int64_t i0 = base + (int64_t)threadIdx.x * SCAN_ITEMS;
    int64_t s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k)
        if (i0 + k < n) s += (int64_t)load(i0 + k);
    int64_t total;
    (void)block_exclusive_scan<int64_t, SCAN_THREADS>(s, &total, smem);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

// One block turns the tile sums into exclusive tile offsets, in place.
__global__ void __launch_bounds__(1024) scan_tile_offsets_kernel(const int32_t* d_n, int64_t cap, int64_t* tile_sums);

template <typename Loader, typename OutT>
__global__ void __launch_bounds__(SCAN_THREADS) scan_tiles_kernel(Loader load, const int32_t* d_n, int64_t cap,
                                                                  const int64_t* tile_offsets, OutT* out,
                                                                  int32_t* d_total) {
    int64_t n = d_n ? (int64_t)*d_n : cap;
    if (n > cap) n = cap;
    int64_t base = (int64_t)blockIdx.x * SCAN_TILE;
    if (n == 0 && blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = 0;
        if (d_total) *d_total = 0;
    }
    if (base >= n) return;
    __shared__ int64_t smem[SCAN_THREADS / 64 + 1];
    int64_t i0 = base + (int64_t)threadIdx.x * SCAN_ITEMS;
    int32_t v[SCAN_ITEMS];
    int64_t s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        v[k] = (i0 + k < n) ? load(i0 + k) : 0;
        s += v[k];
    }
    int64_t total;
    int64_t run = block_exclusive_scan<int64_t, SCAN_THREADS>(s, &total, smem) + tile_offsets[blockIdx.x];
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        if (i0 + k < n) out[i0 + k] = (OutT)run;
        run += v[k];
        if (i0 + k == n - 1) {
            out[n] = (OutT)run;
            if (d_total) *d_total = (int32_t)run;
        }
    }
}

inline size_t scan_ws_bytes_impl(int64_t cap) { return (size_t)(ceil_div(cap, SCAN_TILE) + 1) * sizeof(int64_t); }

// out must hold n+1 entries. ws: scan_ws_bytes(cap).
template <typename Loader, typename OutT>
int32_t exclusive_scan(Loader load, const int32_t* d_n, int64_t cap, OutT* out, int32_t* d_total, void* ws,
                       hipStream_t st) {
    int64_t tiles = ceil_div(cap, SCAN_TILE);
    if (tiles < 1) tiles = 1;
    int64_t* sums = (int64_t*)ws;
    hipLaunchKernelGGL((scan_tile_sums_kernel<Loader>), dim3((unsigned)tiles), dim3(SCAN_THREADS), 0, st, load, d_n, cap,
                       sums);
    hipLaunchKernelGGL(scan_tile_offsets_kernel, dim3(1), dim3(1024), 0, st, d_n, cap, sums);
    hipLaunchKernelGGL((scan_tiles_kernel<Loader, OutT>), dim3((unsigned)tiles), dim3(SCAN_THREADS), 0, st, load, d_n,
                       cap, sums, out, d_total);
    return launch_status("exclusive_scan");
}

// Sum of v over the threads of a block (NT multiple of 64); same value returned to all threads.
template <typename T, int NT>
__device__ __forceinline__ T block_sum(T v, T* smem /* NT/64 entries */) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    if (lane_id() == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    T total = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) total += smem[w];
    __syncthreads();
    return total;
}

// Sum of tile_sums[0 .. n_tiles) computed by the whole block: the "redundant prefix" that lets a
// scan run as two kernels (tile sums, then tile scans) when there are at most a few thousand tiles.
template <int NT>
__device__ __forceinline__ int64_t block_prefix_of_tiles(const int32_t* tile_sums, int64_t n_tiles, int64_t* smem) {
    int64_t s = 0;
    for (int64_t t = threadIdx.x; t < n_tiles; t += NT) s += tile_sums[t];
    return block_sum<int64_t, NT>(s, smem);
}

template <typename Loader>
__global__ void __launch_bounds__(SCAN_THREADS) scan2_tile_sums_kernel(Loader load, const int32_t* d_n, int64_t cap,
                                                                       int32_t* tile_sums) {
    int64_t n = d_n ? (int64_t)*d_n : cap;
    if (n > cap) n = cap;
    int64_t base = (int64_t)blockIdx.x * SCAN_TILE;
    if (base >= n) return;
    __shared__ int32_t smem[SCAN_THREADS / 64];
    int64_t i0 = base + (int64_t)threadIdx.x * SCAN_ITEMS;
    int32_t s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k)
        if (i0 + k < n) s += load(i0 + k);
    s = block_sum<int32_t, SCAN_THREADS>(s, smem);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = s;
}

template <typename Loader>
__global__ void __launch_bounds__(SCAN_THREADS) scan2_tiles_kernel(Loader load, const int32_t* d_n, int64_t cap,
                                                                   const int32_t* tile_sums, int32_t* out,
                                                                   int32_t* d_total) {
    int64_t n = d_n ? (int64_t)*d_n : cap;
    if (n > cap) n = cap;
    int64_t base = (int64_t)blockIdx.x * SCAN_TILE;
    if (n == 0 && blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = 0;
        if (d_total) *d_total = 0;
    }
    if (base >= n) return;
    __shared__ int64_t smem64[SCAN_THREADS / 64 + 1];
    const int64_t tile_off = block_prefix_of_tiles<SCAN_THREADS>(tile_sums, blockIdx.x, smem64);
    int64_t i0 = base + (int64_t)threadIdx.x * SCAN_ITEMS;
    int32_t v[SCAN_ITEMS];
    int64_t s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        v[k] = (i0 + k < n) ? load(i0 + k) : 0;
        s += v[k];
    }
    int64_t total;
    int64_t run = block_exclusive_scan<int64_t, SCAN_THREADS>(s, &total, smem64) + tile_off;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        if (i0 + k < n) out[i0 + k] = (int32_t)run;
        run += v[k];
        if (i0 + k == n - 1) {
            out[n] = (int32_t)run;
            if (d_total) *d_total = (int32_t)run;
        }
    }
}

// Two-kernel exclusive scan for at most a few thousand tiles (cap up to ~8M). ws: int32 per tile.
template <typename Loader>
int32_t exclusive_scan2(Loader load, const int32_t* d_n, int64_t cap, int32_t* out, int32_t* d_total, void* ws,
                        hipStream_t st) {
    int64_t tiles = ceil_div(cap, SCAN_TILE);
    if (tiles < 1) tiles = 1;
    int32_t* sums = (int32_t*)ws;
    hipLaunchKernelGGL((scan2_tile_sums_kernel<Loader>), dim3((unsigned)tiles), dim3(SCAN_THREADS), 0, st, load, d_n, cap,
                       sums);
    hipLaunchKernelGGL((scan2_tiles_kernel<Loader>), dim3((unsigned)tiles), dim3(SCAN_THREADS), 0, st, load, d_n, cap,
                       (const int32_t*)sums, out, d_total);
    return launch_status("exclusive_scan2");
}

struct ArrayLoader {
    const int32_t* p;
    __device__ __forceinline__ int32_t operator()(int64_t i) const { return p[i]; }
};

}  // namespace no
