// Internal helpers shared by the HIP translation units of libneutronorch: error reporting,
// launch arithmetic, device buffers owned by handles.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "neutronorch.h"

namespace no {

void set_error(const char* fmt, ...);
void clear_error();

#define NO_HIP_CHECK(expr)                                                                  \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) {                                                             \
            ::no::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return NO_ERR_HIP;                                                              \
        }                                                                                   \
    } while (0)

#define NO_CHECK(expr)                 \
    do {                               \
        int32_t s_ = (expr);           \
        if (s_ != NO_OK) return s_;    \
    } while (0)

#define NO_REQUIRE(cond, code, ...)            \
    do {                                       \
        if (!(cond)) {                         \
            ::no::set_error(__VA_ARGS__);      \
            return (code);                     \
        }                                      \
    } while (0)

inline int32_t launch_status(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("launch of %s failed: %s", what, hipGetErrorString(e));
        return NO_ERR_HIP;
    }
    return NO_OK;
}

// Launch with an optional pair of events that take the kernel's own start and end times (HIP's extended launch):
// a stage that is a single kernel is then timed like a kernel trace times it, without the dispatch latency and the
// event packets that a record-before / record-after pair on the stream adds.
// Events that only order work between streams of this device: no timing, and a device-scope release when recorded
// (the default is a system-scope fence: cache write-back and invalidation, paid by the record and by the kernels after it).
#define NO_SYNC_EVENT_FLAGS (hipEventDisableTiming | hipEventReleaseToDevice)

#define NO_LAUNCH_TIMED(kernel, grid, block, st, ev0, ev1, ...)                                      \
    do {                                                                                             \
        if (ev0) hipExtLaunchKernelGGL(kernel, grid, block, 0, st, ev0, ev1, 0, __VA_ARGS__);        \
        else hipLaunchKernelGGL(kernel, grid, block, 0, st, __VA_ARGS__);                            \
    } while (0)

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline int ilog2_ceil(uint64_t x) { int b = 0; while ((1ull << b) < x) ++b; return b; }

// A device allocation owned by a handle.
template <typename T>
struct DevBuf {
    T* p = nullptr;
    size_t n = 0;
    int32_t alloc(size_t count) {
        n = count;
        if (count == 0) count = 1;
        hipError_t e = hipMalloc((void**)&p, count * sizeof(T));
        if (e != hipSuccess) {
            p = nullptr;
            set_error("hipMalloc of %zu bytes failed: %s", count * sizeof(T), hipGetErrorString(e));
            return NO_ERR_HIP;
        }
        return NO_OK;
    }
    void release() { if (p) { (void)hipFree(p); p = nullptr; } n = 0; }
};

constexpr int32_t EMPTY = 0x7fffffff;   // vertex -> local id map: no entry

// ---- primitives (scan.hip / radix_sort.hip / fill) ----

// Exclusive prefix sum of n = min(*d_n, cap) int32 values d_in[i] into d_out[0..n] (d_out[n] = total),
// also stored to *d_total if not NULL. Out type int32 or int64. ws needs scan_ws_bytes(cap).
size_t scan_ws_bytes(int64_t cap);
int32_t exclusive_scan_i32(const int32_t* d_in, const int32_t* d_n, int64_t cap, int32_t* d_out,
                           int32_t* d_total, void* ws, hipStream_t st);
int32_t exclusive_scan_i32_to_i64(const int32_t* d_in, int64_t n, int64_t* d_out, void* ws, hipStream_t st);

// Stable LSD radix sort of (key, value) uint32 pairs on the low `bits` bits of the key.
// n = min(*d_n, cap) if d_n != NULL else cap. Result lands in keys_out/vals_out (which may be the
// alt buffers or the inputs depending on the pass count: always returned in *_out).
size_t radix_ws_bytes(int64_t cap);
int32_t radix_sort_pairs(const uint32_t* keys_in, const uint32_t* vals_in, uint32_t* keys_out, uint32_t* vals_out,
                         uint32_t* keys_tmp, uint32_t* vals_tmp, const int32_t* d_n, int64_t cap, int bits,
                         void* ws, hipStream_t st);

int32_t fill_i32(int32_t* d, int32_t value, int64_t n, hipStream_t st);

}  // namespace no
