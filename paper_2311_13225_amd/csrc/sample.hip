// no_sample_blocks: reverse multi-hop fanout sampling over the in-neighbour CSR (the sample()
// loop of Algorithm 1), de-duplication / relabelling of each frontier, the block transpose used
// by the backward pass, and the hot-vertex lookup that removes reusable vertices from the bottom
// hop (Section 4.1.2, Stage 1 of Section 4.2).
//
// One hop is four kernels over a fixed-stride ("padded") edge array, slot q = row * fanout + j:
//   1. sample_rows   a sub-wave group of G lanes (G = 8/16/32/64 >= fanout) serves one destination;
//                    lane j draws slot j with Philox4x32-10 keyed by (stream; vertex, slot, domain,
//                    hop), the group resolves the partial Fisher-Yates swap chain with cross-lane
//                    shuffles, and every sampled id does atomicMin(map[id], n_dst + q): the first
//                    occurrence of an id in (row, slot) order wins, whatever the execution order;
//   2. edge_tile_sums  per 1024-slot tile: number of sampled edges and of first occurrences;
//   3. edge_assign   tile prefix + block scan: compact edge ids, row pointers, new local ids in
//                    first-occurrence order, map[id] = local id;
//   4. edge_indices  indices[e] = map[id]; counts per source for the transpose.
// `map` is a direct-address table int32[V] (HBM is plentiful; no hashing, no probing order to
// reason about). It carries the local ids from one hop to the next and is wiped after the last.
// The transpose (hops above the bottom one) is a counting sort: scan of the per-source counts,
// unordered fill through atomic cursors, then every edge ranks itself inside its (short) column so
// that columns end up in ascending edge id regardless of the fill order.
#include "primitives.hpp"
#include "handles.hpp"
#include "layers.hpp"

namespace no {

// Tiles of the slot scans: 1024 slots (four per thread). Measured on three hops of 15 K / 34 K / 122 K slots: sampling
// stage 232 / 190 / 173 / 171 / 179 us at 4096 / 2048 / 1024 / 512 / 256 slots per tile (a thread's dependent loads and
// its scattered stores are the latency of the kernel; more tiles only lengthen the look-back by one poll per 64).
constexpr int ETHREADS = 256, EITEMS = 4, ETILE = ETHREADS * EITEMS;

// ---------------------------------------------------------------------------- Philox4x32-10

__device__ __forceinline__ uint64_t philox_random64(uint32_t k0, uint32_t k1, uint32_t c0, uint32_t c1, uint32_t c2,
                                                    uint32_t c3) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return ((uint64_t)c1 << 32) | (uint64_t)c0;
}

// ---------------------------------------------------------------------------- 1. sampling

template <int G, typename RowT>
__global__ void __launch_bounds__(256) sample_rows_kernel(const RowT* __restrict__ rowptr, const int32_t* __restrict__ col,
                                                          const int32_t* __restrict__ dst, const int32_t* d_n_dst,
                                                          int32_t n_fixed, int32_t n_cap, int32_t k, uint32_t key0,
                                                          uint32_t key1, uint32_t c3, int32_t* __restrict__ nbr_pad,
                                                          int32_t* __restrict__ src_global, int32_t* map,
                                                          int32_t insert_dst, int32_t* seeds_copy, int32_t* count_out,
                                                          int32_t n_vertices, int32_t* bad_id_flag, int32_t flag_value,
                                                          unsigned long long* scan_status, int32_t n_status) {
    // the tile status words of the scan that follows this launch start out empty
    for (int32_t t = (int32_t)(blockIdx.x * 256 + threadIdx.x); t < n_status; t += (int32_t)(gridDim.x * 256)) scan_status[t] = 0ull;
    int32_t n_dst = d_n_dst ? *d_n_dst : n_fixed;
    if (n_dst > n_cap) n_dst = n_cap;
    if (blockIdx.x == 0 && threadIdx.x == 0) *count_out = n_dst;
    const int32_t i = (int32_t)(blockIdx.x * (256 / G) + threadIdx.x / G);
    const int32_t j = (int32_t)(threadIdx.x % G);
    const bool row_ok = i < n_dst;
    int32_t v = 0;
    int64_t begin = 0, d = 0;
    if (row_ok) {
        v = dst[i];
        if (insert_dst && (uint32_t)v >= (uint32_t)n_vertices) {
            // a caller-supplied seed outside [0, V): stay inside the graph's arrays and report it
            v = 0;
            *bad_id_flag = flag_value;
        }
        begin = (int64_t)rowptr[v];
        d = (int64_t)rowptr[v + 1] - begin;
        if (j == 0) {
            src_global[i] = v;
            if (insert_dst) map[v] = i;       // a plain store and the atomicMin below commute: i is the smaller value
            if (seeds_copy) seeds_copy[i] = v;
        }
    }
    int64_t pos = j;
    const bool take_all = d <= (int64_t)k;
    // The swap partner of slot j: r_j = j + floor(x * (d - j) / 2^64) in [j, d).
    int64_t r = -1 - (int64_t)j;          // distinct negative sentinels for idle lanes
    if (row_ok && !take_all && j < k) {
        uint64_t x = philox_random64(key0, key1, (uint32_t)v, 0u, (uint32_t)j, c3);
        r = (int64_t)j + (int64_t)__umul64hi(x, (uint64_t)(d - j));
    }
    // Whole groups with nothing to shuffle still take part in the cross-lane reads below.
    if (__ballot(row_ok && !take_all) != 0ull) {
        // a = latest earlier step that displaced position j; b = latest earlier step that hit r_j
        int32_t a = -1, b = -1;
        for (int32_t t = 0; t < k; ++t) {
            int64_t rt = __shfl(r, t, G);
            if (t < j) {
                if (rt == (int64_t)j) a = t;
                if (rt == r) b = t;
            }
        }
        // w_j = content of position j just before step j: j itself unless displaced, else w_a.
        int64_t w = j;
        bool done = a < 0;
        while (true) {
            int64_t wa = __shfl(w, a < 0 ? 0 : a, G);
            int da = __shfl((int)done, a < 0 ? 0 : a, G);
            if (!done && da) { w = wa; done = true; }
            if (__ballot(!done) == 0ull) break;
        }
        int64_t wb = __shfl(w, b < 0 ? 0 : b, G);
        if (!take_all) pos = b < 0 ? r : wb;
    }
    const int32_t cnt = d < (int64_t)k ? (int32_t)d : k;
    if (row_ok && j < k) {
        const int32_t q = i * k + j;
        if (j < cnt) {
            int32_t u = col[begin + pos];
            nbr_pad[q] = u;
            atomicMin(&map[u], n_dst + q);   // integer min: order independent
        } else {
            nbr_pad[q] = -1;
        }
    }
}

// ---------------------------------------------------------------------------- 2./3. compaction and new ids

__device__ __forceinline__ int64_t slot_flags(const int32_t* __restrict__ nbr_pad, const int32_t* map, int64_t q,
                                              int32_t n_dst, int32_t* u_out) {
    const int32_t u = nbr_pad[q];
    *u_out = u;
    if (u < 0) return 0;
    return 1ll + ((map[u] == n_dst + (int32_t)q) ? (1ll << 32) : 0ll);    // low word: sampled; high word: first seen
}

// (the two-launch form: the tile sums pass marks the first occurrences in the padded array itself, -2 - id in place of id,
// so that the assignment pass reads its flags with the slots and does not wait for a second probe of the id map)
__device__ __forceinline__ int64_t slot_flags_marked(const int32_t* __restrict__ nbr_pad, int64_t q, int32_t* u_out) {
    const int32_t e = nbr_pad[q];
    *u_out = e <= -2 ? -2 - e : e;
    if (e == -1) return 0;
    return 1ll + (e <= -2 ? (1ll << 32) : 0ll);
}

__global__ void __launch_bounds__(ETHREADS) edge_tile_sums_kernel(int32_t* __restrict__ nbr_pad, const int32_t* map,
                                                                  const int32_t* d_n_dst, int32_t k, int64_t* tile_sums,
                                                                  int32_t* zero_a, int32_t* zero_b, int32_t n_zero) {
    for (int64_t t = (int64_t)blockIdx.x * ETHREADS + threadIdx.x; t < n_zero; t += (int64_t)gridDim.x * ETHREADS) {
        zero_a[t] = 0;
        zero_b[t] = 0;
    }
    const int32_t n_dst = *d_n_dst;
    const int64_t n_pad = (int64_t)n_dst * k;
    const int64_t base = (int64_t)blockIdx.x * ETILE;
    if (base >= n_pad) return;
    __shared__ int64_t smem[ETHREADS / 64];
    const int64_t q0 = base + (int64_t)threadIdx.x * EITEMS;
    int64_t s = 0;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) {
        int32_t u;
        if (q0 + t < n_pad) {
            const int64_t f = slot_flags(nbr_pad, map, q0 + t, n_dst, &u);
            if (f >> 32) nbr_pad[q0 + t] = -2 - u;
            s += f;
        }
    }
    s = block_sum<int64_t, ETHREADS>(s, smem);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = s;
}

__global__ void __launch_bounds__(ETHREADS) edge_assign_kernel(const int32_t* __restrict__ nbr_pad, int32_t* map,
                                                               const int32_t* d_n_dst, int32_t k, uint64_t k_magic,
                                                               const int64_t* __restrict__ tile_sums,
                                                               int32_t* __restrict__ indptr, int32_t* __restrict__ nbr,
                                                               int32_t* __restrict__ edge_row, int32_t* __restrict__ src_global,
                                                               int32_t* counts /* [0]=n_dst (in), [1]=n_src, [2]=nnz */) {
    __shared__ int64_t smem[ETHREADS / 64 + 1];
    const int32_t n_dst = *d_n_dst;
    const int64_t n_pad = (int64_t)n_dst * k;
    const int64_t n_tiles = (n_pad + ETILE - 1) / ETILE;
    if (blockIdx.x == 0) {
        int64_t s = 0;
        for (int64_t t = threadIdx.x; t < n_tiles; t += ETHREADS) s += tile_sums[t];
        s = block_sum<int64_t, ETHREADS>(s, smem);
        if (threadIdx.x == 0) {
            const int32_t nnz = (int32_t)(s & 0xffffffffll), n_new = (int32_t)(s >> 32);
            indptr[n_dst] = nnz;
            counts[1] = n_dst + n_new;
            counts[2] = nnz;
        }
    }
    const int64_t base = (int64_t)blockIdx.x * ETILE;
    if (base >= n_pad) return;
    int64_t tile_off = 0;
    {
        int64_t s = 0;
        for (int64_t t = threadIdx.x; t < (int64_t)blockIdx.x; t += ETHREADS) s += tile_sums[t];
        tile_off = block_sum<int64_t, ETHREADS>(s, smem);
    }
    const int64_t q0 = base + (int64_t)threadIdx.x * EITEMS;
    int64_t f[EITEMS];
    int32_t u[EITEMS];
    int64_t s = 0;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) {
        f[t] = 0;
        u[t] = -1;
        if (q0 + t < n_pad) f[t] = slot_flags_marked(nbr_pad, q0 + t, &u[t]);
        s += f[t];
    }
    int64_t total;
    int64_t run = block_exclusive_scan<int64_t, ETHREADS>(s, &total, smem) + tile_off;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) {
        const int64_t q = q0 + t;
        if (q < n_pad) {
            const int32_t e = (int32_t)(run & 0xffffffffll);
            const int32_t row = k == 1 ? (int32_t)q : (int32_t)__umul64hi((uint64_t)q, k_magic);   // q / k, exact
            if (q - (int64_t)row * k == 0) indptr[row] = e;
            if (f[t] & 1) {
                nbr[e] = u[t];
                edge_row[e] = row;
                if (f[t] >> 32) {
                    const int32_t local = n_dst + (int32_t)(run >> 32);
                    src_global[local] = u[t];
                    map[u[t]] = local;     // only the first occurrence writes; later readers never match n_dst + q
                }
            }
            run += f[t];
        }
    }
}

// One-launch form of the two kernels above (tile sums, then assignment): a single-pass scan. A block publishes its
// tile's sum in a status word, adds up the words of the tiles before it until it meets one that already holds an
// inclusive prefix, publishes its own inclusive prefix and assigns. (Workgroups are handed out in index order, per
// die in turn: an earlier tile is done, running, or the next to start on its die, and a waiting block never holds
// the slot an earlier tile needs.) A word packs both 31-bit counts and a 2-bit state, so it is written and read by one
// 64-bit access at device scope and needs no fence; the words are emptied by the sampling launch before. The wait on
// an earlier tile is bounded: on expiry the block stores the call's id in `fail_flag` and goes on (wrong output, no hang;
// the host reports NO_ERR_TIMEOUT wherever it next reads the blocks' counts).
constexpr unsigned long long SCAN_SUM = 1ull, SCAN_PREFIX = 2ull;
__device__ __forceinline__ unsigned long long scan_pack(int64_t v, unsigned long long state) {
    return ((unsigned long long)(v & 0x7fffffffll)) | ((unsigned long long)((v >> 32) & 0x7fffffffll) << 31) | (state << 62);
}
__device__ __forceinline__ int64_t scan_unpack(unsigned long long w) {
    return (int64_t)(w & 0x7fffffffull) | ((int64_t)((w >> 31) & 0x7fffffffull) << 32);
}

__global__ void __launch_bounds__(ETHREADS) edge_scan_kernel(const int32_t* __restrict__ nbr_pad, int32_t* map,
                                                             const int32_t* d_n_dst, int32_t k, uint64_t k_magic,
                                                             unsigned long long* status, int32_t* __restrict__ indptr,
                                                             int32_t* __restrict__ nbr, int32_t* __restrict__ edge_row,
                                                             int32_t* __restrict__ src_global,
                                                             int32_t* counts /* [0]=n_dst (in), [1]=n_src, [2]=nnz */,
                                                             int32_t* zero_a, int32_t* zero_b, int32_t n_zero, int32_t* fail_flag,
                                                             int32_t flag_value, int32_t spin_limit, int32_t withhold_first,
                                                             unsigned int* done) {
    __shared__ int64_t smem[ETHREADS / 64 + 1];
    __shared__ int64_t prefix_sh;
    __shared__ int cleanup_sh;
    for (int64_t t = (int64_t)blockIdx.x * ETHREADS + threadIdx.x; t < n_zero; t += (int64_t)gridDim.x * ETHREADS) {
        zero_a[t] = 0;
        zero_b[t] = 0;
    }
    const int32_t n_dst = *d_n_dst;
    const int64_t n_pad = (int64_t)n_dst * k;
    if (n_pad == 0) {
        if (blockIdx.x == 0 && threadIdx.x == 0) { indptr[0] = 0; counts[1] = n_dst; counts[2] = 0; }
        return;
    }
    const int64_t base = (int64_t)blockIdx.x * ETILE;
    if (base >= n_pad) return;
    const int64_t q0 = base + (int64_t)threadIdx.x * EITEMS;
    int64_t f[EITEMS];
    int32_t u[EITEMS];
    int64_t s = 0;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) {
        f[t] = 0;
        u[t] = -1;
        if (q0 + t < n_pad) f[t] = slot_flags(nbr_pad, map, q0 + t, n_dst, &u[t]);
        s += f[t];
    }
    int64_t total;
    int64_t run = block_exclusive_scan<int64_t, ETHREADS>(s, &total, smem);
    if (threadIdx.x < 64) {
        // wavefront 0 looks back 64 tiles at a time: lane l reads the word of tile (first - l)
        const int lane = (int)threadIdx.x;
        int64_t prefix = 0;
        if (blockIdx.x > 0) {
            if (lane == 0)
                __hip_atomic_store(&status[blockIdx.x], scan_pack(total, SCAN_SUM), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int64_t first = (int64_t)blockIdx.x - 1;      // nearest tile not yet added
            int spins = 0;
            while (first >= 0) {
                const int64_t j = first - lane;
                unsigned long long w = SCAN_PREFIX << 62;                      // lanes past tile 0: an empty prefix
                if (j >= 0) w = __hip_atomic_load(&status[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const unsigned long long state = w >> 62;
                const unsigned long long is_prefix = __ballot(state == SCAN_PREFIX), is_empty = __ballot(state == 0ull);
                // usable lanes: those before the first empty word; the walk ends at the first prefix among them
                const int n_ok = is_empty ? __builtin_ctzll(is_empty) : 64;
                const int p_at = is_prefix ? __builtin_ctzll(is_prefix) : 64;
                const int take = p_at < n_ok ? p_at + 1 : n_ok;               // lanes [0, take) are added
                int64_t v = lane < take ? scan_unpack(w) : 0;
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
                prefix += v;
                first -= take;
                if (p_at < n_ok) break;                                       // reached an inclusive prefix
                if (take == 0) {
                    if (++spins > spin_limit) {
                        if (lane == 0) __hip_atomic_store(fail_flag, flag_value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
            }
        }
        if (lane == 0) {
            // (withhold_first: test aid; tile 0 keeps its word back, so the tile after it must give up its wait)
            if (!(withhold_first && blockIdx.x == 0))
            __hip_atomic_store(&status[blockIdx.x], scan_pack(prefix + total, SCAN_PREFIX), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            prefix_sh = prefix;
            if (base + ETILE >= n_pad) {      // the last tile holds the totals
                const int64_t all = prefix + total;
                const int32_t nnz = (int32_t)(all & 0xffffffffll), n_new = (int32_t)(all >> 32);
                indptr[n_dst] = nnz;
                counts[1] = n_dst + n_new;
                counts[2] = nnz;
            }
        }
    }
    __syncthreads();
    run += prefix_sh;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) {
        const int64_t q = q0 + t;
        if (q < n_pad) {
            const int32_t e = (int32_t)(run & 0xffffffffll);
            const int32_t row = k == 1 ? (int32_t)q : (int32_t)__umul64hi((uint64_t)q, k_magic);   // q / k, exact
            if (q - (int64_t)row * k == 0) indptr[row] = e;
            if (f[t] & 1) {
                nbr[e] = u[t];
                edge_row[e] = row;
                if (f[t] >> 32) {
                    const int32_t local = n_dst + (int32_t)(run >> 32);
                    src_global[local] = u[t];
                    map[u[t]] = local;     // only the first occurrence writes; later readers never match n_dst + q
                }
            }
            run += f[t];
        }
    }
    // A wait that expired leaves wrong prefixes behind, and kernels after this one would follow them out of their
    // arrays. The tile that finishes last therefore checks the flag and, if it is raised, turns the hop into a
    // consistent empty block: no edges, no new sources, and no entry of this hop left in the id map.
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int n_tiles = (unsigned int)((n_pad + ETILE - 1) / ETILE);
        const bool last = __hip_atomic_fetch_add(done, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == n_tiles - 1;
        cleanup_sh = last && __hip_atomic_load(fail_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == flag_value;
    }
    __syncthreads();
    if (cleanup_sh) {
        for (int64_t q = threadIdx.x; q < n_pad; q += ETHREADS) {
            const int32_t v = nbr_pad[q];
            if (v >= 0 && map[v] >= n_dst) map[v] = EMPTY;      // (entries below n_dst belong to the destinations)
        }
        for (int32_t r = (int32_t)threadIdx.x; r <= n_dst; r += ETHREADS) indptr[r] = 0;
        if (threadIdx.x == 0) { counts[1] = n_dst; counts[2] = 0; }
    }
}

// ---------------------------------------------------------------------------- 4. local indices (+ transpose)

__global__ void edge_indices_kernel(const int32_t* d_nnz, const int32_t* __restrict__ nbr, const int32_t* __restrict__ map,
                                    int32_t* __restrict__ indices, int32_t* csc_cnt) {
    const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= *d_nnz) return;
    const int32_t local = map[nbr[e]];
    indices[e] = local;
    if (csc_cnt) atomicAdd(&csc_cnt[local], 1);     // integer count: order independent
}

__global__ void csc_fill_kernel(const int32_t* d_nnz, const int32_t* __restrict__ indices,
                                const int32_t* __restrict__ csc_indptr, int32_t* cursor, int32_t* __restrict__ unordered) {
    const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= *d_nnz) return;
    const int32_t u = indices[e];
    unordered[csc_indptr[u] + atomicAdd(&cursor[u], 1)] = e;
}

// Every edge finds its rank among the edges of its column; columns are short (a source is sampled by
// few destinations), so the quadratic work is small and needs no sort network or shared memory.
__global__ void csc_rank_kernel(const int32_t* d_nnz, const int32_t* __restrict__ indices,
                                const int32_t* __restrict__ csc_indptr, const int32_t* __restrict__ unordered,
                                const int32_t* __restrict__ edge_row, int32_t* __restrict__ csc_eid,
                                int32_t* __restrict__ csc_dst) {
    const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= *d_nnz) return;
    const int32_t u = indices[e];
    const int32_t b = csc_indptr[u], len = csc_indptr[u + 1] - b;
    int32_t r = 0;
    if (len > 1) {
        const int32_t* col = unordered + b;
        int32_t t = 0;
        for (; t + 8 <= len; t += 8) {       // independent loads: eight compares in flight
            const int32_t x0 = col[t], x1 = col[t + 1], x2 = col[t + 2], x3 = col[t + 3];
            const int32_t x4 = col[t + 4], x5 = col[t + 5], x6 = col[t + 6], x7 = col[t + 7];
            r += (x0 < e) + (x1 < e) + (x2 < e) + (x3 < e) + (x4 < e) + (x5 < e) + (x6 < e) + (x7 < e);
        }
        for (; t < len; ++t) r += col[t] < e ? 1 : 0;
    }
    csc_eid[b + r] = e;
    csc_dst[b + r] = edge_row[e];
}

__global__ void map_wipe_kernel(const int32_t* src_global, const int32_t* d_n_src, int32_t* map) {
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < *d_n_src) map[src_global[i]] = EMPTY;
}

// ---------------------------------------------------------------------------- hot lookup on V^1

struct CacheProbe {
    const int32_t* v1;
    const int32_t* slot_of_vertex;
    const int32_t* version;
    int64_t step;
    int32_t staleness;
    // low word: 1 if the row must be computed; high word: 1 if it is computed AND hot (it will refresh its slot)
    __device__ __forceinline__ int64_t flags(int32_t slot, int32_t ver) const {
        if (slot < 0) return 1;
        const bool hit = ver >= 0 && step - (int64_t)ver <= (int64_t)staleness;
        return hit ? 0 : (1ll + (1ll << 32));
    }
};

// Blocks [0, v1_blocks) probe the cache for a tile of V^1; the remaining blocks write the local indices of
// the hop above (one edge per thread), which must be read out of the id map before the partition re-keys it:
// sharing the launch keeps that pass off the dependency chain of the sampling.
__global__ void __launch_bounds__(ETHREADS) v1_tile_sums_kernel(CacheProbe probe, const int32_t* d_n_v1, int64_t* tile_sums,
                                                                int32_t* __restrict__ probe_slot /* [n]: slot if served from the cache; -1 cold; -2 - slot if hot but to be computed */,
                                                                int32_t* __restrict__ probe_ver /* [n]: the version the probe read (hot vertices) */,
                                                                uint32_t v1_blocks, const int32_t* d_nnz,
                                                                const int32_t* __restrict__ nbr, const int32_t* map,
                                                                int32_t* __restrict__ indices, int32_t* csc_cnt) {
    if (blockIdx.x >= v1_blocks) {
        const int32_t e = (int32_t)((blockIdx.x - v1_blocks) * ETHREADS + threadIdx.x);
        if (e >= *d_nnz) return;
        const int32_t local = map[nbr[e]];
        indices[e] = local;
        if (csc_cnt) atomicAdd(&csc_cnt[local], 1);     // integer count: order independent
        return;
    }
    const int64_t n = *d_n_v1;
    const int64_t base = (int64_t)blockIdx.x * ETILE;
    if (base >= n) return;
    __shared__ int64_t smem[ETHREADS / 64];
    const int64_t i0 = base + (int64_t)threadIdx.x * EITEMS;
    // three dependent loads per vertex; each level is issued for all items before the next is needed
    int32_t v[EITEMS], slot[EITEMS], ver[EITEMS];
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) v[t] = i0 + t < n ? probe.v1[i0 + t] : -1;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) slot[t] = v[t] >= 0 ? probe.slot_of_vertex[v[t]] : -1;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) ver[t] = slot[t] >= 0 ? probe.version[slot[t]] : -1;
    int64_t s = 0;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) {
        if (i0 + t < n) {
            const int64_t f = probe.flags(slot[t], ver[t]);
            probe_slot[i0 + t] = (f & 1) ? (slot[t] >= 0 ? -2 - slot[t] : -1) : slot[t];
            probe_ver[i0 + t] = ver[t];
            s += f;
        }
    }
    s = block_sum<int64_t, ETHREADS>(s, smem);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = s;
}

// Stable split of V^1 into rows to compute and rows served from the cache; re-keys the id map for
// the bottom hop (computed vertex -> its index in the compute list, reusable vertex -> no entry).
__global__ void __launch_bounds__(ETHREADS) v1_partition_kernel(const int32_t* __restrict__ v1, const int32_t* __restrict__ probe_slot,
                                                                const int32_t* __restrict__ probe_ver,
                                                                const int32_t* d_n_v1,
                                                                const int64_t* __restrict__ tile_sums, int32_t* map,
                                                                int32_t* compute_list, int32_t* compute_pos, int32_t* compute_inv,
                                                                int32_t* refresh_slot, int32_t* hit_pos,
                                                                int32_t* hit_slot, int32_t* extra /* n_compute, n_hit, -, -, n_refresh */,
                                                                int32_t* version, int32_t stamp, int32_t* refresh_old) {
    // version != NULL: the slot of a hot vertex that will be recomputed is stamped with the step right here (the row
    // itself arrives with the step's layer-1 product), so that the split of the next batch depends on this split only
    // and not on that product; the version it replaces is kept, in case the batch is never trained on.
    __shared__ int64_t smem[ETHREADS / 64 + 1];
    const int64_t n = *d_n_v1;
    const int64_t n_tiles = (n + ETILE - 1) / ETILE;
    if (blockIdx.x == 0) {
        int64_t s = 0;
        for (int64_t t = threadIdx.x; t < n_tiles; t += ETHREADS) s += tile_sums[t];
        s = block_sum<int64_t, ETHREADS>(s, smem);
        if (threadIdx.x == 0) {
            const int32_t n_compute = (int32_t)(s & 0xffffffffll);
            extra[0] = n_compute;
            extra[1] = (int32_t)n - n_compute;
            extra[4] = (int32_t)(s >> 32);
        }
    }
    const int64_t base = (int64_t)blockIdx.x * ETILE;
    if (base >= n) return;
    int64_t tile_off = 0;
    {
        int64_t s = 0;
        for (int64_t t = threadIdx.x; t < (int64_t)blockIdx.x; t += ETHREADS) s += tile_sums[t] & 0xffffffffll;
        tile_off = block_sum<int64_t, ETHREADS>(s, smem);
    }
    const int64_t i0 = base + (int64_t)threadIdx.x * EITEMS;
    int32_t c[EITEMS], slot[EITEMS], vv[EITEMS], pv[EITEMS];
    int64_t s = 0;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) {
        c[t] = 0;
        slot[t] = -1;
        vv[t] = 0;
        pv[t] = -1;
        if (i0 + t < n) { slot[t] = probe_slot[i0 + t]; vv[t] = v1[i0 + t]; pv[t] = probe_ver[i0 + t]; c[t] = slot[t] < 0 ? 1 : 0; }
        s += c[t];
    }
    int64_t total;
    int64_t run = block_exclusive_scan<int64_t, ETHREADS>(s, &total, smem) + tile_off;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) {
        const int64_t i = i0 + t;
        if (i < n) {
            const int32_t v = vv[t];
            if (c[t]) {
                compute_pos[run] = (int32_t)i;
                compute_inv[i] = (int32_t)run;
                const int32_t rslot = slot[t] <= -2 ? -2 - slot[t] : -1;
                refresh_slot[run] = rslot;
                if (version && rslot >= 0) {
                    refresh_old[run] = pv[t];      // (what the probe read: nothing writes the versions in between)
                    version[rslot] = stamp;
                }
                compute_list[run] = v;
                map[v] = (int32_t)run;
            } else {
                const int64_t p = i - run;
                hit_pos[p] = (int32_t)i;
                compute_inv[i] = -1;
                hit_slot[p] = slot[t];
                map[v] = EMPTY;
            }
            run += c[t];
        }
    }
}

// One-launch form of the two kernels above (a single-pass scan like edge_scan_kernel, with the same status words,
// emptied by the sampling launch of the hop above, and the same bounded waits): a block probes the cache for its tile,
// publishes the tile's counts, adds up the tiles before it and writes its part of the split from the probe results it
// still holds in registers. The first idx_blocks blocks write the local indices of the hop above out of the id map;
// the split re-keys that map, so every tile block waits, before its map writes, until a counter says that all index
// blocks with work have read (they come first in index order and take two round trips, the probe takes four: the
// wait is there for correctness, not because it is ever long).
__global__ void __launch_bounds__(ETHREADS) v1_split_kernel(CacheProbe probe, const int32_t* d_n_v1, unsigned long long* status,
                                                            uint32_t idx_blocks, const int32_t* d_nnz,
                                                            const int32_t* __restrict__ nbr, int32_t* map,
                                                            int32_t* __restrict__ indices, int32_t* csc_cnt,
                                                            unsigned int* idx_done, int32_t* compute_list,
                                                            int32_t* compute_pos, int32_t* compute_inv, int32_t* refresh_slot,
                                                            int32_t* hit_pos, int32_t* hit_slot,
                                                            int32_t* extra /* n_compute, n_hit, -, -, n_refresh */,
                                                            int32_t* version, int32_t stamp, int32_t* refresh_old,
                                                            int32_t* fail_flag, int32_t flag_value, int32_t spin_limit,
                                                            int32_t withhold_first, unsigned int* done, int32_t csc_len,
                                                            int32_t* above_nnz, int32_t* above_indptr,
                                                            const int32_t* above_n_dst) {
    if (blockIdx.x < idx_blocks) {
        const int64_t e = (int64_t)blockIdx.x * ETHREADS + threadIdx.x;
        const int32_t nnz = *d_nnz;
        if ((int64_t)blockIdx.x * ETHREADS >= nnz) return;      // (whole block: no work, no signal)
        if (e < nnz) {
            const int32_t local = map[nbr[e]];
            indices[e] = local;
            // (the range check only matters after an expired wait, when the split may have re-keyed the map already)
            if (csc_cnt && (uint32_t)local < (uint32_t)csc_len) atomicAdd(&csc_cnt[local], 1);     // integer count: order independent
        }
        __syncthreads();      // every map read of the block has returned (its value went into a store)
        if (threadIdx.x == 0) __hip_atomic_fetch_add(idx_done, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    const uint32_t tile = blockIdx.x - idx_blocks;
    __shared__ int64_t smem[ETHREADS / 64 + 1];
    __shared__ int64_t prefix_sh;
    __shared__ int cleanup_sh;
    const int64_t n = *d_n_v1;
    const int64_t base = (int64_t)tile * ETILE;
    if (base >= n) return;
    const int64_t i0 = base + (int64_t)threadIdx.x * EITEMS;
    // three dependent loads per vertex; each level is issued for all items before the next is needed
    int32_t v[EITEMS], slot[EITEMS], ver[EITEMS];
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) v[t] = i0 + t < n ? probe.v1[i0 + t] : -1;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) slot[t] = v[t] >= 0 ? probe.slot_of_vertex[v[t]] : -1;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) ver[t] = slot[t] >= 0 ? probe.version[slot[t]] : -1;
    int64_t f[EITEMS];
    int64_t s = 0;
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) {
        f[t] = i0 + t < n ? probe.flags(slot[t], ver[t]) : 0;
        s += f[t];
    }
    int64_t total;
    int64_t run = block_exclusive_scan<int64_t, ETHREADS>(s, &total, smem);
    if (threadIdx.x < 64) {
        const int lane = (int)threadIdx.x;
        int64_t prefix = 0;
        if (tile > 0) {
            if (lane == 0)
                __hip_atomic_store(&status[tile], scan_pack(total, SCAN_SUM), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int64_t first = (int64_t)tile - 1;
            int spins = 0;
            while (first >= 0) {
                const int64_t j = first - lane;
                unsigned long long w = SCAN_PREFIX << 62;
                if (j >= 0) w = __hip_atomic_load(&status[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const unsigned long long state = w >> 62;
                const unsigned long long is_prefix = __ballot(state == SCAN_PREFIX), is_empty = __ballot(state == 0ull);
                const int n_ok = is_empty ? __builtin_ctzll(is_empty) : 64;
                const int p_at = is_prefix ? __builtin_ctzll(is_prefix) : 64;
                const int take = p_at < n_ok ? p_at + 1 : n_ok;
                int64_t val = lane < take ? scan_unpack(w) : 0;
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) val += __shfl_xor(val, o, 64);
                prefix += val;
                first -= take;
                if (p_at < n_ok) break;
                if (take == 0) {
                    if (++spins > spin_limit) {
                        if (lane == 0) __hip_atomic_store(fail_flag, flag_value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
            }
        }
        if (lane == 0) {
            if (!(withhold_first && tile == 0))
            __hip_atomic_store(&status[tile], scan_pack(prefix + total, SCAN_PREFIX), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            prefix_sh = prefix;
            if (base + ETILE >= n) {      // the last tile holds the totals
                const int64_t all = prefix + total;
                const int32_t n_compute = (int32_t)(all & 0xffffffffll);
                extra[0] = n_compute;
                extra[1] = (int32_t)n - n_compute;
                extra[4] = (int32_t)(all >> 32);
            }
        }
    }
    if (threadIdx.x == 0) {
        const int32_t nnz = *d_nnz;
        const unsigned int expected = (unsigned int)((nnz + ETHREADS - 1) / ETHREADS);
        int spins = 0;
        while (__hip_atomic_load(idx_done, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < expected) {
            if (++spins > spin_limit) { __hip_atomic_store(fail_flag, flag_value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break; }
            __builtin_amdgcn_s_sleep(1);
        }
    }
    __syncthreads();
    run = (run & 0xffffffffll) + (prefix_sh & 0xffffffffll);
#pragma unroll
    for (int t = 0; t < EITEMS; ++t) {
        const int64_t i = i0 + t;
        if (i < n) {
            const int32_t c = (int32_t)(f[t] & 1);
            if (c) {
                compute_pos[run] = (int32_t)i;
                compute_inv[i] = (int32_t)run;
                const int32_t rslot = slot[t] >= 0 ? slot[t] : -1;       // hot but to be computed
                refresh_slot[run] = rslot;
                if (version && rslot >= 0) {
                    refresh_old[run] = ver[t];
                    version[rslot] = stamp;
                }
                compute_list[run] = v[t];
                map[v[t]] = (int32_t)run;
            } else {
                const int64_t p = i - run;
                hit_pos[p] = (int32_t)i;
                compute_inv[i] = -1;
                hit_slot[p] = slot[t];
                map[v[t]] = EMPTY;
            }
            run += c;
        }
    }
    // After an expired wait the split (and possibly the local indices of the hop above, if the map was re-keyed under
    // their readers) cannot be trusted. The tile that finishes last then leaves a consistent state that no later
    // kernel can follow out of its arrays: nothing to compute, nothing reused, no edges in the hop above, and no
    // entry of V^1 left in the id map. (Versions already stamped stay stamped: the caller is told to invalidate.)
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int n_tiles = (unsigned int)((n + ETILE - 1) / ETILE);
        const bool last = __hip_atomic_fetch_add(done, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == n_tiles - 1;
        cleanup_sh = last && __hip_atomic_load(fail_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == flag_value;
    }
    __syncthreads();
    if (cleanup_sh) {
        for (int64_t i = threadIdx.x; i < n; i += ETHREADS) map[probe.v1[i]] = EMPTY;
        const int32_t nd = *above_n_dst;
        for (int32_t r = (int32_t)threadIdx.x; r <= nd; r += ETHREADS) above_indptr[r] = 0;
        if (threadIdx.x == 0) { extra[0] = 0; extra[1] = 0; extra[4] = 0; *above_nnz = 0; }
    }
}

__global__ void set_counts_kernel(int32_t* p, int32_t a, int32_t b, int32_t c) { p[0] = a; p[1] = b; p[4] = c; }

// Takes back the stamps of a split whose batch is not trained on.
__global__ void unstamp_kernel(const int32_t* __restrict__ refresh_slot, const int32_t* __restrict__ refresh_old,
                               const int32_t* d_n_compute, int32_t n_cap, int32_t* version) {
    const int32_t n = min(*d_n_compute, n_cap);
    for (int32_t i = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x); i < n; i += (int32_t)(gridDim.x * blockDim.x)) {
        const int32_t slot = refresh_slot[i];
        if (slot >= 0) version[slot] = refresh_old[i];
    }
}

// ---------------------------------------------------------------------------- host side

static inline int64_t edge_tiles(int64_t n_pad_cap) { int64_t t = ceil_div(n_pad_cap, ETILE); return t < 1 ? 1 : t; }
// does this hop count the edges that leave each source (for its transpose, or for the symmetric normalisation)?
static inline bool counts_sources(const no_blocks_s* b, const HopBuffers& H) { return H.has_csc || b->count_sources; }

template <typename RowT>
static int32_t sample_hop(const RowT* rowptr, const int32_t* col, no_blocks_s* b, int32_t h, const int32_t* d_dst,
                          const int32_t* d_n_dst_in, int32_t n_fixed, bool insert_dst, uint32_t key0, uint32_t key1,
                          uint32_t domain, hipStream_t st, bool indices_now, int32_t extra_status = 0) {
    HopBuffers& H = b->hop[h];
    int32_t* cnt = b->counts.p + 4 * h;              // n_dst, n_src, nnz
    const int32_t k = H.fanout;
    const int T = 256;
    H.d_dst = d_dst;
    H.d_n_dst = cnt;
    int64_t* tile_sums = (int64_t*)b->ws.p;
    const uint32_t c3 = (domain << 8) | (uint32_t)h;
    int32_t* seeds_copy = (h == 0) ? b->seeds.p : nullptr;
    hipEvent_t tev0 = nullptr, tev1 = nullptr;
    if (b->time_hop == h && b->time_ev0) { tev0 = b->time_ev0; tev1 = b->time_ev1; b->time_ev0 = b->time_ev1 = nullptr; b->time_hop = -1; }
#define NO_LAUNCH_SAMPLE(G)                                                                                            \
    NO_LAUNCH_TIMED((sample_rows_kernel<G, RowT>), dim3((unsigned)ceil_div(H.n_dst_cap, 256 / G)), dim3(256), st, tev0, tev1, \
                       rowptr, col, d_dst, d_n_dst_in, n_fixed, H.n_dst_cap, k, key0, key1, c3, H.nbr_pad.p,               \
                       H.src_global.p, b->map.p, insert_dst ? 1 : 0, seeds_copy, cnt, (int32_t)b->n_vertices,               \
                       b->counts.p + 4 * b->n_layers + 5, b->call_id, (unsigned long long*)b->ws.p,                          \
                       (int32_t)edge_tiles(H.nnz_cap) + 1 + extra_status)
    if (k <= 8) NO_LAUNCH_SAMPLE(8);
    else if (k <= 16) NO_LAUNCH_SAMPLE(16);
    else if (k <= 32) NO_LAUNCH_SAMPLE(32);
    else NO_LAUNCH_SAMPLE(64);
#undef NO_LAUNCH_SAMPLE
    const unsigned tiles = (unsigned)edge_tiles(H.nnz_cap);
    const uint64_t k_magic = k > 1 ? (~0ull / (uint64_t)k) + 1ull : 0ull;     // ceil(2^64 / k)
    // One launch where the sampling has the chip to itself or nearly so; two where it runs beside another batch's
    // products (sampling ahead): there the single-pass blocks, which wait on their predecessors while holding a slot,
    // measured slower than two short launches.
    const bool two_pass = b->scan_two_pass;
    const ScanWaitDebug dbg = scan_wait_debug();
    if (two_pass) {
        hipLaunchKernelGGL(edge_tile_sums_kernel, dim3(tiles), dim3(ETHREADS), 0, st, H.nbr_pad.p,
                           (const int32_t*)b->map.p, (const int32_t*)cnt, k, tile_sums, H.csc_cnt.p, H.csc_cur.p,
                           counts_sources(b, H) ? H.n_src_cap + 1 : 0);
        hipLaunchKernelGGL(edge_assign_kernel, dim3(tiles), dim3(ETHREADS), 0, st, (const int32_t*)H.nbr_pad.p, b->map.p,
                           (const int32_t*)cnt, k, k_magic, (const int64_t*)tile_sums, H.indptr.p, H.nbr_global.p, H.edge_row.p,
                           H.src_global.p, cnt);
    } else {
        hipLaunchKernelGGL(edge_scan_kernel, dim3(tiles), dim3(ETHREADS), 0, st, (const int32_t*)H.nbr_pad.p, b->map.p,
                           (const int32_t*)cnt, k, k_magic, (unsigned long long*)b->ws.p, H.indptr.p, H.nbr_global.p,
                           H.edge_row.p, H.src_global.p, cnt, H.csc_cnt.p, H.csc_cur.p, counts_sources(b, H) ? H.n_src_cap + 1 : 0,
                           b->counts.p + 4 * b->n_layers + 6, b->call_id, dbg.spin_limit, dbg.withhold_first_tile,
                           (unsigned int*)((unsigned long long*)b->ws.p + tiles));
    }
    if (indices_now)
        hipLaunchKernelGGL(edge_indices_kernel, dim3((unsigned)ceil_div(H.nnz_cap, T)), dim3(T), 0, st,
                           (const int32_t*)(cnt + 2), (const int32_t*)H.nbr_global.p, (const int32_t*)b->map.p, H.indices.p,
                           counts_sources(b, H) ? H.csc_cnt.p : nullptr);
    return launch_status("sample_hop");
}

// Work that nothing on the caller's stream needs before the join, queued on the side stream behind ONE
// fork event recorded after the last hop's ids are final: the local indices of the hops that do not have
// them yet (the bottom layer aggregates through the global ids; a vertex keeps its local id from the hop
// that first saw it, so the map still answers for the hops above unless the cache split re-keyed it),
// the transposes of the upper hops, and the wipe of the id map.
static int32_t launch_side_work(no_blocks_s* b, int32_t n_hops, const int32_t* d_n_src_last, hipStream_t st,
                                const SideGather* gather, const bool* indices_done) {
    const int T = 256;
    hipStream_t sd = b->side;
    NO_HIP_CHECK(hipEventRecord(b->ev_fork[0], st));
    NO_HIP_CHECK(hipStreamWaitEvent(sd, b->ev_fork[0], 0));
    // the dense copy of the bottom destinations' rows goes first when the forward pass waits for it, else last
    // (then it runs next to the matrix products instead of next to the bandwidth-bound aggregation)
    auto copy_rows = [&]() -> int32_t {
        const HopBuffers& lastg = b->hop[n_hops - 1];
        NO_CHECK(gather_rows(gather->table, gather->row_bytes, gather->row_bytes, lastg.src_global.p,
                             b->counts.p + 4 * (n_hops - 1), lastg.n_dst_cap, gather->out, gather->row_bytes, sd));
        NO_HIP_CHECK(hipEventRecord(b->ev_gather_done, sd));
        return NO_OK;
    };
    const bool have_copy = gather && gather->table;
    if (have_copy && gather->needed_by_forward) NO_CHECK(copy_rows());
    // local indices first: the forward pass of the layers above the bottom one aggregates through them, so it
    // waits for ev_indices_done (not for the whole side stream) when they were left to this stream
    b->upper_indices_deferred = false;
    for (int32_t h = 0; h < n_hops; ++h) {
        HopBuffers& H = b->hop[h];
        int32_t* cnt = b->counts.p + 4 * h;
        if (indices_done[h]) continue;
        hipLaunchKernelGGL(edge_indices_kernel, dim3((unsigned)ceil_div(H.nnz_cap, T)), dim3(T), 0, sd,
                           (const int32_t*)(cnt + 2), (const int32_t*)H.nbr_global.p, (const int32_t*)b->map.p,
                           H.indices.p, counts_sources(b, H) ? H.csc_cnt.p : nullptr);
        if (h < n_hops - 1) b->upper_indices_deferred = true;
    }
    NO_HIP_CHECK(hipEventRecord(b->ev_indices_done, sd));
    for (int32_t h = 0; h < n_hops; ++h) {
        HopBuffers& H = b->hop[h];
        int32_t* cnt = b->counts.p + 4 * h;
        if (!H.has_csc) continue;
        NO_CHECK(exclusive_scan2(ArrayLoader{H.csc_cnt.p}, cnt + 1, H.n_src_cap, H.csc_indptr.p, nullptr, b->ws_side.p, sd));
        hipLaunchKernelGGL(csc_fill_kernel, dim3((unsigned)ceil_div(H.nnz_cap, T)), dim3(T), 0, sd, (const int32_t*)(cnt + 2),
                           (const int32_t*)H.indices.p, (const int32_t*)H.csc_indptr.p, H.csc_cur.p, b->tmp_a.p);
        hipLaunchKernelGGL(csc_rank_kernel, dim3((unsigned)ceil_div(H.nnz_cap, T)), dim3(T), 0, sd, (const int32_t*)(cnt + 2),
                           (const int32_t*)H.indices.p, (const int32_t*)H.csc_indptr.p, (const int32_t*)b->tmp_a.p,
                           (const int32_t*)H.edge_row.p, H.csc_eid.p, H.csc_dst.p);
    }
    HopBuffers& last = b->hop[n_hops - 1];
    hipLaunchKernelGGL(map_wipe_kernel, dim3((unsigned)ceil_div(last.n_src_cap, T)), dim3(T), 0, sd,
                       (const int32_t*)last.src_global.p, d_n_src_last, b->map.p);
    if (have_copy && !gather->needed_by_forward) NO_CHECK(copy_rows());
    b->side_pending = true;
    return launch_status("side work");
}

int32_t blocks_join(no_blocks_s* b, hipStream_t st) {
    if (!b->side_pending) return NO_OK;
    NO_HIP_CHECK(hipEventRecord(b->ev_side_done, b->side));
    NO_HIP_CHECK(hipStreamWaitEvent(st, b->ev_side_done, 0));
    b->side_pending = false;
    return NO_OK;
}

// One launch for the V^1 split where the sampling has the chip to itself, two launches where it runs beside another
// batch's products, as for the edge compaction and for the same reason (measured on a V^1 of five tiles: sampling alone
// 72 -> 68 us in one launch, but 2 % fewer steps per second when sampling ahead).
static bool v1_one_launch(const no_blocks_s* b, unsigned tiles) {
    (void)tiles;
    return !b->scan_two_pass;
}

int32_t sample_blocks_impl(no_graph_s* g, const int32_t* d_seeds, int32_t n_seeds, uint64_t stream_key, uint32_t domain,
                           int32_t n_hops, no_cache_s* cache, int64_t step, no_blocks_s* b, hipStream_t st, bool join,
                           const SideGather* gather, bool stamp_refresh) {
    NO_CHECK(blocks_join(b, st));      // a previous call that was never joined
    b->stamped_cache = nullptr;
    b->call_id = b->call_id % 0x3fffffff + 1;      // flag words written by this call's kernels carry this value
    const int32_t L = b->n_layers;
    int32_t* extra = b->counts.p + 4 * L;     // n_compute, n_hit, -, -, n_refresh
    const uint32_t key0 = (uint32_t)stream_key, key1 = (uint32_t)(stream_key >> 32);
    const int32_t* d_dst = d_seeds;
    const int32_t* d_n = nullptr;
    const bool use_cache = cache != nullptr && L >= 2 && n_hops == L && cache->n_hot > 0;
    b->last_used_cache = use_cache;
    bool indices_done[NO_MAX_LAYERS] = {};
    for (int32_t h = 0; h < n_hops; ++h) {
        if (h == L - 1 && use_cache) {
            // split V^1 (= sources of hop L-2) into reusable rows and rows to compute; the same launch writes
            // hop L-2's local indices, which the re-keyed map could no longer give
            HopBuffers& P = b->hop[h - 1];
            CacheProbe probe{d_dst, cache->slot_of_vertex.p, cache->version.p, step, cache->staleness};
            const unsigned tiles = (unsigned)edge_tiles(P.n_src_cap);
            const unsigned idx_blocks = (unsigned)ceil_div(P.nnz_cap, ETHREADS);
            int64_t* tile_sums = (int64_t*)b->ws.p;
            if (v1_one_launch(b, tiles)) {
                const ScanWaitDebug dbg = scan_wait_debug();
                // (status words and the counter behind them: emptied by the sampling launch of hop L-2, past its own)
                // (word edge_tiles(P.nnz_cap) is the completion counter of hop L-2's edge scan)
                unsigned long long* v1_status = (unsigned long long*)b->ws.p + edge_tiles(P.nnz_cap) + 1;
                hipLaunchKernelGGL(v1_split_kernel, dim3(idx_blocks + tiles), dim3(ETHREADS), 0, st, probe, d_n, v1_status,
                                   idx_blocks, (const int32_t*)(b->counts.p + 4 * (h - 1) + 2), (const int32_t*)P.nbr_global.p,
                                   b->map.p, P.indices.p, counts_sources(b, P) ? P.csc_cnt.p : nullptr, (unsigned int*)(v1_status + tiles),
                                   b->compute_list.p, b->compute_pos.p, b->compute_inv.p, b->refresh_slot.p, b->hit_pos.p,
                                   b->hit_slot.p, extra, stamp_refresh ? cache->version.p : nullptr, (int32_t)step,
                                   b->refresh_old.p, b->counts.p + 4 * b->n_layers + 6, b->call_id, dbg.spin_limit,
                                   dbg.withhold_first_tile, (unsigned int*)(v1_status + tiles + 1), P.n_src_cap + 1,
                                   b->counts.p + 4 * (h - 1) + 2, P.indptr.p, (const int32_t*)(b->counts.p + 4 * (h - 1)));
            } else {
            hipLaunchKernelGGL(v1_tile_sums_kernel, dim3(tiles + idx_blocks), dim3(ETHREADS), 0, st, probe, d_n, tile_sums,
                               b->probe_slot.p, b->probe_ver.p, tiles, (const int32_t*)(b->counts.p + 4 * (h - 1) + 2),
                               (const int32_t*)P.nbr_global.p, (const int32_t*)b->map.p, P.indices.p,
                               counts_sources(b, P) ? P.csc_cnt.p : nullptr);
            indices_done[h - 1] = true;
            hipLaunchKernelGGL(v1_partition_kernel, dim3(tiles), dim3(ETHREADS), 0, st, d_dst,
                               (const int32_t*)b->probe_slot.p, (const int32_t*)b->probe_ver.p, d_n, (const int64_t*)tile_sums, b->map.p, b->compute_list.p, b->compute_pos.p, b->compute_inv.p, b->refresh_slot.p, b->hit_pos.p,
                               b->hit_slot.p, extra, stamp_refresh ? cache->version.p : nullptr, (int32_t)step,
                               b->refresh_old.p);
            }
            indices_done[h - 1] = true;
            b->stamped_cache = stamp_refresh ? cache : nullptr;
            b->stamped_uid = cache->uid;
            b->stamped_contents = cache->contents;
            d_dst = b->compute_list.p;
            d_n = extra + 0;
        }
        // with the cache split ahead, the hops above L-2 read the map before the split re-keys it; every other
        // hop's indices wait for the side stream
        const bool indices_now = use_cache && h < L - 2;
        // the hop above the bottom one also empties the status words of the V^1 split that follows it
        const int32_t extra_status = (use_cache && h == L - 2 && v1_one_launch(b, (unsigned)edge_tiles(b->hop[h].n_src_cap)))
                                         ? (int32_t)edge_tiles(b->hop[h].n_src_cap) + 2 : 0;
        if (g->rowptr_bits == 64)
            NO_CHECK(sample_hop<int64_t>(g->rowptr64.p, g->col.p, b, h, d_dst, d_n, n_seeds, h == 0, key0, key1, domain, st,
                                         indices_now, extra_status));
        else
            NO_CHECK(sample_hop<int32_t>(g->rowptr32.p, g->col.p, b, h, d_dst, d_n, n_seeds, h == 0, key0, key1, domain, st,
                                         indices_now, extra_status));
        if (indices_now) indices_done[h] = true;
        d_dst = b->hop[h].src_global.p;
        d_n = b->counts.p + 4 * h + 1;
    }
    if (!use_cache) hipLaunchKernelGGL(set_counts_kernel, dim3(1), dim3(1), 0, st, extra, 0, 0, 0);
    NO_CHECK(launch_side_work(b, n_hops, d_n, st, gather, indices_done));
    NO_CHECK(launch_status("sample_blocks"));
    if (join) NO_CHECK(blocks_join(b, st));
    return NO_OK;
}

int32_t blocks_unstamp(no_blocks_s* b, hipStream_t st) {
    if (!b->stamped_cache) return NO_OK;
    // nothing to restore when the cache was destroyed since (its address may already name another cache), or when all
    // its versions were replaced (refresh commit: the stamps sit in the copy that is now the pending one; invalidate)
    if (!cache_is_live(b->stamped_cache) || b->stamped_cache->uid != b->stamped_uid ||
        b->stamped_cache->contents != b->stamped_contents) {
        b->stamped_cache = nullptr;
        return NO_OK;
    }
    const int32_t L = b->n_layers;
    const int32_t cap = b->hop[L - 1].n_dst_cap;
    hipLaunchKernelGGL(unstamp_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(cap, 256), 1024)), dim3(256), 0, st,
                       (const int32_t*)b->refresh_slot.p, (const int32_t*)b->refresh_old.p, (const int32_t*)(b->counts.p + 4 * L), cap,
                       b->stamped_cache->version.p);
    b->stamped_cache = nullptr;
    return launch_status("blocks_unstamp");
}

int32_t blocks_create_impl(no_graph_s* g, int32_t n_seeds_cap, const int32_t* fanouts, int32_t n_layers,
                           bool build_csc, no_blocks_s** out) {
    *out = nullptr;
    no_blocks_s* b = new no_blocks_s();
    struct Guard { no_blocks_s* b; ~Guard() { if (b) { b->release(); delete b; } } } guard{b};
    b->n_layers = n_layers;
    b->n_seeds_cap = n_seeds_cap;
    b->n_vertices = g->n_vertices;
    b->build_csc = build_csc;
    int64_t dst_cap = n_seeds_cap;
    int64_t max_pad = 1, max_sort = 1, max_src = 1;
    for (int32_t h = 0; h < n_layers; ++h) {
        HopBuffers& H = b->hop[h];
        int64_t nnz_cap = dst_cap * fanouts[h];
        int64_t src_cap = dst_cap + nnz_cap;
        if (src_cap > g->n_vertices) src_cap = g->n_vertices;
        NO_REQUIRE(nnz_cap + dst_cap < (1ll << 31) - 1, NO_ERR_OVERFLOW, "blocks: hop %d capacity exceeds int32", h);
        H.fanout = fanouts[h];
        H.n_dst_cap = (int32_t)dst_cap;
        H.nnz_cap = (int32_t)nnz_cap;
        H.n_src_cap = (int32_t)src_cap;
        H.has_csc = build_csc && h < n_layers - 1;
        NO_CHECK(H.src_global.alloc((size_t)src_cap));
        NO_CHECK(H.indptr.alloc((size_t)dst_cap + 1));
        NO_CHECK(H.nbr_pad.alloc((size_t)nnz_cap));
        NO_CHECK(H.nbr_global.alloc((size_t)nnz_cap));
        NO_CHECK(H.indices.alloc((size_t)nnz_cap));
        NO_CHECK(H.edge_row.alloc((size_t)nnz_cap));
        NO_CHECK(H.csc_cnt.alloc((size_t)src_cap + 1));       // (every hop: the bottom hop's counts serve the symmetric
        NO_CHECK(H.csc_cur.alloc((size_t)src_cap + 1));       //  normalisation; the two arrays are emptied together)
        if (H.has_csc) {
            NO_CHECK(H.csc_indptr.alloc((size_t)src_cap + 1));
            NO_CHECK(H.csc_dst.alloc((size_t)nnz_cap));
            NO_CHECK(H.csc_eid.alloc((size_t)nnz_cap));
            if (nnz_cap > max_sort) max_sort = nnz_cap;
        }
        if (nnz_cap > max_pad) max_pad = nnz_cap;
        if (src_cap > max_src) max_src = src_cap;
        dst_cap = src_cap;
    }
    NO_CHECK(b->counts.alloc((size_t)4 * n_layers + 8));
    NO_HIP_CHECK(hipMemset(b->counts.p, 0, ((size_t)4 * n_layers + 8) * 4));
    NO_CHECK(b->seeds.alloc((size_t)n_seeds_cap));
    NO_CHECK(b->map.alloc((size_t)g->n_vertices));
    NO_CHECK(fill_i32(b->map.p, EMPTY, g->n_vertices, nullptr));
    NO_CHECK(b->tmp_a.alloc((size_t)max_sort));
    const int64_t max_items = max_pad > max_src ? max_pad : max_src;
    NO_CHECK(b->ws.alloc((size_t)(2 * edge_tiles(max_items + 1) + 8) * sizeof(int64_t)));      // two sets of status words and their counters
    NO_CHECK(b->ws_side.alloc((size_t)(edge_tiles(max_items + 1) + 2) * sizeof(int64_t)));
    NO_HIP_CHECK(hipStreamCreateWithFlags(&b->side, hipStreamNonBlocking));
    for (int32_t h = 0; h < n_layers; ++h) NO_HIP_CHECK(hipEventCreateWithFlags(&b->ev_fork[h], NO_SYNC_EVENT_FLAGS));
    NO_HIP_CHECK(hipEventCreateWithFlags(&b->ev_side_done, NO_SYNC_EVENT_FLAGS));
    NO_HIP_CHECK(hipEventCreateWithFlags(&b->ev_gather_done, NO_SYNC_EVENT_FLAGS));
    NO_HIP_CHECK(hipEventCreateWithFlags(&b->ev_indices_done, NO_SYNC_EVENT_FLAGS));
    if (n_layers >= 2) {
        size_t v1_cap = (size_t)b->hop[n_layers - 2].n_src_cap;
        NO_CHECK(b->compute_list.alloc(v1_cap));
        NO_CHECK(b->compute_pos.alloc(v1_cap));
        NO_CHECK(b->compute_inv.alloc(v1_cap));
        NO_CHECK(b->refresh_slot.alloc(v1_cap));
        NO_CHECK(b->refresh_old.alloc(v1_cap));
        NO_CHECK(b->hit_pos.alloc(v1_cap));
        NO_CHECK(b->hit_slot.alloc(v1_cap));
        NO_CHECK(b->probe_slot.alloc(v1_cap));
        NO_CHECK(b->probe_ver.alloc(v1_cap));
    }
    NO_HIP_CHECK(hipDeviceSynchronize());
    guard.b = nullptr;
    *out = b;
    return NO_OK;
}

void fill_block_view(const no_blocks_s* b, int32_t h, no_block_view* v) {
    const HopBuffers& H = b->hop[h];
    const int32_t* cnt = b->counts.p + 4 * h;
    const int32_t* extra = b->counts.p + 4 * b->n_layers;
    v->n_dst_cap = H.n_dst_cap;
    v->n_src_cap = H.n_src_cap;
    v->nnz_cap = H.nnz_cap;
    v->d_n_dst = cnt;
    v->d_n_src = cnt + 1;
    v->d_nnz = cnt + 2;
    v->d_dst_global = H.src_global.p;     // the first n_dst sources are the destinations
    v->d_src_global = H.src_global.p;
    v->d_indptr = H.indptr.p;
    v->d_nbr_global = H.nbr_global.p;
    v->d_indices = H.indices.p;
    v->d_csc_indptr = H.has_csc ? H.csc_indptr.p : nullptr;
    v->d_csc_dst = H.has_csc ? H.csc_dst.p : nullptr;
    v->d_csc_eid = H.has_csc ? H.csc_eid.p : nullptr;
    const bool bottom_cached = (h == b->n_layers - 1) && b->last_used_cache;
    v->d_compute_pos = bottom_cached ? b->compute_pos.p : nullptr;
    v->d_hit_pos = bottom_cached ? b->hit_pos.p : nullptr;
    v->d_hit_slot = bottom_cached ? b->hit_slot.p : nullptr;
    v->d_n_compute = bottom_cached ? extra + 0 : nullptr;
    v->d_n_hit = bottom_cached ? extra + 1 : nullptr;
}

}  // namespace no

using namespace no;

static int32_t check_fanouts(const int32_t* f, int32_t n_layers, const char* who) {
    NO_REQUIRE(f != nullptr, NO_ERR_INVALID_ARG, "%s: fanouts is NULL", who);
    NO_REQUIRE(n_layers >= 1 && n_layers <= NO_MAX_LAYERS, NO_ERR_INVALID_ARG, "%s: n_layers must be in [1, %d]", who,
               NO_MAX_LAYERS);
    for (int32_t h = 0; h < n_layers; ++h)
        NO_REQUIRE(f[h] >= 1 && f[h] <= NO_MAX_FANOUT, NO_ERR_INVALID_ARG, "%s: fanout[%d] must be in [1, %d]", who, h,
                   NO_MAX_FANOUT);
    return NO_OK;
}

extern "C" int32_t no_blocks_create(no_graph_t g, int32_t n_seeds_cap, const int32_t* h_fanouts, int32_t n_layers,
                                    no_blocks_t* out) {
    clear_error();
    NO_REQUIRE(out != nullptr, NO_ERR_INVALID_ARG, "no_blocks_create: out is NULL");
    *out = nullptr;
    NO_REQUIRE(g != nullptr, NO_ERR_INVALID_ARG, "no_blocks_create: graph is NULL");
    NO_REQUIRE(n_seeds_cap >= 1, NO_ERR_INVALID_ARG, "no_blocks_create: n_seeds_cap must be positive");
    NO_REQUIRE(n_seeds_cap <= g->n_vertices, NO_ERR_INVALID_ARG, "no_blocks_create: more seeds than vertices");
    NO_CHECK(check_fanouts(h_fanouts, n_layers, "no_blocks_create"));
    return blocks_create_impl(g, n_seeds_cap, h_fanouts, n_layers, true, out);
}

extern "C" int32_t no_sample_blocks(no_graph_t g, const int32_t* d_seeds, int32_t n_seeds, uint64_t seed, int64_t step,
                                    no_cache_t cache, no_blocks_t blocks, void* stream) {
    clear_error();
    NO_REQUIRE(g && blocks && d_seeds, NO_ERR_INVALID_ARG, "no_sample_blocks: NULL argument");
    NO_REQUIRE(n_seeds >= 1, NO_ERR_INVALID_ARG, "no_sample_blocks: n_seeds must be positive");
    NO_REQUIRE(n_seeds <= blocks->n_seeds_cap, NO_ERR_CAPACITY, "no_sample_blocks: %d seeds exceed the capacity %d",
               n_seeds, blocks->n_seeds_cap);
    NO_REQUIRE(blocks->n_vertices == g->n_vertices, NO_ERR_INVALID_ARG, "no_sample_blocks: blocks belong to another graph");
    NO_REQUIRE(step >= 0, NO_ERR_INVALID_ARG, "no_sample_blocks: step must be >= 0");
    NO_REQUIRE(!cache || cache->n_vertices == g->n_vertices, NO_ERR_INVALID_ARG,
               "no_sample_blocks: cache belongs to another graph");
    return sample_blocks_impl(g, d_seeds, n_seeds, seed + (uint64_t)step, 0u, blocks->n_layers, cache, step, blocks,
                              (hipStream_t)stream);
}

extern "C" int32_t no_blocks_view(no_blocks_t blocks, int32_t hop, no_block_view* out) {
    clear_error();
    NO_REQUIRE(blocks && out, NO_ERR_INVALID_ARG, "no_blocks_view: NULL argument");
    NO_REQUIRE(hop >= 0 && hop < blocks->n_layers, NO_ERR_INVALID_ARG, "no_blocks_view: hop out of range");
    fill_block_view(blocks, hop, out);
    return NO_OK;
}

extern "C" int32_t no_blocks_sizes(no_blocks_t blocks, void* stream, int32_t* h_sizes) {
    clear_error();
    NO_REQUIRE(blocks && h_sizes, NO_ERR_INVALID_ARG, "no_blocks_sizes: NULL argument");
    const int32_t L = blocks->n_layers;
    int32_t tmp[4 * NO_MAX_LAYERS + 8];
    NO_HIP_CHECK(hipMemcpyAsync(tmp, blocks->counts.p, ((size_t)4 * L + 8) * 4, hipMemcpyDeviceToHost, (hipStream_t)stream));
    NO_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
    for (int32_t h = 0; h < L; ++h) {
        h_sizes[4 * h + 0] = tmp[4 * h + 0];
        h_sizes[4 * h + 1] = tmp[4 * h + 1];
        h_sizes[4 * h + 2] = tmp[4 * h + 2];
        h_sizes[4 * h + 3] = (h == L - 1 && blocks->last_used_cache) ? tmp[4 * L + 1] : 0;
    }
    const int32_t id = blocks->call_id;
    NO_REQUIRE(id == 0 || tmp[4 * L + 6] != id, NO_ERR_TIMEOUT,
               "no_blocks_sizes: a scan of the last sampling call gave up waiting for an earlier tile; the blocks are invalid");
    NO_REQUIRE(id == 0 || tmp[4 * L + 5] != id, NO_ERR_OUT_OF_RANGE,
               "no_blocks_sizes: the last sampling call met a seed id outside [0, V) (read as vertex 0)");
    return NO_OK;
}

namespace no {
static ScanWaitDebug g_scan_wait_debug{1 << 20, 0};
ScanWaitDebug scan_wait_debug() { return g_scan_wait_debug; }
}  // namespace no

extern "C" int32_t no_debug_scan_wait(int32_t spin_limit, int32_t withhold_first_tile) {
    clear_error();
    NO_REQUIRE(spin_limit >= 0, NO_ERR_INVALID_ARG, "no_debug_scan_wait: spin_limit must be >= 0");
    g_scan_wait_debug.spin_limit = spin_limit > 0 ? spin_limit : (1 << 20);
    g_scan_wait_debug.withhold_first_tile = withhold_first_tile ? 1 : 0;
    return NO_OK;
}

extern "C" int32_t no_blocks_destroy(no_blocks_t blocks) {
    clear_error();
    if (!blocks) return NO_OK;
    blocks->release();
    delete blocks;
    return NO_OK;
}
