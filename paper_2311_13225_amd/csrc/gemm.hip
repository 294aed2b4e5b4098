// LDS-tiled fp32 MFMA matrix products (see gemm.hpp). Block tile BM x BN x 32 with BM, BN in
// {64, 128}, 256 threads = 2 x 2 wavefronts, each owning a (BM/2) x (BN/2) sub-tile as
// v_mfma_f32_32x32x2_f32 accumulators. The tile shape is picked per call so that tall-skinny
// problems whose row count is a device scalar still spread over the 256 compute units.
//
// Operand tiles sit in LDS in one of two layouts, chosen by how the operand lies in memory:
//   KC (reduction index contiguous in memory): T[x][k], pitch 36 floats; a lane fetches the four
//       k values it needs for four consecutive MFMAs with one 16-byte LDS read, conflict free.
//   XC (tile row/column index contiguous): T[k][x], pitch = tile width; four 4-byte LDS reads.
// Within each group of 8 reduction indices lanes 0-31 take indices 0-3 and lanes 32-63 take 4-7
// for MFMA 0-3; both operands use the same assignment, so every index is summed exactly once.
#include "gemm.hpp"

#include <stdlib.h>

namespace no {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 32;
constexpr int PITCH_KC = 36;

template <bool KC, int BX> struct TileShape {
    static constexpr int FLOATS = KC ? BX * PITCH_KC : BK * BX;
    static constexpr int PASSES = BX / 32;
};

// 16-byte load from a 4-byte aligned address (rows of 602 floats start on 8-byte boundaries only).
typedef float float4_a4 __attribute__((ext_vector_type(4), aligned(4)));
__device__ __forceinline__ float4 load4_fast(const float* p) {
    float4_a4 v = *reinterpret_cast<const float4_a4*>(p);
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float4 load4_guarded(const float* p, int valid) {
    if (valid >= 4) return load4_fast(p);      // only the lanes that straddle an edge go element by element
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (valid > 0) v.x = p[0];
    if (valid > 1) v.y = p[1];
    if (valid > 2) v.z = p[2];
    return v;
}

// Global -> registers for one BX x 32 operand tile. x = tile row/column index, k = reduction index.
// FAST: the whole tile lies inside the operand (no guards, no branches: the hot path).
// Otherwise every element is guarded and out-of-range elements read as zero; ones_col >= 0 (XC only)
// adds a virtual column of ones at index `ones_col`, which makes row `ones_col` of the product the
// column sums of the other operand (the bias gradient).
// KC tiles take the memory row of tile row (xr + 32 * pass) from xrow[pass] (the tile row itself, or an entry
// of a row index when the operand is a set of rows of a larger table).
template <bool KC, int BX, bool FAST>
__device__ __forceinline__ void tile_fetch(float4 (&reg)[BX / 32], const float* src, int64_t ld, int x0, int x_lim, int k0,
                                           int k_lim, const int32_t (&xrow)[BX / 32], int ones_col = -1) {
    const int tid = (int)threadIdx.x;
    if (KC) {
        const int kq = tid & 7, xr = tid >> 3;
#pragma unroll
        for (int pass = 0; pass < BX / 32; ++pass) {
            const int gx = x0 + xr + 32 * pass, gk = k0 + kq * 4;
            if (FAST) reg[pass] = load4_fast(src + (int64_t)xrow[pass] * ld + gk);
            else reg[pass] = load4_guarded(src + (int64_t)xrow[pass] * ld + gk, gx < x_lim ? k_lim - gk : 0);
        }
    } else {
        constexpr int XQ = BX / 4, ROWS = 256 / XQ;
        const int xq = tid % XQ, kr = tid / XQ;
#pragma unroll
        for (int pass = 0; pass < BX / 32; ++pass) {
            const int gk = k0 + kr + ROWS * pass, gx = x0 + xq * 4;
            if (FAST) reg[pass] = load4_fast(src + (int64_t)gk * ld + gx);
            else {
                float4 v = load4_guarded(src + (int64_t)gk * ld + gx, gk < k_lim ? x_lim - gx : 0);
                if (ones_col >= 0 && gk < k_lim && ones_col >= gx && ones_col < gx + 4) {
                    const int c = ones_col - gx;
                    if (c == 0) v.x = 1.f; else if (c == 1) v.y = 1.f; else if (c == 2) v.z = 1.f; else v.w = 1.f;
                }
                reg[pass] = v;
            }
        }
    }
}

template <bool KC, int BX>
__device__ __forceinline__ void tile_store(const float4 (&reg)[BX / 32], float* S) {
    const int tid = (int)threadIdx.x;
    if (KC) {
        const int kq = tid & 7, xr = tid >> 3;
#pragma unroll
        for (int pass = 0; pass < BX / 32; ++pass)
            *reinterpret_cast<float4*>(&S[(xr + 32 * pass) * PITCH_KC + kq * 4]) = reg[pass];
    } else {
        constexpr int XQ = BX / 4, ROWS = 256 / XQ;
        const int xq = tid % XQ, kr = tid / XQ;
#pragma unroll
        for (int pass = 0; pass < BX / 32; ++pass)
            *reinterpret_cast<float4*>(&S[(kr + ROWS * pass) * BX + xq * 4]) = reg[pass];
    }
}

// The four reduction values (chunk of 8, this lane's half) of tile row/column x.
template <bool KC, int BX>
__device__ __forceinline__ float4 tile_frag(const float* S, int x, int chunk, int half) {
    if (KC) return *reinterpret_cast<const float4*>(&S[x * PITCH_KC + chunk * 8 + half * 4]);
    const float* p = &S[(chunk * 8 + half * 4) * BX + x];
    return make_float4(p[0], p[BX], p[2 * BX], p[3 * BX]);
}

// Number of independent accumulator sets per wave tile: with a single 32x32 accumulator every MFMA would
// depend on the one before it, so small wave tiles keep two sets (even / odd reduction indices) that
// are summed in the epilogue; larger tiles already interleave 2-4 accumulators.
template <int BM, int BN> struct AccSets { static constexpr int N = ((BM / 64) * (BN / 64) >= 4) ? 1 : 2; };

struct NoSideWork { __device__ __forceinline__ void operator()(int) const {} };

// side(chunk) is issued right after the MFMAs of `chunk` (4 chunks per step): the wave issues in order, so LDS stores
// and global loads placed there run while the matrix pipe works through the MFMAs just queued, instead of after the
// whole step's MFMAs have been issued.
template <bool A_KC, bool B_KC, int BM, int BN, class Side = NoSideWork>
__device__ __forceinline__ void tile_mma(const float* As, const float* Bs,
                                         floatx16 (&acc)[AccSets<BM, BN>::N][BM / 64][BN / 64], int wm, int wn,
                                         Side side = Side()) {
    constexpr int MI = BM / 64, NI = BN / 64, SETS = AccSets<BM, BN>::N;
    const int lane = (int)(threadIdx.x & 63);
    const int half = lane >> 5, l32 = lane & 31;
    // the fragments of chunk c + 1 are requested from LDS before the MFMAs of chunk c are issued, so the
    // matrix pipe is not left idle for an LDS round trip between chunks
    float4 a[2][MI], b[2][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i) a[0][i] = tile_frag<A_KC, BM>(As, wm * (BM / 2) + i * 32 + l32, 0, half);
#pragma unroll
    for (int i = 0; i < NI; ++i) b[0][i] = tile_frag<B_KC, BN>(Bs, wn * (BN / 2) + i * 32 + l32, 0, half);
#pragma unroll
    for (int chunk = 0; chunk < BK / 8; ++chunk) {
        const int cb = chunk & 1, nb = cb ^ 1;
        if (chunk + 1 < BK / 8) {
#pragma unroll
            for (int i = 0; i < MI; ++i) a[nb][i] = tile_frag<A_KC, BM>(As, wm * (BM / 2) + i * 32 + l32, chunk + 1, half);
#pragma unroll
            for (int i = 0; i < NI; ++i) b[nb][i] = tile_frag<B_KC, BN>(Bs, wn * (BN / 2) + i * 32 + l32, chunk + 1, half);
        }
        __builtin_amdgcn_sched_barrier(0);      // keep the LDS reads ahead of this chunk's MFMAs
        // index-major order: consecutive MFMAs go to different accumulators
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const int set = kk % SETS;
                    const float av = kk == 0 ? a[cb][mi].x : kk == 1 ? a[cb][mi].y : kk == 2 ? a[cb][mi].z : a[cb][mi].w;
                    const float bv = kk == 0 ? b[cb][ni].x : kk == 1 ? b[cb][ni].y : kk == 2 ? b[cb][ni].z : b[cb][ni].w;
                    acc[set][mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[set][mi][ni], 0, 0, 0);
                }
        __builtin_amdgcn_sched_barrier(0);
        side(chunk);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Accumulator element r of lane: row = 8*(r/4) + 4*(lane/32) + r%4, column = lane%32 of the 32x32 tile.
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

template <int SETS, int MI, int NI>
__device__ __forceinline__ void acc_zero(floatx16 (&acc)[SETS][MI][NI]) {
#pragma unroll
    for (int s = 0; s < SETS; ++s)
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[s][i][j][r] = 0.f;
}

// Sum of the accumulator sets for element r of tile (mi, ni).
template <int SETS, int MI, int NI>
__device__ __forceinline__ float acc_get(const floatx16 (&acc)[SETS][MI][NI], int mi, int ni, int r) {
    float v = acc[0][mi][ni][r];
    if (SETS > 1) v += acc[SETS - 1][mi][ni][r];
    return v;
}

// A block's reduction is a flat list of steps of 32 indices, possibly spanning two operand pairs
// (phases). LDS holds two copies of the operand tiles: while step t is multiplied out of one copy, the
// global loads of later steps land in registers and are stored into the other copy, so a step costs one
// barrier.
struct StepSource {
    const float* A; int64_t lda; const float* B; int64_t ldb;
    const int32_t* a_rows;   // KC layout only: tile row x of A is memory row a_rows[x] (NULL: row x)
    int k_begin, k_lim;      // reduction range of this phase
    int n_steps, n_fast;     // steps in this phase; the first n_fast lie wholly inside the reduction range
    int ones_col;            // virtual column of ones in A (XC layout only), or -1
};

// Guarded or unguarded fetch of step t of the flat list (any step; used outside the pipelined loop).
template <bool A_KC, bool B_KC, int BM, int BN>
__device__ __forceinline__ void fetch_step(float4 (&ra)[BM / 32], float4 (&rb)[BN / 32], const StepSource& p0,
                                           const StepSource& p1, int t, int am0, int a_lim, int bn0, int b_lim,
                                           const int32_t (&arow)[2][BM / 32], const int32_t (&brow)[BN / 32]) {
    const bool second = t >= p0.n_steps;
    const StepSource& p = second ? p1 : p0;
    const int s = second ? t - p0.n_steps : t;
    const int k0 = p.k_begin + s * BK;
    int32_t ar[BM / 32];
#pragma unroll
    for (int i = 0; i < BM / 32; ++i) ar[i] = second ? arow[1][i] : arow[0][i];
    if (s < p.n_fast) {
        tile_fetch<A_KC, BM, true>(ra, p.A, p.lda, am0, a_lim, k0, p.k_lim, ar);
        tile_fetch<B_KC, BN, true>(rb, p.B, p.ldb, bn0, b_lim, k0, p.k_lim, brow);
    } else {
        tile_fetch<A_KC, BM, false>(ra, p.A, p.lda, am0, a_lim, k0, p.k_lim, ar, p.ones_col);
        tile_fetch<B_KC, BN, false>(rb, p.B, p.ldb, bn0, b_lim, k0, p.k_lim, brow);
    }
}

// The steps that lie wholly inside the operands ("fast" steps: all but the last step of a phase whose length is
// no multiple of 32) run first, through a pipeline with R register stages and C = 2 G LDS copies, G being the number
// of steps between two barriers. Step f is multiplied out of copy f % C; meanwhile stage f % R, which holds step
// f + G, is stored into copy (f + G) % C and refilled with step f + G + R, so a load has R steps to arrive. A
// barrier closes every G-th step: the copies written during a group of G steps are those read in the next group,
// and those read in the previous one. With G = 2 a block meets half as many barriers, at twice the LDS.
// The loop body holds no branch around a load: every step issues the same loads (past the last pipelined step
// they re-read that step and the values are dropped), so the wait before an LDS store counts exactly the loads
// issued after the ones it needs instead of draining them all. The pipeline takes a multiple of U = lcm(C, R)
// steps (the loop is unrolled U times, since registers and LDS copies are indexed statically). The steps left over
// (up to U - 1 fast ones and the at most two guarded ones) are multiplied after the loop. Tile rows beyond the
// operand are clamped to its last row in the KC layout (their products belong to output rows that are never
// stored); in the XC layout an edge tile has no fast steps and takes the plain loop.
constexpr int lcm_small(int a, int b) { int m = a; while (m % b) m += a; return m; }

template <bool A_KC, bool B_KC, int BM, int BN, int GRP, int STG>
__device__ __forceinline__ void run_steps(StepSource p0, StepSource p1, int am0, int a_lim, int bn0, int b_lim, float* As,
                                          float* Bs, floatx16 (&acc)[AccSets<BM, BN>::N][BM / 64][BN / 64], int wm, int wn) {
    constexpr int A_FLOATS = TileShape<A_KC, BM>::FLOATS, B_FLOATS = TileShape<B_KC, BN>::FLOATS;
    constexpr int PA = BM / 32, PB = BN / 32;
    const int total_steps = p0.n_steps + p1.n_steps;
    if (total_steps <= 0) return;
    const int tid = (int)threadIdx.x;
    const bool x_fast = (A_KC || am0 + BM <= a_lim) && (B_KC || bn0 + BN <= b_lim);
    if (!x_fast) p0.n_fast = p1.n_fast = 0;
    const int F0 = p0.n_fast, F = p0.n_fast + p1.n_fast;
    // memory rows of this thread's tile rows (loop invariant; used by the KC layout only)
    int32_t arow[2][PA], brow[PB];
#pragma unroll
    for (int i = 0; i < PA; ++i) {
        const int gx = min(am0 + (tid >> 3) + 32 * i, a_lim - 1);
        arow[0][i] = (A_KC && p0.a_rows) ? p0.a_rows[gx] : gx;
        arow[1][i] = (A_KC && p1.a_rows) ? p1.a_rows[gx] : gx;
    }
#pragma unroll
    for (int i = 0; i < PB; ++i) brow[i] = min(bn0 + (tid >> 3) + 32 * i, b_lim - 1);

    if (F == 0) {
        // plain loop, one register stage, every step through the guarded fetch
        float4 ra[PA], rb[PB];
        fetch_step<A_KC, B_KC, BM, BN>(ra, rb, p0, p1, 0, am0, a_lim, bn0, b_lim, arow, brow);
        tile_store<A_KC, BM>(ra, As);
        tile_store<B_KC, BN>(rb, Bs);
        __syncthreads();
        for (int t = 0; t < total_steps; ++t) {
            const int cur = t & 1;
            const bool more = t + 1 < total_steps;
            if (more) fetch_step<A_KC, B_KC, BM, BN>(ra, rb, p0, p1, t + 1, am0, a_lim, bn0, b_lim, arow, brow);
            tile_mma<A_KC, B_KC, BM, BN>(As + cur * A_FLOATS, Bs + cur * B_FLOATS, acc, wm, wn);
            if (more) {
                tile_store<A_KC, BM>(ra, As + (cur ^ 1) * A_FLOATS);
                tile_store<B_KC, BN>(rb, Bs + (cur ^ 1) * B_FLOATS);
            }
            __syncthreads();
        }
        return;
    }

    constexpr int G = GRP, R = STG, C = 2 * G, U = lcm_small(C, R);
    const int Fp = F - F % U;
    // flat step index of leftover i: first the fast steps the pipeline does not take, then the guarded ones
    constexpr int NT = U + 1;
    const int n_left = F - Fp;
    const int g0 = p0.n_fast < p0.n_steps ? p0.n_fast : -1;
    const int g1 = p1.n_fast < p1.n_steps ? p0.n_steps + p1.n_fast : -1;
    const int n_tail = n_left + (g0 >= 0) + (g1 >= 0);
    auto tail_step = [&](int i) {
        if (i < n_left) { const int f = Fp + i; return f < F0 ? f : p0.n_steps + (f - F0); }
        if (i == n_left && g0 >= 0) return g0;
        return g1;
    };
    // per-thread load addresses of the next fast step, advanced step by step
    constexpr int XQ_A = BM / 4, ROWS_A = 256 / XQ_A, XQ_B = BN / 4, ROWS_B = 256 / XQ_B;
    const float* pa[PA];
    const float* pb[PB];
    int64_t inc_a, inc_b;
    auto point_a = [&](const StepSource& p, bool second) {
#pragma unroll
        for (int i = 0; i < PA; ++i)
            pa[i] = A_KC ? p.A + (int64_t)(second ? arow[1][i] : arow[0][i]) * p.lda + p.k_begin + (tid & 7) * 4
                         : p.A + (int64_t)(p.k_begin + tid / XQ_A + ROWS_A * i) * p.lda + am0 + (tid % XQ_A) * 4;
        inc_a = A_KC ? BK : BK * p.lda;
    };
    auto point_b = [&](const StepSource& p) {
#pragma unroll
        for (int i = 0; i < PB; ++i)
            pb[i] = B_KC ? p.B + (int64_t)brow[i] * p.ldb + p.k_begin + (tid & 7) * 4
                         : p.B + (int64_t)(p.k_begin + tid / XQ_B + ROWS_B * i) * p.ldb + bn0 + (tid % XQ_B) * 4;
        inc_b = B_KC ? BK : BK * p.ldb;
    };
    if (F0 > 0) { point_a(p0, false); point_b(p0); } else { point_a(p1, true); point_b(p1); }
    int fa = 0, fb = 0;      // fast steps whose A / B loads have been issued, less one
    auto fetch_a = [&](float4 (&r)[PA]) {
#pragma unroll
        for (int i = 0; i < PA; ++i) r[i] = load4_fast(pa[i]);
        if (fa + 1 < Fp) {
            ++fa;
            if (fa == F0) point_a(p1, true);
            else {
#pragma unroll
                for (int i = 0; i < PA; ++i) pa[i] += inc_a;
            }
        }
    };
    auto fetch_b = [&](float4 (&r)[PB]) {
#pragma unroll
        for (int i = 0; i < PB; ++i) r[i] = load4_fast(pb[i]);
        if (fb + 1 < Fp) {
            ++fb;
            if (fb == F0) point_b(p1);
            else {
#pragma unroll
                for (int i = 0; i < PB; ++i) pb[i] += inc_b;
            }
        }
    };

    float4 ra[R][PA], rb[R][PB];
    if (Fp > 0) {
        // steps 0 .. G-1 go to copies 0 .. G-1, steps G .. G+R-1 wait in stages 0 .. R-1
#pragma unroll
        for (int i = 0; i < G; ++i) {
            fetch_a(ra[0]); fetch_b(rb[0]);
            tile_store<A_KC, BM>(ra[0], As + i * A_FLOATS);
            tile_store<B_KC, BN>(rb[0], Bs + i * B_FLOATS);
        }
#pragma unroll
        for (int i = 0; i < R; ++i) { fetch_a(ra[i]); fetch_b(rb[i]); }
        __syncthreads();
        for (int f = 0; f < Fp; f += U) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int cur = u % C, nx = (u + G) % C, rs = u % R;
                // the stores and loads are issued between the MFMA groups of the current step
                tile_mma<A_KC, B_KC, BM, BN>(As + cur * A_FLOATS, Bs + cur * B_FLOATS, acc, wm, wn, [&](int chunk) {
                    if (chunk == 0) tile_store<A_KC, BM>(ra[rs], As + nx * A_FLOATS);
                    if (chunk == 1) tile_store<B_KC, BN>(rb[rs], Bs + nx * B_FLOATS);
                    if (chunk == 2) fetch_a(ra[rs]);
                    if (chunk == 3) fetch_b(rb[rs]);
                });
                if ((u + 1) % G == 0) __syncthreads();
            }
        }
    }
    // Every LDS copy is free here: the last barrier followed the last reads. Leftover i goes through copy i % C;
    // by the time copy i % C is written again (leftover i + C) C >= 2 barriers have passed since it was read.
    // (Requesting the leftovers before the loop costs registers for its whole length: measured slower.)
    float4 rta[NT][PA], rtb[NT][PB];
#pragma unroll
    for (int i = 0; i < NT; ++i)
        if (i < n_tail) fetch_step<A_KC, B_KC, BM, BN>(rta[i], rtb[i], p0, p1, tail_step(i), am0, a_lim, bn0, b_lim, arow, brow);
#pragma unroll
    for (int i = 0; i < NT; ++i)
        if (i < n_tail) {
            tile_store<A_KC, BM>(rta[i], As + (i % C) * A_FLOATS);
            tile_store<B_KC, BN>(rtb[i], Bs + (i % C) * B_FLOATS);
            __syncthreads();
            tile_mma<A_KC, B_KC, BM, BN>(As + (i % C) * A_FLOATS, Bs + (i % C) * B_FLOATS, acc, wm, wn);
        }
}

// Epilogue staging: the block's BM x BN accumulator tile goes to LDS (row pitch BN + 4 floats, over the operand
// copies, which are no longer read), so that the tile leaves as 16-byte stores along rows, four row segments per
// wavefront instruction, instead of 4-byte stores of the MFMA register layout.
template <int BM, int BN> struct OutTile {
    static constexpr int PITCH = BN + 4, QC = BN / 4, ROWS_PER_PASS = 256 / QC, PASSES = BM / ROWS_PER_PASS;
    static constexpr int FLOATS = BM * PITCH;
};
template <int BM, int BN>
__device__ __forceinline__ void acc_to_lds(float* Cs, const floatx16 (&acc)[AccSets<BM, BN>::N][BM / 64][BN / 64], int wm, int wn) {
    constexpr int MI = BM / 64, NI = BN / 64, SETS = AccSets<BM, BN>::N;
    const int lane = (int)(threadIdx.x & 63);
    __syncthreads();      // every wavefront has finished reading the operand copies
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                Cs[(wm * (BM / 2) + mi * 32 + acc_row(r, lane)) * OutTile<BM, BN>::PITCH + wn * (BN / 2) + ni * 32 + (lane & 31)] =
                    acc_get<SETS, MI, NI>(acc, mi, ni, r);
    __syncthreads();
}

// Workgroups are handed to the 8 accelerator dies (XCDs, each with its own L2) round-robin by linear
// id. The tiles that share an operand panel (all column tiles of one row tile; all tiles of one
// reduction slice) get consecutive *logical* ids, and logical ids are dealt out in chunks per XCD, so
// a panel is fetched into one L2 once instead of into several.
constexpr int N_XCD = 8;
__device__ __forceinline__ int64_t xcd_logical_id(int64_t total_padded) {
    const int64_t id = blockIdx.x;
    return (id % N_XCD) * (total_padded / N_XCD) + id / N_XCD;
}
static inline unsigned xcd_padded(int64_t total) { return (unsigned)(ceil_div(total, N_XCD) * N_XCD); }

// ------------------------------------------------------------------------------------------ NN

template <bool B_KC, int BM, int BN, int GRP = 1, int STG = 2, int OCC = 2>
__global__ void __launch_bounds__(256, OCC) gemm_nn_kernel(GemmNNArgs g) {
    constexpr int MI = BM / 64, NI = BN / 64;
    constexpr int A_TOTAL = 2 * GRP * TileShape<true, BM>::FLOATS, B_TOTAL = 2 * GRP * TileShape<B_KC, BN>::FLOATS;
    // the output tile is staged over the operand copies
    constexpr int SMEM = A_TOTAL + B_TOTAL > OutTile<BM, BN>::FLOATS ? A_TOTAL + B_TOTAL : OutTile<BM, BN>::FLOATS;
    __shared__ __attribute__((aligned(16))) float smem[SMEM];
    float* As = smem;
    float* Bs = smem + A_TOTAL;
    int M = *g.d_M;
    if (M > g.M_cap) M = g.M_cap;
    // the grid covers the row capacity; only the tiles of the actual M rows are dealt out to the XCDs
    const int gx = (g.N + BN - 1) / BN, gy = (M + BM - 1) / BM, gz = g.accumulate ? 1 : g.n_problems;
    const int64_t total = (int64_t)gx * gy * gz;
    if ((int64_t)blockIdx.x >= (total + N_XCD - 1) / N_XCD * N_XCD) return;
    const int64_t lid = xcd_logical_id((total + N_XCD - 1) / N_XCD * N_XCD);
    if (lid >= total) return;
    const int bx = (int)(lid % gx), by = (int)((lid / gx) % gy), bz = (int)(lid / ((int64_t)gx * gy));
    const int m0 = by * BM, n0 = bx * BN;
    if (m0 >= M) return;
    const int prob = g.accumulate ? 0 : bz;
    const int n_phases = g.accumulate ? g.n_problems : 1;
    const int wave = (int)(threadIdx.x >> 6), wm = wave >> 1, wn = wave & 1;
    constexpr int SETS = AccSets<BM, BN>::N;
    floatx16 acc[SETS][MI][NI];
    acc_zero<SETS, MI, NI>(acc);
    // What the epilogue needs per output row is requested here, ahead of the operands, so that it arrives behind
    // them instead of costing a memory round trip after the last product.
    using OT = OutTile<BM, BN>;
    float* C = g.C[prob];
    const int64_t ldc = g.ldc[prob];
    const int32_t* sp = g.row_scale_indptr[prob];
    const int32_t* c_rows = prob == 0 ? g.c_rows : nullptr;
    const int32_t* c_keep_rows = prob == 0 ? g.c_keep_rows : nullptr;
    const int tid = (int)threadIdx.x, cq = tid % OT::QC, tr = tid / OT::QC;
    const int col = n0 + cq * 4;
    // 16-byte stores need aligned rows; otherwise (e.g. 41 classes) the four elements go one by one
    const bool vec = (ldc % 4 == 0) && ((reinterpret_cast<uintptr_t>(C) & 15) == 0) &&
                     (!c_keep_rows || (reinterpret_cast<uintptr_t>(g.c_keep) & 15) == 0) && col + 4 <= g.N;
    // the per-row indices and scales of this thread's rows are requested before the first store waits for one of them
    int32_t crow[OT::PASSES], krow[OT::PASSES];
    float scale[OT::PASSES];
    float bias_v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) bias_v[i] = g.bias ? g.bias[min(col + i, g.N - 1)] : 0.f;
#pragma unroll
    for (int j = 0; j < OT::PASSES; ++j) {
        const int row = min(m0 + tr + OT::ROWS_PER_PASS * j, M - 1);
        crow[j] = c_rows ? c_rows[row] : row;
        krow[j] = c_keep_rows ? c_keep_rows[row] : -1;
        scale[j] = 1.f;
        if (sp) {
            const int len = sp[row + 1] - sp[row] + g.row_scale_plus;
            scale[j] = len > 0 ? (g.row_scale_rsqrt ? 1.f / sqrtf((float)len) : 1.f / (float)len) : 0.f;
        }
    }
    {
        const int q0 = g.accumulate ? 0 : prob, q1 = g.accumulate && n_phases > 1 ? 1 : q0;
        StepSource p0{g.A[q0], g.lda[q0], g.B[q0], g.ldb[q0], g.a_rows[q0], 0, g.K[q0], (g.K[q0] + BK - 1) / BK,
                      g.K[q0] / BK, -1};
        StepSource p1{g.A[q1], g.lda[q1], g.B[q1], g.ldb[q1], g.a_rows[q1], 0, g.K[q1],
                      n_phases > 1 ? (g.K[q1] + BK - 1) / BK : 0, n_phases > 1 ? g.K[q1] / BK : 0, -1};
        run_steps<true, B_KC, BM, BN, GRP, STG>(p0, p1, m0, M, n0, g.N, As, Bs, acc, wm, wn);
    }
    acc_to_lds<BM, BN>(smem, acc, wm, wn);
    // One explicit wait for every load above (vmcnt 0; the other counters left alone): the stores below sit in
    // divergent branches, and a wait placed after them would have to drain the stores as well, row after row.
    __builtin_amdgcn_s_waitcnt(0x0F70);
#pragma unroll
    for (int j = 0; j < OT::PASSES; ++j) {
        const int lr = tr + OT::ROWS_PER_PASS * j, row = m0 + lr;
        if (row >= M || col >= g.N) continue;
        const float4 t = *reinterpret_cast<const float4*>(&smem[lr * OT::PITCH + cq * 4]);
        float v[4] = {t.x + bias_v[0], t.y + bias_v[1], t.z + bias_v[2], t.w + bias_v[3]};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (g.relu) v[i] = v[i] > 0.f ? v[i] : 0.f;
            v[i] *= scale[j];
        }
        float* dst = C + (int64_t)crow[j] * ldc + col;
        float* keep = krow[j] >= 0 ? g.c_keep + (int64_t)krow[j] * ldc + col : nullptr;
        if (vec) {
            *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
            if (keep) *reinterpret_cast<float4*>(keep) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (col + i < g.N) {
                    dst[i] = v[i];
                    if (keep) keep[i] = v[i];
                }
        }
        if (keep && col == 0 && g.c_keep_stamp) g.c_keep_stamp[krow[j]] = g.stamp;
    }
}

// Small products (few output tiles, e.g. the classifier layer over the seeds and its input gradient): a block owns a 32x32 output
// tile and its four wavefronts split the reduction, chunk c of 32 indices going to wave c % 4. Operands go
// from memory straight into MFMA registers with several chunks of loads in flight, so the product takes a
// few memory round trips instead of one per 32 indices; the four partial tiles are summed in wave order
// through LDS. Out-of-range rows and columns are clamped to valid addresses and dropped at the store.
template <bool B_KC>
__global__ void __launch_bounds__(256) gemm_nn_small_kernel(GemmNNArgs g) {
    __shared__ float red[4][16][64];
    int M = *g.d_M;
    if (M > g.M_cap) M = g.M_cap;
    const int m0 = (int)blockIdx.y * 32, n0 = (int)blockIdx.x * 32;
    if (m0 >= M) return;
    const int prob = g.accumulate ? 0 : (int)blockIdx.z;
    const int n_phases = g.accumulate ? g.n_problems : 1;
    const int lane = (int)(threadIdx.x & 63), wave = (int)(threadIdx.x >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int row_c = min(m0 + l32, M - 1), col_c = min(n0 + l32, g.N - 1);
    float* C = g.C[prob];
    const int64_t ldc = g.ldc[prob];
    const int32_t* sp = g.row_scale_indptr[prob];
    const int32_t* c_rows = prob == 0 ? g.c_rows : nullptr;
    const int32_t* c_keep_rows = prob == 0 ? g.c_keep_rows : nullptr;
    int32_t crow[4], krow[4];
    float scale[4], bias_v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {       // indices and scales of this thread's four output elements, requested before the
                                        // operands so that they arrive behind them instead of after the products
        const int e = (int)threadIdx.x + 256 * i;
        const int r = e >> 6, ln = e & 63;
        const int row = min(m0 + acc_row(r, ln), M - 1), col = min(n0 + (ln & 31), g.N - 1);
        crow[i] = c_rows ? c_rows[row] : row;
        krow[i] = c_keep_rows ? c_keep_rows[row] : -1;
        bias_v[i] = g.bias ? g.bias[col] : 0.f;
        scale[i] = 1.f;
        if (sp) {
            const int len = sp[row + 1] - sp[row] + g.row_scale_plus;
            scale[i] = len > 0 ? (g.row_scale_rsqrt ? 1.f / sqrtf((float)len) : 1.f / (float)len) : 0.f;
        }
    }
    floatx16 acc, acc2;                       // two sets, so consecutive MFMAs of a round do not depend on each other
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = acc2[r] = 0.f;
    int chunk_base = 0;                       // chunks of earlier phases
    for (int ph = 0; ph < n_phases; ++ph) {
        const int q = g.accumulate ? ph : prob;
        const int K = g.K[q];
        const float* A = g.A[q] + (int64_t)(g.a_rows[q] ? g.a_rows[q][row_c] : row_c) * g.lda[q];
        const float* B = g.B[q];
        const int64_t ldb = g.ldb[q];
        const int n_chunks = (K + 31) / 32;
        // first chunk of this phase that belongs to this wave
        int c = ((wave - chunk_base) % 4 + 4) % 4;
        for (; c + 4 < n_chunks && (c + 4) * 32 + 32 <= K; c += 8) {     // two full chunks per round
            float4 av[2][4];
            float bv[2][4][4];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int sc = 0; sc < 4; ++sc) {
                    const int k = (c + 4 * u) * 32 + sc * 8 + half * 4;
                    av[u][sc] = load4_fast(A + k);
                    if (B_KC) {
                        const float4 t = load4_fast(B + (int64_t)col_c * ldb + k);
                        bv[u][sc][0] = t.x; bv[u][sc][1] = t.y; bv[u][sc][2] = t.z; bv[u][sc][3] = t.w;
                    } else {
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk) bv[u][sc][kk] = B[(int64_t)(k + kk) * ldb + col_c];
                    }
                }
#pragma unroll
            for (int sc = 0; sc < 4; ++sc) {
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[0][sc].x, bv[0][sc][0], acc, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(av[1][sc].x, bv[1][sc][0], acc2, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[0][sc].y, bv[0][sc][1], acc, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(av[1][sc].y, bv[1][sc][1], acc2, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[0][sc].z, bv[0][sc][2], acc, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(av[1][sc].z, bv[1][sc][2], acc2, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[0][sc].w, bv[0][sc][3], acc, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(av[1][sc].w, bv[1][sc][3], acc2, 0, 0, 0);
            }
        }
        for (; c < n_chunks; c += 4) {                                    // remaining chunks, guarded in k
#pragma unroll
            for (int sc = 0; sc < 4; ++sc) {
                const int k = c * 32 + sc * 8 + half * 4;
                const float4 a4 = load4_guarded(A + k, K - k);
                float b4[4];
                if (B_KC) {
                    const float4 t = load4_guarded(B + (int64_t)col_c * ldb + k, K - k);
                    b4[0] = t.x; b4[1] = t.y; b4[2] = t.z; b4[3] = t.w;
                } else {
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) b4[kk] = k + kk < K ? B[(int64_t)(k + kk) * ldb + col_c] : 0.f;
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.x, b4[0], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.y, b4[1], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.z, b4[2], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.w, b4[3], acc, 0, 0, 0);
            }
        }
        chunk_base += n_chunks;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) red[wave][r][lane] = acc[r] + acc2[r];
    __syncthreads();
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt 0: see gemm_nn_kernel
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = (int)threadIdx.x + 256 * i;
        const int r = e >> 6, ln = e & 63;
        const int row = m0 + acc_row(r, ln), col = n0 + (ln & 31);
        if (row >= M || col >= g.N) continue;
        float v = ((red[0][r][ln] + red[1][r][ln]) + red[2][r][ln]) + red[3][r][ln] + bias_v[i];
        if (g.relu) v = v > 0.f ? v : 0.f;
        C[(int64_t)crow[i] * ldc + col] = v * scale[i];
        if (krow[i] >= 0) {
            g.c_keep[(int64_t)krow[i] * ldc + col] = v * scale[i];
            if (col == 0 && g.c_keep_stamp) g.c_keep_stamp[krow[i]] = g.stamp;
        }
    }
}

// 64 x 64 tiles at every size: with the branch-free pipeline and the scattered epilogue they measured as fast as or
// faster than 64 x 128 and 128 x 64 from 8 K to 70 K rows (e.g. 27 K rows: 151 vs 165 us), and they quantise best;
// register budget for three blocks per compute unit.
template <bool B_KC>
static void launch_nn(const GemmNNArgs& a, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    const int64_t z = a.accumulate ? 1 : a.n_problems;
    dim3 grid(xcd_padded(ceil_div(a.N, 64) * ceil_div(a.M_cap, 64) * z));
    NO_LAUNCH_TIMED((gemm_nn_kernel<B_KC, 64, 64, 1, 2, 3>), grid, dim3(256), st, ev0, ev1, a);
}

int32_t gemm_nn(const GemmNNArgs& a, bool b_transposed, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    if (a.M_cap <= 0 || a.N <= 0) return NO_OK;
    const int64_t z = a.accumulate ? 1 : a.n_problems;
    if (ceil_div(a.M_cap, 64) * ceil_div(a.N, 64) * z <= 128) {
        dim3 grid((unsigned)ceil_div(a.N, 32), (unsigned)ceil_div(a.M_cap, 32), (unsigned)z);
        if (b_transposed) NO_LAUNCH_TIMED((gemm_nn_small_kernel<true>), grid, dim3(256), st, ev0, ev1, a);
        else NO_LAUNCH_TIMED((gemm_nn_small_kernel<false>), grid, dim3(256), st, ev0, ev1, a);
        return launch_status("gemm_nn_small");
    }
    if (b_transposed) launch_nn<true>(a, st, ev0, ev1);
    else launch_nn<false>(a, st, ev0, ev1);
    return launch_status("gemm_nn");
}

// ------------------------------------------------------------------------------------------ TN

// The jobs of one launch (by value in the kernel arguments): job j owns the linear block ids [end_block[j-1], end_block[j]).
struct TNLaunch { GemmTNArgs job[NO_MAX_LAYERS]; uint32_t end_block[NO_MAX_LAYERS]; int32_t n; };

template <int BM, int BN, int GRP = 1, int STG = 2, int OCC = 2>
__global__ void __launch_bounds__(256, OCC) gemm_tn_kernel(TNLaunch launch) {
    int job = 0;
    uint32_t first = 0;
    while (job + 1 < launch.n && blockIdx.x >= launch.end_block[job]) first = launch.end_block[job++];
    const GemmTNArgs& g = launch.job[job];
    constexpr int MI = BM / 64, NI = BN / 64;
    constexpr int A_TOTAL = 2 * GRP * TileShape<false, BM>::FLOATS, B_TOTAL = 2 * GRP * TileShape<false, BN>::FLOATS;
    // the output tile is staged over the operand copies
    constexpr int SMEM = A_TOTAL + B_TOTAL > OutTile<BM, BN>::FLOATS ? A_TOTAL + B_TOTAL : OutTile<BM, BN>::FLOATS;
    __shared__ __attribute__((aligned(16))) float smem[SMEM];
    float* As = smem;
    float* Bs = smem + A_TOTAL;
    int R = *g.d_R;
    if (R > g.R_cap) R = g.R_cap;
    // a job's blocks in the order of a plain 3-D grid (column tile fastest, then row tile, then problem x slice): dealing
    // the slices out per XCD measured slower here (the partial tiles are written once and the operand slices are small),
    // so the tiles of a slice stay spread over the dies
    const uint32_t id = blockIdx.x - first;
    const uint32_t gx = (uint32_t)((g.N + BN - 1) / BN), gy = (uint32_t)((g.Kp + 1 + BM - 1) / BM);
    const int bx = (int)(id % gx), by = (int)((id / gx) % gy), bz = (int)(id / (gx * gy));
    const int prob = bz / g.splits, split = bz % g.splits;
    const int used = tn_used_splits(R, g.splits, g.rows_per_split);
    if (split >= used) return;                 // (the reduction reads the first `used` partials only)
    int chunk = (R + used - 1) / used;
    chunk = (chunk + BK - 1) / BK * BK;
    const int r0 = split * chunk;
    const int r1 = min(R, r0 + chunk);
    const int m0 = by * BM, n0 = bx * BN;
    if (m0 >= g.Kp) {
        // Kp is a multiple of the tile height: this row tile holds nothing but row Kp, the column sums of G that product
        // 0 carries (the bias gradient). A tile of matrix products for one row would be a third of the launch's work at
        // Kp = 128: the sums are taken directly, in a fixed order (row r0 + i by thread group i mod 4, groups combined in
        // order). Product 1 has no such row (the reduction never reads it).
        if (prob != 0) return;
        float* red = smem;                                   // [4][BN]
        const int c = (int)(threadIdx.x % BN), part = (int)(threadIdx.x / BN);
        constexpr int PARTS = 256 / BN;
        float s = 0.f;
        if (n0 + c < g.N)
            for (int r = r0 + part; r < r1; r += PARTS) s += g.G[(int64_t)r * g.ldg + n0 + c];
        red[part * BN + c] = s;
        __syncthreads();
        if (part == 0 && n0 + c < g.N) {
            float t = red[c];
#pragma unroll
            for (int q = 1; q < PARTS; ++q) t += red[q * BN + c];
            g.P[((int64_t)prob * g.splits + split) * (int64_t)(g.Kp + 1) * g.N + (int64_t)g.Kp * g.N + n0 + c] = t;
        }
        return;
    }
    const int wave = (int)(threadIdx.x >> 6), wm = wave >> 1, wn = wave & 1;
    constexpr int SETS = AccSets<BM, BN>::N;
    floatx16 acc[SETS][MI][NI];
    acc_zero<SETS, MI, NI>(acc);
    const float* A = g.A[prob];
    const int64_t lda = g.lda[prob];
    const int ones_col = prob == 0 ? g.Kp : -1;       // product 0 carries the column sums of G in row Kp
    if (r0 < r1) {
        StepSource p0{A, lda, g.G, g.ldg, nullptr, r0, r1, (r1 - r0 + BK - 1) / BK, (r1 - r0) / BK, ones_col};
        StepSource p1 = p0;
        p1.n_steps = p1.n_fast = 0;
        run_steps<false, false, BM, BN, GRP, STG>(p0, p1, m0, g.Kp, n0, g.N, As, Bs, acc, wm, wn);
    }
    using OT = OutTile<BM, BN>;
    acc_to_lds<BM, BN>(smem, acc, wm, wn);
    const int rows_out = g.Kp + 1;
    float* P = g.P + ((int64_t)prob * g.splits + split) * (int64_t)rows_out * g.N;
    const int tid = (int)threadIdx.x, cq = tid % OT::QC, tr = tid / OT::QC;
    const int col = n0 + cq * 4;
    const bool vec = (g.N % 4 == 0) && ((reinterpret_cast<uintptr_t>(P) & 15) == 0) && col + 4 <= g.N;
#pragma unroll
    for (int j = 0; j < OT::PASSES; ++j) {
        const int lr = tr + OT::ROWS_PER_PASS * j, row = m0 + lr;
        if (row >= rows_out || col >= g.N) continue;
        const float4 t = *reinterpret_cast<const float4*>(&smem[lr * OT::PITCH + cq * 4]);
        float* dst = P + (int64_t)row * g.N + col;
        if (vec) *reinterpret_cast<float4*>(dst) = t;
        else {
            const float v[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (col + i < g.N) dst[i] = v[i];
        }
    }
}

int32_t gemm_tn_partials(const GemmTNArgs* jobs, int32_t n_jobs, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    // 64x64 tiles: the output of one split is small, so the chip is filled by many small blocks over a
    // moderate number of splits rather than by few large blocks over many splits (fewer partials to reduce).
    constexpr int bm = 64, bn = 64;
    TNLaunch launch{};
    uint64_t blocks = 0;
    for (int32_t j = 0; j < n_jobs && launch.n < NO_MAX_LAYERS; ++j) {
        const GemmTNArgs& a = jobs[j];
        if (a.Kp <= 0 || a.N <= 0) continue;
        blocks += (uint64_t)ceil_div(a.N, bn) * (uint64_t)ceil_div(a.Kp + 1, bm) * (uint64_t)(a.n_problems * a.splits);
        NO_REQUIRE(blocks < (1ull << 31), NO_ERR_CAPACITY, "gemm_tn: too many blocks");
        launch.job[launch.n] = a;
        launch.end_block[launch.n] = (uint32_t)blocks;
        ++launch.n;
    }
    if (launch.n == 0) return NO_OK;
    dim3 grid((unsigned)blocks);
    NO_LAUNCH_TIMED((gemm_tn_kernel<64, 64, 1, 2, 3>), grid, dim3(256), st, ev0, ev1, launch);
    return launch_status("gemm_tn");
}

// Sums the split partial products in split order: g_self = rows [0,Kp) of product 0, g_bias = row Kp of
// product 0, g_neigh = rows [0,Kp) of product 1. With lr != 0 the parameters take their SGD step in the
// same pass (W <- W - lr * g), after every kernel that read them.
__device__ void write_step_stats(const StatsJob& j) {
    __shared__ float sm[256];
    float s = 0.f;
    for (int i = (int)threadIdx.x; i < j.n; i += 256) s += j.row_loss[i];
    sm[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) sm[threadIdx.x] += sm[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        no_step_stats* stats = j.stats;
        const int32_t* counts = j.counts;
        const int n_layers = j.n_layers;
        stats->loss = sm[0] / (float)j.n;
        for (int h = 0; h < NO_MAX_LAYERS; ++h) {
            stats->n_dst[h] = h < n_layers ? counts[4 * h] : 0;
            stats->n_src[h] = h < n_layers ? counts[4 * h + 1] : 0;
            stats->nnz[h] = h < n_layers ? counts[4 * h + 2] : 0;
        }
        stats->n_hit = j.used_cache ? counts[4 * n_layers + 1] : 0;
        stats->n_refresh = j.used_cache ? counts[4 * n_layers + 4] : 0;
        stats->n_v1 = n_layers >= 2 ? counts[4 * (n_layers - 2) + 1] : counts[0];
        stats->bad_seed = counts[4 * n_layers + 5] == j.call_id ? 1 : 0;
        stats->scan_timeout = counts[4 * n_layers + 6] == j.call_id ? 1 : 0;
        stats->bad_label = counts[4 * n_layers + 7] == j.call_id ? 1 : 0;
        stats->n_miss_hot = stats->n_refresh;      // every computed hot vertex refreshes its slot
        stats->n_cold = stats->n_v1 - stats->n_hit - stats->n_miss_hot;
        stats->bytes_gathered_features = (int64_t)counts[4 * (n_layers - 1) + 1] * j.feat_row_bytes;
        stats->bytes_gathered_embeddings = (int64_t)stats->n_hit * j.emb_row_bytes;
    }
}

struct ReduceLaunch { ReduceArgs job[NO_MAX_LAYERS]; uint32_t end_block[NO_MAX_LAYERS]; int32_t n; };

__global__ void __launch_bounds__(256) reduce_grads_kernel(ReduceLaunch launch, StatsJob stats) {
    if (stats.stats && blockIdx.x == gridDim.x - 1) {      // the extra block of the launch
        if (blockIdx.y == 0) write_step_stats(stats);
        return;
    }
    int job = 0;
    uint32_t first = 0;
    while (job + 1 < launch.n && blockIdx.x >= launch.end_block[job]) first = launch.end_block[job++];
    const ReduceArgs& a = launch.job[job];
    const int32_t Kp = a.Kp, N = a.N;
    int32_t splits = a.splits;
    if (a.d_R) {
        int32_t R = *a.d_R;
        if (R > a.R_cap) R = a.R_cap;
        splits = tn_used_splits(R, a.splits, a.rows_per_split);
    }
    const int64_t per = (int64_t)(Kp + 1) * N;
    const int64_t i = (int64_t)(blockIdx.x - first) * blockDim.x + threadIdx.x;
    const int q = (int)blockIdx.y;
    if (i >= per || q >= a.n_problems) return;
    const bool bias_row = i >= (int64_t)Kp * N;
    if (q == 1 && bias_row) return;
    const float* p = a.P + (int64_t)q * a.splits * per + i;
    // eight partials are requested before the first add; the adds stay in split order
    float s = 0.f;
    int32_t k = 0;
    for (; k + 8 <= splits; k += 8) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = p[(int64_t)(k + j) * per];
#pragma unroll
        for (int j = 0; j < 8; ++j) s += v[j];
    }
    for (; k < splits; ++k) s += p[(int64_t)k * per];
    float* gout = bias_row ? a.g_bias + (i - (int64_t)Kp * N) : (q == 0 ? a.g_self + i : a.g_neigh + i);
    *gout = s;
    float* w = a.w_self ? (bias_row ? a.w_bias + (i - (int64_t)Kp * N) : (q == 0 ? a.w_self + i : a.w_neigh + i)) : nullptr;
    if (a.lr != 0.f && w) *w -= a.lr * s;
    if (a.wt_self && w && !bias_row) {
        // the parameter's bf16 copy for the next step's products (transposed: [N][Kpad]), round-to-nearest-even
        const uint32_t u = __float_as_uint(*w);
        const int32_t k = (int32_t)(i / N), n = (int32_t)(i - (int64_t)k * N);
        (q == 0 ? a.wt_self : a.wt_neigh)[(int64_t)n * a.Kpad + k] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
    }
}

int32_t reduce_grads(const ReduceArgs* jobs, int32_t n_jobs, hipStream_t st, const StatsJob* stats_job) {
    ReduceLaunch launch{};
    uint64_t blocks = 0;
    for (int32_t j = 0; j < n_jobs && launch.n < NO_MAX_LAYERS; ++j) {
        const ReduceArgs& a = jobs[j];
        if (a.Kp <= 0 || a.N <= 0) continue;
        blocks += (uint64_t)ceil_div((int64_t)(a.Kp + 1) * a.N, 256);
        NO_REQUIRE(blocks < (1ull << 31), NO_ERR_CAPACITY, "reduce_grads: too many blocks");
        launch.job[launch.n] = a;
        launch.end_block[launch.n] = (uint32_t)blocks;
        ++launch.n;
    }
    const StatsJob job = stats_job ? *stats_job : StatsJob{};
    if (launch.n == 0 && !job.stats) return NO_OK;
    hipLaunchKernelGGL(reduce_grads_kernel, dim3((unsigned)blocks + (job.stats ? 1u : 0u), 2u), dim3(256), 0, st, launch, job);
    return launch_status("reduce_grads");
}

}  // namespace no
