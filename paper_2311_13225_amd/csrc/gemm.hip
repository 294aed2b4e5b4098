// LDS-tiled fp32 MFMA matrix products (see gemm.hpp). Block tile 128x128x32, 256 threads =
// 4 wavefronts, each owning a 64x64 sub-tile as 2x2 v_mfma_f32_32x32x2_f32 accumulators.
//
// Operand tiles sit in LDS in one of two layouts, chosen by how the operand lies in memory:
//   KC (reduction index contiguous in memory): T[x][k], pitch 36 floats; a lane fetches the four
//       k values it needs for four consecutive MFMAs with one 16-byte LDS read, conflict free.
//   XC (tile row/column index contiguous): T[k][x], pitch 128; four 4-byte LDS reads.
// Within each group of 8 reduction indices lanes 0-31 take indices 0-3 and lanes 32-63 take 4-7
// for MFMA 0-3; both operands use the same assignment, so every index is summed exactly once.
#include "gemm.hpp"

namespace no {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int PITCH_KC = 36, PITCH_XC = 128;
constexpr int TILE_FLOATS = 128 * PITCH_KC;   // >= 32 * PITCH_XC

__device__ __forceinline__ float4 load4(const float* p, int valid, int align) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (valid >= 4) {
        if (align == 4) v = *reinterpret_cast<const float4*>(p);
        else if (align == 2) {
            float2 a = *reinterpret_cast<const float2*>(p), b = *reinterpret_cast<const float2*>(p + 2);
            v = make_float4(a.x, a.y, b.x, b.y);
        } else v = make_float4(p[0], p[1], p[2], p[3]);
    } else {
        if (valid > 0) v.x = p[0];
        if (valid > 1) v.y = p[1];
        if (valid > 2) v.z = p[2];
    }
    return v;
}

// Global -> registers for one 128 x 32 operand tile. x = tile row/column index, k = reduction index.
template <bool KC>
__device__ __forceinline__ void tile_fetch(float4 (&reg)[4], const float* src, int64_t ld, int x0, int x_lim, int k0,
                                           int k_lim, int align) {
    const int tid = (int)threadIdx.x;
    if (KC) {
        const int kq = tid & 7, xr = tid >> 3;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int gx = x0 + xr + 32 * pass, gk = k0 + kq * 4;
            int valid = gx < x_lim ? k_lim - gk : 0;
            reg[pass] = valid > 0 ? load4(src + (int64_t)gx * ld + gk, valid, align) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    } else {
        const int xq = tid & 31, kr = tid >> 5;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int gk = k0 + kr + 8 * pass, gx = x0 + xq * 4;
            int valid = gk < k_lim ? x_lim - gx : 0;
            reg[pass] = valid > 0 ? load4(src + (int64_t)gk * ld + gx, valid, align) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
}

template <bool KC>
__device__ __forceinline__ void tile_store(const float4 (&reg)[4], float* S) {
    const int tid = (int)threadIdx.x;
    if (KC) {
        const int kq = tid & 7, xr = tid >> 3;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass)
            *reinterpret_cast<float4*>(&S[(xr + 32 * pass) * PITCH_KC + kq * 4]) = reg[pass];
    } else {
        const int xq = tid & 31, kr = tid >> 5;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass)
            *reinterpret_cast<float4*>(&S[(kr + 8 * pass) * PITCH_XC + xq * 4]) = reg[pass];
    }
}

// The four reduction values (chunk of 8, this lane's half) of tile row/column x.
template <bool KC>
__device__ __forceinline__ float4 tile_frag(const float* S, int x, int chunk, int half) {
    if (KC) return *reinterpret_cast<const float4*>(&S[x * PITCH_KC + chunk * 8 + half * 4]);
    const float* p = &S[(chunk * 8 + half * 4) * PITCH_XC + x];
    return make_float4(p[0], p[PITCH_XC], p[2 * PITCH_XC], p[3 * PITCH_XC]);
}

template <bool A_KC, bool B_KC>
__device__ __forceinline__ void tile_mma(const float* As, const float* Bs, floatx16 (&acc)[2][2], int wm, int wn) {
    const int lane = (int)(threadIdx.x & 63);
    const int half = lane >> 5, l32 = lane & 31;
#pragma unroll
    for (int chunk = 0; chunk < BK / 8; ++chunk) {
        float4 a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            a[i] = tile_frag<A_KC>(As, wm * 64 + i * 32 + l32, chunk, half);
            b[i] = tile_frag<B_KC>(Bs, wn * 64 + i * 32 + l32, chunk, half);
        }
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mi].x, b[ni].x, acc[mi][ni], 0, 0, 0);
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mi].y, b[ni].y, acc[mi][ni], 0, 0, 0);
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mi].z, b[ni].z, acc[mi][ni], 0, 0, 0);
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mi].w, b[ni].w, acc[mi][ni], 0, 0, 0);
            }
    }
}

// Accumulator element r of lane: row = 8*(r/4) + 4*(lane/32) + r%4, column = lane%32 of the 32x32 tile.
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// ------------------------------------------------------------------------------------------ NN

template <bool B_KC>
__global__ void __launch_bounds__(256) gemm_nn_kernel(GemmNNArgs g) {
    __shared__ __attribute__((aligned(16))) float As[TILE_FLOATS];
    __shared__ __attribute__((aligned(16))) float Bs[TILE_FLOATS];
    int M = *g.d_M;
    if (M > g.M_cap) M = g.M_cap;
    const int m0 = (int)blockIdx.y * BM, n0 = (int)blockIdx.x * BN;
    if (m0 >= M) return;
    const int prob = g.accumulate ? 0 : (int)blockIdx.z;
    const int n_phases = g.accumulate ? g.n_problems : 1;
    const int wave = (int)(threadIdx.x >> 6), wm = wave >> 1, wn = wave & 1;
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    for (int ph = 0; ph < n_phases; ++ph) {
        const int q = g.accumulate ? ph : prob;
        const float* A = g.A[q];
        const float* B = g.B[q];
        const int64_t lda = g.lda[q], ldb = g.ldb[q];
        const int K = g.K[q], aal = g.a_align[q], bal = g.b_align[q];
        float4 ra[4], rb[4];
        tile_fetch<true>(ra, A, lda, m0, M, 0, K, aal);
        tile_fetch<B_KC>(rb, B, ldb, n0, g.N, 0, K, bal);
        for (int k0 = 0; k0 < K; k0 += BK) {
            __syncthreads();
            tile_store<true>(ra, As);
            tile_store<B_KC>(rb, Bs);
            __syncthreads();
            if (k0 + BK < K) {
                tile_fetch<true>(ra, A, lda, m0, M, k0 + BK, K, aal);
                tile_fetch<B_KC>(rb, B, ldb, n0, g.N, k0 + BK, K, bal);
            }
            tile_mma<true, B_KC>(As, Bs, acc, wm, wn);
        }
    }
    const int lane = (int)(threadIdx.x & 63);
    float* C = g.C[prob];
    const int64_t ldc = g.ldc[prob];
    const int32_t* sp = g.row_scale_indptr[prob];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = m0 + wm * 64 + mi * 32 + acc_row(r, lane);
            if (row >= M) continue;
            float scale = 1.f;
            if (sp) { int len = sp[row + 1] - sp[row]; scale = len > 0 ? 1.f / (float)len : 0.f; }
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                const int col = n0 + wn * 64 + ni * 32 + (lane & 31);
                if (col >= g.N) continue;
                float v = acc[mi][ni][r];
                if (g.bias) v += g.bias[col];
                if (g.relu) v = v > 0.f ? v : 0.f;
                C[(int64_t)row * ldc + col] = v * scale;
            }
        }
}

int32_t gemm_nn(const GemmNNArgs& a, bool b_transposed, hipStream_t st) {
    dim3 grid((unsigned)ceil_div(a.N, BN), (unsigned)ceil_div(a.M_cap, BM), (unsigned)(a.accumulate ? 1 : a.n_problems));
    if (a.M_cap <= 0 || a.N <= 0) return NO_OK;
    if (b_transposed) hipLaunchKernelGGL(gemm_nn_kernel<true>, grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(gemm_nn_kernel<false>, grid, dim3(256), 0, st, a);
    return launch_status("gemm_nn");
}

// ------------------------------------------------------------------------------------------ TN

__global__ void __launch_bounds__(256) gemm_tn_kernel(GemmTNArgs g) {
    __shared__ __attribute__((aligned(16))) float As[TILE_FLOATS];
    __shared__ __attribute__((aligned(16))) float Bs[TILE_FLOATS];
    int R = *g.d_R;
    if (R > g.R_cap) R = g.R_cap;
    const int prob = (int)blockIdx.z / g.splits, split = (int)blockIdx.z % g.splits;
    int chunk = (R + g.splits - 1) / g.splits;
    chunk = (chunk + BK - 1) / BK * BK;
    const int r0 = split * chunk;
    const int r1 = min(R, r0 + chunk);
    const int m0 = (int)blockIdx.y * BM, n0 = (int)blockIdx.x * BN;
    const int wave = (int)(threadIdx.x >> 6), wm = wave >> 1, wn = wave & 1;
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    const float* A = g.A[prob];
    const int64_t lda = g.lda[prob];
    const int aal = g.a_align[prob];
    if (r0 < r1) {
        float4 ra[4], rb[4];
        tile_fetch<false>(ra, A, lda, m0, g.Kp, r0, r1, aal);
        tile_fetch<false>(rb, g.G, g.ldg, n0, g.N, r0, r1, g.g_align);
        for (int k0 = r0; k0 < r1; k0 += BK) {
            __syncthreads();
            tile_store<false>(ra, As);
            tile_store<false>(rb, Bs);
            __syncthreads();
            if (k0 + BK < r1) {
                tile_fetch<false>(ra, A, lda, m0, g.Kp, k0 + BK, r1, aal);
                tile_fetch<false>(rb, g.G, g.ldg, n0, g.N, k0 + BK, r1, g.g_align);
            }
            tile_mma<false, false>(As, Bs, acc, wm, wn);
        }
    }
    const int lane = (int)(threadIdx.x & 63);
    float* P = g.P + ((int64_t)prob * g.splits + split) * (int64_t)g.Kp * g.N;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = m0 + wm * 64 + mi * 32 + acc_row(r, lane);
            if (row >= g.Kp) continue;
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                const int col = n0 + wn * 64 + ni * 32 + (lane & 31);
                if (col < g.N) P[(int64_t)row * g.N + col] = acc[mi][ni][r];
            }
        }
}

int32_t gemm_tn_partials(const GemmTNArgs& a, hipStream_t st) {
    if (a.Kp <= 0 || a.N <= 0) return NO_OK;
    dim3 grid((unsigned)ceil_div(a.N, BN), (unsigned)ceil_div(a.Kp, BM), (unsigned)(2 * a.splits));
    hipLaunchKernelGGL(gemm_tn_kernel, grid, dim3(256), 0, st, a);
    return launch_status("gemm_tn");
}

struct ReduceOuts { float* p[4]; };

__global__ void reduce_partials_kernel(const float* __restrict__ P, int32_t splits, int64_t elems, ReduceOuts outs) {
    const int q = (int)blockIdx.y;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= elems) return;
    const float* p = P + (int64_t)q * splits * elems + i;
    float s = 0.f;
    for (int32_t k = 0; k < splits; ++k) s += p[(int64_t)k * elems];
    outs.p[q][i] = s;
}

int32_t reduce_partials(const float* P, int32_t n_out, int32_t splits, int64_t elems, float* const* outs, hipStream_t st) {
    if (elems <= 0 || n_out <= 0) return NO_OK;
    ReduceOuts o{};
    for (int q = 0; q < n_out && q < 4; ++q) o.p[q] = outs[q];
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)ceil_div(elems, 256), (unsigned)n_out), dim3(256), 0, st, P,
                       splits, elems, o);
    return launch_status("reduce_partials");
}

}  // namespace no
