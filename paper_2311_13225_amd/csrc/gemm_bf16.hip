// The dense UPDATE of Eq. 2 for a layer fed by a bf16 feature table, and its weight gradients, with bf16 operands on
// the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation): the features are bf16 as stored, everything
// else that enters a product (the fp32 mean, the weights, the output gradient) is rounded to bf16, nearest-even, on
// its way into the product. At 16 times the fp32 matrix rate these products are bound by their operands' bytes, so
// the kernels are plain: one LDS stage per operand tile, fragments of the (small, cache-resident) weights straight
// from memory, no deep pipeline.
//   NN: C[M,N] = X[x_rows[m], 0:K] * Ws + round(Mn[m, 0:K]) * Wn + bias (ReLU, scattered rows, cache refresh rows)
//   TN: P[q][s][0:K, 0:N] = A_q[rows of slice s]^T * round(G[rows of slice s]), A_0 = X (bf16), A_1 = round(Mn);
//       row K of P[0][s] = column sums of G over the slice in fp32 (the bias gradient takes no rounding)
#include "gemm.hpp"

namespace no {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) { return f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16); }

__device__ __forceinline__ f32x16_t mfma_bf16(const uint4& a, const uint4& b, f32x16_t c) {
    bf16x8_t av, bv;
    __builtin_memcpy(&av, &a, 16);
    __builtin_memcpy(&bv, &b, 16);
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, c, 0, 0, 0);
}

// row of the 32x32 accumulator tile held in register r of lane ln (the column is ln % 32)
__device__ __forceinline__ int acc_tile_row(int r, int ln) { return 8 * (r >> 2) + 4 * (ln >> 5) + (r & 3); }

// ------------------------------------------------------------------------------------------ weights

// w fp32 [K][N] row-major -> out bf16 [N][Kpad] (k contiguous, zeros from K to Kpad): the layout in which a lane's
// eight consecutive k of one output column are 16 contiguous bytes
__global__ void weights_to_bf16_t_kernel(const float* __restrict__ w, int32_t K, int32_t N, int32_t Kpad, uint16_t* __restrict__ out) {
    const int64_t total = (int64_t)N * Kpad;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t n = (int32_t)(i / Kpad), k = (int32_t)(i - (int64_t)n * Kpad);
        out[i] = k < K ? (uint16_t)f32_to_bf16_rne(w[(int64_t)k * N + n]) : (uint16_t)0;
    }
}

int32_t weights_to_bf16_t(const float* w, int32_t K, int32_t N, int32_t Kpad, uint16_t* out, hipStream_t st) {
    int64_t blocks = ceil_div((int64_t)N * Kpad, 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(weights_to_bf16_t_kernel, dim3((unsigned)blocks), dim3(256), 0, st, w, K, N, Kpad, out);
    return launch_status("weights_to_bf16_t");
}

// ------------------------------------------------------------------------------------------ NN

constexpr int NN_BM = 64;            // rows per block (32-row blocks, twice as many, measured slower: 34 vs 28 us at 24 K rows,
                                     // each block re-reads both weight matrices)
constexpr int NN_KC = 128;           // reduction indices staged at a time
constexpr int NN_PITCH = NN_KC + 8;  // bf16 elements per LDS row (16 bytes of padding: rows start 4 banks apart)
constexpr int NN_CPITCH = 64 + 4;    // floats per LDS row of a staged output tile

// Stages rows [m0, m0 + 64) x reduction indices [k0, k0 + 128) of one operand into LDS as bf16 (zeros past K or M).
// A thread's four units are requested together (row indices, then rows) before the first is stored.
__device__ __forceinline__ void stage_rows_bf16(uint16_t* As, const uint16_t* X, int64_t ldx, const int32_t* x_rows,
                                                const float* Mn, int64_t ldm, int m0, int M, int k0, int K) {
    constexpr int UNITS = NN_KC / 8, IT = NN_BM * UNITS / 256;
    const int tid = (int)threadIdx.x;
    int r[IT], u[IT];
    bool on[IT];
#pragma unroll
    for (int i = 0; i < IT; ++i) {
        const int id = tid + 256 * i;
        r[i] = id / UNITS;
        u[i] = id % UNITS;
        on[i] = m0 + r[i] < M && k0 + u[i] * 8 < K;
    }
    if (X) {
        const bool vec = ((reinterpret_cast<uintptr_t>(X) & 15) == 0) && (ldx % 8 == 0) && (K % 8 == 0);
        int64_t src_row[IT];
#pragma unroll
        for (int i = 0; i < IT; ++i) src_row[i] = on[i] ? (int64_t)(x_rows ? x_rows[m0 + r[i]] : m0 + r[i]) : 0;
        uint4 v[IT];
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            v[i] = make_uint4(0u, 0u, 0u, 0u);
            if (!on[i]) continue;
            const int k = k0 + u[i] * 8;
            const uint16_t* src = X + src_row[i] * ldx + k;
            if (vec) v[i] = *reinterpret_cast<const uint4*>(src);
            else {
                uint16_t e[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) e[q] = k + q < K ? src[q] : (uint16_t)0;
                v[i] = make_uint4(e[0] | ((uint32_t)e[1] << 16), e[2] | ((uint32_t)e[3] << 16), e[4] | ((uint32_t)e[5] << 16),
                                  e[6] | ((uint32_t)e[7] << 16));
            }
        }
#pragma unroll
        for (int i = 0; i < IT; ++i) *reinterpret_cast<uint4*>(As + r[i] * NN_PITCH + u[i] * 8) = v[i];
    } else {
        const bool vec = ((reinterpret_cast<uintptr_t>(Mn) & 15) == 0) && (ldm % 4 == 0) && (K % 8 == 0);
        float f[IT][8];
#pragma unroll
        for (int i = 0; i < IT; ++i) {
#pragma unroll
            for (int q = 0; q < 8; ++q) f[i][q] = 0.f;
            if (!on[i]) continue;
            const int k = k0 + u[i] * 8;
            const float* src = Mn + (int64_t)(m0 + r[i]) * ldm + k;
            if (vec) {
                const float4 a = *reinterpret_cast<const float4*>(src), b = *reinterpret_cast<const float4*>(src + 4);
                f[i][0] = a.x; f[i][1] = a.y; f[i][2] = a.z; f[i][3] = a.w; f[i][4] = b.x; f[i][5] = b.y; f[i][6] = b.z; f[i][7] = b.w;
            } else {
#pragma unroll
                for (int q = 0; q < 8; ++q) f[i][q] = k + q < K ? src[q] : 0.f;
            }
        }
#pragma unroll
        for (int i = 0; i < IT; ++i)
            *reinterpret_cast<uint4*>(As + r[i] * NN_PITCH + u[i] * 8) =
                make_uint4(pack_bf16(f[i][0], f[i][1]), pack_bf16(f[i][2], f[i][3]), pack_bf16(f[i][4], f[i][5]), pack_bf16(f[i][6], f[i][7]));
    }
}

// Block: NN_BM rows x 256 columns; wavefront w owns the 64 columns [256*blockIdx.y + 64*w, +64) as tiles of 32 x 32.
__global__ void __launch_bounds__(256) gemm_bf16_nn_kernel(GemmBf16NNArgs g) {
    __shared__ __attribute__((aligned(16))) uint16_t As[NN_BM * NN_PITCH];
    __shared__ int32_t crow_sh[NN_BM], krow_sh[NN_BM];
    __shared__ __attribute__((aligned(16))) float Cs[4 * 32 * NN_CPITCH];       // per wavefront: one 32 x 64 output tile
    int M = *g.d_M;
    if (M > g.M_cap) M = g.M_cap;
    const int m0 = (int)blockIdx.x * NN_BM;
    if (m0 >= M) return;
    const int lane = (int)(threadIdx.x & 63), wave = (int)(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int c0 = ((int)blockIdx.y * 4 + wave) * 64;
    const bool wave_on = c0 < g.N;
    const int Kpad = g.Kpad;
    if (threadIdx.x < NN_BM) {
        const int row = min(m0 + (int)threadIdx.x, M - 1);
        crow_sh[threadIdx.x] = g.c_rows ? g.c_rows[row] : row;
        krow_sh[threadIdx.x] = g.c_keep_rows ? g.c_keep_rows[row] : -1;
    }
    constexpr int RT = NN_BM / 32;
    f32x16_t acc[RT][2];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    for (int phase = 0; phase < 2; ++phase) {
        const uint16_t* Wt = g.Wt[phase];
        for (int k0 = 0; k0 < g.K; k0 += NN_KC) {
            __syncthreads();          // the previous tile has been read
            stage_rows_bf16(As, phase == 0 ? g.X : nullptr, g.ldx, g.x_rows, g.Mn, g.ldm, m0, M, k0, g.K);
            // this wavefront's weight fragments for the tile, straight from memory (zeros past N; Kpad covers the tile)
            uint4 bw[NN_KC / 16][2];
#pragma unroll
            for (int ks = 0; ks < NN_KC / 16; ++ks)
#pragma unroll
                for (int ct = 0; ct < 2; ++ct) {
                    const int col = c0 + ct * 32 + l32, k = k0 + ks * 16 + half * 8;
                    bw[ks][ct] = (wave_on && col < g.N && k < Kpad) ? *reinterpret_cast<const uint4*>(Wt + (int64_t)col * Kpad + k)
                                                                     : make_uint4(0u, 0u, 0u, 0u);
                }
            __syncthreads();
            if (wave_on) {
#pragma unroll
                for (int ks = 0; ks < NN_KC / 16; ++ks) {
                    if (k0 + ks * 16 >= g.K) break;
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        const uint4 a = *reinterpret_cast<const uint4*>(As + (rt * 32 + l32) * NN_PITCH + ks * 16 + half * 8);
#pragma unroll
                        for (int ct = 0; ct < 2; ++ct) acc[rt][ct] = mfma_bf16(a, bw[ks][ct], acc[rt][ct]);
                    }
                }
            }
        }
    }
    // Epilogue: a wavefront's 32 x 64 tiles go through LDS so that a lane stores 16 contiguous bytes of an output row
    // (a quarter of the store instructions of the accumulators' own layout, whole 256-byte row segments per 16 lanes).
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        float* Ct = Cs + wave * 32 * NN_CPITCH;
        if (wave_on) {
#pragma unroll
            for (int ct = 0; ct < 2; ++ct) {
                const int col = c0 + ct * 32 + l32;
                const float bias = (g.bias && col < g.N) ? g.bias[col] : 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v = acc[rt][ct][r] + bias;
                    if (g.relu) v = fmaxf(v, 0.f);
                    Ct[acc_tile_row(r, lane) * NN_CPITCH + ct * 32 + l32] = v;
                }
            }
        }
        __syncthreads();
        if (wave_on) {
            const int c4 = (lane & 15) * 4, col = c0 + c4;
            const bool vec = (g.ldc % 4 == 0) && ((reinterpret_cast<uintptr_t>(g.C) & 15) == 0) &&
                             (!g.c_keep || (reinterpret_cast<uintptr_t>(g.c_keep) & 15) == 0) && col + 4 <= g.N;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int lr = i * 4 + (lane >> 4), row = rt * 32 + lr;
                if (m0 + row >= M || col >= g.N) continue;
                const float4 t = *reinterpret_cast<const float4*>(Ct + lr * NN_CPITCH + c4);
                float* dst = g.C + (int64_t)crow_sh[row] * g.ldc + col;
                const int kr = krow_sh[row];
                float* keep = kr >= 0 ? g.c_keep + (int64_t)kr * g.ldc + col : nullptr;
                if (vec) {
                    *reinterpret_cast<float4*>(dst) = t;
                    if (keep) *reinterpret_cast<float4*>(keep) = t;
                } else {
                    const float v[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (col + q < g.N) { dst[q] = v[q]; if (keep) keep[q] = v[q]; }
                }
            }
        }
        if (rt + 1 < RT) __syncthreads();
    }
}

int32_t gemm_bf16_nn(const GemmBf16NNArgs& a, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    if (a.M_cap <= 0 || a.N <= 0 || a.K <= 0) return NO_OK;
    dim3 grid((unsigned)ceil_div(a.M_cap, NN_BM), (unsigned)ceil_div(a.N, 256));
    NO_LAUNCH_TIMED(gemm_bf16_nn_kernel, grid, dim3(256), st, ev0, ev1, a);
    return launch_status("gemm_bf16_nn");
}

// ------------------------------------------------------------------------------------------ TN

constexpr int TN_T = 128;            // output tile: 128 rows (operand columns) ...
constexpr int TN_W = 64;             // ... x 64 columns of G (128 x 128 tiles, half as many blocks, measured slower)
constexpr int TN_RS = 32;            // slice rows staged at a time
constexpr int TN_PITCH = TN_T + 8;   // bf16 elements per LDS row (a staged slice row)

// A 32-row x 128-column tile held in registers between its request and its store to LDS.
struct TnTileRegs { uint4 raw[2]; float4 f[4]; };      // (a 128-column tile; a 64-column one uses half of f)

__device__ __forceinline__ void tn_request_bf16(TnTileRegs& t, const uint16_t* X, int64_t ldx, int rs, int r1, int c0, int C, bool vec) {
    const int tid = (int)threadIdx.x;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int id = tid + 256 * i, r = id / (TN_T / 8), u = id % (TN_T / 8);
        const int row = rs + r, c = c0 + u * 8;
        t.raw[i] = make_uint4(0u, 0u, 0u, 0u);
        if (row < r1 && c < C) {
            const uint16_t* src = X + (int64_t)row * ldx + c;
            if (vec) t.raw[i] = *reinterpret_cast<const uint4*>(src);
            else {
                uint16_t e[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) e[q] = c + q < C ? src[q] : (uint16_t)0;
                t.raw[i] = make_uint4(e[0] | ((uint32_t)e[1] << 16), e[2] | ((uint32_t)e[3] << 16), e[4] | ((uint32_t)e[5] << 16),
                                      e[6] | ((uint32_t)e[7] << 16));
            }
        }
    }
}
__device__ __forceinline__ void tn_store_bf16(const TnTileRegs& t, uint16_t* T) {
    const int tid = (int)threadIdx.x;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int id = tid + 256 * i, r = id / (TN_T / 8), u = id % (TN_T / 8);
        *reinterpret_cast<uint4*>(T + r * TN_PITCH + u * 8) = t.raw[i];
    }
}
template <int W>
__device__ __forceinline__ void tn_request_f32(TnTileRegs& t, const float* A, int64_t lda, int rs, int r1, int c0, int C, bool vec) {
    const int tid = (int)threadIdx.x;
#pragma unroll
    for (int i = 0; i < TN_RS * (W / 4) / 256; ++i) {
        const int id = tid + 256 * i, r = id / (W / 4), u = id % (W / 4);
        const int row = rs + r, c = c0 + u * 4;
        t.f[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < r1 && c < C) {
            const float* src = A + (int64_t)row * lda + c;
            if (vec) t.f[i] = *reinterpret_cast<const float4*>(src);
            else {
                t.f[i].x = src[0];
                if (c + 1 < C) t.f[i].y = src[1];
                if (c + 2 < C) t.f[i].z = src[2];
                if (c + 3 < C) t.f[i].w = src[3];
            }
        }
    }
}
template <int W>
__device__ __forceinline__ void tn_store_f32(const TnTileRegs& t, uint16_t* T) {
    const int tid = (int)threadIdx.x;
#pragma unroll
    for (int i = 0; i < TN_RS * (W / 4) / 256; ++i) {
        const int id = tid + 256 * i, r = id / (W / 4), u = id % (W / 4);
        *reinterpret_cast<uint2*>(T + r * TN_PITCH + u * 4) = make_uint2(pack_bf16(t.f[i].x, t.f[i].y), pack_bf16(t.f[i].z, t.f[i].w));
    }
}
// The matrix unit wants, per lane, eight consecutive slice rows of ONE column: a column of the staged (row-major) tile.
// Read as eight 2-byte LDS loads (two lanes share a bank word: no conflicts) and packed.
__device__ __forceinline__ uint4 tn_column_fragment(const uint16_t* T, int row0, int col) {
    uint32_t e[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) e[q] = T[(row0 + q) * TN_PITCH + col];
    return make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
}

// Block = (slice, product, 128 x 64 tile of the product), or (slice, 256 columns of the bias row).
__global__ void __launch_bounds__(256) gemm_bf16_tn_kernel(GemmBf16TNArgs g, int32_t tiles_m, int32_t tiles_n, int32_t bias_blocks) {
    __shared__ __attribute__((aligned(16))) uint16_t At[TN_RS * TN_PITCH];     // At[r][m]: slice row r, operand column m
    __shared__ __attribute__((aligned(16))) uint16_t Gt[TN_RS * TN_PITCH];     // Gt[r][n]
    int R = *g.d_R;
    if (R > g.R_cap) R = g.R_cap;
    const int per_split = 2 * tiles_m * tiles_n + bias_blocks;
    const int used = tn_used_splits(R, g.splits, g.rows_per_split);
    // The blocks of a slice (two products x tiles, and the bias row) read the same rows of G and of the operands: they
    // get consecutive logical ids, and logical ids are dealt to the eight dies in chunks (a workgroup's die is its id
    // modulo 8), so that a slice is fetched into one L2 once instead of into several.
    const int64_t total = (int64_t)used * per_split, padded = (total + 7) / 8 * 8;
    if ((int64_t)blockIdx.x >= padded) return;
    const int64_t lid = ((int64_t)blockIdx.x % 8) * (padded / 8) + (int64_t)blockIdx.x / 8;
    if (lid >= total) return;
    const int split = (int)(lid / per_split), rem = (int)(lid % per_split);
    int chunk = (R + used - 1) / used;
    chunk = (chunk + TN_RS - 1) / TN_RS * TN_RS;
    const int r0 = split * chunk, r1 = min(R, r0 + chunk);
    const int64_t per = (int64_t)(g.Kp + 1) * g.N;
    const int tid = (int)threadIdx.x;
    if (rem >= 2 * tiles_m * tiles_n) {
        // bias gradient: column sums of G over the slice, fp32, fixed order (no rounding of the addends)
        const int c = (rem - 2 * tiles_m * tiles_n) * 256 + tid;
        if (c < g.N) {
            float s = 0.f;
            int r = r0;
            for (; r + 8 <= r1; r += 8) {
                float v[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) v[q] = g.G[(int64_t)(r + q) * g.ldg + c];
#pragma unroll
                for (int q = 0; q < 8; ++q) s += v[q];
            }
            for (; r < r1; ++r) s += g.G[(int64_t)r * g.ldg + c];
            g.P[(int64_t)split * per + (int64_t)g.Kp * g.N + c] = s;
        }
        return;
    }
    const int prob = rem / (tiles_m * tiles_n), tile = rem % (tiles_m * tiles_n);
    const int mb = (tile / tiles_n) * TN_T, nb = (tile % tiles_n) * TN_W;
    const int lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
    constexpr int NJ = TN_W / 32;
    f32x16_t acc[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    const bool xvec = ((reinterpret_cast<uintptr_t>(g.X) & 15) == 0) && (g.ldx % 8 == 0) && (g.Kp % 8 == 0);
    const bool mvec = ((reinterpret_cast<uintptr_t>(g.Mn) & 15) == 0) && (g.ldm % 4 == 0) && (g.Kp % 4 == 0);
    const bool gvec = ((reinterpret_cast<uintptr_t>(g.G) & 15) == 0) && (g.ldg % 4 == 0) && (g.N % 4 == 0);
    TnTileRegs ta, tg;
    auto request = [&](int rs) {
        if (prob == 0) tn_request_bf16(ta, g.X, g.ldx, rs, r1, mb, g.Kp, xvec);
        else tn_request_f32<TN_T>(ta, g.Mn, g.ldm, rs, r1, mb, g.Kp, mvec);
        tn_request_f32<TN_W>(tg, g.G, g.ldg, rs, r1, nb, g.N, gvec);
    };
    if (r0 < r1) request(r0);
    for (int rs = r0; rs < r1; rs += TN_RS) {
        __syncthreads();                     // the previous tile pair has been read
        if (prob == 0) tn_store_bf16(ta, At); else tn_store_f32<TN_T>(ta, At);
        tn_store_f32<TN_W>(tg, Gt);
        if (rs + TN_RS < r1) request(rs + TN_RS);      // the next tile pair is in flight during the products of the current one
        __syncthreads();
        // wavefront w: operand columns [mb + 32 w, +32) against the 32-column groups of the tile
#pragma unroll
        for (int ks = 0; ks < TN_RS / 16; ++ks) {
            const uint4 a = tn_column_fragment(At, ks * 16 + half * 8, wave * 32 + l32);
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const uint4 b = tn_column_fragment(Gt, ks * 16 + half * 8, j * 32 + l32);
                acc[j] = mfma_bf16(a, b, acc[j]);
            }
        }
    }
    float* P = g.P + ((int64_t)prob * g.splits + split) * per;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int n = nb + j * 32 + l32;
        if (n >= g.N) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = mb + wave * 32 + acc_tile_row(r, lane);
            if (m < g.Kp) P[(int64_t)m * g.N + n] = acc[j][r];
        }
    }
}

int32_t gemm_bf16_tn_partials(const GemmBf16TNArgs& a, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    if (a.Kp <= 0 || a.N <= 0 || a.splits <= 0) return NO_OK;
    const int32_t tiles_m = (int32_t)ceil_div(a.Kp, TN_T), tiles_n = (int32_t)ceil_div(a.N, TN_W);
    const int32_t bias_blocks = (int32_t)ceil_div(a.N, 256);
    const int64_t blocks = ((int64_t)a.splits * (2 * tiles_m * tiles_n + bias_blocks) + 7) / 8 * 8;
    NO_REQUIRE(blocks < (1ll << 31), NO_ERR_CAPACITY, "gemm_bf16_tn: too many blocks");
    NO_LAUNCH_TIMED(gemm_bf16_tn_kernel, dim3((unsigned)blocks), dim3(256), st, ev0, ev1, a, tiles_m, tiles_n, bias_blocks);
    return launch_status("gemm_bf16_tn");
}

}  // namespace no
