// Matrix-core gradient and evaluation kernels for general shapes: any order N <= 8, any J_n <= 16 P,
// any R <= 16 P with P in {1, 2, 4} (ranks are zero-padded to 16 P).  Same method as the J = R = 16
// kernel (see ftk_kernels_mfma16.hpp for the operand layouts), with every 16 P x 16 P contraction
// cut into P x P blocks of v_mfma_f32_16x16x4_f32 and the core factors B^(n) (and their
// transposes) held in LDS instead of registers:
//
//   projections    C^T[rb] [r x sample]   = sum_jb  B^T[rb][jb] . a^T[jb]
//   A gradient     -e GS[jb] [sample x j] = sum_rb  (-e W)[rb] . B^T[rb][jb]
//   core gradient  GB[jb][rb] [j x r]    += a^T[jb] . (-e W)[rb]            (contracts the tile's samples)
//   top rows       TOP[jb] [row x j]     += ONEHOT [row x sample] . GRAD[jb] [sample x j]
//
// One wave owns 64 sampled entries at a time (four tiles of 16), draws their positions with Philox
// in registers and parks the records in a private LDS buffer.  Factor-row gradients take the same
// three routes as in the J = R = 16 kernel: rows 0..15 of a mode through the one-hot product, rows
// [16, K_n) into an LDS table per workgroup (compare-and-swap adds), all other rows through float
// atomics issued by every lane with out-of-range offsets for lanes that have nothing to add.
// The core gradient lives in matrix-core accumulators for the whole kernel and leaves each wave
// as one table of plain stores.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftk_kernels_mfma16.hpp"

namespace ftk {

struct TiledArgs {
    Coo coo;                     // records in the order the sampling rule reads them
    SampleRule rule;
    uint64_t seed;
    long long M;                 // |Psi|
    const float* A;
    const float* B;
    float* dA;                   // accumulator (synchronous mode) or A itself (in-place mode)
    long long A_off[kMaxOrder];
    int B_off[kMaxOrder];
    int J[kMaxOrder];
    int R;
    int K[kMaxOrder];            // rows [0, K[n]) of mode n live in the LDS table
    int top[kMaxOrder];          // 16 if rows 0..15 go through the one-hot product, else 0
    int hot_off[kMaxOrder];      // first LDS table row of mode n
    int H;                       // rows in the LDS table
    float* hot_partial;          // [gridDim.x][H][16 P]
    float* gb_partial;           // [gridDim.x * waves][B_total]
    int B_total;
    unsigned int mode_bytes[kMaxOrder];   // I_n * J_n * 4
    float lambda_A;
    float scale;                 // 1, or -lr_A in in-place mode
};

__host__ __device__ constexpr int tiled_wave_scratch(int order) { return (order + 1) * 64 + kTransposeFloats; }
__host__ __device__ constexpr size_t tiled_lds_floats(int order, int P, int waves, int H) {
    return (size_t)2 * order * 256 * P * P + (size_t)H * 16 * P + (size_t)waves * tiled_wave_scratch(order);
}

template <int N, int P, int WAVES>
__global__ void __launch_bounds__(WAVES * 64) grad_tiled_kernel(TiledArgs g) {
    extern __shared__ float lds[];
    constexpr int W4 = (N + 1 + 3) / 4;
    constexpr int D = 16 * P;            // padded rank
    constexpr int THREADS = WAVES * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g4 = lane >> 4;
    float* Bl = lds;                                 // [N][D][D]   Bl[n][j][r] = B^(n)[j][r] (zero padded)
    float* Bt = Bl + N * D * D;                      // [N][D][D]   Bt[n][r][j]
    float* hot = Bt + N * D * D;                     // [H][D]
    float* wave_lds = hot + (size_t)g.H * D + wave * tiled_wave_scratch(N);
    int* sidx = reinterpret_cast<int*>(wave_lds);    // [N][64]
    float* sval = wave_lds + N * 64;                 // [64]
    float* tbuf = wave_lds + (N + 1) * 64;           // [16][20]

    for (int q = tid; q < N * D * D; q += THREADS) {
        const int n = q / (D * D), rem = q - n * D * D, j = rem / D, r = rem - j * D;
        const float b = (j < g.J[n] && r < g.R) ? g.B[g.B_off[n] + j * g.R + r] : 0.0f;
        Bl[q] = b;
        Bt[n * D * D + r * D + j] = b;
    }
    for (int q = tid; q < g.H * D; q += THREADS) hot[q] = 0.0f;

    floatx4 GBacc[N][P][P];
    floatx4 Top[N][P];
#pragma unroll
    for (int n = 0; n < N; ++n)
#pragma unroll
        for (int jb = 0; jb < P; ++jb) {
            Top[n][jb] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int rb = 0; rb < P; ++rb) GBacc[n][jb][rb] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
        }
    __syncthreads();

    __amdgpu_buffer_rsrc_t rsrc_A[N], rsrc_dA[N];
#pragma unroll
    for (int n = 0; n < N; ++n) {
        rsrc_A[n] = make_rsrc(g.A + g.A_off[n], g.mode_bytes[n]);
        rsrc_dA[n] = make_rsrc(g.dA + g.A_off[n], g.mode_bytes[n]);
    }

    const long long M = g.M;
    const long long n_groups = (M + 63) / 64;
    const long long group_stride = (long long)gridDim.x * WAVES;
    const uint4* rec4 = reinterpret_cast<const uint4*>(g.coo.rec);
    auto load_record = [&](long long grp, uint4 (&rec)[W4]) {
        const long long k = grp * 64 + lane;
        const uint32_t p = k < M ? sample_place(g.seed, (uint64_t)k, g.rule) : 0u;
#pragma unroll
        for (int q = 0; q < W4; ++q) rec[q] = rec4[(size_t)p * W4 + q];
    };

    uint4 rec[W4];
    long long group = (long long)blockIdx.x * WAVES + wave;
    if (group < n_groups) load_record(group, rec);

#pragma unroll 1
    for (; group < n_groups; group += group_stride) {
        {
            const bool act = group * 64 + lane < M;
            uint32_t flat[4 * W4];
#pragma unroll
            for (int q = 0; q < W4; ++q) {
                flat[4 * q + 0] = rec[q].x;
                flat[4 * q + 1] = rec[q].y;
                flat[4 * q + 2] = rec[q].z;
                flat[4 * q + 3] = rec[q].w;
            }
#pragma unroll
            for (int n = 0; n < N; ++n) sidx[n * 64 + lane] = act ? (int)flat[n] : 0;
            sval[lane] = act ? __uint_as_float(flat[N]) : 0.0f;
        }
        lds_wave_sync();
        if (group + group_stride < n_groups) load_record(group + group_stride, rec);

#pragma unroll 1
        for (int sub = 0; sub < 4; ++sub) {
            const long long base = group * 64 + sub * 16;
            bool actY[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) actY[v] = base + 4 * g4 + v < M;

            // rows in layout Y: aY[n][jb][v] = component 16 jb + c of the row of sample 4g + v
            // (components past J_n and samples past the end of Psi read as zero: out-of-range offset)
            float aY[N][P][4];
            int iY[N][4];
            const float x = sval[sub * 16 + c];
#pragma unroll
            for (int n = 0; n < N; ++n) {
                const int4 r = *reinterpret_cast<const int4*>(sidx + n * 64 + sub * 16 + 4 * g4);
                iY[n][0] = r.x;
                iY[n][1] = r.y;
                iY[n][2] = r.z;
                iY[n][3] = r.w;
#pragma unroll
                for (int jb = 0; jb < P; ++jb) {
                    const int col = 16 * jb + c;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const bool ok = col < g.J[n] && actY[v];
                        const int off = ok ? (iY[n][v] * g.J[n] + col) * 4 : (int)g.mode_bytes[n];
                        aY[n][jb][v] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc_A[n], off, 0, 0));
                    }
                }
            }

            // projections (layout X): s[n][rb][v] = c^(n)_{r = 16 rb + 4g + v} of sample c
            floatx4 s[N][P];
#pragma unroll
            for (int n = 0; n < N; ++n) {
#pragma unroll
                for (int rb = 0; rb < P; ++rb) s[n][rb] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int jb = 0; jb < P; ++jb) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) tbuf[(4 * g4 + v) * 20 + c] = aY[n][jb][v];
                    lds_wave_sync();
                    const float4 ax4 = *reinterpret_cast<const float4*>(tbuf + c * 20 + 4 * g4);
                    lds_wave_sync();
                    const float ax[4] = {ax4.x, ax4.y, ax4.z, ax4.w};
                    const float* Bn = Bl + n * D * D + (16 * jb + 4 * g4) * D + c;
#pragma unroll
                    for (int rb = 0; rb < P; ++rb)
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            s[n][rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(Bn[k * D + 16 * rb], ax[k], s[n][rb], 0, 0, 0);
                }
            }

            // leave-one-out products, prediction, error
            floatx4 w[N][P];
            float xhat = 0.0f;
#pragma unroll
            for (int rb = 0; rb < P; ++rb) {
                floatx4 run = {1.0f, 1.0f, 1.0f, 1.0f};
#pragma unroll
                for (int n = 0; n < N; ++n) {
                    w[n][rb] = run;
                    run *= s[n][rb];
                }
                xhat += (run[0] + run[1]) + (run[2] + run[3]);
                run = floatx4{1.0f, 1.0f, 1.0f, 1.0f};
#pragma unroll
                for (int n = N - 1; n >= 0; --n) {
                    w[n][rb] *= run;
                    run *= s[n][rb];
                }
            }
            xhat += __shfl_xor(xhat, 16);
            xhat += __shfl_xor(xhat, 32);
            const float neg_e = xhat - x;

#pragma unroll
            for (int n = 0; n < N; ++n) {
                // -e w^(n) (layout X), -e GS^(n) (layout Y), and -e w^(n) in layout Y through LDS
                floatx4 gs[P];
                float wY[P][4];
#pragma unroll
                for (int jb = 0; jb < P; ++jb) gs[jb] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int rb = 0; rb < P; ++rb) {
                    const floatx4 wp = w[n][rb] * neg_e;
                    *reinterpret_cast<float4*>(tbuf + c * 20 + 4 * g4) = make_float4(wp[0], wp[1], wp[2], wp[3]);
                    const float* Btn = Bt + n * D * D + (16 * rb + 4 * g4) * D + c;
#pragma unroll
                    for (int jb = 0; jb < P; ++jb)
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            gs[jb] = __builtin_amdgcn_mfma_f32_16x16x4f32(wp[k], Btn[k * D + 16 * jb], gs[jb], 0, 0, 0);
                    lds_wave_sync();
#pragma unroll
                    for (int v = 0; v < 4; ++v) wY[rb][v] = tbuf[(4 * g4 + v) * 20 + c];
                    lds_wave_sync();
                }

                // factor-row gradients: three routes by row number (see the header comment)
#pragma unroll
                for (int jb = 0; jb < P; ++jb) {
                    const int col = 16 * jb + c;
                    float grad[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = iY[n][v];
                        const bool ok = col < g.J[n] && actY[v];
                        grad[v] = ok ? g.scale * fmaf(g.lambda_A, aY[n][jb][v], gs[jb][v]) : 0.0f;
                        const bool cold = ok && row >= g.K[n];
                        __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(
                            grad[v], rsrc_dA[n], cold ? (row * g.J[n] + col) * 4 : (int)g.mode_bytes[n] + c * 4, 0, 0);
                        if (ok && row < g.K[n] && row >= g.top[n])
                            lds_float_add(hot + (size_t)(g.hot_off[n] + row) * D + col, grad[v]);
                    }
                    if (g.top[n] > 0) {
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const float onehot = (iY[n][k] == c && actY[k]) ? 1.0f : 0.0f;
                            Top[n][jb] = __builtin_amdgcn_mfma_f32_16x16x4f32(onehot, grad[k], Top[n][jb], 0, 0, 0);
                        }
                    }
                    // core gradient block: GB[j = 16 jb + 4g + v'][r = 16 rb + c]
#pragma unroll
                    for (int rb = 0; rb < P; ++rb)
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            GBacc[n][jb][rb] =
                                __builtin_amdgcn_mfma_f32_16x16x4f32(aY[n][jb][v], wY[rb][v], GBacc[n][jb][rb], 0, 0, 0);
                }
            }
        }
    }

    // rows 0..15 of each mode: from the wave's accumulators into the workgroup's LDS table
#pragma unroll
    for (int n = 0; n < N; ++n)
        if (g.top[n] > 0) {
#pragma unroll
            for (int jb = 0; jb < P; ++jb)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    lds_float_add(hot + (size_t)(g.hot_off[n] + 4 * g4 + v) * D + 16 * jb + c, Top[n][jb][v]);
        }
    // core gradient: one table per wave, plain stores (entries outside J_n x R are padding, not stored)
    float* gb_out = g.gb_partial + ((size_t)blockIdx.x * WAVES + wave) * g.B_total;
#pragma unroll
    for (int n = 0; n < N; ++n)
#pragma unroll
        for (int jb = 0; jb < P; ++jb)
#pragma unroll
            for (int rb = 0; rb < P; ++rb)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int j = 16 * jb + 4 * g4 + v, r = 16 * rb + c;
                    if (j < g.J[n] && r < g.R) gb_out[g.B_off[n] + j * g.R + r] = GBacc[n][jb][rb][v];
                }
    __syncthreads();
    float* hot_out = g.hot_partial + (size_t)blockIdx.x * g.H * D;
    for (int q = tid; q < g.H * D; q += THREADS) hot_out[q] = hot[q];
}

// ---------------------------------------------------------------------------------------------
// Evaluation pass over all stored entries (RMSE / MAE) for the same shapes: records streamed,
// rows gathered 16 lanes per 64 bytes, projections on the matrix core, errors summed in double.
// ---------------------------------------------------------------------------------------------
template <int N, int P>
__global__ void __launch_bounds__(256) errors_tiled_kernel(Coo coo, uint64_t nnz, const float* __restrict__ A,
                                                           const float* __restrict__ B, Layout L,
                                                           double* __restrict__ sums /* [2]: sse, sae */) {
    extern __shared__ float lds[];
    constexpr int W4 = (N + 1 + 3) / 4;
    constexpr int D = 16 * P;
    __shared__ double red[2][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g4 = lane >> 4;
    float* Bl = lds;                                                    // [N][D][D]
    float* wave_lds = lds + N * D * D + wave * tiled_wave_scratch(N);
    int* sidx = reinterpret_cast<int*>(wave_lds);
    float* tbuf = wave_lds + (N + 1) * 64;
    for (int q = tid; q < N * D * D; q += 256) {
        const int n = q / (D * D), rem = q - n * D * D, j = rem / D, r = rem - j * D;
        Bl[q] = (j < L.J[n] && r < L.R) ? B[L.B_off[n] + j * L.R + r] : 0.0f;
    }
    __syncthreads();

    const uint4* rec4 = reinterpret_cast<const uint4*>(coo.rec);
    const uint64_t n_groups = (nnz + 63) / 64;
    double sse = 0.0, sae = 0.0;
#pragma unroll 1
    for (uint64_t group = (uint64_t)blockIdx.x * 4 + wave; group < n_groups; group += (uint64_t)gridDim.x * 4) {
        const uint64_t p = group * 64 + lane;
        const bool act = p < nnz;
        uint32_t flat[4 * W4];
#pragma unroll
        for (int q = 0; q < W4; ++q) {
            const uint4 r = rec4[(act ? p : 0) * W4 + q];
            flat[4 * q + 0] = r.x;
            flat[4 * q + 1] = r.y;
            flat[4 * q + 2] = r.z;
            flat[4 * q + 3] = r.w;
        }
#pragma unroll
        for (int n = 0; n < N; ++n) sidx[n * 64 + lane] = act ? (int)flat[n] : 0;
        const float xval = act ? __uint_as_float(flat[N]) : 0.0f;
        lds_wave_sync();
#pragma unroll 1
        for (int sub = 0; sub < 4; ++sub) {
            floatx4 prod[P];
#pragma unroll
            for (int rb = 0; rb < P; ++rb) prod[rb] = floatx4{1.0f, 1.0f, 1.0f, 1.0f};
#pragma unroll
            for (int n = 0; n < N; ++n) {
                const int4 r = *reinterpret_cast<const int4*>(sidx + n * 64 + sub * 16 + 4 * g4);
                const int rows[4] = {r.x, r.y, r.z, r.w};
                const float* An = A + L.A_off[n];
                floatx4 sacc[P];
#pragma unroll
                for (int rb = 0; rb < P; ++rb) sacc[rb] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int jb = 0; jb < P; ++jb) {
                    const int col = 16 * jb + c;
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        tbuf[(4 * g4 + v) * 20 + c] = col < L.J[n] ? An[(size_t)rows[v] * L.J[n] + col] : 0.0f;
                    lds_wave_sync();
                    const float4 ax4 = *reinterpret_cast<const float4*>(tbuf + c * 20 + 4 * g4);
                    lds_wave_sync();
                    const float ax[4] = {ax4.x, ax4.y, ax4.z, ax4.w};
                    const float* Bn = Bl + n * D * D + (16 * jb + 4 * g4) * D + c;
#pragma unroll
                    for (int rb = 0; rb < P; ++rb)
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            sacc[rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(Bn[k * D + 16 * rb], ax[k], sacc[rb], 0, 0, 0);
                }
#pragma unroll
                for (int rb = 0; rb < P; ++rb) prod[rb] *= sacc[rb];
            }
            // padded r (>= R) have c = 0 in every mode, so their products are 0 for N >= 1
            float xhat = 0.0f;
#pragma unroll
            for (int rb = 0; rb < P; ++rb) xhat += (prod[rb][0] + prod[rb][1]) + (prod[rb][2] + prod[rb][3]);
            xhat += __shfl_xor(xhat, 16);
            xhat += __shfl_xor(xhat, 32);
            const float x = __shfl(xval, sub * 16 + c);
            if (g4 == 0 && group * 64 + sub * 16 + c < nnz) {
                const double e = (double)x - (double)xhat;
                sse += e * e;
                sae += fabs(e);
            }
        }
    }
    sse = wave_sum(sse);
    sae = wave_sum(sae);
    if (lane == 0) {
        red[0][wave] = sse;
        red[1][wave] = sae;
    }
    __syncthreads();
    if (tid == 0) {
        atomicAdd(sums + 0, (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]));
        atomicAdd(sums + 1, (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]));
    }
}

}  // namespace ftk
