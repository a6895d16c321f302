// Fused sampling + gradient pass for J_n = R = 16 (order N <= 6), built on the fp32 matrix cores.
//
// One wavefront draws 64 positions of Psi at a time (one Philox position and one random record
// read per lane), parks the 64 records in a private LDS buffer, and then works through them as
// four tiles of 16 sampled entries.  The three contractions of the method are 16x16 matrix
// products per mode and run as v_mfma_f32_16x16x4_f32 (four K-steps each):
//
//   projections   C^T  [r x sample] = B^T [r x j]      . a^T [j x sample]      (contract j)
//   A gradient    GS   [sample x j] = W   [sample x r] . B^T [r x j]           (contract r)
//   core gradient GB   [j x r]     += a^T [j x sample] . (-e W) [sample x r]   (contract the tile's samples)
//
// Operand layout of the instruction (lane l, c = l % 16, g = l / 16):
//   A operand: Aop(l) = M[row c][k = g]      B operand: Bop(l) = M[k = g][col c]
//   accumulator register v: D(l, v) = M[row 4g + v][col c]
// A contracted index has to sit in the (g, K-step) position of both operands, so per-sample data
// exists in two register layouts:
//   X: lane (c, g) holds sample c, components 4g..4g+3
//   Y: lane (c, g) holds component c of samples 4g..4g+3   (16 lanes cover one 64-byte row)
// Rows are gathered in layout Y only (four full 64-byte rows per load instruction) and reach
// layout X through a per-wave LDS buffer; -e w goes the other way.  The A gradient comes out of
// the matrix core directly in layout Y, which lets a row be added with ONE 64-byte atomic request.
// The row gather of the next tile is issued before the current tile is computed, and the record
// reads of the next 64 samples are in flight during the whole current group of four tiles.
//
// Rows are numbered by descending frequency, so the rows most samples hit are rows [0, K_n) of
// each mode: their gradient sums are kept in an LDS table (one per workgroup) and leave the
// workgroup once, as plain stores; only the remaining rows use global float atomics.  The core
// gradient is accumulated in matrix-core accumulators over all tiles of a wave, reduced across
// the workgroup's waves in LDS, and also leaves the workgroup as one table of plain stores.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftk_kernels_generic.hpp"

namespace ftk {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kMfmaWaves = 8;                  // waves per workgroup (one workgroup per CU)
constexpr int kMfmaThreads = kMfmaWaves * 64;
constexpr int kTransposeFloats = 16 * 20;      // 16x16 tile, rows padded to 20 floats
__host__ __device__ constexpr int mfma16_wave_scratch(int order) {
    // floats per wave: N index columns + values of 64 samples | transpose buffer | 16 errors
    return (order + 1) * 64 + kTransposeFloats + 16;
}

struct Mfma16Args {
    Coo coo;
    uint64_t nnz;
    uint64_t seed;
    long long M;              // |Psi|
    const float* A;
    const float* B;
    float* dA;
    long long A_off[kMaxOrder];
    int B_off[kMaxOrder];
    int K[kMaxOrder];         // rows [0, K[n]) of mode n live in the LDS table
    int hot_off[kMaxOrder];   // first LDS table row of mode n
    int H;                    // rows in the LDS table (>= sum K[n])
    float* hot_partial;       // [gridDim.x][H][16]
    float* gb_partial;        // [gridDim.x][N * 256]
    float lambda_A;
};

__device__ __forceinline__ void lds_wave_sync() {
    // LDS requests of one wave complete in order; this keeps the compiler from moving LDS reads
    // above the writes of other lanes they depend on, and waits for outstanding LDS traffic.
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}

// LDS float add by compare-and-swap.  The native LDS float add (ds_add_f32) retires about one
// lane every three clocks on this chip, ~30x slower than integer LDS atomics; a CAS loop on the
// value's bits runs at integer-atomic speed and only repeats for lanes that lost a race.
__device__ __forceinline__ void lds_float_add(float* p, float v) {
    unsigned int* u = reinterpret_cast<unsigned int*>(p);
    unsigned int seen = *u, expect;
    do {
        expect = seen;
        seen = atomicCAS(u, expect, __float_as_uint(__uint_as_float(expect) + v));
    } while (seen != expect);
}

template <int N>
struct TileRows {
    float aY[N][4];   // layout Y: component c of the rows of samples 4g..4g+3
    int iY[N][4];     // their row numbers
    float x;          // value of sample c (layout X)
};

template <int N>
__global__ void __launch_bounds__(kMfmaThreads) grad_mfma16_kernel(Mfma16Args g) {
    extern __shared__ float lds[];
    constexpr int W4 = (N + 1 + 3) / 4;   // 16-byte words per record
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g4 = lane >> 4;
    float* hot = lds;
    float* wave_lds = lds + (size_t)g.H * 16 + wave * mfma16_wave_scratch(N);
    int* sidx = reinterpret_cast<int*>(wave_lds);           // [N][64]
    float* sval = wave_lds + N * 64;                         // [64]
    float* tbuf = wave_lds + (N + 1) * 64;                   // [16][20]
    float* ebuf = tbuf + kTransposeFloats;                   // [16]
    float* gbred = lds + (size_t)g.H * 16 + kMfmaWaves * mfma16_wave_scratch(N);

    for (int q = tid; q < g.H * 16; q += kMfmaThreads) hot[q] = 0.0f;
    for (int q = tid; q < N * 256; q += kMfmaThreads) gbred[q] = 0.0f;

    // B^(n) in the two operand layouts:  Bq[n][k] = B[4g+k][c],  Br[n][k] = B[c][4g+k]
    float Bq[N][4], Br[N][4];
#pragma unroll
    for (int n = 0; n < N; ++n) {
        const float* Bn = g.B + g.B_off[n];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            Bq[n][k] = Bn[(4 * g4 + k) * 16 + c];
            Br[n][k] = Bn[c * 16 + 4 * g4 + k];
        }
    }
    floatx4 GBacc[N];
#pragma unroll
    for (int n = 0; n < N; ++n) GBacc[n] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
    __syncthreads();

    const long long M = g.M;
    const long long n_groups = (M + 63) / 64;
    const long long group_stride = (long long)gridDim.x * kMfmaWaves;
    const uint4* rec4 = reinterpret_cast<const uint4*>(g.coo.rec);

    // record of sample (group * 64 + lane): N row numbers and the value's bits
    auto load_record = [&](long long group, uint4 (&rec)[W4]) {
        const long long k = group * 64 + lane;
        const uint32_t p = k < M ? sample_position(g.seed, (uint64_t)k, g.nnz) : 0u;
#pragma unroll
        for (int q = 0; q < W4; ++q) rec[q] = rec4[(size_t)p * W4 + q];
    };
    // rows of tile `sub` (0..3) of the group parked in LDS, gathered in layout Y
    auto gather = [&](long long group, int sub, TileRows<N>& t) {
        const long long base = group * 64 + sub * 16;
        t.x = sval[sub * 16 + c];
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const int4 r = *reinterpret_cast<const int4*>(sidx + n * 64 + sub * 16 + 4 * g4);
            t.iY[n][0] = r.x;
            t.iY[n][1] = r.y;
            t.iY[n][2] = r.z;
            t.iY[n][3] = r.w;
            const float* An = g.A + g.A_off[n];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                // samples past the end of Psi were parked as row 0 with value 0; their rows are
                // forced to zero so that every contribution of theirs is exactly zero
                const float a = An[(long long)t.iY[n][v] * 16 + c];
                t.aY[n][v] = (base + 4 * g4 + v < M) ? a : 0.0f;
            }
        }
    };

    uint4 rec[W4];
    long long group = (long long)blockIdx.x * kMfmaWaves + wave;
    if (group < n_groups) load_record(group, rec);

    for (; group < n_groups; group += group_stride) {
        // park the 64 records (struct of arrays) for this wave
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

        TileRows<N> cur, nxt;
        gather(group, 0, nxt);
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) {
            cur = nxt;
            if (sub < 3) gather(group, sub + 1, nxt);
            const long long base = group * 64 + sub * 16;

            // rows: layout Y -> LDS -> layout X, then projections s[n][v] = c^(n)_{r = 4g+v} of sample c
            floatx4 s[N];
#pragma unroll
            for (int n = 0; n < N; ++n) {
#pragma unroll
                for (int v = 0; v < 4; ++v) tbuf[(4 * g4 + v) * 20 + c] = cur.aY[n][v];
                lds_wave_sync();
                const float4 ax = *reinterpret_cast<const float4*>(tbuf + c * 20 + 4 * g4);
                lds_wave_sync();
                floatx4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(Bq[n][0], ax.x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(Bq[n][1], ax.y, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(Bq[n][2], ax.z, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(Bq[n][3], ax.w, acc, 0, 0, 0);
                s[n] = acc;
            }

            // leave-one-out products (prefix sweep, then suffix sweep), prediction, error
            floatx4 w[N];
            floatx4 run = {1.0f, 1.0f, 1.0f, 1.0f};
#pragma unroll
            for (int n = 0; n < N; ++n) {
                w[n] = run;
                run *= s[n];
            }
            float xhat = (run[0] + run[1]) + (run[2] + run[3]);
            xhat += __shfl_xor(xhat, 16);
            xhat += __shfl_xor(xhat, 32);
            const float e = cur.x - xhat;
            run = floatx4{1.0f, 1.0f, 1.0f, 1.0f};
#pragma unroll
            for (int n = N - 1; n >= 0; --n) {
                w[n] *= run;
                run *= s[n];
            }

            // errors of samples 4g..4g+3 for layout Y
            if (g4 == 0) ebuf[c] = e;
            lds_wave_sync();
            const float4 eY4 = *reinterpret_cast<const float4*>(ebuf + 4 * g4);
            const float eY[4] = {eY4.x, eY4.y, eY4.z, eY4.w};

#pragma unroll
            for (int n = 0; n < N; ++n) {
                // GS^(n) in layout Y:  gs[v] = GS_{j = c} of sample 4g+v
                floatx4 gs = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int k = 0; k < 4; ++k) gs = __builtin_amdgcn_mfma_f32_16x16x4f32(w[n][k], Br[n][k], gs, 0, 0, 0);

                // -e w: layout X -> LDS -> layout Y
                const floatx4 wp = w[n] * (-e);
                *reinterpret_cast<float4*>(tbuf + c * 20 + 4 * g4) = make_float4(wp[0], wp[1], wp[2], wp[3]);
                lds_wave_sync();
                float wY[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) wY[v] = tbuf[(4 * g4 + v) * 20 + c];
                lds_wave_sync();

                // factor-row gradient -e GS + lambda_A a, one 64-byte row per 16 lanes
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if (base + 4 * g4 + v < M) {
                        const float grad = fmaf(-eY[v], gs[v], g.lambda_A * cur.aY[n][v]);
                        const int row = cur.iY[n][v];
                        if (row < g.K[n])
                            lds_float_add(hot + (size_t)(g.hot_off[n] + row) * 16 + c, grad);
                        else
                            atomicAdd(g.dA + g.A_off[n] + (long long)row * 16 + c, grad);
                    }
                }

                // core gradient: GB[j = 4g+v'][r = c] += sum_samples a_j (-e w_r)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    GBacc[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(cur.aY[n][v], wY[v], GBacc[n], 0, 0, 0);
            }
        }
    }

    // workgroup reduction of the core gradient, then one table of plain stores per workgroup
#pragma unroll
    for (int n = 0; n < N; ++n)
#pragma unroll
        for (int v = 0; v < 4; ++v) lds_float_add(gbred + n * 256 + (4 * g4 + v) * 16 + c, GBacc[n][v]);
    __syncthreads();
    float* gb_out = g.gb_partial + (size_t)blockIdx.x * (N * 256);
    for (int q = tid; q < N * 256; q += kMfmaThreads) gb_out[q] = gbred[q];
    float* hot_out = g.hot_partial + (size_t)blockIdx.x * g.H * 16;
    for (int q = tid; q < g.H * 16; q += kMfmaThreads) hot_out[q] = hot[q];
}

// ---------------------------------------------------------------------------------------------
// A <- A - lr_A dA.  Blocks [0, dense_blocks) scan the dense accumulator (rows updated with global
// atomics); the remaining blocks sum the per-workgroup LDS tables of the frequently hit rows.
// ---------------------------------------------------------------------------------------------
struct ApplyHotArgs {
    const float* hot_partial;   // [parts][H][J]
    int parts;
    int H;
    int J;
    int order;
    int K[kMaxOrder];
    int hot_off[kMaxOrder];
    long long A_off[kMaxOrder];
};

__global__ void __launch_bounds__(256) apply_A_hot_kernel(float* __restrict__ A, float* __restrict__ dA, long long n4,
                                                          float lr_A, int dense_blocks, ApplyHotArgs h) {
    if ((int)blockIdx.x < dense_blocks) {
        float4* A4 = reinterpret_cast<float4*>(A);
        float4* D4 = reinterpret_cast<float4*>(dA);
        for (long long q = (long long)blockIdx.x * blockDim.x + threadIdx.x; q < n4;
             q += (long long)dense_blocks * blockDim.x) {
            const float4 d = D4[q];
            if (d.x != 0.0f || d.y != 0.0f || d.z != 0.0f || d.w != 0.0f) {
                float4 a = A4[q];
                a.x = fmaf(-lr_A, d.x, a.x);
                a.y = fmaf(-lr_A, d.y, a.y);
                a.z = fmaf(-lr_A, d.z, a.z);
                a.w = fmaf(-lr_A, d.w, a.w);
                A4[q] = a;
                D4[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
        }
        return;
    }
    const int q = ((int)blockIdx.x - dense_blocks) * blockDim.x + threadIdx.x;
    const int table = h.H * h.J;
    if (q >= table) return;
    const int hrow = q / h.J, j = q - hrow * h.J;
    int n = -1;
    for (int m = 0; m < h.order; ++m)
        if (hrow >= h.hot_off[m] && hrow < h.hot_off[m] + h.K[m]) n = m;
    if (n < 0) return;
    float d0 = 0.0f, d1 = 0.0f, d2 = 0.0f, d3 = 0.0f;
    int b = 0;
    for (; b + 4 <= h.parts; b += 4) {
        d0 += h.hot_partial[(size_t)(b + 0) * table + q];
        d1 += h.hot_partial[(size_t)(b + 1) * table + q];
        d2 += h.hot_partial[(size_t)(b + 2) * table + q];
        d3 += h.hot_partial[(size_t)(b + 3) * table + q];
    }
    for (; b < h.parts; ++b) d0 += h.hot_partial[(size_t)b * table + q];
    const float d = (d0 + d1) + (d2 + d3);
    if (d != 0.0f) {
        float* a = A + h.A_off[n] + (long long)(hrow - h.hot_off[n]) * h.J + j;
        *a = fmaf(-lr_A, d, *a);
    }
}

}  // namespace ftk
