// Shape-generic kernels: any order N <= 10, any J_n, any R within the LDS budget.
// One lane owns one sampled nonzero.  These are the reference-speed path; shapes with a
// specialised kernel never run grad_generic in the default configuration.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftk_philox.hpp"

namespace ftk {

constexpr int kMaxOrder = 10;

// Everything a kernel needs to find the parameters.  A^(n) for all modes share one allocation
// (mode n starts at float offset A_off[n]); so do dA^(n) (same offsets), B^(n) and GB^(n)
// (float offset B_off[n], row-major J_n x R).
struct Layout {
    int order;
    int R;
    int J[kMaxOrder];
    int B_off[kMaxOrder];
    long long A_off[kMaxOrder];
    int B_total;   // sum_n J_n * R
};

struct Batch {
    const int32_t* idx;   // [order][cap]: idx[n * cap + k] = i_n of sample k
    const float* val;     // [cap]
    long long count;      // M = |Psi|
    long long cap;
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// ---------------------------------------------------------------------------------------------
// The tensor in device memory: one record per stored entry, `words` 32-bit words each
// (N mode indices, then the value's bits, padded to a multiple of 4 words), so that a random
// position costs one 16-byte-aligned access instead of N + 1 scattered ones.  Mode indices
// are the library's internal row numbers (rows renumbered by descending frequency).
// ---------------------------------------------------------------------------------------------
struct Coo {
    const uint32_t* rec;
    int words;
};

__host__ __device__ inline int record_words(int order) { return ((order + 1 + 3) / 4) * 4; }

// Kernels that are no templates are defined once, in the host file's translation unit: the units that hold the
// instances of the matrix-core kernel templates define FTK_TEMPLATE_KERNELS_ONLY and skip them.
#ifndef FTK_TEMPLATE_KERNELS_ONLY
// ---------------------------------------------------------------------------------------------
// Psi: positions from Philox, and the sampled entries gathered into a dense batch
// (step a1 + a2: the only place the tensor is read with random access).
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) sample_gather_kernel(Coo coo, int order, SampleRule rule, uint64_t seed,
                                                            long long M, long long cap, uint32_t* __restrict__ pos,
                                                            int32_t* __restrict__ bidx, float* __restrict__ bval) {
    const long long k = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= M) return;
    const uint32_t p = sample_place(seed, (uint64_t)k, rule);
    pos[k] = caller_position(p, rule);
    const uint4* r4 = reinterpret_cast<const uint4*>(coo.rec + (size_t)p * coo.words);
    uint32_t w[kMaxOrder + 4];
    for (int q = 0; q < coo.words / 4; ++q) {
        const uint4 t = r4[q];
        w[4 * q + 0] = t.x;
        w[4 * q + 1] = t.y;
        w[4 * q + 2] = t.z;
        w[4 * q + 3] = t.w;
    }
    for (int n = 0; n < order; ++n) bidx[(long long)n * cap + k] = (int32_t)w[n];
    bval[k] = __uint_as_float(w[order]);
}

// ---------------------------------------------------------------------------------------------
// gradient pass, one lane per sample
//   LDS: c[N*R][T] | w[N*R][T] | per-wave GB partial sums [T/64][B_total] | (optional) B [B_total]
// ---------------------------------------------------------------------------------------------
struct GradArgs {
    Layout L;
    Batch batch;
    const float* A;
    const float* B;
    float* dA;         // where factor-row gradients are added: the accumulator (synchronous mode) or A itself
    float* GB;
    float lambda_A;
    float scale;       // 1 (synchronous: the update pass applies -lr_A) or -lr_A (in-place mode)
    int b_in_lds;
    int core_only;     // 1: accumulate the core gradient only, leave the factor rows alone
};

__global__ void grad_generic_kernel(GradArgs g) {
    extern __shared__ float lds[];
    const int N = g.L.order, R = g.L.R, T = blockDim.x, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, BT = g.L.B_total;
    float* c_l = lds;
    float* w_l = c_l + (size_t)N * R * T;
    float* gb_w = w_l + (size_t)N * R * T + (size_t)wave * BT;
    float* b_l = w_l + (size_t)N * R * T + (size_t)(T >> 6) * BT;

    for (int q = lane; q < BT; q += 64) gb_w[q] = 0.0f;
    if (g.b_in_lds)
        for (int q = tid; q < BT; q += T) b_l[q] = g.B[q];
    __syncthreads();
    const float* Bm = g.b_in_lds ? b_l : g.B;

    const long long M = g.batch.count, cap = g.batch.cap;
    for (long long base = (long long)blockIdx.x * T; base < M; base += (long long)gridDim.x * T) {
        const long long k = base + tid;
        const bool act = k < M;
        float e = 0.0f;
        if (act) {
            // c^(n)_r = a^(n) . B^(n)[:, r]
            for (int n = 0; n < N; ++n) {
                const int Jn = g.L.J[n];
                const float* row = g.A + g.L.A_off[n] + (long long)g.batch.idx[(long long)n * cap + k] * Jn;
                const float* Bn = Bm + g.L.B_off[n];
                for (int r = 0; r < R; ++r) {
                    float acc = 0.0f;
                    for (int j = 0; j < Jn; ++j) acc = fmaf(row[j], Bn[j * R + r], acc);
                    c_l[(size_t)(n * R + r) * T + tid] = acc;
                }
            }
            // leave-one-out products by a prefix and a suffix sweep over the modes
            float xhat = 0.0f;
            for (int r = 0; r < R; ++r) {
                float run = 1.0f;
                for (int n = 0; n < N; ++n) {
                    w_l[(size_t)(n * R + r) * T + tid] = run;
                    run *= c_l[(size_t)(n * R + r) * T + tid];
                }
                xhat += run;
                run = 1.0f;
                for (int n = N - 1; n >= 0; --n) {
                    w_l[(size_t)(n * R + r) * T + tid] *= run;
                    run *= c_l[(size_t)(n * R + r) * T + tid];
                }
            }
            e = g.batch.val[k] - xhat;
            // factor-row gradient: -e GS^(n) + lambda_A a^(n), accumulated into dA
            for (int n = 0; n < N && !g.core_only; ++n) {
                const int Jn = g.L.J[n];
                const long long roff = g.L.A_off[n] + (long long)g.batch.idx[(long long)n * cap + k] * Jn;
                const float* Bn = Bm + g.L.B_off[n];
                for (int j = 0; j < Jn; ++j) {
                    float gs = 0.0f;
                    for (int r = 0; r < R; ++r) gs = fmaf(Bn[j * R + r], w_l[(size_t)(n * R + r) * T + tid], gs);
                    atomicAdd(g.dA + roff + j, g.scale * fmaf(-e, gs, g.lambda_A * g.A[roff + j]));
                }
            }
        }
        // core gradient: sum over the wave's samples of -e a_j w_r, kept per wave in LDS
        for (int n = 0; n < N; ++n) {
            const int Jn = g.L.J[n];
            const float* row = g.A + g.L.A_off[n];
            if (act) row += (long long)g.batch.idx[(long long)n * cap + k] * Jn;
            for (int j = 0; j < Jn; ++j) {
                const float ea = act ? -e * row[j] : 0.0f;
                for (int r = 0; r < R; ++r) {
                    float v = act ? ea * w_l[(size_t)(n * R + r) * T + tid] : 0.0f;
                    v = wave_sum(v);
                    if (lane == 0) gb_w[g.L.B_off[n] + j * R + r] += v;
                }
            }
        }
    }
    __syncthreads();
    for (int q = lane; q < BT; q += 64) {
        const float v = gb_w[q];
        if (v != 0.0f) atomicAdd(g.GB + q, v);
    }
}

// ---------------------------------------------------------------------------------------------
// Factor phase of Algorithm 1 in the order it is printed (lines 1-16), one lane per sampled entry,
// all lanes running at once: inside a sample the modes are taken one after the other, and mode n
// already sees what modes < n of the same sample have just done to their rows (their projections
// c^(m) are advanced by the change, c^(m)_r += sum_j delta_j B^(m)[j,r], which is the projection
// of the row the lane has just written).  Each row is changed in place with M = 1,
//     a <- a - lr_A ( -e GS^(n) + lambda_A a ),
// as a float atomic add of the difference, so that samples which share a row do not lose each
// other's updates.  The core phase (lines 17-39) is a second launch of grad_generic_kernel with
// core_only set, over the same samples and the rows this kernel leaves.
//   LDS: c[N*R][T] | w[R][T] | (optional) B [B_total]; the launch reserves grad_generic's layout.
// ---------------------------------------------------------------------------------------------
__global__ void factor_phase_generic_kernel(GradArgs g, float* A_rw, float lr_A) {
    extern __shared__ float lds[];
    const int N = g.L.order, R = g.L.R, T = blockDim.x, tid = threadIdx.x;
    const int BT = g.L.B_total;
    float* c_l = lds;
    float* w_l = c_l + (size_t)N * R * T;
    float* b_l = w_l + (size_t)N * R * T + (size_t)(T >> 6) * BT;
    if (g.b_in_lds)
        for (int q = tid; q < BT; q += T) b_l[q] = g.B[q];
    __syncthreads();
    const float* Bm = g.b_in_lds ? b_l : g.B;

    const long long M = g.batch.count, cap = g.batch.cap;
    for (long long k = (long long)blockIdx.x * T + tid; k < M; k += (long long)gridDim.x * T) {
        const float x = g.batch.val[k];
        for (int m = 0; m < N; ++m) {
            const int Jm = g.L.J[m];
            const float* row = A_rw + g.L.A_off[m] + (long long)g.batch.idx[(long long)m * cap + k] * Jm;
            const float* Bn = Bm + g.L.B_off[m];
            for (int r = 0; r < R; ++r) {
                float acc = 0.0f;
                for (int j = 0; j < Jm; ++j) acc = fmaf(row[j], Bn[j * R + r], acc);
                c_l[(size_t)(m * R + r) * T + tid] = acc;
            }
        }
        for (int n = 0; n < N; ++n) {
            float xhat = 0.0f;
            for (int r = 0; r < R; ++r) {
                float prod = 1.0f;
                for (int m = 0; m < N; ++m)
                    if (m != n) prod *= c_l[(size_t)(m * R + r) * T + tid];
                w_l[(size_t)r * T + tid] = prod;
                xhat = fmaf(prod, c_l[(size_t)(n * R + r) * T + tid], xhat);
            }
            const float e = x - xhat;
            const int Jn = g.L.J[n];
            float* row = A_rw + g.L.A_off[n] + (long long)g.batch.idx[(long long)n * cap + k] * Jn;
            const float* Bn = Bm + g.L.B_off[n];
            for (int j = 0; j < Jn; ++j) {
                float gs = 0.0f;
                for (int r = 0; r < R; ++r) gs = fmaf(Bn[j * R + r], w_l[(size_t)r * T + tid], gs);
                const float delta = -lr_A * fmaf(-e, gs, g.lambda_A * row[j]);
                atomicAdd(row + j, delta);
                if (n + 1 < N)
                    for (int r = 0; r < R; ++r) c_l[(size_t)(n * R + r) * T + tid] += delta * Bn[j * R + r];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// whole-tensor error sums (RMSE / MAE): one lane per stored nonzero, streaming over Omega
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) errors_generic_kernel(Coo coo, Layout L, uint64_t nnz,
                                                             const float* __restrict__ A,
                                                             const float* __restrict__ B, int b_in_lds,
                                                             double* __restrict__ sums /* [2]: sse, sae */) {
    extern __shared__ float lds[];
    __shared__ double red[2][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (b_in_lds) {
        for (int q = tid; q < L.B_total; q += blockDim.x) lds[q] = B[q];
        __syncthreads();
    }
    const float* Bm = b_in_lds ? lds : B;
    double sse = 0.0, sae = 0.0;
    for (uint64_t p = (uint64_t)blockIdx.x * blockDim.x + tid; p < nnz; p += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t* rec = coo.rec + (size_t)p * coo.words;
        float xhat = 0.0f;
        for (int r = 0; r < L.R; ++r) {
            float prod = 1.0f;
            for (int n = 0; n < L.order; ++n) {
                const int Jn = L.J[n];
                const float* row = A + L.A_off[n] + (long long)rec[n] * Jn;
                const float* Bn = Bm + L.B_off[n];
                float acc = 0.0f;
                for (int j = 0; j < Jn; ++j) acc = fmaf(row[j], Bn[j * L.R + r], acc);
                prod *= acc;
            }
            xhat += prod;
        }
        const double e = (double)__uint_as_float(rec[L.order]) - (double)xhat;
        sse += e * e;
        sae += fabs(e);
    }
    sse = wave_sum(sse);
    sae = wave_sum(sae);
    if (lane == 0) {
        red[0][wave] = sse;
        red[1][wave] = sae;
    }
    __syncthreads();
    if (tid == 0) {
        double a = 0.0, b = 0.0;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) {
            a += red[0][w];
            b += red[1][w];
        }
        atomicAdd(sums + 0, a);
        atomicAdd(sums + 1, b);
    }
}

// ---------------------------------------------------------------------------------------------
// set-up kernels
// ---------------------------------------------------------------------------------------------
// Initial values are a function of the element's position in the CALLER's arrays (row-major, J or R
// floats per row); `stride` is the row length of the library's own copy, whose padding stays zero.
__global__ void __launch_bounds__(256) init_uniform_kernel(float* __restrict__ out, long long rows, int cols, int stride,
                                                           uint64_t init_seed, uint32_t array_id) {
    const long long total = rows * cols;
    for (long long q = (long long)blockIdx.x * blockDim.x + threadIdx.x; q < total;
         q += (long long)gridDim.x * blockDim.x) {
        const long long i = q / cols;
        out[i * stride + (q - i * cols)] = init_value(init_seed, array_id, (uint64_t)q);
    }
}

__global__ void __launch_bounds__(256) check_range_kernel(const int32_t* __restrict__ idx, uint64_t nnz, int32_t dim,
                                                          unsigned int* __restrict__ bad) {
    unsigned int mine = 0;
    for (uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += (uint64_t)gridDim.x * blockDim.x) {
        const int32_t v = idx[p];
        mine += (v < 0 || v >= dim) ? 1u : 0u;
    }
    if (mine) atomicAdd(bad, mine);
}

// Per-row occurrence counts of one mode over all stored entries.  In a skewed mode a handful of
// rows hold a tenth of all entries each, and global atomics on one address serialise; so every
// workgroup counts through a small direct-mapped cache in LDS (a slot belongs to the first row
// number that hashes there) and only rows that find their slot taken go to memory one by one.
// The cache is added to the global counters once, when the workgroup is done.
constexpr int kHistSlots = 4096;
__global__ void __launch_bounds__(256) histogram_kernel(const int32_t* __restrict__ idx, uint64_t nnz,
                                                        unsigned int* __restrict__ counts) {
    __shared__ int owner[kHistSlots];
    __shared__ unsigned int cached[kHistSlots];
    for (int q = threadIdx.x; q < kHistSlots; q += 256) {
        owner[q] = -1;
        cached[q] = 0u;
    }
    __syncthreads();
    for (uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += (uint64_t)gridDim.x * blockDim.x) {
        const int row = idx[p];
        const unsigned int slot = ((unsigned int)row * 2654435761u) >> 20;   // top 12 bits of a multiplicative hash
        int who = owner[slot];
        if (who == -1) {
            who = atomicCAS(&owner[slot], -1, row);
            if (who == -1) who = row;
        }
        if (who == row)
            atomicAdd(&cached[slot], 1u);
        else
            atomicAdd(counts + row, 1u);
    }
    __syncthreads();
    for (int q = threadIdx.x; q < kHistSlots; q += 256)
        if (cached[q] != 0u) atomicAdd(counts + owner[q], cached[q]);
}

// word `slot` of every record <- new_of_old[idx[p]]  (or the value's bits when new_of_old == nullptr)
__global__ void __launch_bounds__(256) pack_records_kernel(const uint32_t* __restrict__ src, uint64_t nnz,
                                                           const int32_t* __restrict__ new_of_old,
                                                           uint32_t* __restrict__ rec, int words, int slot) {
    for (uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t v = src[p];
        rec[p * words + slot] = new_of_old ? (uint32_t)new_of_old[v] : v;
    }
}

// records in the pseudo-random order of the tile-sampling rule: dst[q] = src[(a q + b) mod nnz]
__global__ void __launch_bounds__(256) reorder_records_kernel(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst,
                                                              uint64_t nnz, int words, uint64_t a, uint64_t b) {
    const int w4 = words / 4;
    const uint4* s4 = reinterpret_cast<const uint4*>(src);
    uint4* d4 = reinterpret_cast<uint4*>(dst);
    for (uint64_t q = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nnz; q += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t p = (a * q + b) % nnz;
        for (int i = 0; i < w4; ++i) d4[q * w4 + i] = s4[p * w4 + i];
    }
}

// Parameter rows between the caller's numbering and the internal one:
// to_internal:  dst[new_of_old[i]][:] = src[i][:]      from_internal:  dst[i][:] = src[new_of_old[i]][:]
// Rows between the caller's numbering (J floats per row) and the library's (renumbered, `stride`
// floats per row, padding untouched).
__global__ void __launch_bounds__(256) permute_rows_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                           const int32_t* __restrict__ new_of_old, long long rows,
                                                           int J, int stride, int to_internal) {
    const long long total = rows * J;
    for (long long q = (long long)blockIdx.x * blockDim.x + threadIdx.x; q < total;
         q += (long long)gridDim.x * blockDim.x) {
        const long long i = q / J;
        const int j = (int)(q - i * J);
        const long long m = new_of_old[i];
        if (to_internal)
            dst[m * stride + j] = src[q];
        else
            dst[q] = src[m * stride + j];
    }
}

__global__ void __launch_bounds__(256) init_factor_kernel(float* __restrict__ out, long long rows, int J, int stride,
                                                          const int32_t* __restrict__ new_of_old, uint64_t init_seed,
                                                          uint32_t array_id) {
    const long long total = rows * J;
    for (long long q = (long long)blockIdx.x * blockDim.x + threadIdx.x; q < total;
         q += (long long)gridDim.x * blockDim.x) {
        const long long i = q / J;
        const int j = (int)(q - i * J);
        out[(long long)new_of_old[i] * stride + j] = init_value(init_seed, array_id, (uint64_t)q);
    }
}

__global__ void __launch_bounds__(256) fill_zero_kernel(float* __restrict__ out, long long count) {
    for (long long q = (long long)blockIdx.x * blockDim.x + threadIdx.x; q < count;
         q += (long long)gridDim.x * blockDim.x)
        out[q] = 0.0f;
}

__global__ void __launch_bounds__(256) widen_positions_kernel(const uint32_t* __restrict__ pos, long long count,
                                                              long long* __restrict__ out) {
    const long long k = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < count) out[k] = (long long)pos[k];
}

#endif  // FTK_TEMPLATE_KERNELS_ONLY

}  // namespace ftk
