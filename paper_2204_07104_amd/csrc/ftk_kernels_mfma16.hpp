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
// Rows are gathered in layout X (one 16-byte load per lane and mode: a quarter of a row) and feed
// the projections straight from the registers they arrive in; layout Y, which the core gradient
// and the regulariser term need later in the tile, is reached through a per-wave LDS buffer, and
// -e w takes the same route.  The A gradient (with the -e factor already folded into w) comes out
// of the matrix core directly in layout Y, which lets a row be added with ONE 64-byte atomic
// request per 16 lanes.
// A random 64-byte row read takes a few microseconds to come back on a loaded chip, far longer
// than a tile's arithmetic, and a workgroup that owns a whole CU's LDS runs only two waves per
// SIMD.  So every wave keeps a deep software pipeline of its own: the rows of the next THREE
// tiles are always in flight (a ring of four register tiles, crossing group boundaries), the
// records of the next group are already parked in LDS, and the records of the group after that
// are on their way.
//
// Rows are numbered by descending frequency, so the rows most samples hit are rows [0, K_n) of
// each mode: their gradient sums are kept in an LDS table (one per workgroup) and leave the
// workgroup once, as plain stores; only the remaining rows use global float atomics.  The 16
// most frequent rows of a mode do not even touch LDS per sample: the tile's gradients are summed
// per row by one more matrix product, ONEHOT [row x sample] . GRAD [sample x j], into
// accumulators that live in registers for the whole kernel.  The core
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
// One parked group of 64 samples, per wave, in 32-bit words:
//   [N][64] row words | [64] values | [4][4][4N] atomic list | [4][4][4N] table list | [8] list lengths (+8 unused)
// The lists are per tile and hold, compacted, the (sample, mode) pairs of the tile whose gradient
// row goes to a global atomic resp. to the workgroup's LDS table; list position p sits at
// [p % 4][p / 4], so that the 16 lanes of quarter g = p % 4 find their entries side by side.
__host__ __device__ constexpr int mfma16_list_words(int order) { return 4 * 16 * order; }   // 16 N positions per tile
__host__ __device__ constexpr int mfma16_group_words(int order) {
    return (order + 1) * 64 + 2 * mfma16_list_words(order) + 16;
}
__host__ __device__ constexpr int mfma16_wave_scratch(int order) {
    // floats per wave: two parked groups | one transpose buffer per mode
    return 2 * mfma16_group_words(order) + order * kTransposeFloats;
}
constexpr int kSinkRows = 4;   // rows of +inf behind the LDS table (see the scatter stage)

// A row word describes one (sample, mode):
//   bits 0..29  row * 64, the byte offset of the row inside its mode (rows < 2^24)
//   bits 30..31 route of its gradient: 0 global atomic, 1 LDS table, 2 one of the 16 most frequent rows
constexpr unsigned int kRouteShift = 30;
constexpr unsigned int kRowMask = (1u << kRouteShift) - 1u;
// An atomic-list entry is (row number counted over the whole packed parameter array) << 7 | slot,
// a table-list entry is slot << 20 | byte offset of the row's cell in the LDS table; slot = 16 n + s
// names the tile's staged gradient row of mode n, sample s.  An unused atomic entry names a row far
// past the end of the array.
constexpr unsigned int kNoAtomic = 0xffffff80u;   // slot 0, row far past the end

constexpr int kMfma16MaxOrder = 6;   // orders this kernel is instantiated for
struct Mfma16Args {
    Coo coo;                  // records in the order the sampling rule reads them
    SampleRule rule;
    uint64_t seed;
    long long M;              // |Psi|
    const float* A;
    const float* B;
    float* dA;                // where rows [K, I_n) are added: the accumulator (synchronous mode) or A itself
    long long A_off[kMfma16MaxOrder];
    int B_off[kMfma16MaxOrder];
    int K[kMfma16MaxOrder];         // rows [0, K[n]) of mode n live in the LDS table
    int top[kMfma16MaxOrder];       // 16 if K[n] >= 16 (rows 0..15 go through the one-hot matrix product), else 0
    int hot_off[kMfma16MaxOrder];   // first LDS table row of mode n
    int H;                    // rows in the LDS table (>= sum K[n])
    float* hot_partial;       // [gridDim.x][H][16]
    float* gb_partial;        // [gridDim.x][N * 256]
    unsigned int row_bytes[kMfma16MaxOrder];   // I_n * 64: size of mode n's rows in A and dA
    unsigned int all_bytes;              // size of the whole packed A (and dA), below 2^31 - 64
    unsigned int first_row[kMfma16MaxOrder];   // A_off[n] / 16: number of mode n's row 0 counted over the packed array
    float lambda_A;
    float scale;              // 1 (synchronous: the update pass applies -lr_A) or -lr_A (in-place mode)
    int pair_turns;           // entry-sampling rule: a wave's turns come in pairs that share their Philox blocks (see the kernel)
    int tiles_each, tiles_more;   // ceil(M / 16) tiles over the launch's workgroups: each gets tiles_each, the first tiles_more one more
};

__device__ __forceinline__ void lds_wave_sync() {
    // Lanes of one wave exchange data through LDS without a workgroup barrier.  The LDS unit
    // executes the requests of a wave in the order they were issued, so a read issued after
    // another lane's write already sees it; all that is needed is that the COMPILER keeps the
    // program order of the accesses (it reasons per thread and could otherwise move a read above a
    // write to a different address).  No wait is issued here: the compiler waits for each read
    // where its value is first used, which leaves the round trip free to overlap other work.
    asm volatile("" ::: "memory");
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

// LDS accessed by its 32-bit address (what the parked cell words hold).
typedef __attribute__((address_space(3))) unsigned int lds_u32;
__device__ __forceinline__ unsigned int lds_address(const void* p) {
    return (unsigned int)(uintptr_t)reinterpret_cast<const __attribute__((address_space(3))) char*>(
        (const __attribute__((address_space(3))) void*)p);
}
__device__ __forceinline__ unsigned int lds_cas(unsigned int addr, unsigned int expect, unsigned int desired) {
    lds_u32* q = (lds_u32*)(uintptr_t)addr;
    __atomic_compare_exchange_n(q, &expect, desired, false, __ATOMIC_RELAXED, __ATOMIC_RELAXED);
    return expect;   // the value that was there
}

// Everything a wave keeps across tiles.
template <int N>
struct WaveState {
    float Bq[N][4], Br[N][4];   // B^(n) in the two operand layouts: Bq[n][k] = B[4g+k][c], Br[n][k] = B[c][4g+k]
    floatx4 GBacc[N];           // core gradient, D layout: GB[j = 4g+v][r = c]
    floatx4 Top[N];             // gradient sums of rows 0..15 of each mode, D layout: [row 4g+v][j = c]
    floatx4 ring[4][N];         // rows in flight, layout X: slot t % 4 holds tile t (components 4g..4g+3 of sample c)
};

// Buffer resource over `bytes` bytes at p (raw buffer, 32-bit data).  Accesses at offsets past
// `bytes` are dropped by the hardware: loads return 0 and atomics do nothing.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned int bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}

// Issue the row gather of tile `t` (0..3) of the group parked at `sbuf` into a ring slot:
// layout X, lane (c, g) reads bytes [16g, 16g + 16) of sample c's row.
template <int N>
__device__ __forceinline__ void gather_rows(const __amdgpu_buffer_rsrc_t (&rsrc_A)[N], const unsigned int* sbuf, int t,
                                            int c, int g4, floatx4 (&dst)[N]) {
    typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int n = 0; n < N; ++n) {
        const unsigned int word = sbuf[n * 64 + t * 16 + c];
        const uintx4 q = __builtin_amdgcn_raw_buffer_load_b128(rsrc_A[n], (int)((word & kRowMask) | (unsigned int)(g4 * 16)), 0, 0);
        dst[n] = floatx4{__uint_as_float(q[0]), __uint_as_float(q[1]), __uint_as_float(q[2]), __uint_as_float(q[3])};
    }
}

// One group of 64 samples parked at `scur` (row words, values, scatter lists): four tiles of 16 (the
// first n_tiles of them in the last group of a wave's share).
// While tile t is computed, the rows of tile t + 3 are requested: tile 3 of this group during
// tile 0, then tiles 0..2 of the wave's next group (parked at `snxt`).  The requests are
// unconditional, so that the compiler's count of outstanding memory operations is exact.
// A sample slot with no sample behind it (the ragged end of Psi, or a whole group past it) is
// parked as value 0 and, in every mode, as the row just past the mode's last one: the buffer
// range check makes that row read as zeros, so the slot's projections, prediction, error and
// gradients are all exact zeros, and it is on neither scatter list.  No masks in the arithmetic.
// MODE: what one pass over Psi does.
//   kSyncPass     all gradients at the rows as gathered; rows outside the tables are added to the accumulator g.dA
//   kInPlacePass  the same gradients scaled by g.scale = -lr_A and added straight into A (g.dA is A)
//   kFactorPhase  Algorithm 1, lines 1-16, for the 16 samples of a tile at once: the modes of a sample are taken in
//                 turn, and after mode n's row has moved by delta = -lr_A (-e GS^(n) + lambda_A a^(n)) the sample's
//                 projections of that mode are advanced, c^(n) += delta B^(n) (one more 16x16 product), so that the
//                 next mode's prediction, error and GS see the row mode n has just written; rows are updated as in
//                 kInPlacePass; no core gradient
//   kCorePhase    Algorithm 1, lines 17-39: only the core gradient, at the rows the factor phase left
constexpr int kSyncPass = 0, kInPlacePass = 1, kFactorPhase = 2, kCorePhase = 3;

template <int N, int MODE>
__device__ __forceinline__ void process_group(const Mfma16Args& g, WaveState<N>& st, unsigned int hot_addr,
                                              unsigned int top_key, const unsigned int* scur, const unsigned int* snxt,
                                              float* tbuf, int c, int g4, int n_tiles) {
    __amdgpu_buffer_rsrc_t rsrc_A[N];
#pragma unroll
    for (int n = 0; n < N; ++n) rsrc_A[n] = make_rsrc(g.A + g.A_off[n], g.row_bytes[n]);
    const __amdgpu_buffer_rsrc_t rsrc_dA = make_rsrc(g.dA, g.all_bytes);
    const float* sval = reinterpret_cast<const float*>(scur + N * 64);
    const unsigned int* atomic_list = scur + (N + 1) * 64;
    const unsigned int* table_list = atomic_list + mfma16_list_words(N);
    const unsigned int* list_len = table_list + mfma16_list_words(N);
    const unsigned int c4 = (unsigned int)c * 4u;

#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
        // (wave-uniform) only the last group of a wave's share holds fewer than four tiles (n_tiles >= 1)
        if (sub > 0 && sub >= n_tiles) break;
        // The tile's scatter lists were written when the group was parked: their first batches and
        // lengths are asked for now, long before they are used.
        // (Up to order 3, where the registers allow it; above, everything is read where it is used.)
        constexpr bool AHEAD = N <= 3;
        const unsigned int* alist = atomic_list + sub * (16 * N) + g4 * (4 * N);
        const unsigned int* tlist = table_list + sub * (16 * N) + g4 * (4 * N);
        uint4 a_first = {0u, 0u, 0u, 0u}, a_second = {0u, 0u, 0u, 0u}, t_first = {0u, 0u, 0u, 0u};
        unsigned int len_atomic = 0u, len_table = 0u;
        if constexpr (AHEAD) {
            a_first = *reinterpret_cast<const uint4*>(alist);
            a_second = N > 1 ? *reinterpret_cast<const uint4*>(alist + 4) : a_first;
            t_first = *reinterpret_cast<const uint4*>(tlist);
            len_atomic = list_len[sub];
            len_table = list_len[4 + sub];
        }

        if (sub == 0)
            gather_rows<N>(rsrc_A, scur, 3, c, g4, st.ring[3]);
        else
            gather_rows<N>(rsrc_A, snxt, sub - 1, c, g4, st.ring[sub - 1]);

        floatx4 aX[N];
#pragma unroll
        for (int n = 0; n < N; ++n) aX[n] = st.ring[sub][n];
        const float x = sval[sub * 16 + c];

        // rows of all modes: layout X -> LDS -> layout Y (read back further down)
#pragma unroll
        for (int n = 0; n < N; ++n)
            *reinterpret_cast<float4*>(tbuf + n * kTransposeFloats + c * 20 + 4 * g4) =
                make_float4(aX[n][0], aX[n][1], aX[n][2], aX[n][3]);

        // projections, layout X:  s[n][v] = c^(n)_{r = 4g+v} of sample c
        floatx4 s[N];
#pragma unroll
        for (int n = 0; n < N; ++n) s[n] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int n = 0; n < N; ++n) s[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(st.Bq[n][0], aX[n][0], s[n], 0, 0, 0);
#pragma unroll
        for (int n = 0; n < N; ++n) s[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(st.Bq[n][1], aX[n][1], s[n], 0, 0, 0);
#pragma unroll
        for (int n = 0; n < N; ++n) s[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(st.Bq[n][2], aX[n][2], s[n], 0, 0, 0);
#pragma unroll
        for (int n = 0; n < N; ++n) s[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(st.Bq[n][3], aX[n][3], s[n], 0, 0, 0);

        float aY[N][4], wY[N][4], grad[N][4];
        if constexpr (MODE == kFactorPhase) {
            // rows in layout Y (for the regulariser term), out of the buffer before the gradients go into it
            lds_wave_sync();
#pragma unroll
            for (int n = 0; n < N; ++n)
#pragma unroll
                for (int v = 0; v < 4; ++v) aY[n][v] = tbuf[n * kTransposeFloats + (4 * g4 + v) * 20 + c];
            lds_wave_sync();
#pragma unroll
            for (int n = 0; n < N; ++n) {
                // w^(n) from the projections as they stand: those of modes < n already advanced
                floatx4 wn = {1.0f, 1.0f, 1.0f, 1.0f};
#pragma unroll
                for (int k = 0; k < N; ++k)
                    if (k != n) wn *= s[k];
                const floatx4 full = wn * s[n];
                const float part_n = (full[0] + full[1]) + (full[2] + full[3]);
                const floatx4 xsum_n = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, part_n, floatx4{0.0f, 0.0f, 0.0f, 0.0f}, 0, 0, 0);
                wn *= xsum_n[0] - x;   // -e w^(n)
                floatx4 gsn = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int k = 0; k < 4; ++k) gsn = __builtin_amdgcn_mfma_f32_16x16x4f32(wn[k], st.Br[n][k], gsn, 0, 0, 0);
                // delta of the row (layout Y), staged for the scatter below ...
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    grad[n][v] = g.scale * fmaf(g.lambda_A, aY[n][v], gsn[v]);
                    tbuf[n * kTransposeFloats + (4 * g4 + v) * 20 + c] = grad[n][v];
                }
                // ... and read back in layout X to advance the sample's projections of this mode
                if (n + 1 < N) {
                    lds_wave_sync();
                    const float4 dx = *reinterpret_cast<const float4*>(tbuf + n * kTransposeFloats + c * 20 + 4 * g4);
                    s[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(st.Bq[n][0], dx.x, s[n], 0, 0, 0);
                    s[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(st.Bq[n][1], dx.y, s[n], 0, 0, 0);
                    s[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(st.Bq[n][2], dx.z, s[n], 0, 0, 0);
                    s[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(st.Bq[n][3], dx.w, s[n], 0, 0, 0);
                }
            }
        } else {
        // leave-one-out products (prefix sweep, then suffix sweep), prediction, error
        floatx4 w[N];
        floatx4 run = {1.0f, 1.0f, 1.0f, 1.0f};
#pragma unroll
        for (int n = 0; n < N; ++n) {
            w[n] = run;
            run *= s[n];
        }
        // x^ of sample c = sum over r: four components here, the other twelve in the lanes of the
        // other three g.  A product with an all-ones matrix adds across g and leaves the sum in
        // every lane of column c, without a trip through LDS.
        const float part = (run[0] + run[1]) + (run[2] + run[3]);
        const floatx4 xsum = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, part, floatx4{0.0f, 0.0f, 0.0f, 0.0f}, 0, 0, 0);
        const float neg_e = xsum[0] - x;
        run = floatx4{1.0f, 1.0f, 1.0f, 1.0f};
#pragma unroll
        for (int n = N - 1; n >= 0; --n) {
            w[n] *= run;
            run *= s[n];
        }

        // rows in layout Y, out of the buffer before -e w goes into it
        lds_wave_sync();
#pragma unroll
        for (int n = 0; n < N; ++n)
#pragma unroll
            for (int v = 0; v < 4; ++v) aY[n][v] = tbuf[n * kTransposeFloats + (4 * g4 + v) * 20 + c];
        lds_wave_sync();

        // -e w of all modes: layout X -> LDS -> layout Y
#pragma unroll
        for (int n = 0; n < N; ++n) {
            w[n] *= neg_e;
            *reinterpret_cast<float4*>(tbuf + n * kTransposeFloats + c * 20 + 4 * g4) =
                make_float4(w[n][0], w[n][1], w[n][2], w[n][3]);
        }
        // -e GS^(n) straight into layout Y:  gs[n][v] = -e GS_{j = c} of sample 4g+v
        floatx4 gs[N];
#pragma unroll
        for (int n = 0; n < N; ++n) gs[n] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
        if constexpr (MODE != kCorePhase) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int n = 0; n < N; ++n)
                    gs[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(w[n][k], st.Br[n][k], gs[n], 0, 0, 0);
        }
        lds_wave_sync();
#pragma unroll
        for (int n = 0; n < N; ++n)
#pragma unroll
            for (int v = 0; v < 4; ++v) wY[n][v] = tbuf[n * kTransposeFloats + (4 * g4 + v) * 20 + c];

        // Factor-row gradients -e GS + lambda_A a (layout Y: one 64-byte row per 16 lanes).
#pragma unroll
        for (int n = 0; n < N; ++n)
#pragma unroll
            for (int v = 0; v < 4; ++v) grad[n][v] = fmaf(g.lambda_A, aY[n][v], gs[n][v]);
        if constexpr (MODE == kInPlacePass) {   // in-place mode adds -lr_A * gradient
#pragma unroll
            for (int n = 0; n < N; ++n)
#pragma unroll
                for (int v = 0; v < 4; ++v) grad[n][v] *= g.scale;
        }
        }   // MODE != kFactorPhase
        // Where each row goes was decided when the group was parked:
        //   the 16 most frequent rows of a mode: summed over the tile by the matrix core against a
        //     one-hot operand, straight from the registers
        //   every other row: staged in the wave's LDS buffer (the -e w reads above are done), then
        //     fetched again through the tile's two compacted lists, four rows per instruction:
        //     rows of the workgroup's LDS table by compare-and-swap float adds, the rest by global
        //     float atomics.
        // A global float atomic instruction costs this chip the same ~110 clocks of a per-CU unit
        // whether one or all four of its 16-lane rows are in range, so the lists matter: without
        // them nearly every instruction of every (mode, quarter) would carry at least one such row.
        if constexpr (MODE == kCorePhase) {
            // core gradient only: GB[j = 4g+v'][r = c] += sum_samples a_j (-e w_r)
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int n = 0; n < N; ++n)
                    st.GBacc[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(aY[n][v], wY[n][v], st.GBacc[n], 0, 0, 0);
            lds_wave_sync();   // the next tile overwrites the buffer
            continue;
        }
        if constexpr (MODE != kFactorPhase) {   // (the factor phase has staged its rows mode by mode)
#pragma unroll
            for (int n = 0; n < N; ++n)
#pragma unroll
                for (int v = 0; v < 4; ++v) tbuf[n * kTransposeFloats + (4 * g4 + v) * 20 + c] = grad[n][v];
        }
        lds_wave_sync();

        auto atomics4 = [&](int first) {
            const uint4 e4 = *reinterpret_cast<const uint4*>(alist + first);
            const unsigned int e[4] = {e4.x, e4.y, e4.z, e4.w};
            float val[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) val[i] = tbuf[(e[i] & 127u) * 20u + (unsigned int)c];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(val[i], rsrc_dA, (int)(((e[i] >> 1) & ~63u) | c4), 0, 0);
        };
        // LDS table, four list positions (16 rows) per batch.  Entries past the end of the list aim
        // at a row of +inf, which absorbs any finite addend: their swaps succeed and change nothing.
        int n_table = 0;
        auto swap4 = [&](int first, const float (&val)[4], const unsigned int (&cl)[4], const unsigned int (&sn)[4]) {
            unsigned int got[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                got[i] = lds_cas(cl[i], sn[i], __float_as_uint(__uint_as_float(sn[i]) + val[i]));
            __builtin_amdgcn_sched_barrier(0);   // all four swaps go out before the first result is waited for
            bool lost = false;
#pragma unroll
            for (int i = 0; i < 4; ++i) lost = lost || got[i] != sn[i];
            // Rarely, another wave (or another quarter of this instruction) changed a word between
            // the read and the swap: the lanes that lost go round again for their listed rows.
            if (__builtin_amdgcn_ballot_w64(lost) != 0) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    bool again = got[i] != sn[i] && (first + i) * 4 + g4 < n_table;
                    while (again) {
                        const unsigned int expect = got[i];
                        got[i] = lds_cas(cl[i], expect, __float_as_uint(__uint_as_float(expect) + val[i]));
                        again = got[i] != expect;
                    }
                }
            }
        };
        auto table4 = [&](int first) {   // one batch, read where it is used
            const uint4 e4 = *reinterpret_cast<const uint4*>(tlist + first);
            const unsigned int e[4] = {e4.x, e4.y, e4.z, e4.w};
            float val[4];
            unsigned int cl[4], sn[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                val[i] = tbuf[(e[i] >> 20) * 20u + (unsigned int)c];
                cl[i] = hot_addr + (e[i] & 0xfffffu) + c4;
                sn[i] = *(lds_u32*)(uintptr_t)cl[i];
            }
            swap4(first, val, cl, sn);
        };
        auto core_gradient = [&]() {   // GB[j = 4g+v'][r = c] += sum_samples a_j (-e w_r)
            if constexpr (MODE != kFactorPhase) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int n = 0; n < N; ++n)
                        st.GBacc[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(aY[n][v], wY[n][v], st.GBacc[n], 0, 0, 0);
            }
        };

        if constexpr (AHEAD) {
            // Everything the scatter reads from the staged rows is asked for in one go: the values of the
            // first eight atomic-list positions and of the first four table-list positions.
            const unsigned int ea[8] = {a_first.x, a_first.y, a_first.z, a_first.w, a_second.x, a_second.y, a_second.z, a_second.w};
            const unsigned int et[4] = {t_first.x, t_first.y, t_first.z, t_first.w};
            float aval[8], tval[4];
            unsigned int cell[4], seen[4];
#pragma unroll
            for (int i = 0; i < (N > 1 ? 8 : 4); ++i) aval[i] = tbuf[(ea[i] & 127u) * 20u + (unsigned int)c];
#pragma unroll
            for (int i = 0; i < 4; ++i) tval[i] = tbuf[(et[i] >> 20) * 20u + (unsigned int)c];
            // one-hot operands of the 16 most frequent rows: all compares first, then the products
            float onehot[N][4];
#pragma unroll
            for (int n = 0; n < N; ++n)
                if (g.top[n] > 0) {
                    const uint4 r = *reinterpret_cast<const uint4*>(scur + n * 64 + sub * 16 + 4 * g4);
                    onehot[n][0] = r.x == top_key ? 1.0f : 0.0f;
                    onehot[n][1] = r.y == top_key ? 1.0f : 0.0f;
                    onehot[n][2] = r.z == top_key ? 1.0f : 0.0f;
                    onehot[n][3] = r.w == top_key ? 1.0f : 0.0f;
                }
            const int n_atomic = __builtin_amdgcn_readfirstlane((int)len_atomic);
            n_table = __builtin_amdgcn_readfirstlane((int)len_table);

            // Global atomics.  Eight instructions go out whatever the list holds (entries past its end
            // aim beyond the array and are dropped by the hardware, cheaply): a fixed count lets the
            // compiler wait for prefetched rows without waiting for atomics issued after them.
#pragma unroll
            for (int i = 0; i < (N > 1 ? 8 : 4); ++i)
                __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(aval[i], rsrc_dA, (int)(((ea[i] >> 1) & ~63u) | c4), 0, 0);
            // the table cells of the first batch are read while the matrix core is busy below
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                cell[i] = hot_addr + (et[i] & 0xfffffu) + c4;
                seen[i] = *(lds_u32*)(uintptr_t)cell[i];
            }
#pragma unroll
            for (int b = 2; b < N; ++b)
                if (n_atomic > 16 * b) atomics4(4 * b);
#pragma unroll
            for (int n = 0; n < N; ++n)
                if (g.top[n] > 0) {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        st.Top[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(onehot[n][k], grad[n][k], st.Top[n], 0, 0, 0);
                }
            core_gradient();
            if (n_table > 0) swap4(0, tval, cell, seen);
#pragma unroll
            for (int b = 1; b < N; ++b)
                if (n_table > 16 * b) table4(4 * b);
        } else {
            // the same steps with everything read where it is used (fewer values alive at once)
#pragma unroll
            for (int n = 0; n < N; ++n)
                if (g.top[n] > 0) {
                    const uint4 r = *reinterpret_cast<const uint4*>(scur + n * 64 + sub * 16 + 4 * g4);
                    const unsigned int rw[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const float onehot = rw[k] == top_key ? 1.0f : 0.0f;
                        st.Top[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(onehot, grad[n][k], st.Top[n], 0, 0, 0);
                    }
                }
            const int n_atomic = __builtin_amdgcn_readfirstlane((int)list_len[sub]);
            n_table = __builtin_amdgcn_readfirstlane((int)list_len[4 + sub]);
            atomics4(0);
            if (N > 1) atomics4(4);
#pragma unroll
            for (int b = 2; b < N; ++b)
                if (n_atomic > 16 * b) atomics4(4 * b);
            core_gradient();
#pragma unroll
            for (int b = 0; b < N; ++b)
                if (n_table > 16 * b) table4(4 * b);
        }
        lds_wave_sync();   // the next tile overwrites the staged rows
    }
}

// TILES: Psi is drawn by the tile-sampling rule (runs of 64 neighbouring records) instead of entry
// by entry.  MODE: see process_group (in the synchronous pass g.scale is 1 and not looked at).
template <int N, bool TILES, int MODE>
__global__ void __launch_bounds__(kMfmaThreads) grad_mfma16_kernel(Mfma16Args g) {
    extern __shared__ float lds[];
    constexpr int W4 = (N + 1 + 3) / 4;   // 16-byte words per record
    constexpr int kGroupWords = mfma16_group_words(N);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
    const int c = lane & 15, g4 = lane >> 4;
    float* hot = lds;
    float* wave_lds = lds + (size_t)(g.H + kSinkRows) * 16 + wave * mfma16_wave_scratch(N);
    unsigned int* sbuf = reinterpret_cast<unsigned int*>(wave_lds);   // two parked groups
    float* tbuf = wave_lds + 2 * kGroupWords;                          // [N][16][20]
    float* gbred = lds + (size_t)(g.H + kSinkRows) * 16 + kMfmaWaves * mfma16_wave_scratch(N);

    WaveState<N> st;
#pragma unroll
    for (int n = 0; n < N; ++n) {
        const float* Bn = g.B + g.B_off[n];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            st.Bq[n][k] = Bn[(4 * g4 + k) * 16 + c];
            st.Br[n][k] = Bn[c * 16 + 4 * g4 + k];
        }
        st.GBacc[n] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
        st.Top[n] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int t = 0; t < 4; ++t) st.ring[t][n] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
    }

    const long long M = g.M;
    const uint4* rec4 = reinterpret_cast<const uint4*>(g.coo.rec);
    const unsigned int hot_addr = lds_address(hot);
    // row word of "row c, one of the 16 most frequent" (kept opaque so that the match below is one compare)
    unsigned int top_key = (2u << kRouteShift) + (unsigned int)c * 64u;
    asm volatile("" : "+v"(top_key));

    // Which samples a wave takes: a share [s0, s_end) of Psi made of whole tiles of 16 samples.  The kernel lasts as long
    // as its slowest wave, so the tiles are dealt out evenly: to the workgroups, inside a workgroup to its four pairs of
    // waves w, w + 4 -- the two that share a SIMD -- and inside a pair 9 : 7, because the SIMD serves its older wave
    // first: measured on the benchmark shape, wave w takes 2.5 us per tile and wave w + 4 takes 3.0 us while both run
    // (with |Psi| = 1e6 on 2048 waves: 35 and 26 tiles, where whole groups dealt round-robin gave most waves 32).
    // Which wave sits where is the hardware's choice; a wrong guess costs balance, not correctness.
    // The wave's turns are numbered t = 0, 1, 2, ...:
    //   paired turns (entry rule, when every wave has several turns: g.pair_turns), as long as 128 samples are left:
    //     turns 2u and 2u + 1 share the samples [s0 + 128 u, s0 + 128 u + 128): lane l takes the (2 l)-th of them in
    //     the even turn and the (2 l + 1)-th in the odd one.  Both come out of ONE Philox block (s0 is even: low
    //     and high pair of words), evaluated in the even turn only.
    //   then, and otherwise: turn t is the 64 samples from s0 + 64 t on, lane l its l-th sample; the last turn of
    //     the share may hold fewer than four tiles.
    // Which lane and turn a sample lands in changes the order of the sums only.
    const bool paired = !TILES && g.pair_turns != 0;
    long long s0, s_end;
    int n_pair_turns, n_turns, last_tiles;
    {
        // (the host has done the division: no 64-bit divide on the way to the first record)
        static_assert(kMfmaWaves == 8, "the shares are dealt to four pairs of waves");
        const int b = (int)blockIdx.x;
        const int Tb = g.tiles_each + (b < g.tiles_more ? 1 : 0);              // the workgroup's tiles, from tile b0 on
        const long long b0 = (long long)b * g.tiles_each + (b < g.tiles_more ? b : g.tiles_more);
        const int pr = wave & 3;
        const int Tp = (Tb >> 2) + (pr < (Tb & 3) ? 1 : 0);                    // the pair's tiles, from tile p0 on
        const long long p0 = b0 + pr * (Tb >> 2) + (pr < (Tb & 3) ? pr : (Tb & 3));
        const int older = Tp >= 16 ? (9 * Tp + 15) >> 4 : (Tp + 1) >> 1;
        const int tiles = wave < 4 ? older : Tp - older;
        s0 = (wave < 4 ? p0 : p0 + older) * 16;
        s_end = s0 + tiles * 16 < M ? s0 + tiles * 16 : M;
        n_pair_turns = paired ? 2 * (tiles >> 3) : 0;
        const int rest = tiles - 4 * n_pair_turns;                // tiles of the turns that are not paired
        n_turns = n_pair_turns + ((rest + 3) >> 2);
        last_tiles = (rest & 3) == 0 ? 4 : (rest & 3);
    }
    auto sample_of = [&](long long t) -> long long {   // this lane's sample number in turn t
        if (t < n_pair_turns) return s0 + 128 * (t >> 1) + 2 * lane + (t & 1);
        return s0 + 64 * t + lane;
    };
    auto turn_exists = [&](long long t) -> bool { return t < n_turns; };   // wave-uniform
    auto tiles_of = [&](long long t) -> int { return t == n_turns - 1 ? last_tiles : 4; };
    uint32_t odd_place = 0u;   // entry rule: where the odd turn's sample is read, kept from the even turn

    // record of this lane's sample in turn t: N row numbers and the value's bits.  A slot with no
    // sample of the share behind it reads record 0 and is parked as an empty slot.
    auto load_record = [&](long long t, uint4 (&rec)[W4]) {
        const long long k = sample_of(t);
        uint32_t p;
        if constexpr (TILES) {
            p = tile_place(g.seed, (uint64_t)k, g.rule);
        } else if (t >= n_pair_turns) {
            p = sample_position(g.seed, (uint64_t)k, g.rule.nnz);
        } else {
            if ((t & 1) == 0) {
                const uint64_t ctr = (uint64_t)k >> 1;
                const U4 o = philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), 0u, 0u, (uint32_t)g.seed, (uint32_t)(g.seed >> 32));
                p = (uint32_t)__umul64hi(((uint64_t)o.y << 32) | (uint64_t)o.x, g.rule.nnz);
                odd_place = (uint32_t)__umul64hi(((uint64_t)o.w << 32) | (uint64_t)o.z, g.rule.nnz);
            } else {
                p = odd_place;
            }
        }
        if (k >= s_end) p = 0u;
#pragma unroll
        for (int q = 0; q < W4; ++q) rec[q] = rec4[(size_t)p * W4 + q];
    };
    // Park a group (lane = sample): row words, values, and the two compacted lists of each tile.
    const int my_tile = lane >> 4, my_s = lane & 15;
    const unsigned long long tile_lanes = 0xffffull << (16 * my_tile);
    const unsigned long long lanes_below = tile_lanes & ((1ull << lane) - 1ull);   // of my tile
    auto park_record = [&](long long t, const uint4 (&rec)[W4], unsigned int* dst) {
        const bool act = sample_of(t) < s_end;
        uint32_t flat[4 * W4];
#pragma unroll
        for (int q = 0; q < W4; ++q) {
            flat[4 * q + 0] = rec[q].x;
            flat[4 * q + 1] = rec[q].y;
            flat[4 * q + 2] = rec[q].z;
            flat[4 * q + 3] = rec[q].w;
        }
        unsigned int* atomic_list = dst + (N + 1) * 64 + my_tile * (16 * N);
        unsigned int* table_list = atomic_list + mfma16_list_words(N);
        // every list position starts out unused: lane (tile, quarter q, j) clears positions [q][j], [q][j+4], ...
        {
            const int q = (lane >> 2) & 3, j = lane & 3;
            const unsigned int unused_cell = (unsigned int)(g.H + q) * 64u;   // a row of +inf, one per quarter
#pragma unroll
            for (int i = 0; i < 4 * N; i += 4) {
                atomic_list[q * (4 * N) + j + i] = kNoAtomic;
                table_list[q * (4 * N) + j + i] = unused_cell;
            }
        }
        lds_wave_sync();
        int n_atomic = 0, n_table = 0;   // entries of my tile's lists so far
#pragma unroll
        for (int n = 0; n < N; ++n) {
            // an empty slot: the row just past the mode's last one (reads as zeros), on no list
            const int row = act ? (int)flat[n] : (int)(g.row_bytes[n] >> 6);
            const bool to_table = act && row >= g.top[n] && row < g.K[n];
            const bool to_atomic = act && row >= g.K[n];
            const unsigned int route = (to_atomic || !act) ? 0u : to_table ? 1u : 2u;
            dst[n * 64 + lane] = (unsigned int)row * 64u + (route << kRouteShift);
            const unsigned long long atomic_lanes = __builtin_amdgcn_ballot_w64(to_atomic);
            const unsigned long long table_lanes = __builtin_amdgcn_ballot_w64(to_table);
            const unsigned int slot = (unsigned int)(n * 16 + my_s);
            if (to_atomic) {
                const int p = n_atomic + __popcll(atomic_lanes & lanes_below);
                atomic_list[(p & 3) * (4 * N) + (p >> 2)] = ((g.first_row[n] + (unsigned int)row) << 7) | slot;
            }
            if (to_table) {
                const int p = n_table + __popcll(table_lanes & lanes_below);
                table_list[(p & 3) * (4 * N) + (p >> 2)] = (slot << 20) | ((unsigned int)(g.hot_off[n] + row) * 64u);
            }
            n_atomic += __popcll(atomic_lanes & tile_lanes);
            n_table += __popcll(table_lanes & tile_lanes);
        }
        dst[N * 64 + lane] = act ? flat[N] : 0u;
        if (my_s == 0) {
            dst[(N + 1) * 64 + 2 * mfma16_list_words(N) + my_tile] = (unsigned int)n_atomic;
            dst[(N + 1) * 64 + 2 * mfma16_list_words(N) + 4 + my_tile] = (unsigned int)n_table;
        }
    };

    // fill the pipeline: the records of the wave's first two turns are on their way while the workgroup clears its tables
    uint4 rec[W4], rec0[W4];
    const bool has_turns = turn_exists(0);
    if (has_turns) {
        load_record(0, rec0);
        load_record(1, rec);
    }
    for (int q = tid; q < g.H * 4; q += kMfmaThreads) reinterpret_cast<float4*>(hot)[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int q = tid; q < kSinkRows * 16; q += kMfmaThreads) hot[g.H * 16 + q] = __uint_as_float(0x7f800000u);
    for (int q = tid; q < N * 256; q += kMfmaThreads) gbred[q] = 0.0f;
    __syncthreads();
    if (has_turns) {
        __amdgpu_buffer_rsrc_t rsrc_A[N];
#pragma unroll
        for (int n = 0; n < N; ++n) rsrc_A[n] = make_rsrc(g.A + g.A_off[n], g.row_bytes[n]);

        // ... then the rows of the first three tiles
        park_record(0, rec0, sbuf);
        lds_wave_sync();
#pragma unroll
        for (int t = 0; t < 3; ++t) gather_rows<N>(rsrc_A, sbuf, t, c, g4, st.ring[t]);

        // One turn: park the next turn's records (requested a whole turn ago), request the
        // records of the turn after it, then the four tiles.  Turns past the wave's last one hold
        // only empty slots.
        auto one_turn = [&](long long t, int parity) {
            unsigned int* scur = sbuf + parity * kGroupWords;
            unsigned int* snxt = sbuf + (parity ^ 1) * kGroupWords;
            park_record(t + 1, rec, snxt);
            load_record(t + 2, rec);
            lds_wave_sync();
            process_group<N, MODE>(g, st, hot_addr, top_key, scur, snxt, tbuf, c, g4, tiles_of(t));
        };
        // From order 4 on the first turn is peeled off the loop: the loop proper is then entered with the same sequence
        // of outstanding memory operations as its own back edge, and the compiler's wait counts in the steady state
        // are exact instead of the minimum over both entries (order 5, 1e6 samples: 270 us against 273 us).  Up to order
        // 3 there is one copy of the loop body: a wave has less than ten turns on the benchmark shape, and a second
        // copy of 40 KB of code has to be fetched before it runs (100.1 us against 100.9 us).
        long long t = 0;
        int parity = 0;
        if constexpr (N >= 4) {
            one_turn(0, 0);
            t = 1;
            parity = 1;
        }
        for (; turn_exists(t); ++t, parity ^= 1) one_turn(t, parity);
    }

    // rows 0..15 of each mode: from the wave's accumulators into the workgroup's LDS table (a mode whose table
    // holds fewer than 16 rows never used its accumulator: its zeros aim at the rows of +inf), and the workgroup
    // reduction of the core gradient.  All cells are read, then all swaps issued, then the lost ones repeated, so that
    // the round trips of a wave overlap.  Then one table of plain stores per workgroup.
    {
        unsigned int cell[8 * N], seen[8 * N], got[8 * N];
        float val[8 * N];
#pragma unroll
        for (int n = 0; n < N; ++n)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = g.top[n] > 0 ? g.hot_off[n] + 4 * g4 + v : g.H + v;
                cell[8 * n + v] = hot_addr + (unsigned int)(row * 16 + c) * 4u;
                val[8 * n + v] = st.Top[n][v];
                cell[8 * n + 4 + v] = lds_address(gbred + n * 256 + (4 * g4 + v) * 16 + c);
                val[8 * n + 4 + v] = st.GBacc[n][v];
            }
#pragma unroll
        for (int i = 0; i < 8 * N; ++i) seen[i] = *(lds_u32*)(uintptr_t)cell[i];
#pragma unroll
        for (int i = 0; i < 8 * N; ++i) got[i] = lds_cas(cell[i], seen[i], __float_as_uint(__uint_as_float(seen[i]) + val[i]));
#pragma unroll
        for (int i = 0; i < 8 * N; ++i) {
            bool again = got[i] != seen[i];
            while (again) {
                const unsigned int expect = got[i];
                got[i] = lds_cas(cell[i], expect, __float_as_uint(__uint_as_float(expect) + val[i]));
                again = got[i] != expect;
            }
        }
    }
    __syncthreads();
    float* gb_out = g.gb_partial + (size_t)blockIdx.x * (N * 256);
    for (int q = tid; q < N * 256; q += kMfmaThreads) gb_out[q] = gbred[q];
    float* hot_out = g.hot_partial + (size_t)blockIdx.x * g.H * 16;
    for (int q = tid; q < g.H * 4; q += kMfmaThreads) reinterpret_cast<float4*>(hot_out)[q] = reinterpret_cast<const float4*>(hot)[q];
}

// ---------------------------------------------------------------------------------------------
// Evaluation pass over a set of entries (RMSE / MAE, Section 5.1) for J_n = R = 16: a streaming
// version of the forward half of the gradient kernel.  A wave reads 64 consecutive records
// (coalesced), parks their row numbers, gathers the rows of a 16-entry tile in layout X (16-byte
// loads, the next tile requested while the current one is multiplied) and runs the projections
// on the matrix core; the sum over r is one more product with an all-ones matrix.  Squared and
// absolute errors are summed in double.  No transposes: only layout X is needed here.
// ---------------------------------------------------------------------------------------------
struct ModeBytes {
    unsigned int v[kMfma16MaxOrder];   // I_n * 64: size of mode n's rows in A
};

template <int N>
__global__ void __launch_bounds__(256) errors_mfma16_kernel(Coo coo, uint64_t nnz, const float* __restrict__ A,
                                                            const float* __restrict__ B, Layout L, ModeBytes row_bytes,
                                                            double* __restrict__ sums /* [2]: sse, sae */) {
    typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
    constexpr int W4 = (N + 1 + 3) / 4;
    __shared__ int sidx_all[4][(N + 1) * 64];   // per wave: [N][64] row byte offsets | [64] values
    __shared__ double red[2][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g4 = lane >> 4;
    int* sidx = sidx_all[wave];
    const float* sval = reinterpret_cast<const float*>(sidx + N * 64);
    float Bq[N][4];
    __amdgpu_buffer_rsrc_t rsrc_A[N];
#pragma unroll
    for (int n = 0; n < N; ++n) {
#pragma unroll
        for (int k = 0; k < 4; ++k) Bq[n][k] = B[L.B_off[n] + (4 * g4 + k) * 16 + c];
        rsrc_A[n] = make_rsrc(A + L.A_off[n], row_bytes.v[n]);
    }

    auto gather = [&](int t, floatx4 (&dst)[N]) {
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const uintx4 q = __builtin_amdgcn_raw_buffer_load_b128(rsrc_A[n], sidx[n * 64 + t * 16 + c] + g4 * 16, 0, 0);
            dst[n] = floatx4{__uint_as_float(q[0]), __uint_as_float(q[1]), __uint_as_float(q[2]), __uint_as_float(q[3])};
        }
    };

    const uint4* rec4 = reinterpret_cast<const uint4*>(coo.rec);
    const uint64_t n_groups = (nnz + 63) / 64;
    double sse = 0.0, sae = 0.0;
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
        lds_wave_sync();   // the previous group's reads of the parked words come first
#pragma unroll
        for (int n = 0; n < N; ++n) sidx[n * 64 + lane] = act ? (int)(flat[n] * 64u) : 0;
        sidx[N * 64 + lane] = act ? (int)flat[N] : 0;
        lds_wave_sync();
        floatx4 cur[N], nxt[N];
        gather(0, nxt);
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) {
#pragma unroll
            for (int n = 0; n < N; ++n) cur[n] = nxt[n];
            if (sub < 3) gather(sub + 1, nxt);
            floatx4 acc[N];
#pragma unroll
            for (int n = 0; n < N; ++n) acc[n] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int n = 0; n < N; ++n) acc[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(Bq[n][k], cur[n][k], acc[n], 0, 0, 0);
            floatx4 prod = acc[0];
#pragma unroll
            for (int n = 1; n < N; ++n) prod *= acc[n];
            // xhat of entry (sub * 16 + c): four of its r here, the rest in the other three lane groups
            const float part = (prod[0] + prod[1]) + (prod[2] + prod[3]);
            const floatx4 xsum = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, part, floatx4{0.0f, 0.0f, 0.0f, 0.0f}, 0, 0, 0);
            if (g4 == 0 && group * 64 + sub * 16 + c < nnz) {
                const double e = (double)sval[sub * 16 + c] - (double)xsum[0];
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

// ---------------------------------------------------------------------------------------------
// The update pass, one launch:
//   blocks [0, dense_blocks)                 A <- A - lr_A dA over the dense accumulator (rows that
//                                            were updated with global atomics), clearing it
//   next hot_blocks blocks                   A <- A - lr_A sum_b hot_partial[b] for the rows kept in
//                                            the workgroups' LDS tables (64 elements per block,
//                                            4 threads striding over the partial tables of each)
//   last B_blocks blocks                     B <- B - lr_B (sum_b GB[b] / M + lambda_B B)
// ---------------------------------------------------------------------------------------------
struct ApplyArgs {
    float* A;
    float* dA;
    long long n4;               // float4 elements of the packed A / dA allocation
    int dense_blocks;
    // frequently hit rows
    float* hot_partial;         // [hot_parts][H][J]
    int hot_clear;              // zero the tables as they are read (tables that the next gradient pass adds to with atomics)
    int hot_parts;
    int hot_blocks;             // ceil(H * J / 64)
    int H;
    int J;                      // floats per table row (J_n padded to a multiple of 16)
    int Jn[kMaxOrder];          // floats per row of A^(n)
    int order;
    int K[kMaxOrder];
    int hot_off[kMaxOrder];
    long long A_off[kMaxOrder];
    // core factors
    float* B;
    float* GB;                  // [gb_parts][B_total]
    int B_total;
    int gb_parts;
    int gb_clear;               // zero GB[0] afterwards (single atomically accumulated table)
    float lr_A, lr_B, lambda_B, inv_M;
    unsigned int* clear_word;   // a counter to reset for the next step (or NULL)
};

#ifndef FTK_TEMPLATE_KERNELS_ONLY   // no template: defined in the host file's translation unit only
__global__ void __launch_bounds__(256) apply_kernel(ApplyArgs p) {
    __shared__ float red[4][64];
    const int tid = threadIdx.x;
    int blk = (int)blockIdx.x;
    if (blk < p.dense_blocks) {
        float4* A4 = reinterpret_cast<float4*>(p.A);
        float4* D4 = reinterpret_cast<float4*>(p.dA);
        for (long long q = (long long)blk * 256 + tid; q < p.n4; q += (long long)p.dense_blocks * 256) {
            const float4 d = D4[q];
            const bool nx = d.x != 0.0f, ny = d.y != 0.0f, nz = d.z != 0.0f, nw = d.w != 0.0f;
            if (nx && ny && nz && nw) {
                float4 a = A4[q];
                a.x = fmaf(-p.lr_A, d.x, a.x);
                a.y = fmaf(-p.lr_A, d.y, a.y);
                a.z = fmaf(-p.lr_A, d.z, a.z);
                a.w = fmaf(-p.lr_A, d.w, a.w);
                A4[q] = a;
                D4[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            } else if (nx || ny || nz || nw) {
                // Only the elements with a sum of their own are written.  Four consecutive floats can
                // belong to two rows (J_n need not be a multiple of 4), and the neighbour may be a row
                // of the workgroup tables, which the blocks further down update in this same launch:
                // writing its unchanged value back from here would race with them.
                float* a = p.A + 4 * q;
                if (nx) a[0] = fmaf(-p.lr_A, d.x, a[0]);
                if (ny) a[1] = fmaf(-p.lr_A, d.y, a[1]);
                if (nz) a[2] = fmaf(-p.lr_A, d.z, a[2]);
                if (nw) a[3] = fmaf(-p.lr_A, d.w, a[3]);
                D4[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
        }
        return;
    }
    blk -= p.dense_blocks;
    // 64 consecutive elements per block (256 contiguous bytes of every partial table), four
    // threads per element striding over the tables
    const int ql = tid & 63, sub = tid >> 6;
    const bool is_hot = blk < p.hot_blocks;
    if (!is_hot) blk -= p.hot_blocks;
    const int count = is_hot ? p.H * p.J : p.B_total;
    const int parts = is_hot ? p.hot_parts : p.gb_parts;
    float* src = is_hot ? p.hot_partial : p.GB;
    const bool clear = is_hot && p.hot_clear;
    const int q = blk * 64 + ql;
    float acc0 = 0.0f, acc1 = 0.0f;
    if (q < count) {
        // eight independent loads in flight per thread
        int b = sub;
        for (; b + 28 < parts; b += 32) {
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = src[(size_t)(b + 4 * u) * count + q];
            if (clear) {
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (t[u] != 0.0f) src[(size_t)(b + 4 * u) * count + q] = 0.0f;
            }
            acc0 += (t[0] + t[2]) + (t[4] + t[6]);
            acc1 += (t[1] + t[3]) + (t[5] + t[7]);
        }
        for (; b < parts; b += 4) {
            const float t = src[(size_t)b * count + q];
            if (clear && t != 0.0f) src[(size_t)b * count + q] = 0.0f;
            acc0 += t;
        }
    }
    red[sub][ql] = acc0 + acc1;
    __syncthreads();
    if (tid >= 64 || q >= count) return;
    const float total = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
    if (is_hot) {
        const int hrow = q / p.J, j = q - hrow * p.J;
        int n = -1;
        for (int m = 0; m < p.order; ++m)
            if (hrow >= p.hot_off[m] && hrow < p.hot_off[m] + p.K[m]) n = m;
        if (n >= 0 && j < p.Jn[n] && total != 0.0f) {
            float* a = p.A + p.A_off[n] + (long long)(hrow - p.hot_off[n]) * p.Jn[n] + j;
            *a = fmaf(-p.lr_A, total, *a);
        }
    } else {
        const float b0 = p.B[q];
        p.B[q] = b0 - p.lr_B * fmaf(total, p.inv_M, p.lambda_B * b0);
        if (p.gb_clear) p.GB[q] = 0.0f;
        if (q == 0 && p.clear_word) *p.clear_word = 0u;
    }
}
#endif

}  // namespace ftk
