// Matrix-core gradient and evaluation kernels for general shapes: any order N <= 8 (N <= 10 at P = 1), any J_n <= 16 P,
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
// in registers and parks the records in a private LDS buffer (two of them, used in turn, so the
// rows of a group's first tile can be requested while the group before it is still being worked
// on).  The factor rows of a tile are requested one tile ahead.  Where every J_n is a multiple of
// four (X4) a lane fetches 16 bytes of its sample's row, which is the operand layout of the
// projections, and the other layout comes from an LDS transpose; otherwise lanes fetch single
// floats in the layout of the gradient and the transpose runs the other way.
// Factor-row gradients take the same three routes as in the J = R = 16 kernel: rows 0..15 of a
// mode through the one-hot product, rows [16, K_n) into a table per workgroup, all other rows
// through float atomics.  The atomic is issued by every lane for every element, without a test: an
// element that takes another route gets an out-of-range buffer offset.  The workgroup's table is
//   P <= 2  in LDS (compare-and-swap adds, issued for every element of a tile that has a table row,
//           those of other routes at an LDS row nobody reads): these shapes are bound by the float
//           atomic instructions, and every row summed on chip is an atomic request less;
//   P = 4   in global memory, in the same allocation as the accumulator, and its rows are added by
//           the very atomics that are issued anyway (another offset, nothing else): this shape is
//           bound by instruction issue with one wave per SIMD, the atomic unit has room, and what a
//           table row is for is to keep the most frequent rows from queueing on one address across
//           all workgroups.
// The core gradient lives in matrix-core accumulators for the whole kernel, is summed over the
// workgroup's waves in LDS at the end and leaves the workgroup as one table of plain stores.
//
// ROWS (thread-block strategy (1) of Section 4.2: the rows of a mode are owned by thread blocks, and
// the row update sums over the samples of Psi that hit the row, Eq. Gradient_low_rank): rows outside
// the tables are not added to memory with atomics.  The rows of every mode are cut into buckets of
// 2^shift rows; a workgroup of this kernel keeps one list per bucket, and the gradient row of a
// (sample, mode) is appended to the list of its row's bucket as J_n floats + a word that names the row (padded to
// a multiple of 16 bytes, so that the owner can read an entry with 16-byte loads), with plain stores
// (list positions come from LDS counters).  rows_apply_kernel then gives every bucket to
// one workgroup, which sums the bucket's lists of all gradient workgroups in an LDS table and updates
// the bucket's rows of A^(n) with plain stores: no atomics on A or on an accumulator.  A list that is
// full (their capacities follow the expected counts, with slack) sends the row through the float
// atomic into the accumulator after all, and counts it; the bucket owners fold the accumulator in
// when that counter is not zero.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftk_kernels_mfma16.hpp"

namespace ftk {

// Where element (k, m) of a zero-padded 16 P x 16 P matrix of mode n sits in LDS so that the lane
// (c, g) of a wave finds the four values (k = 16 kb + 4 g + 0..3, m = 16 mb + c) it feeds to four
// consecutive 16x16x4 products in one 16-byte read, and a wave's read covers 1 KB without gaps.
template <int P>
__device__ __forceinline__ int operand_slot(int n, int k, int m) {
    const int kb = k >> 4, g = (k >> 2) & 3, kk = k & 3, mb = m >> 4, c = m & 15;
    return ((n * P + kb) * P + mb) * 256 + (16 * g + c) * 4 + kk;
}

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
    int K[kMaxOrder];            // rows [0, K[n]) of mode n are summed per workgroup (one-hot product or table)
    int top[kMaxOrder];          // 16 if rows 0..15 go through the one-hot product, else 0
    int hot_off[kMaxOrder];      // first table row of mode n
    int H;                       // rows in a workgroup's table
    float* hot_partial;          // [gridDim.x][H][16 P]: the workgroups' tables as the update pass reads them
    float* gb_partial;           // [gridDim.x][B_total]
    int B_total;
    unsigned int mode_bytes[kMaxOrder];   // I_n * J_n * 4
    // P = 4: rows [top[n], K[n]) are added, by the same float atomics as all other rows, to this workgroup's rows
    // of hot_partial, which then sits in the same allocation as dA, behind it:
    unsigned int table_off[kMaxOrder];    // bytes from row 0 of mode n in dA to hot_partial
    unsigned int table_stride;            // bytes of one workgroup's table, H * 16 P * 4
    unsigned int dA_bytes[kMaxOrder];     // bytes from row 0 of mode n in dA to the end of the launch's tables (or mode_bytes[n])
    float lambda_A;
    float scale;                 // 1, or -lr_A in in-place mode
    int sort_mode;               // P <= 2: the samples of a group are parked sorted by their route in this mode (-1: as drawn)
    int tiles_each, tiles_more;  // ceil(M / 16) tiles over the launch's workgroups: each gets tiles_each, the first tiles_more one more
    // ROWS only: the per-workgroup lists of gradient rows (see the header comment)
    float* lists;                // [gridDim.x][list_words]
    unsigned int* list_fill;     // [n_buckets][gridDim.x]: entries in each list when the kernel ends
    const uint2* bucket_info;    // [n_buckets]: x = first word of the bucket's list in a workgroup's area, y = capacity in entries
    unsigned int* overflow;      // entries that found their list full
    unsigned int list_words;     // words in one workgroup's area
    int n_buckets;
    int bucket0[kMaxOrder];      // first bucket of mode n
    int bucket_shift[kMaxOrder]; // rows per bucket of mode n = 1 << shift
};

// words of one list entry of a mode with J floats per row: the row's gradient, the word that names the row (its
// byte offset inside the mode, row * J * 4), padding to 16 bytes
__host__ __device__ constexpr int rows_entry_words(int J) { return (J + 1 + 3) & ~3; }

// one parked group of 64 samples, in words.  Evaluation pass: [order][64] row numbers | [64] values.
__host__ __device__ constexpr int tiled_park_words(int order) { return (order + 1) * 64; }
// Gradient pass: [order][64] byte offsets of the rows inside their modes (for the gathers) | [order][64] route words
// (where the row's gradient goes, decided once per sample when the group is parked) | [64] values
__host__ __device__ constexpr int tiled_grad_park_words(int order) { return (2 * order + 1) * 64; }
// A route word is what the tile adds its column offset to for the float atomic: a byte offset below 2^30 lands (the
// row in the accumulator; P = 4: also the row of the workgroup's table behind it), anything else is out of range:
//   kRouteTable | byte offset of the row in the workgroup's LDS table   (P <= 2)
//   kRouteOneHot | 4 row (row 0..15): summed by the one-hot product;  kRouteNone: nothing to add (no sample)
//   kRouteList | byte offset, in the workgroup's list area, of the entry the row's gradient is written to   (ROWS)
// Every word is a multiple of four (the atomic's address has to be aligned even where it is out of range) and below
// 0xc0000000 (the marker 2^30 of a padded column is added to it and must not wrap).
constexpr unsigned int kRouteTable = 0x40000000u, kRouteOneHot = 0x80000000u, kRouteNone = kRouteOneHot | (0xffu << 2);
constexpr unsigned int kRouteList = 0xa0000000u, kRouteListMask = 0xe0000000u;   // list areas stay below 2^29 bytes
// ROWS: behind the ordinary layout, LDS holds three arrays of n_buckets words (rounded up to a multiple of
// four): list counters | first words | capacities; then per wave and parked group one word, "a list was full"
__host__ __device__ constexpr size_t tiled_rows_lds_words(int order, int waves, int n_buckets) {
    return (size_t)3 * ((n_buckets + 3) & ~3) + (size_t)waves * 2;
}
// per wave: two parked groups, the transpose buffer, and 4 x 16 P words nobody reads (see `sink`)
__host__ __device__ constexpr int tiled_wave_scratch(int order, int P) {
    return 2 * tiled_grad_park_words(order) + kTransposeFloats + 64 * P;
}
__host__ __device__ constexpr size_t tiled_lds_floats(int order, int P, int waves, int H) {
    return (size_t)2 * order * 256 * P * P + (size_t)H * 16 * P + (size_t)waves * tiled_wave_scratch(order, P);
}

// MODE (see process_group in ftk_kernels_mfma16.hpp): kSyncPass serves the synchronous and the fused in-place step
// (g.scale tells them apart); kFactorPhase and kCorePhase are the two passes of Algorithm 1's printed order: in the
// factor phase a tile takes its modes in turn, each with the prediction and GS^(n) at the projections as the modes
// before it left them, adds the row's change to A (scatter as in the in-place step) and advances the samples'
// projections of that mode by the change, c^(n) += delta B^(n) (P x P more products); the core phase takes only the core
// gradient, at the rows the factor phase left.
template <int N, int P, int WAVES, bool X4, bool ROWS, int MODE = kSyncPass>
__global__ void __launch_bounds__(WAVES * 64) grad_tiled_kernel(TiledArgs g) {
    static_assert(MODE == kSyncPass || ((MODE == kFactorPhase || MODE == kCorePhase) && !ROWS), "the passes of the printed order keep no lists");
    extern __shared__ float lds[];
    constexpr int W4 = (N + 1 + 3) / 4;
    constexpr int D = 16 * P;            // padded rank
    constexpr int THREADS = WAVES * 64;
    // Rows [top, K) of a mode: summed in the workgroup's LDS table (P <= 2, where the float atomics are what bounds
    // the pass), or in the workgroup's table in global memory through the atomics every element issues anyway
    // (P = 4, where instruction issue bounds the pass and a swap with its round trip costs more than it saves).
    constexpr bool LDS_TABLE = P < 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g4 = lane >> 4;
    float* Bl = lds;                                 // B^(n) (zero padded) as operands of the projections, see operand_slot
    float* Bt = Bl + N * D * D;                      // its transpose as operands of the A gradient
    float* hot = Bt + N * D * D;                     // [H][D]
    float* wave_lds = hot + (size_t)g.H * D + wave * tiled_wave_scratch(N, P);
    // two parked groups (see tiled_grad_park_words); tbuf [16][20]
    float* tbuf = wave_lds + 2 * tiled_grad_park_words(N);
    // Table updates are issued for every element; those of samples that take another route aim at a
    // row of their own that nobody reads (one per 16-lane group, so they never collide).
    float* sink = tbuf + kTransposeFloats;
    const unsigned int sink_addr = lds_address(sink + g4 * D), hot_addr = lds_address(hot);
    const unsigned int sink_rel = sink_addr - hot_addr;          // beyond every row of the table
    const unsigned int top_key = kRouteOneHot | ((unsigned int)c << 2);   // the route word of row c of the one-hot product
    // Out-of-range marker for buffer offsets: added to anything below 2^30 (every mode is smaller,
    // checked by the host) or to itself it stays beyond the end of the buffer as an unsigned offset.
    constexpr unsigned int kDropped = 0x40000000u;

    for (int q = tid; q < N * D * D; q += THREADS) {
        const int n = q / (D * D), rem = q - n * D * D, j = rem / D, r = rem - j * D;
        const float b = (j < g.J[n] && r < g.R) ? g.B[g.B_off[n] + j * g.R + r] : 0.0f;
        Bl[operand_slot<P>(n, j, r)] = b;
        // the factor every row gradient carries (1, or -lr_A in in-place mode) rides in the operand of the A-gradient
        // products, the only place Bt is used: -e GS comes out of the matrix cores already scaled
        Bt[operand_slot<P>(n, r, j)] = g.scale * b;
    }
    for (int q = tid; q < g.H * D; q += THREADS) hot[q] = 0.0f;
    for (int q = lane; q < 4 * D; q += 64) sink[q] = __builtin_inff();
    // ROWS: list counters, bucket info and the parked entry words behind everything else
    const int nb4 = (g.n_buckets + 3) & ~3;
    unsigned int* list_count = reinterpret_cast<unsigned int*>(hot + (size_t)g.H * D + WAVES * tiled_wave_scratch(N, P));
    unsigned int* list_first = list_count + nb4;
    unsigned int* list_cap = list_first + nb4;
    unsigned int* wave_full = list_cap + nb4 + wave * 2;   // per parked group: a list was full
    if constexpr (ROWS) {
        for (int q = tid; q < g.n_buckets; q += THREADS) {
            const uint2 info = g.bucket_info[q];
            list_count[q] = 0u;
            list_first[q] = info.x;
            list_cap[q] = info.y;
        }
    }

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
        rsrc_dA[n] = make_rsrc(g.dA + g.A_off[n], LDS_TABLE ? g.mode_bytes[n] : g.dA_bytes[n]);
    }
    // ROWS: this workgroup's list area (the host keeps list_words below 2^27, so byte offsets stay below 2^29)
    const __amdgpu_buffer_rsrc_t rsrc_lists =
        make_rsrc(ROWS ? (const void*)(g.lists + (size_t)blockIdx.x * g.list_words) : (const void*)g.A, ROWS ? g.list_words * 4u : 0u);

    const long long M = g.M;
    const float lambda_scaled = g.lambda_A * g.scale;
    // Every wave takes a contiguous share of Psi made of whole tiles: the launch's ceil(M / 16) tiles go evenly to the
    // workgroups (the host has done that division), a workgroup's tiles evenly to its four SIMDs, so that the work
    // differs by one tile at most, where whole groups of 64 dealt round-robin leave up to four tiles between the waves.
    // The wave goes through its share in groups of 64; the last group may hold fewer than four tiles, and the tiles it
    // does not hold are not run.
    // Eight waves: waves w and w + 4 share a SIMD, which serves the older one (w) first, so the two split the SIMD's
    // tiles 9 : 7 and finish together (measured: 1 % of the pass on C3, C4 and the order sweep; 10 : 6 is too much).
    // Which wave sits where is the hardware's choice; a wrong guess costs balance, not correctness.
    static_assert(WAVES == 4 || WAVES == 8, "one or two waves per SIMD");
    const int wg = (int)blockIdx.x;
    const int wg_tiles = g.tiles_each + (wg < g.tiles_more ? 1 : 0);
    const long long wg_first = (long long)wg * g.tiles_each + (wg < g.tiles_more ? wg : g.tiles_more);
    const int simd = wave & 3;
    const int simd_tiles = (wg_tiles >> 2) + (simd < (wg_tiles & 3) ? 1 : 0);
    long long first_tile = wg_first + simd * (wg_tiles >> 2) + (simd < (wg_tiles & 3) ? simd : (wg_tiles & 3));
    int my_tiles = simd_tiles;
    if constexpr (WAVES == 8) {
        const int older = simd_tiles >= 16 ? (9 * simd_tiles + 15) >> 4 : (simd_tiles + 1) >> 1;
        my_tiles = wave < 4 ? older : simd_tiles - older;
        first_tile += wave < 4 ? 0 : older;
    }
    const long long first = first_tile * 16;
    const int mine = first < M ? (int)min((long long)my_tiles * 16, M - first) : 0;   // this wave's samples are [first, first + mine)
    const int n_groups = (mine + 63) / 64;
    const uint4* rec4 = reinterpret_cast<const uint4*>(g.coo.rec);
    auto load_record = [&](int grp, uint4 (&rec)[W4]) {
        const int local = grp * 64 + lane;
        const uint32_t p = local < mine ? sample_place(g.seed, (uint64_t)(first + local), g.rule) : 0u;
#pragma unroll
        for (int q = 0; q < W4; ++q) rec[q] = rec4[(size_t)p * W4 + q];
    };

    // Park a group's records: per (sample, mode) the byte offset of the row inside its mode (lanes past the end of Psi:
    // the end of the mode, which reads as zeros) and the route word; per sample the value (lanes past the end: 0).
    // ROWS: every (sample, mode) whose row is outside the tables also takes its place in the list of
    // its row's bucket here (one LDS counter increment per lane and mode); its route word names that place.
    auto park_record = [&](int grp, const uint4 (&rec)[W4], float* park, unsigned int* was_full) {
        const bool act = grp * 64 + lane < mine;
        uint32_t flat[4 * W4];
#pragma unroll
        for (int q = 0; q < W4; ++q) {
            flat[4 * q + 0] = rec[q].x;
            flat[4 * q + 1] = rec[q].y;
            flat[4 * q + 2] = rec[q].z;
            flat[4 * q + 3] = rec[q].w;
        }
        unsigned int* words = reinterpret_cast<unsigned int*>(park);
        unsigned int list_word[N];   // ROWS: the route word of a row whose gradient goes to a list, else 0
#pragma unroll
        for (int n = 0; n < N; ++n) list_word[n] = 0u;
        if constexpr (ROWS) {
            bool full = false;
#pragma unroll
            for (int n = 0; n < N; ++n) {
                const int row = (int)flat[n];
                if (act && row >= g.K[n]) {
                    const int b = g.bucket0[n] + ((row - g.K[n]) >> g.bucket_shift[n]);
                    const unsigned int place = atomicAdd(&list_count[b], 1u);
                    if (place < list_cap[b]) {
                        list_word[n] = kRouteList | ((list_first[b] + place * (unsigned int)rows_entry_words(g.J[n])) * 4u);
                    } else {   // the row goes through the float atomic after all
                        full = true;
                        atomicAdd(g.overflow, 1u);
                    }
                }
            }
            const unsigned long long any_full = __builtin_amdgcn_ballot_w64(full);
            if (lane == 0) *was_full = any_full != 0ull ? 1u : 0u;
        }
        unsigned int in_mode[N], route[N];
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const int row = (int)flat[n];
            in_mode[n] = act ? (unsigned int)(row * g.J[n] * 4) : g.mode_bytes[n];
            if (!act)
                route[n] = kRouteNone;
            else if (list_word[n] != 0u)
                route[n] = list_word[n];
            else if (row < g.top[n])
                route[n] = kRouteOneHot | ((unsigned int)row << 2);
            else if (row < g.K[n])
                route[n] = LDS_TABLE ? kRouteTable | (unsigned int)((g.hot_off[n] + row) * D * 4)
                                     : g.table_off[n] + (unsigned int)blockIdx.x * g.table_stride + (unsigned int)((g.hot_off[n] + row) * D * 4);
            else
                route[n] = in_mode[n];
        }
        // Where the sample is parked.  The order of the samples inside a group of 64 is free (it changes the order of
        // the sums only).  P <= 2: the group is sorted by the kind of route its row takes in the mode the host names
        // (the one whose routes are most mixed), so that a tile tends to hold one kind: the table swaps and the one-hot
        // products of that mode are skipped in the tiles without such a row, and the atomic instructions of the other
        // tiles carry no request.  Equal keys keep their order, so the lanes past the end of Psi (largest key) stay last.
        int slot = lane;
        if constexpr (LDS_TABLE) {
            if (g.sort_mode >= 0) {
                unsigned int key = 0u;
#pragma unroll
                for (int n = 0; n < N; ++n) key = n == g.sort_mode ? route[n] >> 30 : key;
                if (!act) key = 3u;
                slot = 0;
#pragma unroll
                for (unsigned int k = 0; k < 4; ++k) {
                    const unsigned long long same = __builtin_amdgcn_ballot_w64(key == k);
                    const int before = (int)__builtin_amdgcn_mbcnt_hi((unsigned int)(same >> 32), __builtin_amdgcn_mbcnt_lo((unsigned int)same, 0u));
                    slot += key > k ? __builtin_popcountll(same) : key == k ? before : 0;
                }
            }
        }
#pragma unroll
        for (int n = 0; n < N; ++n) {
            words[n * 64 + slot] = in_mode[n];
            words[(N + n) * 64 + slot] = route[n];
        }
        park[2 * N * 64 + slot] = act ? __uint_as_float(flat[N]) : 0.0f;
    };
    // Request the factor rows of tile `sub` of a parked group whose first sample is number `first`.
    //   X4: rows[n][jb] = components 16 jb + 4g .. +3 of the row of sample c           (layout X)
    //  !X4: rows[n][jb][v] = component 16 jb + c of the row of sample 4g + v            (layout Y)
    // Components past J_n and samples past the end of Psi read as zero (out-of-range offset).
    auto gather_rows = [&](const float* park, int sub, floatx4 (&rows)[N][P]) {
        const int* in_mode = reinterpret_cast<const int*>(park);   // byte offsets of the rows; the end of the mode for no sample
        if constexpr (X4) {
#pragma unroll
            for (int n = 0; n < N; ++n) {
                const int row_off = in_mode[n * 64 + sub * 16 + c];
#pragma unroll
                for (int jb = 0; jb < P; ++jb) {
                    const int col = 16 * jb + 4 * g4;
                    const int off = col < g.J[n] ? row_off + col * 4 : (int)g.mode_bytes[n];
                    rows[n][jb] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rsrc_A[n], off, 0, 0));
                }
            }
        } else {
#pragma unroll
            for (int n = 0; n < N; ++n) {
                const int4 r = *reinterpret_cast<const int4*>(in_mode + n * 64 + sub * 16 + 4 * g4);
                const int rr[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
                for (int jb = 0; jb < P; ++jb) {
                    const int col = 16 * jb + c;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int off = col < g.J[n] ? rr[v] + col * 4 : (int)g.mode_bytes[n];
                        rows[n][jb][v] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc_A[n], off, 0, 0));
                    }
                }
            }
        }
    };

    uint4 rec[W4];
    int group = 0;
    floatx4 cur[N][P];
    int buf = 0;
    if (group < n_groups) {
        load_record(group, rec);
        park_record(group, rec, wave_lds, wave_full);
        lds_wave_sync();
        if (group + 1 < n_groups) load_record(group + 1, rec);
        gather_rows(wave_lds, 0, cur);
    }

#pragma unroll 1
    for (; group < n_groups; ++group, buf ^= 1) {
        const int tiles = min(4, (mine - 64 * group + 15) / 16);   // four, but for the last group of the share
        const float* park = wave_lds + buf * tiled_grad_park_words(N);
        float* park_next = wave_lds + (buf ^ 1) * tiled_grad_park_words(N);
        const unsigned int* routes = reinterpret_cast<const unsigned int*>(park) + N * 64;
        const float* sval = park + 2 * N * 64;
        const unsigned int* was_full = wave_full + buf;
        unsigned int* was_full_next = wave_full + (buf ^ 1);

#pragma unroll 1
        for (int sub = 0; sub < tiles; ++sub) {
            // Request the next tile's rows (past the last group every lane is past the end of Psi and
            // nothing is read).  X4: into the registers of this tile's rows as soon as the projections
            // have consumed them; otherwise those registers stay in use as the gradient's layout, and
            // the request goes out at the top of the tile into registers of its own.
            auto request_next = [&](floatx4 (&rows)[N][P]) {
                if (sub < 3) {
                    gather_rows(park, sub + 1, rows);
                } else {
                    if (group + 1 < n_groups) {
                        park_record(group + 1, rec, park_next, was_full_next);
                        lds_wave_sync();
                        if (group + 2 < n_groups) load_record(group + 2, rec);
                    }
                    gather_rows(park_next, 0, rows);
                }
            };
            floatx4 nxt[X4 ? 1 : N][X4 ? 1 : P];
            if constexpr (!X4) request_next(nxt);

            const float x = sval[sub * 16 + c];
            // both layouts of the tile's rows: aX[k] = component 16 jb + 4g + k of sample c (only used
            // by the projections), aY[n][jb][v] = component 16 jb + c of sample 4g + v
            float aY[N][P][4];
            // projections (layout X): s[n][rb][v] = c^(n)_{r = 16 rb + 4g + v} of sample c
            // The core-factor operands of a block of products are read from LDS one block ahead of the
            // products that use them (the scheduling barrier keeps the reads where they are written).
            // (Not for P = 4, where the registers are all taken: there each block reads its own.)
            constexpr bool AHEAD = P < 4;
            floatx4 s[N][P];
            float4 bop[P];
            if constexpr (AHEAD) {
#pragma unroll
                for (int rb = 0; rb < P; ++rb) bop[rb] = *reinterpret_cast<const float4*>(Bl + rb * 256 + lane * 4);
            }
#pragma unroll
            for (int n = 0; n < N; ++n) {
#pragma unroll
                for (int rb = 0; rb < P; ++rb) s[n][rb] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int jb = 0; jb < P; ++jb) {
                    float4 bcur[P];
                    if constexpr (AHEAD) {
#pragma unroll
                        for (int rb = 0; rb < P; ++rb) bcur[rb] = bop[rb];
                        if (n * P + jb + 1 < N * P) {
#pragma unroll
                            for (int rb = 0; rb < P; ++rb)
                                bop[rb] = *reinterpret_cast<const float4*>(Bl + ((n * P + jb + 1) * P + rb) * 256 + lane * 4);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    } else {
#pragma unroll
                        for (int rb = 0; rb < P; ++rb)
                            bcur[rb] = *reinterpret_cast<const float4*>(Bl + ((n * P + jb) * P + rb) * 256 + lane * 4);
                    }
                    float ax[4];
                    if constexpr (X4) {
#pragma unroll
                        for (int k = 0; k < 4; ++k) ax[k] = cur[n][jb][k];
                        *reinterpret_cast<float4*>(tbuf + c * 20 + 4 * g4) = make_float4(ax[0], ax[1], ax[2], ax[3]);
                        lds_wave_sync();
#pragma unroll
                        for (int v = 0; v < 4; ++v) aY[n][jb][v] = tbuf[(4 * g4 + v) * 20 + c];
                        lds_wave_sync();
                    } else {
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            aY[n][jb][v] = cur[n][jb][v];
                            tbuf[(4 * g4 + v) * 20 + c] = aY[n][jb][v];
                        }
                        lds_wave_sync();
                        const float4 ax4 = *reinterpret_cast<const float4*>(tbuf + c * 20 + 4 * g4);
                        lds_wave_sync();
                        ax[0] = ax4.x;
                        ax[1] = ax4.y;
                        ax[2] = ax4.z;
                        ax[3] = ax4.w;
                    }
#pragma unroll
                    for (int rb = 0; rb < P; ++rb) {
                        const float bk[4] = {bcur[rb].x, bcur[rb].y, bcur[rb].z, bcur[rb].w};
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            s[n][rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(bk[k], ax[k], s[n][rb], 0, 0, 0);
                    }
                }
            }

            // P = 4: the request waits until the last mode's gradients are under way: the registers it fills are then free
            // for the leave-one-out products and the A-gradient stage, which otherwise shuttle values through the
            // other half of the register file (C5 0.780 -> 0.761 ms per launch); the rows still have a third of the
            // tile's matrix work to arrive in.
            constexpr bool LATE_REQUEST = P == 4;
            if constexpr (X4 && !LATE_REQUEST) request_next(cur);

            // leave-one-out products, prediction, error (factor phase: per mode, further down)
            floatx4 w[N][P];
            float xhat = 0.0f;
#pragma unroll
            for (int rb = 0; rb < (MODE == kFactorPhase ? 0 : P); ++rb) {
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
            float neg_e = xhat - x;

            float4 top_[P];   // operands of the next block of the A-gradient products, read one block ahead
            if constexpr (AHEAD) {
#pragma unroll
                for (int jb = 0; jb < P; ++jb) top_[jb] = *reinterpret_cast<const float4*>(Bt + jb * 256 + lane * 4);
            }
#pragma unroll
            for (int n = 0; n < N; ++n) {
                if constexpr (X4 && LATE_REQUEST) {
                    if (n == N - 1) request_next(cur);
                }
                if constexpr (MODE == kFactorPhase) {
                    // w^(n), prediction and error from the projections as they stand: those of modes < n already advanced
                    float part = 0.0f;
#pragma unroll
                    for (int rb = 0; rb < P; ++rb) {
                        floatx4 wn = {1.0f, 1.0f, 1.0f, 1.0f};
#pragma unroll
                        for (int k = 0; k < N; ++k)
                            if (k != n) wn *= s[k][rb];
                        w[n][rb] = wn;
                        const floatx4 full = wn * s[n][rb];
                        part += (full[0] + full[1]) + (full[2] + full[3]);
                    }
                    part += __shfl_xor(part, 16);
                    part += __shfl_xor(part, 32);
                    neg_e = part - x;
                }
                // -e w^(n) (layout X), -e GS^(n) (layout Y), and -e w^(n) in layout Y through LDS
                floatx4 gs[P];
                float wY[P][4];
#pragma unroll
                for (int jb = 0; jb < P; ++jb) gs[jb] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int rb = 0; rb < P; ++rb) {
                    float4 tcur[P];
                    if constexpr (AHEAD) {
#pragma unroll
                        for (int jb = 0; jb < P; ++jb) tcur[jb] = top_[jb];
                        if (n * P + rb + 1 < N * P) {
#pragma unroll
                            for (int jb = 0; jb < P; ++jb)
                                top_[jb] = *reinterpret_cast<const float4*>(Bt + ((n * P + rb + 1) * P + jb) * 256 + lane * 4);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    } else {
#pragma unroll
                        for (int jb = 0; jb < P; ++jb)
                            tcur[jb] = *reinterpret_cast<const float4*>(Bt + ((n * P + rb) * P + jb) * 256 + lane * 4);
                    }
                    const floatx4 wp = w[n][rb] * neg_e;
                    *reinterpret_cast<float4*>(tbuf + c * 20 + 4 * g4) = make_float4(wp[0], wp[1], wp[2], wp[3]);
                    if constexpr (MODE != kCorePhase) {
#pragma unroll
                        for (int jb = 0; jb < P; ++jb) {
                            const float tk[4] = {tcur[jb].x, tcur[jb].y, tcur[jb].z, tcur[jb].w};
#pragma unroll
                            for (int k = 0; k < 4; ++k)
                                gs[jb] = __builtin_amdgcn_mfma_f32_16x16x4f32(wp[k], tk[k], gs[jb], 0, 0, 0);
                        }
                    }
                    lds_wave_sync();
#pragma unroll
                    for (int v = 0; v < 4; ++v) wY[rb][v] = tbuf[(4 * g4 + v) * 20 + c];
                    lds_wave_sync();
                }

                if constexpr (MODE == kCorePhase) {
#pragma unroll
                    for (int jb = 0; jb < P; ++jb)
#pragma unroll
                        for (int rb = 0; rb < P; ++rb)
#pragma unroll
                            for (int v = 0; v < 4; ++v)
                                GBacc[n][jb][rb] =
                                    __builtin_amdgcn_mfma_f32_16x16x4f32(aY[n][jb][v], wY[rb][v], GBacc[n][jb][rb], 0, 0, 0);
                    continue;
                }
                // factor-row gradients: where each row's goes was decided when the group was parked (route words, see
                // tiled_grad_park_words).  Padding columns and samples past the end of Psi have a = 0 and -e GS = 0, so
                // their gradient is zero without a test; what keeps them out of dA is the offset.
                const uint4 routes4 = *reinterpret_cast<const uint4*>(routes + n * 64 + sub * 16 + 4 * g4);
                const unsigned int abase[4] = {routes4.x, routes4.y, routes4.z, routes4.w};   // samples 4g .. 4g+3
                unsigned int tbase[4];      // P <= 2: LDS address of the sample's table row, or of the row nobody reads
                float onehot[4];
                bool is_top[4];
                // ROWS: the byte offset of each sample's list entry in the workgroup's list area (or the marker), the word that
                // names its row in the entry (the row's byte offset inside its mode), and whether any list of the group was full
                unsigned int entv[4] = {kDropped, kDropped, kDropped, kDropped};
                unsigned int rowv[4] = {0u, 0u, 0u, 0u};
                bool group_had_full_list = false;
                if constexpr (ROWS) {
                    const uint4 r4 = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned int*>(park) + n * 64 + sub * 16 + 4 * g4);
                    rowv[0] = r4.x;
                    rowv[1] = r4.y;
                    rowv[2] = r4.z;
                    rowv[3] = r4.w;
#pragma unroll
                    for (int v = 0; v < 4; ++v) entv[v] = (abase[v] & kRouteListMask) == kRouteList ? abase[v] & ~kRouteListMask : kDropped;
                    group_had_full_list = __builtin_amdgcn_readfirstlane((int)*was_full) != 0;
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    // a table word minus its tag is the row's offset in the table, every other word lands far above it
                    if constexpr (LDS_TABLE) tbase[v] = hot_addr + min(abase[v] - kRouteTable, sink_rel);
                    is_top[v] = abase[v] == top_key;
                    onehot[v] = is_top[v] ? 1.0f : 0.0f;
                }
                // ROWS: the atomics only go out where a row needs them (its list was full; P = 4: a table row)
                bool rows_need_atomics = group_had_full_list;
                if constexpr (ROWS && !LDS_TABLE) {
                    if (g.K[n] > g.top[n])
                        rows_need_atomics = rows_need_atomics || __builtin_amdgcn_ballot_w64(min(min(abase[0], abase[1]), min(abase[2], abase[3])) < kRouteTable) != 0;
                }
                // Table rows (P <= 2): compare-and-swap adds, the reads of all the lane's elements of the mode first,
                // then the swaps, so their round trips overlap.  A swap loses when another wave, another lane of the
                // same instruction or an earlier element of this lane changed the word in between: those go round
                // again.  The rows nobody reads hold +inf, which absorbs any finite addend: swaps aimed there succeed
                // and change nothing, so no lane has to be told apart.
                constexpr int BATCH = LDS_TABLE ? 4 * P : 1;
                unsigned int cell[BATCH];
                float tval[BATCH];
                auto table_batch = [&]() {
                    unsigned int seen[BATCH], got[BATCH];
#pragma unroll
                    for (int i = 0; i < BATCH; ++i) seen[i] = *(lds_u32*)(uintptr_t)cell[i];
#pragma unroll
                    for (int i = 0; i < BATCH; ++i)
                        got[i] = lds_cas(cell[i], seen[i], __float_as_uint(__uint_as_float(seen[i]) + tval[i]));
                    __builtin_amdgcn_sched_barrier(0);
                    bool lost = false;
#pragma unroll
                    for (int i = 0; i < BATCH; ++i) lost = lost || got[i] != seen[i];
                    if (__builtin_amdgcn_ballot_w64(lost) != 0) {
#pragma unroll
                        for (int i = 0; i < BATCH; ++i) {
                            bool again = got[i] != seen[i];
                            while (again) {
                                const unsigned int expect = got[i];
                                got[i] = lds_cas(cell[i], expect, __float_as_uint(__uint_as_float(expect) + tval[i]));
                                again = got[i] != expect;
                            }
                        }
                    }
                };
                // the one-hot products are skipped for a tile in which no sample hits rows 0..15 of this mode, the swaps
                // for a tile in which no sample has a table row (wave-uniform tests)
                const bool any_top = g.top[n] > 0 && __builtin_amdgcn_ballot_w64(is_top[0] || is_top[1] || is_top[2] || is_top[3]) != 0;
                bool any_table = false;
                if constexpr (LDS_TABLE) {
                    if (g.K[n] > g.top[n])
                        any_table = __builtin_amdgcn_ballot_w64(min(min(tbase[0], tbase[1]), min(tbase[2], tbase[3])) < sink_addr) != 0;
                }
#pragma unroll
                for (int jb = 0; jb < P; ++jb) {
                    // byte offset of the lane's column inside a row, or the marker for columns past J_n
                    const unsigned int col4 = 16 * jb + c < g.J[n] ? (unsigned int)((16 * jb + c) * 4) : kDropped;
                    float grad[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        grad[v] = fmaf(lambda_scaled, aY[n][jb][v], gs[jb][v]);
                        if constexpr (ROWS) {
                            // the list entry: components 0 .. J_n - 1, then the word that names the row (its lane may be in
                            // a block of columns of its own when J_n is a multiple of 16: see below)
                            const int col = 16 * jb + c;
                            const unsigned int word = col < g.J[n] ? __float_as_uint(grad[v]) : rowv[v];
                            const unsigned int off = col <= g.J[n] ? entv[v] + (unsigned int)col * 4u : kDropped;
                            __builtin_amdgcn_raw_buffer_store_b32(word, rsrc_lists, (int)off, 0, 0);
                            if (rows_need_atomics)
                                __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(grad[v], rsrc_dA[n], (int)(abase[v] + col4), 0, 0);
                        } else {
                            __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(grad[v], rsrc_dA[n], (int)(abase[v] + col4), 0, 0);
                        }
                        if constexpr (LDS_TABLE) {
                            cell[4 * jb + v] = tbase[v] + (unsigned int)((16 * jb + c) * 4);
                            tval[4 * jb + v] = grad[v];
                        }
                    }
                    if (any_top) {
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            Top[n][jb] = __builtin_amdgcn_mfma_f32_16x16x4f32(onehot[k], grad[k], Top[n][jb], 0, 0, 0);
                    }
                    if constexpr (MODE == kFactorPhase) {
                        // the block of the row's change (layout Y) goes through LDS into layout X and advances the
                        // sample's projections of this mode: c^(n)[rb] += delta[jb] B^(n)[jb][rb]
                        if (n + 1 < N) {
#pragma unroll
                            for (int v = 0; v < 4; ++v) tbuf[(4 * g4 + v) * 20 + c] = grad[v];
                            lds_wave_sync();
                            const float4 dx4 = *reinterpret_cast<const float4*>(tbuf + c * 20 + 4 * g4);
                            lds_wave_sync();
                            const float dx[4] = {dx4.x, dx4.y, dx4.z, dx4.w};
#pragma unroll
                            for (int rb = 0; rb < P; ++rb) {
                                const float4 b4 = *reinterpret_cast<const float4*>(Bl + ((n * P + jb) * P + rb) * 256 + lane * 4);
                                const float bk[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
                                for (int k = 0; k < 4; ++k)
                                    s[n][rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(bk[k], dx[k], s[n][rb], 0, 0, 0);
                            }
                        }
                    } else {
                        // core gradient block: GB[j = 16 jb + 4g + v'][r = 16 rb + c]
#pragma unroll
                        for (int rb = 0; rb < P; ++rb)
#pragma unroll
                            for (int v = 0; v < 4; ++v)
                                GBacc[n][jb][rb] =
                                    __builtin_amdgcn_mfma_f32_16x16x4f32(aY[n][jb][v], wY[rb][v], GBacc[n][jb][rb], 0, 0, 0);
                    }
                }
                if constexpr (LDS_TABLE) {
                    if (any_table) table_batch();
                }
                if constexpr (ROWS) {
                    if (g.J[n] == D) {   // no lane of the blocks above holds column J_n: the rows' words go out on their own
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const unsigned int off = c == 0 ? entv[v] + (unsigned int)D * 4u : kDropped;
                            __builtin_amdgcn_raw_buffer_store_b32(rowv[v], rsrc_lists, (int)off, 0, 0);
                        }
                    }
                }
            }
            if constexpr (!X4) {
#pragma unroll
                for (int n = 0; n < N; ++n)
#pragma unroll
                    for (int jb = 0; jb < P; ++jb) cur[n][jb] = nxt[n][jb];
            }
        }
    }

    // rows 0..15 of each mode: from the wave's accumulators into the workgroup's LDS table
#pragma unroll
    for (int n = 0; n < (MODE == kCorePhase ? 0 : N); ++n)
        if (g.top[n] > 0) {
#pragma unroll
            for (int jb = 0; jb < P; ++jb)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    lds_float_add(hot + (size_t)(g.hot_off[n] + 4 * g4 + v) * D + 16 * jb + c, Top[n][jb][v]);
        }
    // core gradient: summed over the workgroup's waves in LDS, where the operand tables are no longer needed (the
    // waves take turns, so plain adds do), and stored as one table per workgroup (entries outside J_n x R are padding)
    __syncthreads();
    float* gb_sum = lds;   // [N][D][D]
#pragma unroll 1
    for (int turn = 0; turn < (MODE == kFactorPhase ? 0 : WAVES); ++turn) {
        if (wave == turn) {
#pragma unroll
            for (int n = 0; n < N; ++n)
#pragma unroll
                for (int jb = 0; jb < P; ++jb)
#pragma unroll
                    for (int rb = 0; rb < P; ++rb)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            float* cell = gb_sum + ((size_t)n * D + 16 * jb + 4 * g4 + v) * D + 16 * rb + c;
                            *cell = turn == 0 ? GBacc[n][jb][rb][v] : *cell + GBacc[n][jb][rb][v];
                        }
        }
        __syncthreads();
    }
    if constexpr (MODE != kFactorPhase) {
        float* gb_out = g.gb_partial + (size_t)blockIdx.x * g.B_total;
        for (int q = tid; q < N * D * D; q += THREADS) {
            const int n = q / (D * D), rem = q - n * D * D, j = rem / D, r = rem - j * D;
            if (j < g.J[n] && r < g.R) gb_out[g.B_off[n] + j * g.R + r] = gb_sum[q];
        }
        __syncthreads();
    }
    if constexpr (MODE == kCorePhase) return;
    float* hot_out = g.hot_partial + (size_t)blockIdx.x * g.H * D;
    if constexpr (LDS_TABLE) {
        for (int q = tid; q < g.H * D; q += THREADS) hot_out[q] = hot[q];
    } else {
        // only rows 0..15 of a mode were summed on chip; the other table rows of hot_out hold what the atomics added
#pragma unroll
        for (int n = 0; n < N; ++n)
            if (g.top[n] > 0)
                for (int q = tid; q < 16 * D; q += THREADS) hot_out[g.hot_off[n] * D + q] = hot[g.hot_off[n] * D + q];
    }
    if constexpr (ROWS) {
        for (int q = tid; q < g.n_buckets; q += THREADS)
            g.list_fill[(size_t)q * gridDim.x + blockIdx.x] = min(list_count[q], list_cap[q]);
    }
}

// ---------------------------------------------------------------------------------------------
// ROWS, second half: one workgroup per bucket of rows.  It sums, in an LDS table, the gradient rows
// that the gradient workgroups appended to their lists of this bucket, and then updates the bucket's
// rows A^(n)[i,:] <- A^(n)[i,:] - lr_A (sum) with plain stores.  If any list was full during the
// gradient pass (the counter is not zero), the rows that went into the accumulator instead are
// folded in (and the accumulator cleared) first.
// ---------------------------------------------------------------------------------------------
struct RowsApplyArgs {
    const float* lists;              // [n_sources][list_words]
    const unsigned int* list_fill;   // [n_buckets][n_sources]
    const uint2* bucket_info;        // [n_buckets]: first word, capacity
    const int4* bucket_rows;         // [n_buckets]: x = mode, y = first row of the bucket within its mode, z = rows in the bucket
    unsigned int list_words;
    int n_buckets;
    int n_sources;                   // workgroups of the gradient launch
    float* A;
    float* dA;
    long long A_off[kMaxOrder];
    int J[kMaxOrder];
    const unsigned int* overflow;
    float lr_A;
};

constexpr int kRowsApplyThreads = 512;
constexpr int kRowsApplyMaxSources = 1024;   // gradient workgroups (one per CU)
#ifndef FTK_TEMPLATE_KERNELS_ONLY   // no template: defined in the host file's translation unit only
__global__ void __launch_bounds__(kRowsApplyThreads) rows_apply_kernel(RowsApplyArgs p) {
    extern __shared__ float table[];   // [rows][J_n]
    __shared__ unsigned int fill[kRowsApplyMaxSources];
    const int tid = threadIdx.x;
    const int b = (int)blockIdx.x;
    const int4 d = p.bucket_rows[b];
    const int n = d.x, row0 = d.y, rows = d.z, J = p.J[n], stride = rows_entry_words(J);
    const int cells = rows * J;
    const uint2 info = p.bucket_info[b];
    const int cap = (int)info.y;
    for (int q = tid; q < cells; q += kRowsApplyThreads) table[q] = 0.0f;
    for (int w = tid; w < p.n_sources; w += kRowsApplyThreads) fill[w] = p.list_fill[(size_t)b * p.n_sources + w];
    __syncthreads();
    // Every place of every source's list of this bucket is one work item (places past a list's fill
    // are skipped), so that the loads of many lists are in flight at once: a thread takes `kAhead`
    // entries at a time and asks for 16 floats of each, as 16-byte loads, before it adds the first.
    constexpr int kAhead = 4;
    typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
    const unsigned int places = (unsigned int)p.n_sources * (unsigned int)cap;   // below 2^31: checked by the host
    for (unsigned int base = 0; base < places; base += kRowsApplyThreads * kAhead) {
        const float* src[kAhead];
        int row[kAhead];   // first cell of the entry's row in the table, or -1
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const unsigned int i = base + (unsigned int)(u * kRowsApplyThreads + tid);
            const unsigned int w = i / (unsigned int)cap, place = i - w * (unsigned int)cap;
            const bool valid = i < places && place < fill[w < (unsigned int)p.n_sources ? w : 0u];
            src[u] = valid ? p.lists + (size_t)w * p.list_words + info.x + (size_t)place * stride : nullptr;
            // the entry names its row by the row's byte offset inside the mode: the row's first cell in the table
            row[u] = valid ? (int)(__float_as_uint(src[u][J]) >> 2) - row0 * J : -1;
        }
        for (int j0 = 0; j0 < J; j0 += 16) {
            uintx4 v[kAhead][4];
#pragma unroll
            for (int u = 0; u < kAhead; ++u)
#pragma unroll
                for (int k4 = 0; k4 < 4; ++k4)   // words past J inside the entry are the row's word and padding: read, not used
                    v[u][k4] = (src[u] && j0 + 4 * k4 < J) ? *reinterpret_cast<const uintx4*>(src[u] + j0 + 4 * k4) : uintx4{0u, 0u, 0u, 0u};
            // compare-and-swap adds, one entry's 16 floats at a time: all reads, then all swaps, and only
            // the swaps that lost (another thread changed the cell in between) go round again
#pragma unroll
            for (int u = 0; u < kAhead; ++u)
                if (row[u] >= 0 && row[u] < cells) {
                    unsigned int* cell = reinterpret_cast<unsigned int*>(table + row[u] + j0);
                    unsigned int seen[16], got[16];
#pragma unroll
                    for (int k = 0; k < 16; ++k) seen[k] = j0 + k < J ? cell[k] : 0u;
#pragma unroll
                    for (int k = 0; k < 16; ++k)
                        got[k] = j0 + k < J ? atomicCAS(cell + k, seen[k], __float_as_uint(__uint_as_float(seen[k]) + __uint_as_float(v[u][k >> 2][k & 3])))
                                            : 0u;
                    // lanes of one instruction that hit the same row lose together, on every cell of the row:
                    // the lost swaps of a round all go out again before any is waited for
                    bool lost = false;
#pragma unroll
                    for (int k = 0; k < 16; ++k) lost = lost || got[k] != seen[k];
                    while (lost) {
                        unsigned int again[16];
#pragma unroll
                        for (int k = 0; k < 16; ++k)
                            again[k] = got[k] != seen[k]
                                           ? atomicCAS(cell + k, got[k], __float_as_uint(__uint_as_float(got[k]) + __uint_as_float(v[u][k >> 2][k & 3])))
                                           : got[k];
                        lost = false;
#pragma unroll
                        for (int k = 0; k < 16; ++k) {
                            const bool was_lost = got[k] != seen[k];
                            seen[k] = was_lost ? got[k] : seen[k];      // what the retry expected
                            got[k] = was_lost ? again[k] : seen[k];     // settled cells compare equal from now on
                            lost = lost || got[k] != seen[k];
                        }
                    }
                }
        }
    }
    __syncthreads();
    float* A_rows = p.A + p.A_off[n] + (long long)row0 * J;
    if (*p.overflow != 0u) {
        float* dA_rows = p.dA + p.A_off[n] + (long long)row0 * J;
        for (int q = tid; q < cells; q += kRowsApplyThreads) {
            const float extra = dA_rows[q];
            if (extra != 0.0f) {
                table[q] += extra;
                dA_rows[q] = 0.0f;
            }
        }
    }
    for (int q = tid; q < cells; q += kRowsApplyThreads) {
        const float t = table[q];
        if (t != 0.0f) A_rows[q] = fmaf(-p.lr_A, t, A_rows[q]);
    }
}
#endif

// ---------------------------------------------------------------------------------------------
// Evaluation pass over all stored entries (RMSE / MAE) for the same shapes: records streamed,
// rows gathered 16 bytes per lane in the operand layout (X4) or 16 lanes per 64 bytes and
// transposed in LDS, projections on the matrix core, errors summed in double.
// ---------------------------------------------------------------------------------------------
constexpr int kTiledMaxOrder = 10;   // orders 9 and 10 are instantiated for P = 1 only
struct TiledModeBytes {
    unsigned int v[kTiledMaxOrder];   // I_n * J_n * 4: size of mode n's rows in A
};

template <int N, int P, bool X4>
__global__ void __launch_bounds__(256) errors_tiled_kernel(Coo coo, uint64_t nnz, const float* __restrict__ A,
                                                           const float* __restrict__ B, Layout L, TiledModeBytes mode_bytes,
                                                           double* __restrict__ sums /* [2]: sse, sae */) {
    extern __shared__ float lds[];
    constexpr int W4 = (N + 1 + 3) / 4;
    constexpr int D = 16 * P;
    __shared__ double red[2][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g4 = lane >> 4;
    float* Bl = lds;                                                    // [N][D][D], see operand_slot
    float* wave_lds = lds + N * D * D + wave * tiled_wave_scratch(N, P);   // two parked groups, then tbuf
    float* tbuf = wave_lds + 2 * tiled_park_words(N);
    for (int q = tid; q < N * D * D; q += 256) {
        const int n = q / (D * D), rem = q - n * D * D, j = rem / D, r = rem - j * D;
        Bl[operand_slot<P>(n, j, r)] = (j < L.J[n] && r < L.R) ? B[L.B_off[n] + j * L.R + r] : 0.0f;
    }
    __syncthreads();

    const uint4* rec4 = reinterpret_cast<const uint4*>(coo.rec);
    const uint64_t n_groups = (nnz + 63) / 64;
    const uint64_t group_stride = (uint64_t)gridDim.x * 4;
    __amdgpu_buffer_rsrc_t rsrc_A[N];
#pragma unroll
    for (int n = 0; n < N; ++n) rsrc_A[n] = make_rsrc(A + L.A_off[n], mode_bytes.v[n]);

    auto load_record = [&](uint64_t grp, uint4 (&rec)[W4]) {
        const uint64_t p = grp * 64 + lane;
#pragma unroll
        for (int q = 0; q < W4; ++q) rec[q] = rec4[(p < nnz ? p : 0) * W4 + q];
    };
    // row numbers and values of a group, zero for lanes past the end
    auto park_record = [&](uint64_t grp, const uint4 (&rec)[W4], float* park) {
        const bool act = grp * 64 + lane < nnz;
        uint32_t flat[4 * W4];
#pragma unroll
        for (int q = 0; q < W4; ++q) {
            flat[4 * q + 0] = rec[q].x;
            flat[4 * q + 1] = rec[q].y;
            flat[4 * q + 2] = rec[q].z;
            flat[4 * q + 3] = rec[q].w;
        }
        int* sidx = reinterpret_cast<int*>(park);
#pragma unroll
        for (int n = 0; n < N; ++n) sidx[n * 64 + lane] = act ? (int)flat[n] : 0;
        park[N * 64 + lane] = act ? __uint_as_float(flat[N]) : 0.0f;
    };
    // the rows of tile `sub` of a parked group, in the layouts of the gradient kernel's gather_rows;
    // entries past the end read row 0 (they are left out of the sums below)
    auto gather_rows = [&](const float* park, int sub, floatx4 (&rows)[N][P]) {
        const int* sidx = reinterpret_cast<const int*>(park);
        if constexpr (X4) {
#pragma unroll
            for (int n = 0; n < N; ++n) {
                const int row = sidx[n * 64 + sub * 16 + c];
#pragma unroll
                for (int jb = 0; jb < P; ++jb) {
                    const int col = 16 * jb + 4 * g4;
                    const int off = col < L.J[n] ? (row * L.J[n] + col) * 4 : (int)mode_bytes.v[n];
                    rows[n][jb] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rsrc_A[n], off, 0, 0));
                }
            }
        } else {
#pragma unroll
            for (int n = 0; n < N; ++n) {
                const int4 r = *reinterpret_cast<const int4*>(sidx + n * 64 + sub * 16 + 4 * g4);
                const int rr[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
                for (int jb = 0; jb < P; ++jb) {
                    const int col = 16 * jb + c;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int off = col < L.J[n] ? (rr[v] * L.J[n] + col) * 4 : (int)mode_bytes.v[n];
                        rows[n][jb][v] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc_A[n], off, 0, 0));
                    }
                }
            }
        }
    };

    double sse = 0.0, sae = 0.0;
    uint4 rec[W4];
    floatx4 cur[N][P];
    uint64_t group = (uint64_t)blockIdx.x * 4 + wave;
    int buf = 0;
    if (group < n_groups) {
        load_record(group, rec);
        park_record(group, rec, wave_lds);
        lds_wave_sync();
        if (group + group_stride < n_groups) load_record(group + group_stride, rec);
        gather_rows(wave_lds, 0, cur);
    }
#pragma unroll 1
    for (; group < n_groups; group += group_stride, buf ^= 1) {
        const float* park = wave_lds + buf * tiled_park_words(N);
        float* park_next = wave_lds + (buf ^ 1) * tiled_park_words(N);
#pragma unroll 1
        for (int sub = 0; sub < 4; ++sub) {
            floatx4 nxt[N][P];
            if (sub < 3) {
                gather_rows(park, sub + 1, nxt);
            } else if (group + group_stride < n_groups) {
                park_record(group + group_stride, rec, park_next);
                lds_wave_sync();
                if (group + 2 * group_stride < n_groups) load_record(group + 2 * group_stride, rec);
                gather_rows(park_next, 0, nxt);
            } else {
#pragma unroll
                for (int n = 0; n < N; ++n)
#pragma unroll
                    for (int jb = 0; jb < P; ++jb) nxt[n][jb] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
            }

            floatx4 prod[P];
#pragma unroll
            for (int rb = 0; rb < P; ++rb) prod[rb] = floatx4{1.0f, 1.0f, 1.0f, 1.0f};
            // core-factor operands: read one block of products ahead (P < 4), as in the gradient kernel
            constexpr bool AHEAD = P < 4;
            float4 bop[P];
            if constexpr (AHEAD) {
#pragma unroll
                for (int rb = 0; rb < P; ++rb) bop[rb] = *reinterpret_cast<const float4*>(Bl + rb * 256 + lane * 4);
            }
#pragma unroll
            for (int n = 0; n < N; ++n) {
                floatx4 sacc[P];
#pragma unroll
                for (int rb = 0; rb < P; ++rb) sacc[rb] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int jb = 0; jb < P; ++jb) {
                    float4 bcur[P];
                    if constexpr (AHEAD) {
#pragma unroll
                        for (int rb = 0; rb < P; ++rb) bcur[rb] = bop[rb];
                        if (n * P + jb + 1 < N * P) {
#pragma unroll
                            for (int rb = 0; rb < P; ++rb)
                                bop[rb] = *reinterpret_cast<const float4*>(Bl + ((n * P + jb + 1) * P + rb) * 256 + lane * 4);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    } else {
#pragma unroll
                        for (int rb = 0; rb < P; ++rb)
                            bcur[rb] = *reinterpret_cast<const float4*>(Bl + ((n * P + jb) * P + rb) * 256 + lane * 4);
                    }
                    float ax[4];   // components 16 jb + 4g .. +3 of the row of sample c
                    if constexpr (X4) {
#pragma unroll
                        for (int k = 0; k < 4; ++k) ax[k] = cur[n][jb][k];
                    } else {
#pragma unroll
                        for (int v = 0; v < 4; ++v) tbuf[(4 * g4 + v) * 20 + c] = cur[n][jb][v];
                        lds_wave_sync();
                        const float4 ax4 = *reinterpret_cast<const float4*>(tbuf + c * 20 + 4 * g4);
                        lds_wave_sync();
                        ax[0] = ax4.x;
                        ax[1] = ax4.y;
                        ax[2] = ax4.z;
                        ax[3] = ax4.w;
                    }
#pragma unroll
                    for (int rb = 0; rb < P; ++rb) {
                        const float bk[4] = {bcur[rb].x, bcur[rb].y, bcur[rb].z, bcur[rb].w};
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            sacc[rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(bk[k], ax[k], sacc[rb], 0, 0, 0);
                    }
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
            const float x = park[N * 64 + sub * 16 + c];
            if (g4 == 0 && group * 64 + sub * 16 + c < nnz) {
                const double e = (double)x - (double)xhat;
                sse += e * e;
                sae += fabs(e);
            }
#pragma unroll
            for (int n = 0; n < N; ++n)
#pragma unroll
                for (int jb = 0; jb < P; ++jb) cur[n][jb] = nxt[n][jb];
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
