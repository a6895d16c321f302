// Device-side Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) and the two rules built on it:
// the position of sample k in Psi, and the initial value of a parameter element.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ftk {

struct U4 {
    uint32_t x, y, z, w;
};

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1) {
    constexpr uint32_t MUL_A = 0xD2511F53u, MUL_B = 0xCD9E8D57u;
    constexpr uint32_t WEYL_A = 0x9E3779B9u, WEYL_B = 0xBB67AE85u;
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        const uint32_t hiA = __umulhi(MUL_A, c0), loA = MUL_A * c0;
        const uint32_t hiB = __umulhi(MUL_B, c2), loB = MUL_B * c2;
        c0 = hiB ^ c1 ^ k0;
        c2 = hiA ^ c3 ^ k1;
        c1 = loB;
        c3 = loA;
        k0 += WEYL_A;
        k1 += WEYL_B;
    }
    return U4{c0, c1, c2, c3};
}

// p_k = floor(u * nnz / 2^64): sample k uses counter k/2 and the low (even k) or high (odd k)
// pair of output words, low word first.
__device__ __forceinline__ uint32_t sample_position(uint64_t seed, uint64_t k, uint64_t nnz) {
    const uint64_t ctr = k >> 1;
    const U4 o = philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), 0u, 0u, (uint32_t)seed,
                               (uint32_t)(seed >> 32));
    const uint32_t lo = (k & 1) ? o.z : o.x;
    const uint32_t hi = (k & 1) ? o.w : o.y;
    const uint64_t u = ((uint64_t)hi << 32) | (uint64_t)lo;
    return (uint32_t)__umul64hi(u, nnz);   // nnz < 2^32, so the position fits 32 bits
}

// Tile-sampling variant: Psi is made of runs of 64 neighbours in a fixed pseudo-random order of
// the stored entries (stored place q holds the caller's entry (a q + b) mod nnz).  Group g = k / 64
// draws its run with the entry rule above among n_runs = ceil(nnz / 64) runs; sample k sits at
// stored place (64 run + k % 64) mod nnz.
struct SampleRule {
    uint64_t nnz;
    uint64_t n_runs;   // 0: entry sampling (the default rule)
    uint64_t a, b;     // the order of the stored entries in tile mode
};

__device__ __forceinline__ uint32_t tile_place(uint64_t seed, uint64_t k, const SampleRule& r) {
    const uint64_t run = sample_position(seed, k >> 6, r.n_runs);
    uint64_t q = 64 * run + (k & 63);
    if (q >= r.nnz) q %= r.nnz;   // only the last run wraps (several times if nnz < 64)
    return (uint32_t)q;
}

// where sample k is read from: its position among the caller's entries (entry rule, records in the
// caller's order) or its stored place (tile rule, records in the pseudo-random order)
__device__ __forceinline__ uint32_t sample_place(uint64_t seed, uint64_t k, const SampleRule& r) {
    return r.n_runs ? tile_place(seed, k, r) : sample_position(seed, k, r.nnz);
}

// the caller's position of the entry stored at place q (tile rule); a, q < 2^32
__device__ __forceinline__ uint32_t caller_position(uint32_t q, const SampleRule& r) {
    return r.n_runs ? (uint32_t)((r.a * (uint64_t)q + r.b) % r.nnz) : q;
}

// U[0, 0.5): top 24 bits of output word 0, scaled by 2^-25.
__device__ __forceinline__ float init_value(uint64_t init_seed, uint32_t array_id, uint64_t q) {
    const U4 o = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), array_id, 1u, (uint32_t)init_seed,
                               (uint32_t)(init_seed >> 32));
    return (float)(o.x >> 8) * (1.0f / 33554432.0f);
}

}  // namespace ftk
