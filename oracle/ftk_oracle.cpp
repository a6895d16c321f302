// CPU oracle for the sampled-SGD step of sparse Tucker decomposition with a
// Kruskal-approximated core (FastTucker).
//
// THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It exists so that the HIP
// library has something slow and obviously correct to be compared against.
// Only the tests, the smoke check and the benchmark's cpu-baseline leg may
// load it.  It shares no code, header, table or helper with the HIP path.
//
// Style: plain single-threaded C++17, parameters stored in fp32 (as the
// library stores them), every sum and product carried in double, one rounding
// to fp32 when a parameter is written back.  No blocking, no fusion, no
// prefix/suffix trick: the leave-one-out product is the explicit product over
// the other modes, exactly as the closed forms in Section 3.1 / 3.2 print it.
//
// Notation (paper, Section 3):  N = order, I_n = mode size, J_n = Tucker rank
// of mode n, R = R_core = Kruskal rank of the core,
//   A^(n) in R^{I_n x J_n}  row-major,   B^(n) in R^{J_n x R}  row-major,
//   c^(n)_r = b^(n)T_{:,r} a^(n)T_{i_n,:}            (under-braces of the GS^(n) and Q^(n),r derivations)
//   xhat    = sum_r prod_n c^(n)_r                   (Eq. kruskal_approximation + Theorem 1)
//   GS^(n)  = sum_r b^(n)_{:,r} prod_{k!=n} c^(k)_r  (derivation after Theorem 1)
//   Q^(n),r = a^(n)T_{i_n,:} prod_{k!=n} c^(k)_r     (derivation after Theorem 2)
//
// Readings of the paper taken here (each is listed in the design notes too):
//  * loss per nonzero is (1/2) e^2 + (1/2) lambda |.|^2: the printed gradients
//    (Eq. Gradient_low_rank, Eq. Gradient_low_rank_core) carry no factor 2;
//  * factor rows use M = 1 (sum over the samples that hit the row), the core
//    uses M = |Psi| (mean)  -- the input line of Algorithm 1;
//  * lambda_A a is added once per processed sample (Algorithm 1, line 12),
//    lambda_B B once per step;
//  * synchronous (Jacobi) mode: every gradient is evaluated at the parameters
//    the step started with, then all parameters are updated at once; the order
//    Algorithm 1 prints (rows overwritten sample by sample, mode by mode) is a
//    second entry point, fto_sgd_step_hogwild;
//  * Psi: i.i.d. uniform positions with replacement from Philox4x32-10.
//
// Pins (see tests/test_oracle_*.py): Philox known-answer vectors of Salmon et
// al.; brute-force dense-core Tucker contraction (Eq. tucker with the core of
// Eq. kruskal_approximation built explicitly); central finite differences of
// the sampled loss; closed-form special cases; invariants.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
// as 1, 2, 3", SC'11).  Counter 4 x 32 bit, key 2 x 32 bit, ten rounds.
// ---------------------------------------------------------------------------
struct Words4 { uint32_t w[4]; };

Words4 philox_round(const Words4& c, uint32_t k0, uint32_t k1) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c.w[0];
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c.w[2];
    Words4 o;
    o.w[0] = (uint32_t)(p1 >> 32) ^ c.w[1] ^ k0;
    o.w[1] = (uint32_t)p1;
    o.w[2] = (uint32_t)(p0 >> 32) ^ c.w[3] ^ k1;
    o.w[3] = (uint32_t)p0;
    return o;
}

Words4 philox4x32_10(Words4 c, uint32_t k0, uint32_t k1) {
    for (int round = 0; round < 10; ++round) {
        c = philox_round(c, k0, k1);
        k0 += 0x9E3779B9u;   // golden-ratio Weyl increments of the key schedule
        k1 += 0xBB67AE85u;
    }
    return c;
}

// floor(u * n / 2^64) for 64-bit u, n  (unsigned 128-bit product, top half)
uint64_t mulhi_u64(uint64_t u, uint64_t n) {
    return (uint64_t)(((unsigned __int128)u * (unsigned __int128)n) >> 64);
}

// position of sample k: counter (lo32(k/2), hi32(k/2), 0, 0), key = seed;
// even k takes output words 0,1, odd k takes words 2,3 (low word first).
uint64_t sample_position(uint64_t seed, uint64_t k, uint64_t nnz) {
    const uint64_t c = k >> 1;
    Words4 ctr = {{(uint32_t)c, (uint32_t)(c >> 32), 0u, 0u}};
    Words4 o = philox4x32_10(ctr, (uint32_t)seed, (uint32_t)(seed >> 32));
    const uint64_t u = (k & 1u) ? ((uint64_t)o.w[2] | ((uint64_t)o.w[3] << 32))
                                : ((uint64_t)o.w[0] | ((uint64_t)o.w[1] << 32));
    return mulhi_u64(u, nnz);
}

// ---------------------------------------------------------------------------
// model on one nonzero, everything in double
// ---------------------------------------------------------------------------
struct Terms {
    std::vector<std::vector<double>> c;    // c[n][r]
    std::vector<std::vector<double>> w;    // w[n][r]  = prod_{k != n} c[k][r]
    std::vector<std::vector<double>> gs;   // gs[n][j] = sum_r B^(n)[j][r] w[n][r]
    double xhat = 0.0;
};

void nonzero_terms(int N, const int32_t* J, int R, const float* const* a,
                   const float* const* B, Terms& t) {
    t.c.assign(N, std::vector<double>(R, 0.0));
    t.w.assign(N, std::vector<double>(R, 0.0));
    t.gs.resize(N);
    for (int n = 0; n < N; ++n)
        for (int r = 0; r < R; ++r) {
            double acc = 0.0;
            for (int j = 0; j < J[n]; ++j)
                acc += (double)a[n][j] * (double)B[n][(size_t)j * R + r];
            t.c[n][r] = acc;
        }
    t.xhat = 0.0;
    for (int r = 0; r < R; ++r) {
        double prod = 1.0;
        for (int n = 0; n < N; ++n) prod *= t.c[n][r];
        t.xhat += prod;
    }
    for (int n = 0; n < N; ++n) {
        for (int r = 0; r < R; ++r) {
            double prod = 1.0;
            for (int k = 0; k < N; ++k)
                if (k != n) prod *= t.c[k][r];
            t.w[n][r] = prod;
        }
        t.gs[n].assign(J[n], 0.0);
        for (int j = 0; j < J[n]; ++j) {
            double acc = 0.0;
            for (int r = 0; r < R; ++r)
                acc += (double)B[n][(size_t)j * R + r] * t.w[n][r];
            t.gs[n][j] = acc;
        }
    }
}

bool bad_shape(int N, const int32_t* J, int R) {
    if (N < 1 || N > 16 || R < 1 || !J) return true;
    for (int n = 0; n < N; ++n)
        if (J[n] < 1) return true;
    return false;
}

}  // namespace

extern "C" {

// Raw generator, exposed so the known-answer vectors can be checked.
void fto_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    Words4 c = {{ctr[0], ctr[1], ctr[2], ctr[3]}};
    Words4 o = philox4x32_10(c, key[0], key[1]);
    for (int i = 0; i < 4; ++i) out[i] = o.w[i];
}

// Psi: n_samples positions in [0, nnz), i.i.d. uniform with replacement.
int fto_sample_positions(uint64_t seed, int64_t n_samples, int64_t nnz, int64_t* pos_out) {
    if (n_samples < 0 || nnz < 1 || !pos_out) return -1;
    for (int64_t k = 0; k < n_samples; ++k)
        pos_out[k] = (int64_t)sample_position(seed, (uint64_t)k, (uint64_t)nnz);
    return 0;
}

// Tile sampling, a VARIANT of the rule above (the paper only says Psi is drawn at random from
// Omega, Section 4.1): Psi is made of whole runs of 64 entries that are neighbours in a fixed
// pseudo-random order of Omega, so that a run can be fetched with one contiguous read.
//   order of Omega:   stored place q holds the caller's entry  pi(q) = (a q + b) mod nnz,
//                     b = floor(nnz / 3),  a = the largest integer <= max(1, floor(nnz * 618034 / 1000000))
//                     with gcd(a, nnz) = 1  (so pi is a bijection of [0, nnz))
//   run of group g:   T_g = the position the entry rule above draws for sample g among
//                     n_runs = ceil(nnz / 64) places (same seed, counter g / 2, halves by parity of g)
//   sample k:         g = k / 64,  q_k = (64 T_g + k mod 64) mod nnz,  p_k = pi(q_k)
int fto_tile_order_constants(int64_t nnz, int64_t* a_out, int64_t* b_out) {
    if (nnz < 1 || !a_out || !b_out) return -1;
    uint64_t a = (uint64_t)nnz * 618034ull / 1000000ull;   // nnz < 2^32: no overflow
    if (a < 1) a = 1;
    for (; a > 1; --a) {
        uint64_t x = a, y = (uint64_t)nnz;
        while (y) {
            const uint64_t t = x % y;
            x = y;
            y = t;
        }
        if (x == 1) break;
    }
    *a_out = (int64_t)a;
    *b_out = nnz / 3;
    return 0;
}

int fto_sample_positions_tiles(uint64_t seed, int64_t n_samples, int64_t nnz, int64_t* pos_out) {
    if (n_samples < 0 || nnz < 1 || nnz >= (1ll << 32) || !pos_out) return -1;
    int64_t a = 0, b = 0;
    fto_tile_order_constants(nnz, &a, &b);
    const uint64_t n_runs = ((uint64_t)nnz + 63) / 64;
    for (int64_t k = 0; k < n_samples; ++k) {
        const uint64_t g = (uint64_t)k / 64;
        const uint64_t run = sample_position(seed, g, n_runs);
        const uint64_t q = (64 * run + (uint64_t)k % 64) % (uint64_t)nnz;
        pos_out[k] = (int64_t)(((uint64_t)a * q + (uint64_t)b) % (uint64_t)nnz);   // a, q < 2^32
    }
    return 0;
}

// Initial parameters U[0, 0.5): element q of parameter array `array_id`
// (n for A^(n), N + n for B^(n)) is 0.5 * 2^-24 * (top 24 bits of word 0 of
// Philox(counter = (lo32 q, hi32 q, array_id, 1), key = init_seed)).
int fto_init_uniform(uint64_t init_seed, int32_t array_id, int64_t count, float* out) {
    if (count < 0 || !out) return -1;
    for (int64_t q = 0; q < count; ++q) {
        Words4 ctr = {{(uint32_t)(uint64_t)q, (uint32_t)((uint64_t)q >> 32), (uint32_t)array_id, 1u}};
        Words4 o = philox4x32_10(ctr, (uint32_t)init_seed, (uint32_t)(init_seed >> 32));
        out[q] = (float)((double)(o.w[0] >> 8) * (0.5 / 16777216.0));
    }
    return 0;
}

// Everything the method derives from one nonzero: c, w (leave-one-out), GS, xhat.
// a_rows[n] -> J[n] floats (the gathered row), B[n] -> J[n]*R floats row-major.
// c_out, w_out: N*R doubles (mode-major); gs_out[n] -> J[n] doubles.
int fto_nonzero_terms(int32_t order, const int32_t* J, int32_t R, const float* const* a_rows,
                      const float* const* B, double* xhat_out, double* c_out, double* w_out,
                      double* const* gs_out) {
    if (bad_shape(order, J, R) || !a_rows || !B) return -1;
    Terms t;
    nonzero_terms(order, J, R, a_rows, B, t);
    if (xhat_out) *xhat_out = t.xhat;
    for (int n = 0; n < order; ++n) {
        for (int r = 0; r < R; ++r) {
            if (c_out) c_out[(size_t)n * R + r] = t.c[n][r];
            if (w_out) w_out[(size_t)n * R + r] = t.w[n][r];
        }
        if (gs_out && gs_out[n])
            for (int j = 0; j < J[n]; ++j) gs_out[n][j] = t.gs[n][j];
    }
    return 0;
}

// One synchronous step (Algorithm 1 with every gradient taken at the starting
// parameters).  A[n] (I_n x J_n) and B[n] (J_n x R) are updated in place.
//   dA^(n)[i_n,:] += -e GS^(n) + lambda_A a^(n)        for every sample occurrence
//   GB^(n)[j,r]   += -e a^(n)_j w^(n)_r
//   A <- A - lr_A dA          (touched rows; M = 1)
//   B <- B - lr_B (GB / |Psi| + lambda_B B)
int fto_sgd_step_sync(int32_t order, const int64_t* dims, int64_t nnz, const int32_t* const* idx,
                      const float* vals, const int32_t* J, int32_t R, float* const* A,
                      float* const* B, const int64_t* pos, int64_t n_samples, float lr_A,
                      float lr_B, float lambda_A, float lambda_B) {
    if (bad_shape(order, J, R) || !dims || !idx || !vals || !A || !B || nnz < 1) return -1;
    if (n_samples < 1 || !pos) return -1;
    const int N = order;
    std::vector<std::vector<double>> dA(N), GB(N);
    for (int n = 0; n < N; ++n) {
        dA[n].assign((size_t)dims[n] * J[n], 0.0);
        GB[n].assign((size_t)J[n] * R, 0.0);
    }
    std::vector<std::vector<uint8_t>> touched(N);
    for (int n = 0; n < N; ++n) touched[n].assign((size_t)dims[n], 0);

    std::vector<const float*> a(N);
    Terms t;
    for (int64_t k = 0; k < n_samples; ++k) {
        const int64_t p = pos[k];
        if (p < 0 || p >= nnz) return -2;
        for (int n = 0; n < N; ++n) {
            const int64_t i = idx[n][p];
            if (i < 0 || i >= dims[n]) return -3;
            a[n] = A[n] + (size_t)i * J[n];
        }
        nonzero_terms(N, J, R, a.data(), B, t);
        const double e = (double)vals[p] - t.xhat;
        for (int n = 0; n < N; ++n) {
            const size_t i = (size_t)idx[n][p];
            touched[n][i] = 1;
            double* drow = dA[n].data() + i * J[n];
            for (int j = 0; j < J[n]; ++j) {
                drow[j] += -e * t.gs[n][j] + (double)lambda_A * (double)a[n][j];
                for (int r = 0; r < R; ++r)
                    GB[n][(size_t)j * R + r] += -e * (double)a[n][j] * t.w[n][r];
            }
        }
    }
    for (int n = 0; n < N; ++n) {
        for (int64_t i = 0; i < dims[n]; ++i) {
            if (!touched[n][(size_t)i]) continue;
            for (int j = 0; j < J[n]; ++j) {
                const size_t q = (size_t)i * J[n] + j;
                A[n][q] = (float)((double)A[n][q] - (double)lr_A * dA[n][q]);
            }
        }
        for (size_t q = 0; q < (size_t)J[n] * R; ++q)
            B[n][q] = (float)((double)B[n][q] -
                              (double)lr_B * (GB[n][q] / (double)n_samples + (double)lambda_B * (double)B[n][q]));
    }
    return 0;
}

// One step of Algorithm 1 in the order it is printed (the "Hogwild" mode of the library, here
// run sequentially so it is deterministic):
//   factor phase (lines 1-16), sample by sample in the order of Psi, and inside a sample mode by
//   mode: c of the OTHER modes from the CURRENT rows (so mode n already sees the rows that modes
//   < n of the same sample, and all earlier samples, have just written), GS^(n), the three parts,
//   and the row is overwritten at once with M = 1:  a <- a - lr_A (-e GS + lambda_A a);
//   core phase (lines 17-39) over the same samples with the updated factor matrices: the
//   gradients of all b^(n)_{:,r} are accumulated and B is updated once with M = |Psi|
//   (Section 4.2: the b vectors depend on each other and are updated simultaneously).
// Every row write is rounded to fp32, as the library stores fp32.
int fto_sgd_step_hogwild(int32_t order, const int64_t* dims, int64_t nnz, const int32_t* const* idx,
                         const float* vals, const int32_t* J, int32_t R, float* const* A,
                         float* const* B, const int64_t* pos, int64_t n_samples, float lr_A,
                         float lr_B, float lambda_A, float lambda_B) {
    if (bad_shape(order, J, R) || !dims || !idx || !vals || !A || !B || nnz < 1) return -1;
    if (n_samples < 1 || !pos) return -1;
    const int N = order;
    std::vector<const float*> a(N);
    Terms t;
    for (int64_t k = 0; k < n_samples; ++k) {
        const int64_t p = pos[k];
        if (p < 0 || p >= nnz) return -2;
        for (int n = 0; n < N; ++n) {
            if (idx[n][p] < 0 || idx[n][p] >= dims[n]) return -3;
            a[n] = A[n] + (size_t)idx[n][p] * J[n];
        }
        for (int n = 0; n < N; ++n) {
            nonzero_terms(N, J, R, a.data(), B, t);   // everything from the current rows
            const double e = (double)vals[p] - t.xhat;
            float* row = A[n] + (size_t)idx[n][p] * J[n];
            for (int j = 0; j < J[n]; ++j)
                row[j] = (float)((double)row[j] -
                                 (double)lr_A * (-e * t.gs[n][j] + (double)lambda_A * (double)row[j]));
        }
    }
    std::vector<std::vector<double>> GB(N);
    for (int n = 0; n < N; ++n) GB[n].assign((size_t)J[n] * R, 0.0);
    for (int64_t k = 0; k < n_samples; ++k) {
        const int64_t p = pos[k];
        for (int n = 0; n < N; ++n) a[n] = A[n] + (size_t)idx[n][p] * J[n];
        nonzero_terms(N, J, R, a.data(), B, t);
        const double e = (double)vals[p] - t.xhat;
        for (int n = 0; n < N; ++n)
            for (int j = 0; j < J[n]; ++j)
                for (int r = 0; r < R; ++r)
                    GB[n][(size_t)j * R + r] += -e * (double)a[n][j] * t.w[n][r];
    }
    for (int n = 0; n < N; ++n)
        for (size_t q = 0; q < (size_t)J[n] * R; ++q)
            B[n][q] = (float)((double)B[n][q] -
                              (double)lr_B * (GB[n][q] / (double)n_samples + (double)lambda_B * (double)B[n][q]));
    return 0;
}

// Summed squared and absolute error over a list of stored nonzeros
// (positions == nullptr: all nnz).  RMSE = sqrt(sse / count), MAE = sae / count
// (Section 5.1 defines both on a test set Gamma).
int fto_errors(int32_t order, const int64_t* dims, int64_t nnz, const int32_t* const* idx,
               const float* vals, const int32_t* J, int32_t R, const float* const* A,
               const float* const* B, const int64_t* positions, int64_t count, double* rmse_out,
               double* mae_out) {
    if (bad_shape(order, J, R) || !dims || !idx || !vals || !A || !B || nnz < 1) return -1;
    const int N = order;
    const int64_t m = positions ? count : nnz;
    if (m < 1) return -1;
    std::vector<const float*> a(N);
    Terms t;
    double sse = 0.0, sae = 0.0;
    for (int64_t k = 0; k < m; ++k) {
        const int64_t p = positions ? positions[k] : k;
        if (p < 0 || p >= nnz) return -2;
        for (int n = 0; n < N; ++n) {
            const int64_t i = idx[n][p];
            if (i < 0 || i >= dims[n]) return -3;
            a[n] = A[n] + (size_t)i * J[n];
        }
        nonzero_terms(N, J, R, a.data(), B, t);
        const double e = (double)vals[p] - t.xhat;
        sse += e * e;
        sae += std::fabs(e);
    }
    if (rmse_out) *rmse_out = std::sqrt(sse / (double)m);
    if (mae_out) *mae_out = sae / (double)m;
    return 0;
}

}  // extern "C"
