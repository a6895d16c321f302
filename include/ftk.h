/*
 * ftk -- sampled stochastic-gradient step of sparse Tucker decomposition with a
 * Kruskal-approximated core (FastTucker), for one AMD MI355X (gfx950).
 *
 * Problem (Definition "Sparse Tucker Decomposition", Eq. tucker): given an N-order
 * sparse tensor X with stored entries Omega and ranks J_1..J_N, find factor matrices
 * A^(n) in R^{I_n x J_n} and a core G with X ~ G x_1 A^(1) ... x_N A^(N).  The core is
 * held as N small matrices B^(n) in R^{J_n x R} with G ~ sum_r b^(1)_r o ... o b^(N)_r
 * (Eq. kruskal_approximation, R = R_core).  For a stored entry x at (i_1..i_N):
 *
 *   c^(n)_r = sum_j A^(n)[i_n,j] B^(n)[j,r]          (under-braces of the GS and Q derivations)
 *   xhat    = sum_r prod_n c^(n)_r                    (Theorem 1)
 *   w^(n)_r = prod_{k != n} c^(k)_r
 *   GS^(n)_j = sum_r B^(n)[j,r] w^(n)_r               (Section 3.1, after Theorem 1)
 *   Q^(n),r_j = A^(n)[i_n,j] w^(n)_r                  (Section 3.2, after Theorem 2)
 *   e = x - xhat
 *
 * One step (Algorithm 1) over a sample set Psi of M stored entries, all gradients taken
 * at the parameters the step starts from (synchronous mode):
 *
 *   A^(n)[i,:] <- A^(n)[i,:] - lr_A * sum_{k in Psi, i_n(k) = i} ( -e_k GS^(n)_k + lambda_A A^(n)[i,:] )
 *   B^(n)      <- B^(n)      - lr_B * ( (1/M) sum_{k in Psi} -e_k Q^(n)_k  + lambda_B B^(n) )
 *
 * (Eq. Gradient_low_rank with parts (1)+(3) merged, Eq. Gradient_low_rank_core with parts
 * (1)+(3)+(4) merged; "M = 1 for factor matrices, M = |Psi| for core tensor" is the input line
 * of Algorithm 1.  The mean-over-Psi reading of Eq. SGD for the factor rows is the same step
 * with lr_A / M.)  Rows no sample touches do not change.
 *
 * Conventions
 *  - Plain C ABI.  Every call returns an int status (FTK_OK = 0, negative = error), never
 *    throws and never aborts.  ftk_last_error() gives a message for the last failure.
 *  - Indices are 0-based int32; sample positions are int64 at this boundary.
 *  - All matrices are dense row-major fp32: A^(n) is I_n x J_n, B^(n) is J_n x R.
 *  - "host" / "device" is stated for every pointer.  Device pointers must belong to the HIP
 *    device that was current when ftk_create() ran; that device must be current in later calls
 *    (calls that touch device memory return FTK_ESTATE otherwise).
 *  - The library owns copies of the tensor, the parameters and Psi.  Caller buffers can be
 *    released as soon as the call they were passed to returns.
 *  - ftk_sample / ftk_sgd_step only enqueue work on the context's stream (the null stream
 *    unless ftk_set_stream() was called).  ftk_rmse, ftk_mae, ftk_get_*, ftk_set_factors
 *    wait for that stream.
 *  - A context is not thread-safe; different contexts are independent.
 */
#ifndef FTK_H
#define FTK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ftk_ctx ftk_ctx;

enum {
    FTK_OK = 0,
    FTK_EINVAL = -1,       /* bad argument (null pointer, size out of range, index out of range) */
    FTK_ENOMEM = -2,       /* a host or device allocation failed */
    FTK_EDEVICE = -3,      /* a HIP call failed, or no usable gfx950 device */
    FTK_ESTATE = -4,       /* call order (e.g. ftk_sgd_step before ftk_sample), or another HIP device is current */
    FTK_EUNSUPPORTED = -5  /* valid but outside what the kernels are built for */
};

/* ftk_create flags */
enum {
    FTK_PTRS_HOST = 0u,    /* idx[n] and vals point to host memory (default) */
    FTK_PTRS_DEVICE = 1u,  /* idx[n] and vals point to device memory (the idx array itself is host) */
    FTK_LAYOUT_EXACT = 2u  /* keep the library's copy of A^(n), B^(n) at J_n and R floats per row.  Without it
                              ranks up to 16 (order 2..5) are held zero-padded to 16, which costs memory (rows of
                              64 bytes) and buys the fastest kernel; results are the same either way. */
};

/* ftk_set_mode */
enum {
    FTK_SYNC = 0,          /* all gradients at the step's starting parameters, then one update */
    FTK_HOGWILD = 1,       /* in-place factor rows, one fused pass (run concurrently): see ftk_sgd_step */
    FTK_HOGWILD_MODEWISE = 2   /* in-place, Algorithm 1 as printed: modes of a sample in turn, then the core: see ftk_sgd_step */
};

#define FTK_MAX_ORDER 10

/*
 * Create a context for one tensor and initialise the parameters.
 *   out        host; receives the context (NULL on failure)
 *   order      N, 1..FTK_MAX_ORDER
 *   dims       host int64[order]; 1 <= I_n < 2^31
 *   nnz        number of stored entries |Omega|, 1 <= nnz < 2^32; repeated coordinates are allowed
 *   idx        host array of `order` pointers; idx[n] -> int32[nnz] (struct of arrays), host or
 *              device per `flags`; every value must satisfy 0 <= idx[n][p] < dims[n] (checked)
 *   vals       fp32[nnz], host or device per `flags`
 *   J          host int32[order], J_n >= 1;   R >= 1.   R <= J_n is NOT required.
 *   init_seed  A^(n), B^(n) ~ U[0, 0.5): element q (row-major flat index) of parameter array t
 *              (t = n for A^(n), t = N + n for B^(n)) is
 *              0.5 * 2^-24 * (w0 >> 8),  w0 = word 0 of Philox4x32-10(counter = (lo32 q, hi32 q, t, 1),
 *              key = (lo32 init_seed, hi32 init_seed)).      ("Initializing A, B", Algorithm 1)
 * Errors: FTK_EINVAL, FTK_ENOMEM, FTK_EDEVICE, FTK_EUNSUPPORTED (N*R or J_n beyond kernel limits).
 */
int ftk_create(ftk_ctx** out, int32_t order, const int64_t* dims, int64_t nnz,
               const int32_t* const* idx, const float* vals, const int32_t* J, int32_t R,
               uint64_t init_seed, uint32_t flags);

/* Release everything the context owns.  NULL is allowed. */
void ftk_destroy(ftk_ctx* ctx);

/*
 * Draw the sample set Psi for the next step(s) (Definition "SGD": "an M entries set Psi is
 * randomly selected from Omega"; the paper fixes neither generator nor replacement rule).
 * Psi is n_samples i.i.d. uniform positions WITH replacement:
 *   (w0,w1,w2,w3) = Philox4x32-10(counter = (lo32(k/2), hi32(k/2), 0, 0), key = (lo32 seed, hi32 seed))
 *   u = w0 | w1 << 32  for even k,   w2 | w3 << 32  for odd k
 *   p_k = floor(u * nnz / 2^64)
 * Psi stays valid until the next ftk_sample.  1 <= n_samples < 2^31.
 */
int ftk_sample(ftk_ctx* ctx, uint64_t seed, int64_t n_samples);

/* Copy Psi to host int64[n_samples] (waits for the stream).  FTK_ESTATE if nothing was sampled. */
int ftk_get_samples(ftk_ctx* ctx, int64_t* pos_out);

/*
 * One SGD step over the current Psi (formulas at the top of this file).  FTK_ESTATE if no Psi.
 * In FTK_SYNC mode the result is independent of the order in which samples are processed up to
 * fp32 summation order.
 * In FTK_HOGWILD mode there is no accumulator and no separate factor update: every sample adds
 * -lr_A (-e GS^(n) + lambda_A a^(n)) straight into A^(n) while other samples are reading it, as
 * Algorithm 1 lines 1-16 do (M = 1).  Deviations from the printed order, both forced by running
 * samples concurrently: the N gradients of one sample all use the rows as gathered (mode n does
 * not see the row mode n-1 of the same sample just wrote), and the most frequently hit rows are
 * accumulated per workgroup and added at the end of the step.  The core factors are updated once
 * per step from the accumulated gradient, M = |Psi| (Section 4.2).  Results depend on scheduling;
 * this mode is meant to be judged by its RMSE curve.
 * FTK_HOGWILD_MODEWISE follows Algorithm 1 as printed, at the price of a second pass: a factor
 * phase in which every sample takes its modes one after the other, mode n using what modes < n of
 * the same sample have just written (Algorithm 1 lines 1-16: after mode n's row has moved by delta,
 * the sample's projections c^(n) are advanced by delta B^(n), which is the projection of the row it
 * has just written); then a core phase over the same Psi that takes the core gradient at the
 * updated rows (lines 17-39) and updates every B^(n) once.  Samples still run concurrently, so
 * samples that share a row see each other's updates in no fixed order; on a Psi whose samples share
 * no row the result is that of the printed order up to fp32 rounding.
 * It runs on the matrix cores where the "mfma16" or the "tiled" kernel is in use (16 samples at a
 * time; rows outside the workgroup tables are changed by float atomics as they are met, the most
 * frequently hit rows are accumulated per workgroup and added when the factor phase ends), and on the
 * one-lane-per-sample kernels otherwise (every row update a float atomic; FTK_EUNSUPPORTED where they
 * do not fit the shape).
 * Non-finite parameters: the kernels keep the sample slots behind the end of Psi and the padding of
 * short ranks out of the sums by arithmetic (their operands are zero), which holds while A and B
 * are finite.  Once a step has produced inf or NaN (a step size far too large), every later call
 * still returns normally, but which further elements turn NaN is unspecified.
 */
int ftk_sgd_step(ftk_ctx* ctx, float lr_A, float lr_B, float lambda_A, float lambda_B);

/*
 * ftk_sgd_step for callers that must not allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same step, same arguments, same result up to fp32
 * summation order; the difference is where the gradient kernel's per-workgroup partial tables
 * (factor-row sums and core-gradient sums, read back by the update pass of the same call) live:
 * in a static array in device memory that belongs to the library's code, 32 MiB per GPU, held
 * until the process ends, instead of the buffers ftk_create allocated.  The call itself performs
 * no allocation of any kind (no hipMalloc / hipFree, no event creation: per-kernel timing is not
 * recorded for it) -- it only launches the two kernels of a step on the context's stream.
 *  - Matrix-core kernels only ("mfma16", "tiled") in FTK_SYNC or FTK_HOGWILD mode; the
 *    one-lane-per-sample kernels keep Psi in arrays allocated on demand: FTK_EUNSUPPORTED.
 *  - FTK_EUNSUPPORTED, with the sizes in ftk_last_error, if this shape and |Psi| need more than
 *    the 32 MiB (workgroups x (table rows x padded rank + core-gradient floats) x 4 bytes; the
 *    benchmark shape, order 3 with J = R = 16 and |Psi| = 1e6, needs 23 MB).  At ranks above 32
 *    the factor-row tables are part of the context's own parameter allocation (made by
 *    ftk_create) and only the core-gradient tables use the static array.
 *  - Every context on a GPU shares that GPU's array, and nothing in it has to survive from one
 *    call to the next (each workgroup overwrites its part before the update pass reads it), but
 *    two such calls that overlap on one GPU -- different streams, different host threads -- race.
 *  - Inputs and outputs are the context's, as for ftk_sgd_step; the two calls can be mixed freely.
 */
int ftk_sgd_step_noalloc(ftk_ctx* ctx, float lr_A, float lr_B, float lambda_A, float lambda_B);

/*
 * RMSE = sqrt( sum_{Omega} (x - xhat)^2 / |Omega| ) and MAE = sum_{Omega} |x - xhat| / |Omega|
 * over ALL stored entries (Section 5.1 defines both over a test set Gamma; this library's
 * Gamma is Omega).  Squared errors are summed in double.  out: host.  Waits for the stream.
 */
int ftk_rmse(ftk_ctx* ctx, double* out);
int ftk_mae(ftk_ctx* ctx, double* out);

/*
 * RMSE and MAE of the current parameters on a held-out set Gamma of n_eval entries given as
 * coordinates + values (Section 5.1: both accuracy measures are taken over a test set Gamma):
 *   RMSE = sqrt( sum_Gamma (x - xhat)^2 / |Gamma| ),  MAE = sum_Gamma |x - xhat| / |Gamma|.
 * idx: array of `order` pointers to int32[n_eval] (0-based, the caller's row numbers, struct of
 * arrays as for ftk_create), vals: fp32[n_eval]; host memory, or device memory if flags has
 * FTK_PTRS_DEVICE.  Borrowed for the duration of the call only.  Either output may be NULL.
 * The set is copied to the device, checked and evaluated in one streaming pass; errors are summed
 * in double.  Waits for the stream.  FTK_EINVAL: n_eval outside 1..2^32-1, NULL idx / vals, an
 * index outside [0, I_n), unknown flag bits.  FTK_ENOMEM / FTK_EDEVICE as for ftk_create.
 */
int ftk_evaluate(ftk_ctx* ctx, int64_t n_eval, const int32_t* const* idx, const float* vals, uint32_t flags,
                 double* rmse_out, double* mae_out);

/*
 * Step size of iteration t (t = 0, 1, ...) under the decay the paper trains with (Section 5.1):
 *   gamma_t = alpha / (1 + beta * t^1.5).
 * A plain host function: callers pass the result to ftk_sgd_step as lr_A / lr_B.  Returns NaN for
 * t < 0 or a negative denominator.
 */
double ftk_step_size(double alpha, double beta, int64_t t);

/*
 * Copy parameters out / in.  A[n]: host fp32[I_n * J_n] row-major; B[n]: host fp32[J_n * R]
 * row-major.  Either array of pointers may be NULL (skipped), as may single entries.
 */
int ftk_get_factors(ftk_ctx* ctx, float* const* A_out, float* const* B_out);
int ftk_set_factors(ftk_ctx* ctx, const float* const* A_in, const float* const* B_in);

/*
 * How ftk_sample draws Psi.  The paper only says that Psi is selected at random from Omega
 * (Section 4.1); two rules are built:
 * FTK_SAMPLE_ENTRIES (default): M positions i.i.d. uniform over the stored entries, see ftk_sample.
 * FTK_SAMPLE_TILES: Psi is made of runs of 64 entries that are neighbours in a pseudo-random order
 *   of Omega fixed by nnz alone, so that each run is one contiguous read: stored place q holds the
 *   caller's entry pi(q) = (a q + b) mod nnz with b = floor(nnz / 3) and a the largest integer
 *   <= max(1, floor(nnz * 618034 / 1000000)) coprime to nnz; group g = k / 64 draws its run T_g with
 *   the entry rule (same seed, sample number g) among ceil(nnz / 64) runs, and sample k is the
 *   caller's entry pi((64 T_g + k mod 64) mod nnz).  Samples of a run are distinct entries but the
 *   runs overlap nowhere or completely, so Psi is less random than under the default rule; every
 *   entry is still equally likely (exactly, when 64 divides nnz).  The first switch to this rule
 *   allocates a second copy of the stored entries.  ftk_get_samples reports positions in the
 *   caller's numbering under either rule.
 * Takes effect at the next ftk_sample / ftk_sgd_step.  FTK_EINVAL for an unknown rule.
 */
enum { FTK_SAMPLE_ENTRIES = 0, FTK_SAMPLE_TILES = 1 };
int ftk_set_sampling(ftk_ctx* ctx, int rule);

/* FTK_SYNC (default), FTK_HOGWILD or FTK_HOGWILD_MODEWISE. */
int ftk_set_mode(ftk_ctx* ctx, int mode);

/* Use this hipStream_t (passed as void*) for all later work; NULL = the null stream.
 * The caller keeps ownership of the stream and must keep it alive. */
int ftk_set_stream(ftk_ctx* ctx, void* hip_stream);

/*
 * Per-kernel timing with HIP events on the context's stream, for benchmarks.
 * ftk_set_timing(ctx, 1) makes every later ftk_sample / ftk_sgd_step bracket each kernel it
 * launches with events; ftk_get_timing waits for the stream and returns, for kernel slot
 * `which` (FTK_K_*), the summed milliseconds and the number of launches since timing was
 * switched on (or last read with reset != 0).
 */
enum {
    FTK_K_SAMPLE = 0,   /* Psi materialised as arrays (only launched for the generic kernel / ftk_get_samples) */
    FTK_K_GRAD = 1,     /* gradient pass (the specialised variants also draw Psi and fetch the entries in it) */
    FTK_K_APPLY = 2,    /* update pass: A, B */
    FTK_K_COUNT = 3
};
int ftk_set_timing(ftk_ctx* ctx, int enabled);
int ftk_get_timing(ftk_ctx* ctx, int which, double* total_ms, int64_t* launches, int reset);

/*
 * Gradient-kernel variant.  ftk_create picks the fastest variant built for (N, J_n, R)
 * ("auto").  ftk_set_kernel forces one by name; "auto" restores the default.
 * FTK_EUNSUPPORTED if the named variant is not built for this shape.  The variants:
 *   "mfma16"   J_n = R = 16 for every mode, order <= 6, I_n < 2^24, all A^(n) together below 2 GB
 *   "tiled"    order <= 8 with J_n <= 64, R <= 64 (order 9 and 10: J_n <= 16, R <= 16), I_n * J_n < 2^28, and room in LDS for the core
 *              factors padded to multiples of 16 (twice)
 *   "generic"  one lane per sample: any order <= FTK_MAX_ORDER and any ranks for which
 *              512 * order * R + 4 * sum_n J_n R bytes fit in LDS
 *   "rows"     the "tiled" kernel with the factor-row update done by row owners, the first of the two
 *              thread-block strategies of Section 4.2 (the rows of a mode are distributed over thread blocks;
 *              a row's update is the sum over the samples of Psi that hit it, Eq. Gradient_low_rank): rows
 *              that are not summed in the on-chip tables are written to per-workgroup lists, one list per
 *              bucket of rows, and a second kernel gives every bucket to one workgroup, which sums the
 *              bucket's lists on chip and writes the rows of A^(n): no float atomics on A^(n) or on an
 *              accumulator (at ranks above 32 the workgroups' own tables, which hold the most frequent rows,
 *              are in device memory and are still filled by atomics).  Never chosen by "auto" (measured
 *              slower than "tiled" on this GPU).  Synchronous
 *              step only; needs the shapes of "tiled" with every J_n a multiple of 4 and at most 4096
 *              buckets; allocates the lists (sized from |Psi| and the rows' frequencies) on the device.
 *              "rows:tight" is the same with lists of half the expected length, so that many rows take the
 *              fallback (a full list sends the row through a float atomic after all): for tests.
 * All of them compute the same step (same Psi, same formulas); they differ in speed only.
 * ftk_kernel_name: the variant in use (static string, never NULL).
 */
int ftk_set_kernel(ftk_ctx* ctx, const char* name);
const char* ftk_kernel_name(const ftk_ctx* ctx);

/*
 * Which factor rows the current gradient kernel sums per workgroup (on chip; at ranks above 32 in a
 * table of the workgroup's own in device memory) instead of adding them to the shared accumulator
 * one sample at a time (the sum over the samples that hit a row in Eq. Gradient_low_rank is the same
 * either way; this only reports where it is formed).  Rows of a mode are ranked by how often they
 * occur in Omega, most frequent first, ties by ascending row number; for the sample count of the
 * last ftk_sample (or a default before the first) the kernel keeps ranks [0, K_out[n]) of mode n
 * in a per-workgroup table, of which ranks [0, top_out[n]) go through a one-hot matrix product;
 * all other rows are updated with float atomics.  K_out, top_out: host int32[order], either may be
 * NULL.  The one-lane-per-sample variant keeps no table: all zeros.  For tests and tuning.
 */
int ftk_get_table_rows(ftk_ctx* ctx, int32_t* K_out, int32_t* top_out);

/* Message for the most recent failure on this context (ctx == NULL: of ftk_create on this thread). */
const char* ftk_last_error(const ftk_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* FTK_H */
