// Which instances of the matrix-core kernel templates the library holds.  The host file (ftk_api.hip) sees them
// as `extern template` declarations; ftk_instances.hip defines them, one translation unit per (kernel family,
// order) -- selected with -DFTK_INST_FAMILY / -DFTK_INST_ORDER -- so that the build can compile them side by side.
#pragma once
#include "ftk_kernels_mfma16.hpp"
#include "ftk_kernels_tiled.hpp"

// J_n = R = 16 kernel, order N: both sampling rules x the four passes, and the evaluation pass
#define FTK_MFMA16_INSTANCES(X, XE, N)                                                    \
    X(N, false, ftk::kSyncPass) X(N, false, ftk::kInPlacePass) X(N, false, ftk::kFactorPhase) X(N, false, ftk::kCorePhase) \
    X(N, true, ftk::kSyncPass) X(N, true, ftk::kInPlacePass) X(N, true, ftk::kFactorPhase) X(N, true, ftk::kCorePhase)     \
    XE(N)
// general matrix-core kernel, order N, ranks padded to 16 P (WAVES waves per workgroup): rows fetched 16 bytes per
// lane or float by float (one pass, and the two phases of the mode-by-mode order), the row-owner form for the
// former; the evaluation pass for both
#define FTK_TILED_INSTANCES_P(X, XE, N, P, WAVES)                                                                               \
    X(N, P, WAVES, true, false, ftk::kSyncPass) X(N, P, WAVES, false, false, ftk::kSyncPass) X(N, P, WAVES, true, true, ftk::kSyncPass) \
    X(N, P, WAVES, true, false, ftk::kFactorPhase) X(N, P, WAVES, true, false, ftk::kCorePhase)                                 \
    X(N, P, WAVES, false, false, ftk::kFactorPhase) X(N, P, WAVES, false, false, ftk::kCorePhase) XE(N, P, true) XE(N, P, false)
#define FTK_TILED_INSTANCES(X, XE, N) \
    FTK_TILED_INSTANCES_P(X, XE, N, 1, 8) FTK_TILED_INSTANCES_P(X, XE, N, 2, 8) FTK_TILED_INSTANCES_P(X, XE, N, 4, 4)
// orders 9 and 10 (the end of the paper's order sweep): ranks up to 16 only
#define FTK_TILED_INSTANCES_HIGH(X, XE, N) FTK_TILED_INSTANCES_P(X, XE, N, 1, 8)

#define FTK_GRAD_MFMA16(N, T, M) template __global__ void ftk::grad_mfma16_kernel<N, T, M>(ftk::Mfma16Args);
#define FTK_ERRORS_MFMA16(N) \
    template __global__ void ftk::errors_mfma16_kernel<N>(ftk::Coo, uint64_t, const float*, const float*, ftk::Layout, ftk::ModeBytes, double*);
#define FTK_GRAD_TILED(N, P, W, X4, R, M) template __global__ void ftk::grad_tiled_kernel<N, P, W, X4, R, M>(ftk::TiledArgs);
#define FTK_ERRORS_TILED(N, P, X4) \
    template __global__ void ftk::errors_tiled_kernel<N, P, X4>(ftk::Coo, uint64_t, const float*, const float*, ftk::Layout, ftk::TiledModeBytes, double*);

#define FTK_ALL_INSTANCES(PREFIX_GM, PREFIX_EM, PREFIX_GT, PREFIX_ET)                                      \
    FTK_MFMA16_INSTANCES(PREFIX_GM, PREFIX_EM, 1) FTK_MFMA16_INSTANCES(PREFIX_GM, PREFIX_EM, 2)           \
    FTK_MFMA16_INSTANCES(PREFIX_GM, PREFIX_EM, 3) FTK_MFMA16_INSTANCES(PREFIX_GM, PREFIX_EM, 4)           \
    FTK_MFMA16_INSTANCES(PREFIX_GM, PREFIX_EM, 5) FTK_MFMA16_INSTANCES(PREFIX_GM, PREFIX_EM, 6)           \
    FTK_TILED_INSTANCES(PREFIX_GT, PREFIX_ET, 1) FTK_TILED_INSTANCES(PREFIX_GT, PREFIX_ET, 2)             \
    FTK_TILED_INSTANCES(PREFIX_GT, PREFIX_ET, 3) FTK_TILED_INSTANCES(PREFIX_GT, PREFIX_ET, 4)             \
    FTK_TILED_INSTANCES(PREFIX_GT, PREFIX_ET, 5) FTK_TILED_INSTANCES(PREFIX_GT, PREFIX_ET, 6)             \
    FTK_TILED_INSTANCES(PREFIX_GT, PREFIX_ET, 7) FTK_TILED_INSTANCES(PREFIX_GT, PREFIX_ET, 8)             \
    FTK_TILED_INSTANCES_HIGH(PREFIX_GT, PREFIX_ET, 9) FTK_TILED_INSTANCES_HIGH(PREFIX_GT, PREFIX_ET, 10)

#ifdef FTK_INSTANCES_EXTERN
// the host file: every instance is defined elsewhere
#define FTK_X_GM(N, T, M) extern FTK_GRAD_MFMA16(N, T, M)
#define FTK_X_EM(N) extern FTK_ERRORS_MFMA16(N)
#define FTK_X_GT(N, P, W, X4, R, M) extern FTK_GRAD_TILED(N, P, W, X4, R, M)
#define FTK_X_ET(N, P, X4) extern FTK_ERRORS_TILED(N, P, X4)
FTK_ALL_INSTANCES(FTK_X_GM, FTK_X_EM, FTK_X_GT, FTK_X_ET)
#endif
