// Definitions of the matrix-core kernel instances of one (family, order): see ftk_instances.hpp.
//   -DFTK_INST_FAMILY=1 -DFTK_INST_ORDER=N   J_n = R = 16 kernel, order N (1..6)
//   -DFTK_INST_FAMILY=2 -DFTK_INST_ORDER=N   general matrix-core kernel, order N (1..10)
#define FTK_TEMPLATE_KERNELS_ONLY
#include "ftk_instances.hpp"

#if FTK_INST_FAMILY == 1
FTK_MFMA16_INSTANCES(FTK_GRAD_MFMA16, FTK_ERRORS_MFMA16, FTK_INST_ORDER)
#elif FTK_INST_FAMILY == 2
#if FTK_INST_ORDER <= 8
FTK_TILED_INSTANCES(FTK_GRAD_TILED, FTK_ERRORS_TILED, FTK_INST_ORDER)
#else
FTK_TILED_INSTANCES_HIGH(FTK_GRAD_TILED, FTK_ERRORS_TILED, FTK_INST_ORDER)
#endif
#else
#error "FTK_INST_FAMILY must be 1 or 2"
#endif
