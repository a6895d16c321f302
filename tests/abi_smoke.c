/* The boundary from plain C: the header compiles as C99, the library links, and calls that need no
 * device behave as the header says.  Built and run by tests/test_abi_host.py. */
#include <stdio.h>

#include "ftk.h"

int main(void) {
    ftk_ctx* ctx = (ftk_ctx*)&ctx; /* any non-NULL value: ftk_create has to reset it */
    const int rc = ftk_create(&ctx, 0, NULL, 1, NULL, NULL, NULL, 4, 1u, FTK_PTRS_HOST); /* order 0 */
    printf("create rc=%d ctx_is_null=%d error=\"%s\"\n", rc, ctx == NULL, ftk_last_error(NULL));
    printf("null ctx: sample=%d step=%d rmse=%d kernel=%s\n", ftk_sample(NULL, 1u, 1), ftk_sgd_step(NULL, 0.f, 0.f, 0.f, 0.f),
           ftk_rmse(NULL, NULL), ftk_kernel_name(NULL));
    printf("step_size=%.17g\n", ftk_step_size(0.5, 0.25, 4));
    ftk_destroy(NULL);
    return (rc == FTK_EINVAL && ctx == NULL) ? 0 : 1;
}
