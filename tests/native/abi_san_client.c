/* Host-side paths of the library (argument validation, launch planning, Option II arithmetic)
 * driven from C for a build whose HOST code carries AddressSanitizer and UBSan.  No kernel is
 * launched: every call below fails validation (or is pure host arithmetic), so the host arrays
 * passed as pointers are never handed to a kernel, with or without a GPU in the machine. */
#include <stdio.h>
#include <stdint.h>
#include "core.h"
int main(void) {
    float dummy[64];
    uint64_t plan[10];
    unsigned long long acc = 0;
    for (uint64_t d = 1; d <= (1ull << 34); d = d * 3 + 1)
        for (uint32_t m = 1; m < (1u << 22); m = m * 5 + 3)
            for (uint32_t n = 1; n <= 65535; n = n * 7 + 1) {
                if (core_debug_plan(d, m, n, plan) == CORE_OK) acc += plan[2] + plan[5];
                acc += core_workspace_bytes(d, m, n) & 0xff;
            }
    size_t ws = core_workspace_bytes(1024, 16, 4);
    int rc = core_round(1, 0, 1024, 16, 4, dummy, CORE_DTYPE_F32, 1024, dummy, dummy, dummy, ws - 1, NULL);
    printf("round rc %d (%s)\n", rc, core_strerror(rc));
    if (rc != CORE_ERR_WORKSPACE_TOO_SMALL) return 1;
    rc = core_reconstruct_update(1, 0, 16, 4, dummy, 0.25f, 0.1f, dummy + 16, dummy + 20, NULL, 0.0f, NULL, NULL, NULL);
    printf("overlap rc %d\n", rc);
    if (rc != CORE_ERR_INVALID_ARGUMENT) return 2;
    rc = core_accept_trial(16, dummy, dummy + 1, dummy + 16, dummy + 24, (int32_t *)(dummy + 2), NULL);
    printf("accept rc %d\n", rc);
    if (rc != CORE_ERR_INVALID_ARGUMENT) return 3;
    rc = core_reconstruct_trial(1, 0, 16, 4, dummy, 0.25f, dummy + 40, dummy + 16, dummy + 40, NULL, NULL);
    if (rc != CORE_ERR_INVALID_ARGUMENT) return 4;
    rc = core_nonconvex_step(16, 4, dummy, 4.0f, 1.0, 1.0, dummy + 8, dummy + 8, NULL);
    if (rc != CORE_ERR_INVALID_ARGUMENT) return 5;
    rc = core_reconstruct(1, 0, 4, 0xFFFFFFFFu, dummy, 0.25f, dummy + 8, NULL);   /* m above 2^32 - 1024 */
    if (rc != CORE_ERR_INVALID_ARGUMENT) return 7;
    if (core_workspace_bytes(4, 0xFFFFFC01u, 1) != 0 || core_workspace_bytes(4, 0xFFFFFC00u, 1) == 0) return 8;
    double h = 0; rc = core_step_size_option2(1 << 20, 64, 2.0, 0.1, 3.0, 4.0, &h);
    printf("opt2 rc %d h %g acc %llu\n", rc, h, acc);
    if (rc != CORE_OK) return 6;
    double loss = -1.0; rc = core_privacy_loss(32.0, 8, 2.0, 2.0, &loss);   /* equal norms: no loss */
    if (rc != CORE_OK || loss != 0.0) return 9;
    if (core_privacy_loss(32.0, 8, 2.0, 0.0, &loss) != CORE_ERR_INVALID_ARGUMENT) return 10;
    /* the output must not overlap the projections */
    if (core_projection_sqnorms(4, 2, dummy, (double *)(dummy + 6), NULL) != CORE_ERR_INVALID_ARGUMENT) return 11;
    puts("sanitized client ok");
    return 0;
}
