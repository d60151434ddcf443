/* A plain C11 client of include/core.h: proves the header is valid C, that the library links
 * from C, and that bad arguments come back as error codes (no GPU is touched). */
#include <stdio.h>
#include <string.h>
#include "core.h"

int main(void)
{
    float dummy[4];
    if (core_workspace_bytes(0, 1, 1) != 0) return 1;
    const size_t ws = core_workspace_bytes(1024, 16, 4);
    if (ws == 0) return 2;
    if (core_round(1, 0, 1024, 16, 4, NULL, CORE_DTYPE_F32, 1024, dummy, dummy, dummy, ws, NULL)
        != CORE_ERR_INVALID_ARGUMENT) return 3;
    if (core_compress(1, 0, 16, 4, dummy, (core_dtype)9, dummy, dummy, ws, NULL) != CORE_ERR_INVALID_ARGUMENT) return 4;
    if (core_reconstruct(1, 0, 16, 4, dummy, 0.25f, NULL, NULL) != CORE_ERR_INVALID_ARGUMENT) return 5;
    if (core_reconstruct_update(1, 0, 16, 4, dummy, 0.25f, 0.1f, NULL, dummy, NULL, 0.0f, NULL, NULL, NULL)
        != CORE_ERR_INVALID_ARGUMENT) return 6;
    if (core_xi_bytes(5, 3) != 2u * 3u * 16u) return 7;
    if (strlen(core_strerror(CORE_ERR_WORKSPACE_TOO_SMALL)) == 0) return 8;
    if (core_last_hip_error() != 0) return 9;
    {
        double h = 0.0;
        if (core_step_size_option2(16, 16, 1e-9, 1.0, 2.0, 8.0, &h) != CORE_OK) return 10;
        if (h < 0.99 / 3200.0 || h > 1.01 / 3200.0) return 11;
        if (core_accept_trial(16, dummy, dummy + 1, dummy, dummy, NULL, NULL) != CORE_ERR_INVALID_ARGUMENT)
            return 12;
        if (core_nonconvex_step(16, 4, dummy, 4.0f, -1.0, 1.0, NULL, dummy + 1, NULL)
            != CORE_ERR_INVALID_ARGUMENT) return 13;
    }
    puts("c client ok");
    return 0;
}
