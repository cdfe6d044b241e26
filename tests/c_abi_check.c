/* Compiled as C99 by tests/test_headers_are_c_cpu.py: the public headers must be plain C, and a C
 * program must be able to link against the library and reach its host-side entry points. */
#include <stdio.h>
#include <string.h>

#include "lnmod.h"
#include "lnmod_sched.h"
#include "lnmod_tools.h"

int main(void) {
    int shape[7] = {0, 0, 0, 0, 0, 0, 0};   /* K, VPL, R, per_cu, clusters, interleave, flat */
    /* validation runs before any device call, so these work on a host without a GPU */
    if (lnmod_forward(NULL, NULL, NULL, 1, 8, 64, 1e-6f, NULL, NULL, NULL, NULL, LNMOD_BF16, LNMOD_PER_SAMPLE) !=
        LNMOD_EINVAL)
        return 1;
    if (strcmp(lnmod_status_string(LNMOD_OK), lnmod_status_string(LNMOD_EINVAL)) == 0) return 2;
    if (lnmod_backward_workspace_bytes(1, 75600, 5120, LNMOD_PER_SAMPLE) == 0) return 3;
    if (lnmod_table_shape(LNMOD_FAMILY_BACKWARD, 5120, LNMOD_BF16, 0, shape) != LNMOD_OK) return 4;
    if (shape[0] * shape[1] * 64 < 5120 / 8) return 5;
    if (lnmod_backward_workspace_bytes_shaped(NULL, 1, 75600, 5120, LNMOD_PER_SAMPLE) !=
        lnmod_backward_workspace_bytes(1, 75600, 5120, LNMOD_PER_SAMPLE))
        return 6;
    if (lnmod_backward_workspace_bytes_shaped(shape, 1, 75600, 5120, LNMOD_PER_SAMPLE) == 0) return 7;
    printf("backward D=5120 bf16: K=%d VPL=%d R=%d per_cu=%d\n", shape[0], shape[1], shape[2], shape[3]);
    return 0;
}
