/* The public header must be plain C, and the host-only entry points must link and run without a GPU.
 * Built and run by tests/test_host_setup.py (gcc -std=c99 -pedantic -Wall -Werror). */
#include <stdio.h>
#include <string.h>

#include "sdnn.h"

int main(void)
{
    /* 3 x 4 pattern:  row 0: cols 1,3   row 1: (empty)   row 2: cols 0,1,2 */
    const int32_t row_ptr[4] = {0, 2, 2, 5};
    const int32_t col_idx[5] = {1, 3, 0, 1, 2};
    const float values[5] = {1.f, 2.f, 3.f, 4.f, 5.f};
    int32_t t_row_ptr[5], t_row_idx[5], t_perm[5], order[3];
    sdnn_layer layer;
    sdnn_config cfg;
    size_t bytes = 0;

    if (strncmp(sdnn_version(), "sdnn", 4) != 0) return 1;
    if (sdnn_check_csr(3, 4, row_ptr, col_idx) != SDNN_OK) return 2;
    if (sdnn_transpose_pattern(3, 4, row_ptr, col_idx, t_row_ptr, t_row_idx, t_perm) != SDNN_OK) return 3;
    /* column 1 holds the entries (0,1) at position 0 and (2,1) at position 3 */
    if (t_row_ptr[1] != 1 || t_row_ptr[2] != 3 || t_row_idx[1] != 0 || t_row_idx[2] != 2 || t_perm[1] != 0 ||
        t_perm[2] != 3)
        return 4;
    if (sdnn_row_schedule(3, row_ptr, order) != SDNN_OK || order[0] != 2 || order[1] != 0 || order[2] != 1) return 5;

    layer.n_out = 3; layer.n_in = 4; layer.row_ptr = row_ptr; layer.col_idx = col_idx; layer.values = values;
    layer.bias = NULL;
    memset(&cfg, 0, sizeof cfg);
    cfg.act_cap = 32.0f; cfg.max_batch = 8; cfg.training = 1; cfg.update_bias = 1;
    cfg.activation = SDNN_ACT_RELU_CAP; cfg.fuse_gradient = SDNN_FUSE_AUTO;
    if (sdnn_workspace_bytes(&layer, 1, &cfg, &bytes) != SDNN_OK || bytes == 0) return 6;
    cfg.max_batch = 0;
    if (sdnn_workspace_bytes(&layer, 1, &cfg, &bytes) != SDNN_EINVAL || strlen(sdnn_last_error(NULL)) == 0) return 7;
    printf("c abi ok, workspace %lu bytes\n", (unsigned long)bytes);
    return 0;
}
