// Host-only setup pieces: CSR validation, transposed index, row schedule.
// Nothing here touches the GPU, so these entry points can be checked on a
// machine without one.
#include "sdnn_internal.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <numeric>
#include <vector>

static thread_local char g_err[512] = "";

void sdnn_set_global_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}
const char *sdnn_global_error() { return g_err; }

extern "C" int sdnn_check_csr(int32_t n_out, int32_t n_in, const int32_t *row_ptr,
                              const int32_t *col_idx)
{
    if (n_out < 0 || n_in < 0) { sdnn_set_global_error("negative matrix size"); return SDNN_EINVAL; }
    if (!row_ptr) { sdnn_set_global_error("row_ptr is NULL"); return SDNN_EINVAL; }
    if (row_ptr[0] != 0) { sdnn_set_global_error("row_ptr[0] != 0"); return SDNN_EINVAL; }
    for (int32_t j = 0; j < n_out; ++j)
        if (row_ptr[j + 1] < row_ptr[j]) {
            sdnn_set_global_error("row_ptr decreases at row %d", j);
            return SDNN_EINVAL;
        }
    if (row_ptr[n_out] > 0 && !col_idx) { sdnn_set_global_error("col_idx is NULL"); return SDNN_EINVAL; }
    for (int32_t j = 0; j < n_out; ++j)
        for (int32_t p = row_ptr[j]; p < row_ptr[j + 1]; ++p) {
            if (col_idx[p] < 0 || col_idx[p] >= n_in) {
                sdnn_set_global_error("column %d out of range in row %d", col_idx[p], j);
                return SDNN_EINVAL;
            }
            if (p > row_ptr[j] && col_idx[p] <= col_idx[p - 1]) {
                sdnn_set_global_error("columns of row %d are not strictly ascending", j);
                return SDNN_EINVAL;
            }
        }
    return SDNN_OK;
}

// Counting sort by column; visiting the rows in ascending order makes every
// transposed row list its source rows in ascending order, which fixes the
// summation order of the backward product.
extern "C" int sdnn_transpose_pattern(int32_t n_out, int32_t n_in, const int32_t *row_ptr,
                                      const int32_t *col_idx, int32_t *t_row_ptr,
                                      int32_t *t_row_idx, int32_t *t_perm)
{
    if (!row_ptr || !t_row_ptr) { sdnn_set_global_error("NULL pointer"); return SDNN_EINVAL; }
    const int32_t nnz = row_ptr[n_out];
    if (nnz > 0 && (!col_idx || !t_row_idx || !t_perm)) {
        sdnn_set_global_error("NULL pointer");
        return SDNN_EINVAL;
    }
    std::fill(t_row_ptr, t_row_ptr + n_in + 1, 0);
    for (int32_t p = 0; p < nnz; ++p) t_row_ptr[col_idx[p] + 1]++;
    for (int32_t i = 0; i < n_in; ++i) t_row_ptr[i + 1] += t_row_ptr[i];
    try {
        std::vector<int32_t> cursor(t_row_ptr, t_row_ptr + n_in);
        for (int32_t j = 0; j < n_out; ++j)
            for (int32_t p = row_ptr[j]; p < row_ptr[j + 1]; ++p) {
                const int32_t q = cursor[col_idx[p]]++;
                t_row_idx[q] = j;
                t_perm[q] = p;
            }
    } catch (...) { // nothing may cross the C boundary
        sdnn_set_global_error("host allocation failed");
        return SDNN_ENOMEM;
    }
    return SDNN_OK;
}

extern "C" int sdnn_row_schedule(int32_t n_rows, const int32_t *row_ptr, int32_t *order)
{
    if (n_rows < 0 || !row_ptr || (n_rows > 0 && !order)) {
        sdnn_set_global_error("NULL pointer or negative size");
        return SDNN_EINVAL;
    }
    std::iota(order, order + n_rows, 0);
    try {
        std::stable_sort(order, order + n_rows, [&](int32_t a, int32_t b) {
            return row_ptr[a + 1] - row_ptr[a] > row_ptr[b + 1] - row_ptr[b];
        });
    } catch (...) {
        sdnn_set_global_error("host allocation failed");
        return SDNN_ENOMEM;
    }
    return SDNN_OK;
}

extern "C" const char *sdnn_version(void) { return "sdnn 0.1 (gfx950)"; }
