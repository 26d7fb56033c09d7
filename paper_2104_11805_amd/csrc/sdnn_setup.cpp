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

// Greedy clustering of rows by shared columns, one pass over the entries.  Every column remembers
// the cluster of the last row that used it; a row joins the open cluster that most of its columns
// point at (if at least a quarter of them do), otherwise it opens a new cluster.  Clusters are
// closed at max_cluster_rows rows.  The result lists the rows cluster by cluster, clusters by
// decreasing longest row (so the longest-first dealing of the row schedule survives between
// clusters), rows inside a cluster by decreasing length, ties in arrival order.
extern "C" int sdnn_cluster_rows(int32_t n_rows, int32_t n_cols, const int32_t *row_ptr, const int32_t *col_idx,
                                 int32_t max_cluster_rows, int32_t *order, int32_t *cluster_of)
{
    if (n_rows < 0 || n_cols < 0 || !row_ptr || (n_rows > 0 && !order) || max_cluster_rows < 1) {
        sdnn_set_global_error("NULL pointer or bad size");
        return SDNN_EINVAL;
    }
    if (row_ptr[n_rows] > 0 && !col_idx) { sdnn_set_global_error("col_idx is NULL"); return SDNN_EINVAL; }
    try {
        std::vector<int32_t> last((size_t)n_cols, -1);  // column -> cluster of the last row that used it
        std::vector<int32_t> size, longest;             // per cluster
        std::vector<int32_t> votes, touched;            // scratch: votes per cluster of the current row
        std::vector<int32_t> member((size_t)n_rows, -1);
        for (int32_t j = 0; j < n_rows; ++j) {
            const int32_t beg = row_ptr[j], end = row_ptr[j + 1], len = end - beg;
            int32_t best = -1, best_votes = 0;
            touched.clear();
            for (int32_t p = beg; p < end; ++p) {
                const int32_t c = last[col_idx[p]];
                if (c < 0 || size[c] >= max_cluster_rows) continue;
                if (votes[c]++ == 0) touched.push_back(c);
                if (votes[c] > best_votes || (votes[c] == best_votes && c < best)) { best_votes = votes[c]; best = c; }
            }
            for (int32_t c : touched) votes[c] = 0;
            if (best < 0 || 4 * best_votes < len) { // nothing worth joining: a cluster of its own
                best = (int32_t)size.size();
                size.push_back(0);
                longest.push_back(0);
                votes.push_back(0);
            }
            member[j] = best;
            size[best]++;
            longest[best] = std::max(longest[best], len);
            for (int32_t p = beg; p < end; ++p) last[col_idx[p]] = best;
        }
        const int32_t n_clusters = (int32_t)size.size();
        std::vector<int32_t> corder((size_t)n_clusters);
        std::iota(corder.begin(), corder.end(), 0);
        std::stable_sort(corder.begin(), corder.end(), [&](int32_t a, int32_t b) { return longest[a] > longest[b]; });
        std::vector<int32_t> rank((size_t)n_clusters);
        for (int32_t k = 0; k < n_clusters; ++k) rank[corder[k]] = k;
        std::iota(order, order + n_rows, 0);
        std::stable_sort(order, order + n_rows, [&](int32_t a, int32_t b) {
            if (rank[member[a]] != rank[member[b]]) return rank[member[a]] < rank[member[b]];
            return row_ptr[a + 1] - row_ptr[a] > row_ptr[b + 1] - row_ptr[b];
        });
        if (cluster_of)
            for (int32_t j = 0; j < n_rows; ++j) cluster_of[j] = rank[member[j]];
    } catch (...) {
        sdnn_set_global_error("host allocation failed");
        return SDNN_ENOMEM;
    }
    return SDNN_OK;
}

// Deals a row order out to the 8 XCDs.  Workgroups take 4 consecutive rows of the schedule and
// workgroup ids go to the XCDs round-robin, so rows 32q + 4x .. 32q + 4x + 3 of the schedule run on
// XCD x.  The rows of `order` (neighbours share columns) are cut into 8 contiguous stretches of about
// equal numbers of entries, and stretch x fills the places of XCD x: neighbours then run on one XCD
// (one L2) and, four at a time, on one CU at about the same moment.  When the stretches differ in
// length the places left over at the end are filled from the remaining stretches in turn.
extern "C" int sdnn_deal_rows_to_xcds(int32_t n_rows, const int32_t *row_ptr, const int32_t *order, int32_t *dealt)
{
    if (n_rows < 0 || !row_ptr || (n_rows > 0 && (!order || !dealt))) {
        sdnn_set_global_error("NULL pointer or negative size");
        return SDNN_EINVAL;
    }
    const int X = 8, G = 4;
    try {
        // cut points by entries (+1 per row so that empty rows count too)
        int64_t total = 0;
        for (int32_t r = 0; r < n_rows; ++r) total += row_ptr[order[r] + 1] - row_ptr[order[r]] + 1;
        std::vector<int32_t> cut(X + 1, n_rows);
        cut[0] = 0;
        int64_t acc = 0;
        int x = 1;
        for (int32_t r = 0; r < n_rows && x < X; ++r) {
            acc += row_ptr[order[r] + 1] - row_ptr[order[r]] + 1;
            while (x < X && acc * X >= total * x) cut[x++] = r + 1;
        }
        std::vector<int32_t> next(cut.begin(), cut.begin() + X); // read position of every stretch
        for (int32_t pos = 0; pos < n_rows; ++pos) {
            int xcd = (pos / G) % X;
            for (int t = 0; t < X && next[xcd] >= cut[xcd + 1]; ++t) xcd = (xcd + 1) % X; // stretch used up: the next one
            dealt[pos] = order[next[xcd]++];
        }
    } catch (...) {
        sdnn_set_global_error("host allocation failed");
        return SDNN_ENOMEM;
    }
    return SDNN_OK;
}

extern "C" const char *sdnn_version(void) { return "sdnn 0.1 (gfx950)"; }
