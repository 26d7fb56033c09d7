// Host-only setup routines of libsdnn under AddressSanitizer + UBSan (built and run by
// tests/test_host_setup.py with g++; no GPU, no HIP runtime: only sdnn_setup.cpp is linked).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../include/sdnn.h"

static uint32_t rng_state = 12345u;
static uint32_t rnd() { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }

int main()
{
    for (int trial = 0; trial < 200; ++trial) {
        const int n_out = 1 + rnd() % 40, n_in = 1 + rnd() % 40;
        std::vector<int32_t> row_ptr(n_out + 1, 0), col;
        for (int j = 0; j < n_out; ++j) {
            for (int i = 0; i < n_in; ++i)
                if (rnd() % 4 == 0) col.push_back(i);
            row_ptr[j + 1] = (int32_t)col.size();
        }
        const int nnz = (int)col.size();
        if (sdnn_check_csr(n_out, n_in, row_ptr.data(), col.data()) != SDNN_OK) return 1;
        std::vector<int32_t> t_rp(n_in + 1), t_ri(nnz), t_pm(nnz), order(n_out), back_rp(n_out + 1), back_ri(nnz), back_pm(nnz);
        if (sdnn_transpose_pattern(n_out, n_in, row_ptr.data(), col.data(), t_rp.data(), t_ri.data(), t_pm.data())) return 2;
        if (sdnn_transpose_pattern(n_in, n_out, t_rp.data(), t_ri.data(), back_rp.data(), back_ri.data(), back_pm.data())) return 3;
        for (int j = 0; j <= n_out; ++j) if (back_rp[j] != row_ptr[j]) return 4;
        for (int p = 0; p < nnz; ++p) if (back_ri[p] != col[p] || t_pm[back_pm[p]] != p) return 5;
        if (sdnn_row_schedule(n_out, row_ptr.data(), order.data())) return 6;
        for (int r = 1; r < n_out; ++r)
            if (row_ptr[order[r] + 1] - row_ptr[order[r]] > row_ptr[order[r - 1] + 1] - row_ptr[order[r - 1]]) return 7;
        // clustering by shared columns and dealing to the XCDs: both give permutations of the rows
        {
            std::vector<int32_t> corder(n_out), cluster_of(n_out), dealt(n_out), seen(n_out, 0);
            if (sdnn_cluster_rows(n_out, n_in, row_ptr.data(), col.data(), 1 + (int)(rnd() % 9), corder.data(), cluster_of.data())) return 10;
            if (sdnn_deal_rows_to_xcds(n_out, row_ptr.data(), corder.data(), dealt.data())) return 11;
            for (int r = 0; r < n_out; ++r) {
                if (dealt[r] < 0 || dealt[r] >= n_out || seen[dealt[r]]++) return 12;
                if (cluster_of[r] < 0 || cluster_of[r] >= n_out) return 13;
            }
        }
        // malformed inputs must be rejected, not read out of bounds
        if (nnz > 0) {
            std::vector<int32_t> bad(col);
            bad[rnd() % nnz] = n_in + (int)(rnd() % 5);
            if (sdnn_check_csr(n_out, n_in, row_ptr.data(), bad.data()) != SDNN_EINVAL) return 8;
        }
    }
    if (sdnn_check_csr(3, 3, nullptr, nullptr) != SDNN_EINVAL) return 9;
    std::puts("host setup: ok");
    return 0;
}
