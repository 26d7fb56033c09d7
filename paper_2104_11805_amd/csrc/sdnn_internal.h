// Shared between the translation units of libsdnn only.
#pragma once
#include <cstddef>
#include <cstdint>

#include "../../include/sdnn.h"

#include <hip/hip_vector_types.h> // int4

void sdnn_set_global_error(const char *fmt, ...);
const char *sdnn_global_error();

// Per-layer descriptor, readable by the kernels (a copy lives in the workspace).
struct LayerDev {
    int32_t n_out, n_in, nnz, pad_;
    const int32_t *row_ptr;   // [n_out+1]
    const int32_t *col_idx;   // [nnz]
    float *vals;              // [nnz]
    float *bias;              // [n_out]
    const int32_t *t_row_ptr; // [n_in+1]   transposed index (rows of W^T = columns of W)
    const int32_t *t_row_idx; // [nnz]
    const int32_t *t_perm;    // [nnz]      position of the entry in vals
    const int4 *sched;        // [n_out]    {row, first entry, end, 0}, rows of W by decreasing length
    const int4 *t_sched;      // [n_in]     the same for the rows of W^T
    float *X_prev;            // X_{l-1}  [n_in][B]   (training mode)
    float *X;                 // X_l      [n_out][B]  (training mode)
    float *D;                 // Delta_l  [n_out][B]  (training mode)
    float *G[2];              // [nnz] each: gradient of the stored entries over one half of the batch, in the order of
                              // the transposed index (fused backward sweep; training mode)
    const int32_t *t_col;     // [nnz]: the row of W^T (column of W) of each entry of the transposed index; only on nets
                              // created for one sample per step (max_batch == 1) with the fused sweep, NULL otherwise
    float *vals_t;            // [nnz]: the values in the order of the transposed index (vals_t[q] == vals[t_perm[q]]),
                              // read by the fused backward sweep; NULL where that sweep is not set up
    // The way back from the transposed order to the CSR order, in two passes that both move whole runs (NULL with
    // vals_t).  `mid` holds the values grouped by the TR_CHUNK-entry chunk of the CSR array they belong to, inside
    // a chunk in the order of the transposed index, so that chunk c of the CSR array is filled from entries
    // [c TR_CHUNK, (c+1) TR_CHUNK) of mid.  A span of TR_SPAN consecutive entries of the transposed index lands
    // in mid as one run per chunk; the span's workgroup first puts its values into that order in LDS.
    const uint16_t *mid_slot; // [nnz]: rank of entry q among the entries of its span, by place in mid
    const int32_t *mid_dst;   // [nnz]: mid_dst[span start + k] = the place in mid of the span's entry of rank k
    const uint16_t *mid_loc;  // [nnz]: t_perm of the entry at that place of mid, minus its chunk's start
    float *mid;               // [nnz]
    // lane-major copy of W for the LDS-resident forward (small inference nets; NULL otherwise): the rows,
    // longest first, in blocks of 64; block b holds, for k = 0 .. K_b - 1, entry k of its 64 rows side by
    // side (lm[lm_off[b] + 64 k + lane] = {column, weight bits}), padded with {0, 0.0f} up to the block's
    // longest row, so that lane r of a wavefront walks row r with coalesced loads
    int2 *lm;                 // [lm_off[n_blocks]]
    const int32_t *lm_off;    // [n_blocks + 1], multiples of 64
    const int32_t *lm_row;    // [64 n_blocks]: the row of each lane, -1 past the last row
    float *lm_bias;           // [64 n_blocks]: the bias of that row
    int32_t n_blocks, pad2_;
};
