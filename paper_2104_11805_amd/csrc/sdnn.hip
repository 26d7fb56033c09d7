// libsdnn: HIP kernels (gfx950) and the C-ABI entry points that launch them.
//
// Mapping to the hardware (64-wide wavefronts, no matrix cores: none of the
// three passes is a dense contraction):
//   * forward / backward product: one wavefront per matrix row, the 64 lanes
//     walk the row together and each lane owns V consecutive samples, so the
//     row's column indices and weights are wave-uniform (scalar loads) and each
//     gathered activation row is one contiguous 256*V-byte read.  Each lane adds
//     its terms in storage order in fp64: the sum is the same as a sequential
//     CPU loop's, whatever the batch size.
//   * pattern-confined gradient: one wavefront per row, lanes split as
//     4 edge groups x 16 sample lanes, so that only a 16-lane butterfly is
//     needed per 8 edges before the weight is rewritten in place.
//   * W^T: the transposed index lists, per column, the source rows and the
//     positions of the values in the CSR array.
//   * layers of 4096 rows and more: the backward sweep also forms the gradient
//     of the stored entries (k_bwd_grad, gathered rows parked in LDS) and reads
//     the values from a copy in the order of the transposed index; the descent
//     step is then a streaming pass over that copy (k_apply) and a second one
//     that rebuilds the CSR copy (k_spread_vals).
//   * inference on large activation blocks goes through all layers in
//     sub-blocks of samples, so that a layer's output is still in the
//     memory-side cache when the next layer gathers it.
//   * one sample per step (B = 1): lanes over entries / rows instead of samples
//     (k_spmv_stage, k_spmv_wave, k_spmv, k_update_b1).
//   * inference that drops dead samples: flags set by the forward epilogue,
//     in-place packing on the device (k_pack), no host synchronisation.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <functional>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "sdnn_internal.h"

// ---------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------

#define LDS_T 4        // samples a workgroup of the LDS-resident forward carries
#define LDS_MAX_N 4096 // its widest layer: 2 buffers x 4096 x 4 samples x 4 B = 128 KiB of the CU's 160 KiB
#define WAVES_PER_BLOCK 4 // product kernels: 4 rows per workgroup (measured best of 1, 2, 4, 8)
#define UPD_WAVES 1       // update kernel: one wavefront per workgroup (measured best of 1, 2, 4, 8)
#define BLOCK_THREADS (64 * WAVES_PER_BLOCK)

template <int V> __device__ __forceinline__ void ldv(const float *p, float (&x)[V]);
template <> __device__ __forceinline__ void ldv<1>(const float *p, float (&x)[1]) { x[0] = *p; }
template <> __device__ __forceinline__ void ldv<2>(const float *p, float (&x)[2])
{
    const float2 t = *reinterpret_cast<const float2 *>(p);
    x[0] = t.x; x[1] = t.y;
}
template <> __device__ __forceinline__ void ldv<4>(const float *p, float (&x)[4])
{
    const float4 t = *reinterpret_cast<const float4 *>(p);
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
}
template <int V> __device__ __forceinline__ void stv(float *p, const float (&x)[V]);
template <> __device__ __forceinline__ void stv<1>(float *p, const float (&x)[1]) { *p = x[0]; }
template <> __device__ __forceinline__ void stv<2>(float *p, const float (&x)[2])
{
    *reinterpret_cast<float2 *>(p) = make_float2(x[0], x[1]);
}
template <> __device__ __forceinline__ void stv<4>(float *p, const float (&x)[4])
{
    *reinterpret_cast<float4 *>(p) = make_float4(x[0], x[1], x[2], x[3]);
}

// Gather of V consecutive floats of an activation row through a buffer
// descriptor: the address is (uniform base) + (scalar row offset) + (lane
// offset), so a load costs one SGPR and no per-load address VGPRs.  Offsets are
// 32-bit byte offsets: an activation block must stay below 4 GiB (checked by the
// host).  Reads past num_records return 0 instead of faulting.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const float *base, size_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)(unsigned)bytes, 0x00020000);
}
template <int V>
__device__ __forceinline__ void gatherv(__amdgpu_buffer_rsrc_t r, unsigned lane_off, unsigned row_off,
                                        float (&x)[V])
{
    if constexpr (V == 1) {
        x[0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)lane_off, (int)row_off, 0));
    } else if constexpr (V == 2) {
        const u32x2 t = __builtin_amdgcn_raw_buffer_load_b64(r, (int)lane_off, (int)row_off, 0);
        x[0] = __uint_as_float(t.x); x[1] = __uint_as_float(t.y);
    } else {
        const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)row_off, 0);
        x[0] = __uint_as_float(t.x); x[1] = __uint_as_float(t.y);
        x[2] = __uint_as_float(t.z); x[3] = __uint_as_float(t.w);
    }
}

// Activations (the paper's Eq. 3 leaves f open; Section 6.1 trains with the sigmoid).
//   ACT_RELU_CAP: f(z) = min(max(z, 0), cap), f' = [0 < x < cap] from the stored output x
//   ACT_SIGMOID:  f(z) = 1 / (1 + exp(-z)),   f' = x (1 - x)     from the stored output x
#define ACT_RELU_CAP 0
#define ACT_SIGMOID 1
__device__ __forceinline__ float act_apply(int act, double z, float capf)
{
    if (act == ACT_SIGMOID) return (float)(1.0 / (1.0 + exp(-z)));
    const double cap = (double)capf;
    z = z < 0.0 ? 0.0 : z;
    z = z > cap ? cap : z;
    return (float)z;
}
// value * f'(z) with f' taken from the stored output x
__device__ __forceinline__ float act_backprop(int act, double value, float x, float capf)
{
    if (act == ACT_SIGMOID) {
        const double xd = (double)x;
        return (float)(value * (xd * (1.0 - xd)));
    }
    return (x > 0.0f && x < capf) ? (float)value : 0.0f;
}

// Orders the LDS (or in-place global) accesses of the lanes of one wavefront: what the lanes wrote before
// is visible to the other lanes after, and nothing is moved across.  Costs no instruction beyond the wait
// for the outstanding accesses.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup ids are handed to the 8 XCDs round-robin and each XCD has its own
// L2.  Give every XCD whole batch tiles (all row groups of tile x, x+8, ...)
// so that the activation slab of a tile is gathered through one L2 only.  The
// tiles left over when the tile count is not a multiple of 8 are shared.
__device__ __forceinline__ void map_block(unsigned bid, unsigned n_tiles, unsigned n_rg,
                                          unsigned &tile, unsigned &rg)
{
    const unsigned t8 = n_tiles & ~7u;
    const unsigned n8 = t8 * n_rg;
    if (bid < n8) {
        const unsigned xcd = bid & 7u, k = bid >> 3;
        tile = xcd + 8u * (k / n_rg);
        rg = k % n_rg;
    } else {
        const unsigned k = bid - n8;
        tile = t8 + k / n_rg;
        rg = k % n_rg;
    }
}

// ---------------------------------------------------------------------------
// K1 / K2: row-per-wavefront sparse product with fused epilogue
//   MODE 0 (forward, Eq. 3):   out = min(max(sum + bias[row], 0), cap)
//   MODE 1 (backward, Eq. 7):  out = sum * [0 < Xprev[row] < cap]; the values
//                              are read through the transposed index (perm)
// ---------------------------------------------------------------------------
struct SpmmArgs {
    const int32_t *row_ptr;
    const int32_t *idx;
    const float *vals;
    const int32_t *perm;  // MODE 1 only
    const int4 *sched;    // per task: {row, first entry, end of entries, 0}, rows by decreasing length
    const float *in;      // [n_cols][B]
    size_t in_bytes;      // < 4 GiB
    float *out;           // [n_rows][B]
    const float *aux;     // MODE 0: bias [n_rows] (may be NULL); MODE 1: Xprev [n_rows][B]
    int32_t n_rows, B;
    uint32_t n_tiles, n_rg, n_vblocks, tile_base;
    float cap;
    int32_t act;
    const int32_t *n_live; // NULL, or the number of leading columns of the block that still matter (device)
    int32_t *flags;        // NULL, or MODE 0: flags[s] is set to 1 for every sample s with a non-zero output
    float *g_part;         // GRAD kernels: gradient of the stored entries over this launch's samples, in the order of
                           // the transposed index [nnz]
    int32_t store_out;     // GRAD kernels: 0 = only the gradient is wanted (first layer: there is no Delta_0)
};

// The part of a row task that does not depend on the previous layer's output:
// which row, where its entries are, and its first (up to) 64 entries, entry k
// held by lane k.
struct RowMeta {
    int row, beg, end;
    int c_l;
    float w_l;
    int p_l; // MODE 1: position of the entry in the CSR arrays
};

template <int MODE>
__device__ __forceinline__ void load_chunk(const int32_t *idx, const float *vals, const int32_t *perm,
                                           int base, int end, int lane, int &c_l, float &w_l, int &p_l)
{
    c_l = 0;
    w_l = 0.0f;
    p_l = 0;
    if (base + lane < end) {
        c_l = idx[base + lane];
        if (MODE == 1) {
            p_l = perm[base + lane];
            w_l = vals[p_l];
        } else {
            w_l = vals[base + lane];
        }
    }
}

template <int MODE>
__device__ __forceinline__ RowMeta load_meta(const int4 *sched, const int32_t *idx, const float *vals,
                                             const int32_t *perm, int r, int lane)
{
    RowMeta m;
    const int4 t = sched[r]; // one (scalar) load instead of the chain order -> row_ptr
    m.row = t.x;
    m.beg = t.y;
    m.end = t.z;
    load_chunk<MODE>(idx, vals, perm, m.beg, m.end, lane, m.c_l, m.w_l, m.p_l);
    return m;
}

// One row of the product for the 64*V samples of one batch tile.  All 64 lanes
// must be active (lane k's registers are read by readlane); lanes past the end
// of the batch redo sample 0 and do not store.
template <int V, int MODE, int U, int ACT>
__device__ __forceinline__ void spmm_row(RowMeta m, const int32_t *idx, const float *vals,
                                         const int32_t *perm, const float *in, size_t in_bytes,
                                         float *out, const float *aux, int B, float capf, int act,
                                         unsigned tile, int lane, int32_t *flags)
{
    const int s_own = (int)tile * (64 * V) + lane * V;
    const bool live = s_own < B;
    const int s = live ? s_own : 0;
    const size_t ld = (size_t)B;
    const unsigned so = 4u * (unsigned)s;  // byte offset of the lane inside an activation row
    const unsigned ldb = 4u * (unsigned)B; // bytes per activation row
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(in, in_bytes);

    // operands of the epilogue, requested early so that they arrive with the gathers
    float xp[V];
    double b = 0.0;
    if (MODE == 0) {
        if (aux) b = (double)aux[m.row];
    } else {
        ldv<V>(aux + (size_t)m.row * ld + s, xp);
    }

    double acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.0;

    // Long rows (U == 16), forward: a row's entries are the same for all lanes and never change inside a kernel, so they
    // are read through the scalar cache, 16 columns and 16 weights at a time and a group ahead, straight into scalar
    // registers: no lane broadcasts (2 of 11 vector instructions per entry at four samples per lane).
    if constexpr (MODE == 0 && U == 16) {
        typedef int i32x16 __attribute__((ext_vector_type(16)));
        typedef float f32x16 __attribute__((ext_vector_type(16)));
        const int __attribute__((address_space(4))) *sidx = (const int __attribute__((address_space(4))) *)idx;
        const float __attribute__((address_space(4))) *svals = (const float __attribute__((address_space(4))) *)vals;
        int g = m.beg;
        i32x16 c, cn;
        f32x16 w, wn;
        if (g + 16 <= m.end) {
#pragma unroll
            for (int k = 0; k < 16; ++k) { c[k] = sidx[g + k]; w[k] = svals[g + k]; }
        }
        for (; g + 16 <= m.end; g += 16) {
            if (g + 32 <= m.end) {
#pragma unroll
                for (int k = 0; k < 16; ++k) { cn[k] = sidx[g + 16 + k]; wn[k] = svals[g + 16 + k]; }
            }
            float x[16][V];
#pragma unroll
            for (int k = 0; k < 16; ++k) gatherv<V>(rin, so, (unsigned)c[k] * ldb, x[k]);
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const double wk = (double)w[k];
#pragma unroll
                for (int v = 0; v < V; ++v) acc[v] = fma(wk, (double)x[k][v], acc[v]);
            }
            c = cn;
            w = wn;
        }
        if (g < m.end) { // the row's last entries, fewer than 16: same order, every entry guarded (wave-uniform)
            const int n = m.end - g;
            float x[16][V];
#pragma unroll
            for (int k = 0; k < 16; ++k)
                if (k < n) gatherv<V>(rin, so, (unsigned)sidx[g + k] * ldb, x[k]);
#pragma unroll
            for (int k = 0; k < 16; ++k)
                if (k < n) {
                    const double wk = (double)svals[g + k];
#pragma unroll
                    for (int v = 0; v < V; ++v) acc[v] = fma(wk, (double)x[k][v], acc[v]);
                }
        }
    } else {
    // U gathers are in flight per lane before the first of them is consumed
    int c_l = m.c_l, p_l = m.p_l;
    float w_l = m.w_l;
    for (int base = m.beg; base < m.end; base += 64) {
        const int n = min(64, m.end - base);
        // the entries of the next 64 are requested before this chunk's gathers, not after them
        int c_n = 0, p_n = 0;
        float w_n = 0.0f;
        if (base + 64 < m.end) load_chunk<MODE>(idx, vals, perm, base + 64, m.end, lane, c_n, w_n, p_n);
        for (int g = 0; g < n; g += U) {
            float x[U][V];
            if (g + U <= n) {
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    const int c = __builtin_amdgcn_readlane(c_l, g + k);
                    gatherv<V>(rin, so, (unsigned)c * ldb, x[k]);
                }
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    const double wk = (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_l), g + k));
#pragma unroll
                    for (int v = 0; v < V; ++v) acc[v] = fma(wk, (double)x[k][v], acc[v]);
                }
            } else {
                // ragged end of the row: same order, every entry guarded (wave-uniform branches)
#pragma unroll
                for (int k = 0; k < U; ++k)
                    if (g + k < n) {
                        const int c = __builtin_amdgcn_readlane(c_l, g + k);
                        gatherv<V>(rin, so, (unsigned)c * ldb, x[k]);
                    }
#pragma unroll
                for (int k = 0; k < U; ++k)
                    if (g + k < n) {
                        const double wk = (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_l), g + k));
#pragma unroll
                        for (int v = 0; v < V; ++v) acc[v] = fma(wk, (double)x[k][v], acc[v]);
                    }
            }
        }
        c_l = c_n;
        w_l = w_n;
        p_l = p_n;
    }
    }

    float o[V];
    if (MODE == 0) {
#pragma unroll
        for (int v = 0; v < V; ++v) o[v] = act_apply(ACT, acc[v] + b, capf); // compile-time: exp() costs registers
    } else {
#pragma unroll
        for (int v = 0; v < V; ++v) o[v] = act_backprop(act, acc[v], xp[v], capf);
    }
    if (live) stv<V>(out + (size_t)m.row * ld + s, o);
    if (MODE == 0 && flags != nullptr && live) { // other rows store the same 1: no ordering needed
#pragma unroll
        for (int v = 0; v < V; ++v)
            if (o[v] != 0.0f) flags[s + v] = 1;
    }
}

// The grid is sized to what the chip holds at once and every workgroup walks
// "virtual blocks" blockIdx.x, blockIdx.x + gridDim.x, ...: a wavefront that
// handles one short row and exits costs more to dispatch than to run.
// gridDim.x is a multiple of 8, so a workgroup keeps its XCD's tiles.
// ACT: the activation of the forward epilogue, fixed at compile time (the sigmoid's exp() would
// otherwise set the register count, and with it the occupancy, of the ReLU kernels too); the
// backward epilogue reads a.act.
template <int V, int MODE, int U, bool TILES_INNER, int ACT>
__global__ void __launch_bounds__(BLOCK_THREADS) k_spmm(const SpmmArgs a)
{
    const int lane = threadIdx.x & 63;
    const unsigned wave = threadIdx.x >> 6;
    unsigned n_tiles = a.n_tiles, n_vblocks = a.n_vblocks;
    if (a.n_live) { // only the batch tiles that hold live columns
        n_tiles = min(n_tiles, ((unsigned)*a.n_live + 64u * V - 1u) / (64u * V));
        n_vblocks = n_tiles * a.n_rg;
    }
    if constexpr (TILES_INNER) {
        // a few batch tiles shared by all XCDs: a wavefront keeps its row and walks the tiles, so the row's
        // task record and entries are fetched once, and the whole chip gathers from one tile's slab at a time
        for (unsigned rg = blockIdx.x; rg < a.n_rg; rg += gridDim.x) {
            const int r = __builtin_amdgcn_readfirstlane((int)(rg * WAVES_PER_BLOCK + wave));
            if (r >= a.n_rows) continue;
            const RowMeta m = load_meta<MODE>(a.sched, a.idx, a.vals, a.perm, r, lane);
            for (unsigned tile = 0; tile < n_tiles; ++tile)
                spmm_row<V, MODE, U, ACT>(m, a.idx, a.vals, a.perm, a.in, a.in_bytes, a.out, a.aux, a.B, a.cap, a.act,
                                          tile + a.tile_base, lane, a.flags);
        }
        return;
    }
    for (unsigned vb = blockIdx.x; vb < n_vblocks; vb += gridDim.x) {
        unsigned tile, rg;
        map_block(vb, n_tiles, a.n_rg, tile, rg);
        const int r = __builtin_amdgcn_readfirstlane((int)(rg * WAVES_PER_BLOCK + wave));
        if (r >= a.n_rows) continue;
        const RowMeta m = load_meta<MODE>(a.sched, a.idx, a.vals, a.perm, r, lane);
        spmm_row<V, MODE, U, ACT>(m, a.idx, a.vals, a.perm, a.in, a.in_bytes, a.out, a.aux, a.B, a.cap, a.act, tile + a.tile_base, lane, a.flags);
    }
}

// ---------------------------------------------------------------------------
// K1p / K2p: the same product for wide layers with short rows, swept in column panels.
//
// A 64-sample tile of a wide layer's operand (n_cols x 256 B) is several times the 4 MiB L2 of an
// XCD, and a row's 32 or so gathers land all over it, so without further care most gathers miss
// L2.  Here a wavefront owns R rows and keeps their entries (entry k of a row in lane k) and their
// R accumulators in registers; it walks the operand in panels of panel_cols rows, and in each
// panel every one of its rows consumes the entries whose column falls into the panel.  Column
// indices ascend inside a row, so each row still adds its terms in storage order: the sums are the
// same as in k_spmm.  The wavefronts resident on an XCD advance through the panels at about the
// same pace (nothing enforces it: a wavefront that runs ahead or behind only loses L2 hits), so
// an XCD's L2 holds one panel at a time and pulls each operand row in once per launch.
// Rows must have at most 64 entries (checked by the host); one sample per lane.
// ---------------------------------------------------------------------------
#define PANEL_SLOTS 8 // gathers of one row segment that are in flight together; longer segments go round again

// Requests the operand rows of entries k .. min(k + PANEL_SLOTS, ke) - 1 of a row (wave-uniform branches).
__device__ __forceinline__ void panel_issue(__amdgpu_buffer_rsrc_t rin, unsigned so, unsigned ldb, int c_l, int k, int ke,
                                            float (&x)[PANEL_SLOTS])
{
#define PANEL_G(j) x[j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rin, (int)so, (int)((unsigned)__builtin_amdgcn_readlane(c_l, k + j) * ldb), 0))
    const int n = ke - k;
    if (n > 0) { PANEL_G(0);
    if (n > 1) { PANEL_G(1);
    if (n > 2) { PANEL_G(2);
    if (n > 3) { PANEL_G(3);
    if (n > 4) { PANEL_G(4);
    if (n > 5) { PANEL_G(5);
    if (n > 6) { PANEL_G(6);
    if (n > 7) { PANEL_G(7); } } } } } } } }
#undef PANEL_G
}

// Adds the terms of the same entries, in storage order.
__device__ __forceinline__ void panel_consume(float w_l, int k, int ke, const float (&x)[PANEL_SLOTS], double &acc)
{
#define PANEL_F(j) acc = fma((double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_l), k + j)), (double)x[j], acc)
    const int n = ke - k;
    if (n > 0) { PANEL_F(0);
    if (n > 1) { PANEL_F(1);
    if (n > 2) { PANEL_F(2);
    if (n > 3) { PANEL_F(3);
    if (n > 4) { PANEL_F(4);
    if (n > 5) { PANEL_F(5);
    if (n > 6) { PANEL_F(6);
    if (n > 7) { PANEL_F(7); } } } } } } } }
#undef PANEL_F
}

template <int R, int MODE, int ACT>
__global__ void __launch_bounds__(BLOCK_THREADS) k_spmm_panel(const SpmmArgs a, int n_cols, int panel_cols)
{
    const int lane = threadIdx.x & 63;
    const unsigned wave = threadIdx.x >> 6;
    const int B = a.B;
    const size_t ld = (size_t)B;
    const unsigned ldb = 4u * (unsigned)B;
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    for (unsigned vb = blockIdx.x; vb < a.n_vblocks; vb += gridDim.x) {
        unsigned tile, rg;
        map_block(vb, a.n_tiles, a.n_rg, tile, rg); // n_rg counts groups of WAVES_PER_BLOCK * R rows here
        const int r0 = __builtin_amdgcn_readfirstlane((int)((rg * WAVES_PER_BLOCK + wave) * R));
        if (r0 >= a.n_rows) continue;
        const int s_own = (int)(tile + a.tile_base) * 64 + lane;
        const bool live = s_own < B;
        const int s = live ? s_own : 0;
        const unsigned so = 4u * (unsigned)s;

        int row[R], c_l[R], kcur[R];
        float w_l[R], xp[R];
        double acc[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            row[r] = -1;
            c_l[r] = 0x7fffffff; // past every panel: lanes beyond the end of a row, and rows beyond the last
            w_l[r] = 0.0f;
            xp[r] = 0.0f;
            acc[r] = 0.0;
            kcur[r] = 0;
            if (r0 + r < a.n_rows) {
                const int4 t = a.sched[r0 + r];
                row[r] = t.x;
                if (t.y + lane < t.z) {
                    c_l[r] = a.idx[t.y + lane];
                    w_l[r] = MODE == 1 ? a.vals[a.perm[t.y + lane]] : a.vals[t.y + lane];
                }
                if (MODE == 1) xp[r] = a.aux[(size_t)t.x * ld + s];
            }
        }
        for (int pe = panel_cols;; pe += panel_cols) {
            const bool last = pe >= n_cols;
            const int bound = last ? 0x7fffffff : pe;
#pragma unroll
            for (int r = 0; r < R; r += 2) {
                // columns ascend inside a row: the entries below the bound are a prefix of the lanes
                const int ke0 = (int)__popcll(__ballot(c_l[r] < bound));
                int k0 = kcur[r];
                kcur[r] = ke0;
                float x0[PANEL_SLOTS];
                panel_issue(rin, so, ldb, c_l[r], k0, ke0, x0);
                if constexpr (R > 1) {
                    const int ke1 = (int)__popcll(__ballot(c_l[r + 1] < bound));
                    int k1 = kcur[r + 1];
                    kcur[r + 1] = ke1;
                    float x1[PANEL_SLOTS];
                    panel_issue(rin, so, ldb, c_l[r + 1], k1, ke1, x1);
                    panel_consume(w_l[r], k0, ke0, x0, acc[r]);
                    panel_consume(w_l[r + 1], k1, ke1, x1, acc[r + 1]);
                    for (k1 += PANEL_SLOTS; k1 < ke1; k1 += PANEL_SLOTS) {
                        panel_issue(rin, so, ldb, c_l[r + 1], k1, ke1, x1);
                        panel_consume(w_l[r + 1], k1, ke1, x1, acc[r + 1]);
                    }
                } else {
                    panel_consume(w_l[r], k0, ke0, x0, acc[r]);
                }
                for (k0 += PANEL_SLOTS; k0 < ke0; k0 += PANEL_SLOTS) {
                    panel_issue(rin, so, ldb, c_l[r], k0, ke0, x0);
                    panel_consume(w_l[r], k0, ke0, x0, acc[r]);
                }
            }
            if (last) break;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (row[r] < 0) continue;
            float o;
            if (MODE == 0) o = act_apply(ACT, acc[r] + (a.aux ? (double)a.aux[row[r]] : 0.0), a.cap);
            else o = act_backprop(a.act, acc[r], xp[r], a.cap);
            if (live) a.out[(size_t)row[r] * ld + s] = o;
        }
    }
}

// ---------------------------------------------------------------------------
// K1f: the whole feed-forward sweep (Eq. 3 for l = 1..L) in one launch, for nets whose widest layer
// fits in LDS.  The batch vectors are independent (they are the columns of X, Section 5.1), so a
// workgroup takes LDS_T of them through all layers by itself: their activations live in two LDS
// buffers ([neuron][LDS_T] floats, one read and one written per layer, a workgroup barrier between
// layers), and only W is streamed, from its lane-major copy: lane r of a wavefront walks row r of a
// block of 64 rows, one coalesced 8-byte load per entry, one 16-byte LDS read for the LDS_T
// activations the entry points at.  Every lane adds its row's terms in storage order in fp64: the
// same sums as k_spmm.  Slots past the end of a row that is shorter than its block hold weight 0
// and add an exact zero.
// ---------------------------------------------------------------------------
#define LDS_WAVES 16 // wavefronts per workgroup: one workgroup per CU
#define LDS_U 8      // entries in flight per lane
#define LDS_BLOCKS (LDS_MAX_N / 64 / LDS_WAVES) // blocks of 64 rows a wavefront has per layer, at most
template <int ACT>
__global__ void __launch_bounds__(64 * LDS_WAVES)
k_fwd_lds(const LayerDev *__restrict__ layers, int n_layers, const float *__restrict__ X0, float *__restrict__ XL,
          int B, int buf_floats, float cap, int vec_io)
{
    extern __shared__ __attribute__((aligned(16))) float lds_act[];
    float *in = lds_act, *out = lds_act + buf_floats;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int s0 = blockIdx.x * LDS_T;
    const bool full = s0 + LDS_T <= B && vec_io; // all LDS_T samples exist and rows of X are 16-byte aligned

    // X_0: the workgroup's LDS_T columns (zeros past the end of the batch)
    const int n0 = layers[0].n_in;
    for (int i = tid; i < n0; i += 64 * LDS_WAVES) {
        const float *src = X0 + (size_t)i * B + s0;
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (full) {
            v = *reinterpret_cast<const float4 *>(src);
        } else {
            if (s0 + 0 < B) v.x = src[0];
            if (s0 + 1 < B) v.y = src[1];
            if (s0 + 2 < B) v.z = src[2];
            if (s0 + 3 < B) v.w = src[3];
        }
        *reinterpret_cast<float4 *>(in + LDS_T * i) = v;
    }
    __syncthreads();

    // A wavefront takes the blocks wave, wave + LDS_WAVES, ... of every layer: at most LDS_BLOCKS of them.  Where
    // they lie, their rows and biases do not depend on the activations, so all of it is requested at once, a layer
    // ahead: a layer then starts with its first entries, not with a chain of dependent loads per block.
    int off_n[LDS_BLOCKS], end_n[LDS_BLOCKS], row_n[LDS_BLOCKS];
    float bias_n[LDS_BLOCKS];
    auto request_meta = [&](int l) {
        const LayerDev &L = layers[l];
#pragma unroll
        for (int j = 0; j < LDS_BLOCKS; ++j) {
            const int b = wave + LDS_WAVES * j;
            off_n[j] = end_n[j] = 0;
            row_n[j] = -1;
            bias_n[j] = 0.0f;
            if (b < L.n_blocks) {
                off_n[j] = L.lm_off[b];
                end_n[j] = L.lm_off[b + 1];
                row_n[j] = L.lm_row[b * 64 + lane];
                bias_n[j] = L.lm_bias[b * 64 + lane];
            }
        }
    };
    request_meta(0);
    for (int l = 0; l < n_layers; ++l) {
        const LayerDev &L = layers[l];
        const bool last = l == n_layers - 1;
        int off_c[LDS_BLOCKS], end_c[LDS_BLOCKS], row_c[LDS_BLOCKS];
        float bias_c[LDS_BLOCKS];
#pragma unroll
        for (int j = 0; j < LDS_BLOCKS; ++j) { off_c[j] = off_n[j]; end_c[j] = end_n[j]; row_c[j] = row_n[j]; bias_c[j] = bias_n[j]; }
        if (!last) request_meta(l + 1);
#pragma unroll
        for (int j = 0; j < LDS_BLOCKS; ++j) {
            if (wave + LDS_WAVES * j >= L.n_blocks) break;
            const int off = off_c[j];
            const int K = (end_c[j] - off) >> 6; // entries of the block's longest row
            const int row = row_c[j];
            const float bias = bias_c[j];
            const int2 *__restrict__ e = L.lm + off + lane;
            double acc[LDS_T];
#pragma unroll
            for (int t = 0; t < LDS_T; ++t) acc[t] = 0.0;
            for (int k0 = 0; k0 < K; k0 += LDS_U) {
                int2 ent[LDS_U];
                float4 x[LDS_U];
                if (k0 + LDS_U <= K) {
#pragma unroll
                    for (int u = 0; u < LDS_U; ++u) ent[u] = e[(k0 + u) * 64];
                } else { // the block's last entries: the slots past them add an exact zero
#pragma unroll
                    for (int u = 0; u < LDS_U; ++u) ent[u] = k0 + u < K ? e[(k0 + u) * 64] : make_int2(0, 0);
                }
#pragma unroll
                for (int u = 0; u < LDS_U; ++u) x[u] = *reinterpret_cast<const float4 *>(in + LDS_T * ent[u].x);
#pragma unroll
                for (int u = 0; u < LDS_U; ++u) {
                    const double w = (double)__int_as_float(ent[u].y);
                    acc[0] = fma(w, (double)x[u].x, acc[0]);
                    acc[1] = fma(w, (double)x[u].y, acc[1]);
                    acc[2] = fma(w, (double)x[u].z, acc[2]);
                    acc[3] = fma(w, (double)x[u].w, acc[3]);
                }
            }
            if (row >= 0) {
                const double bd = (double)bias;
                const float4 o = make_float4(act_apply(ACT, acc[0] + bd, cap), act_apply(ACT, acc[1] + bd, cap),
                                             act_apply(ACT, acc[2] + bd, cap), act_apply(ACT, acc[3] + bd, cap));
                if (!last) {
                    *reinterpret_cast<float4 *>(out + LDS_T * row) = o;
                } else {
                    float *dst = XL + (size_t)row * B + s0;
                    if (full) {
                        *reinterpret_cast<float4 *>(dst) = o;
                    } else {
                        if (s0 + 0 < B) dst[0] = o.x;
                        if (s0 + 1 < B) dst[1] = o.y;
                        if (s0 + 2 < B) dst[2] = o.z;
                        if (s0 + 3 < B) dst[3] = o.w;
                    }
                }
            }
        }
        __syncthreads(); // the layer is complete before anyone reads it, and read before it is overwritten
        float *t = in; in = out; out = t;
    }
}

// Rewrites the weights and biases of a layer's lane-major copy from the CSR values and the bias array
// (after sdnn_set_weights).
__global__ void __launch_bounds__(64) k_lm_refresh(const LayerDev *__restrict__ layer)
{
    const LayerDev &L = *layer;
    const int b = blockIdx.x, lane = threadIdx.x;
    const int row = L.lm_row[b * 64 + lane];
    if (row < 0) return;
    const int off = L.lm_off[b];
    const int beg = L.row_ptr[row], len = L.row_ptr[row + 1] - beg;
    for (int k = 0; k < len; ++k) L.lm[off + 64 * k + lane].y = __float_as_int(L.vals[beg + k]);
    L.lm_bias[b * 64 + lane] = L.bias[row];
}

// ---------------------------------------------------------------------------
// K2 + K4a: back-propagation through W_l fused with the gradient of W_l's stored entries, for
// launches of at most 64 samples (one sample per lane).  The wavefront of row i of W_l^T gathers
// Delta_l(j, :) for every stored entry (j, i) anyway and holds X_{l-1}(i, :), the two operands of
// Eq. 4 for exactly that entry.  The gathered rows are parked in LDS, 16 entries at a time
// ([entry][sample], padded), and then lane (e, q) sums entry e over quarter q of the samples in fp64;
// the four quarters are added and lane e stores g(j, i) = sum_s Delta_l(j, s) X_{l-1}(i, s) at the
// entry's place in the transposed index.  Every stored entry lies in exactly one row of W_l^T, so the
// launch writes the whole gradient array; nothing is accumulated in memory.  The values are read from
// their copy in the same order (vals_t): the sweep streams through index, values and gradient, and
// only the rows of Delta_l are gathered.  This removes the update's own gather pass over X_{l-1}.
// ---------------------------------------------------------------------------
#define TR_CHUNK 16384 // entries of the CSR array that one workgroup of k_spread_vals fills from LDS (64 KiB)
#define TR_THREADS 512
#define TR_SPAN 8192   // consecutive entries of the transposed index that one workgroup of k_apply takes (32 KiB of LDS)
#define GRAD_LD 68 // floats per parked entry: 64 samples + pad (rows stay 16-byte aligned, banks spread)
#define GRAD_GE 16 // entries parked at a time: 4.6 KB of LDS per wavefront, which keeps 8 wavefronts per SIMD
template <int U>
__device__ __forceinline__ void spmm_row_grad(RowMeta m, const SpmmArgs &a, unsigned tile, int lane,
                                              float *__restrict__ dt, float *__restrict__ xt)
{
    const int B = a.B;
    const int s_own = (int)tile * 64 + lane;
    const bool live = s_own < B;
    const int s = live ? s_own : 0;
    const size_t ld = (size_t)B;
    const unsigned so = 4u * (unsigned)s;
    const unsigned ldb = 4u * (unsigned)B;
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);

    const float xp = a.aux[(size_t)m.row * ld + s]; // X_{l-1}(i, s): mask operand and gradient operand
    xt[lane] = live ? xp : 0.0f;                    // samples outside the launch add nothing to the gradient

    double acc = 0.0;
    int c_l = m.c_l, p_l;
    float w_l = m.w_l;
    const int e = lane & (GRAD_GE - 1), q = lane / GRAD_GE; // reducer of entry e over quarter q of the samples
    for (int base = m.beg; base < m.end; base += 64) {
        const int n = min(64, m.end - base);
        // a.vals is the copy of the values in the order of the transposed index: read like a forward row
        if (base != m.beg) load_chunk<0>(a.idx, a.vals, nullptr, base, m.end, lane, c_l, w_l, p_l);
        for (int g0 = 0; g0 < n; g0 += GRAD_GE) { // GRAD_GE entries are parked at a time
            const int ng = min(GRAD_GE, n - g0);
            for (int g = 0; g < ng; g += U) {
                float x[U];
                if (g + U <= ng) {
#pragma unroll
                    for (int k = 0; k < U; ++k) {
                        const int c = __builtin_amdgcn_readlane(c_l, g0 + g + k);
                        x[k] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rin, (int)so, (int)((unsigned)c * ldb), 0));
                    }
#pragma unroll
                    for (int k = 0; k < U; ++k) {
                        const double wk = (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_l), g0 + g + k));
                        acc = fma(wk, (double)x[k], acc);
                        dt[(g + k) * GRAD_LD + lane] = x[k];
                    }
                } else { // ragged end of the row: same order, every entry guarded (wave-uniform branches)
#pragma unroll
                    for (int k = 0; k < U; ++k)
                        if (g + k < ng) {
                            const int c = __builtin_amdgcn_readlane(c_l, g0 + g + k);
                            x[k] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rin, (int)so, (int)((unsigned)c * ldb), 0));
                        }
#pragma unroll
                    for (int k = 0; k < U; ++k)
                        if (g + k < ng) {
                            const double wk = (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_l), g0 + g + k));
                            acc = fma(wk, (double)x[k], acc);
                            dt[(g + k) * GRAD_LD + lane] = x[k];
                        }
                }
            }
            // entry e of this group, samples 16q .. 16q+15: the lanes now read what other lanes of the
            // wavefront have parked
            wave_lds_sync();
            double sum = 0.0;
            if (e < ng) {
                const float4 *dp = reinterpret_cast<const float4 *>(dt + e * GRAD_LD + 16 * q);
                const float4 *xq = reinterpret_cast<const float4 *>(xt + 16 * q);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float4 d4 = dp[t], x4 = xq[t];
                    sum = fma((double)d4.x, (double)x4.x, sum);
                    sum = fma((double)d4.y, (double)x4.y, sum);
                    sum = fma((double)d4.z, (double)x4.z, sum);
                    sum = fma((double)d4.w, (double)x4.w, sum);
                }
            }
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 32);
            if (q == 0 && e < ng) a.g_part[base + g0 + e] = (float)sum; // the entry's place in the transposed index
            wave_lds_sync(); // the next group's rows are parked over the ones just read
        }
    }
    if (a.store_out && live) a.out[(size_t)m.row * ld + s] = act_backprop(a.act, acc, xp, a.cap);
}
template <int U>
__global__ void __launch_bounds__(BLOCK_THREADS) k_bwd_grad(const SpmmArgs a)
{
    __shared__ __attribute__((aligned(16))) float dt[WAVES_PER_BLOCK][GRAD_GE * GRAD_LD];
    __shared__ __attribute__((aligned(16))) float xt[WAVES_PER_BLOCK][64];
    const int lane = threadIdx.x & 63;
    const unsigned wave = threadIdx.x >> 6;
    for (unsigned vb = blockIdx.x; vb < a.n_vblocks; vb += gridDim.x) {
        unsigned tile, rg;
        map_block(vb, a.n_tiles, a.n_rg, tile, rg);
        const int r = __builtin_amdgcn_readfirstlane((int)(rg * WAVES_PER_BLOCK + wave));
        if (r >= a.n_rows) continue;
        const RowMeta m = load_meta<0>(a.sched, a.idx, a.vals, nullptr, r, lane);
        spmm_row_grad<U>(m, a, tile + a.tile_base, lane, dt[wave], xt[wave]);
    }
}

// The same sweep for long rows and a batch of up to 256 samples in one launch: four samples per lane, as in the long-row
// product kernels, a gathered row of Delta_l being 1 KiB.  Eight entries are parked at a time ([entry][256 samples],
// padded: 8.3 KB per wavefront, four wavefronts per SIMD); lane (e, q) sums entry e over the q-th eighth of the
// samples (32 of them), three shuffles add the eighths.
#define GRAD4_LD 260 // floats per parked entry: 256 samples + pad
#define GRAD4_GE 8
template <int U>
__global__ void __launch_bounds__(BLOCK_THREADS) k_bwd_grad4(const SpmmArgs a)
{
    __shared__ __attribute__((aligned(16))) float dt_all[WAVES_PER_BLOCK][GRAD4_GE * GRAD4_LD];
    __shared__ __attribute__((aligned(16))) float xt_all[WAVES_PER_BLOCK][256];
    const int lane = threadIdx.x & 63;
    const unsigned wave = threadIdx.x >> 6;
    float *__restrict__ dt = dt_all[wave];
    float *__restrict__ xt = xt_all[wave];
    const int B = a.B; // a multiple of 4, at most 256: one tile
    const size_t ld = (size_t)B;
    const unsigned ldb = 4u * (unsigned)B;
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const int s_own = 4 * lane;
    const bool live = s_own < B;
    const int s = live ? s_own : 0;
    const unsigned so = 4u * (unsigned)s;
    const int e = lane & (GRAD4_GE - 1), q = lane / GRAD4_GE; // reducer of entry e over samples 32 q .. 32 q + 31
    for (unsigned vb = blockIdx.x; vb < a.n_vblocks; vb += gridDim.x) {
        const int r = __builtin_amdgcn_readfirstlane((int)(vb * WAVES_PER_BLOCK + wave));
        if (r >= a.n_rows) continue;
        // the row's task record and its entries are the same for all lanes and do not change inside the kernel: they
        // are read through the scalar cache into scalar registers, eight columns and eight weights a group ahead
        typedef int i32x4s __attribute__((ext_vector_type(4)));
        typedef int i32x8 __attribute__((ext_vector_type(8)));
        typedef float f32x8 __attribute__((ext_vector_type(8)));
        const i32x4s task = ((const i32x4s __attribute__((address_space(4))) *)a.sched)[r];
        RowMeta m;
        m.row = task.x; m.beg = task.y; m.end = task.z;
        const int __attribute__((address_space(4))) *sidx = (const int __attribute__((address_space(4))) *)a.idx;
        const float __attribute__((address_space(4))) *svals = (const float __attribute__((address_space(4))) *)a.vals;
        float xp[4];
        ldv<4>(a.aux + (size_t)m.row * ld + s, xp); // X_{l-1}(i, s ..): mask operand and gradient operand
        wave_lds_sync();                            // the previous row's X values have been read
        {
            float4 xz = make_float4(0.0f, 0.0f, 0.0f, 0.0f); // samples outside the batch add nothing to the gradient
            if (live) xz = make_float4(xp[0], xp[1], xp[2], xp[3]);
            *reinterpret_cast<float4 *>(xt + 4 * lane) = xz;
        }
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
        static_assert(U == GRAD4_GE, "a parked group is one batch of gathers");
        // reduces the ng parked entries over the samples and stores their gradients at entries g .. g + ng - 1
        auto reduce_parked = [&](int g, int ng) {
            wave_lds_sync(); // the lanes now read what other lanes of the wavefront have parked
            double sum = 0.0;
            if (e < ng) {
                const float4 *dp = reinterpret_cast<const float4 *>(dt + e * GRAD4_LD + 32 * q);
                const float4 *xq = reinterpret_cast<const float4 *>(xt + 32 * q);
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const float4 d4 = dp[t], x4 = xq[t];
                    sum = fma((double)d4.x, (double)x4.x, sum);
                    sum = fma((double)d4.y, (double)x4.y, sum);
                    sum = fma((double)d4.z, (double)x4.z, sum);
                    sum = fma((double)d4.w, (double)x4.w, sum);
                }
            }
            sum += __shfl_xor(sum, 8);
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 32);
            if (q == 0 && e < ng) a.g_part[g + e] = (float)sum; // the entry's place in the transposed index
            wave_lds_sync(); // the next group's rows are parked over the ones just read
        };
        int g = m.beg;
        i32x8 c, cn;
        f32x8 w, wn;
        if (g + 8 <= m.end) {
#pragma unroll
            for (int k = 0; k < 8; ++k) { c[k] = sidx[g + k]; w[k] = svals[g + k]; }
        }
        for (; g + 8 <= m.end; g += 8) {
            if (g + 16 <= m.end) {
#pragma unroll
                for (int k = 0; k < 8; ++k) { cn[k] = sidx[g + 8 + k]; wn[k] = svals[g + 8 + k]; }
            }
            float x[8][4];
#pragma unroll
            for (int k = 0; k < 8; ++k) gatherv<4>(rin, so, (unsigned)c[k] * ldb, x[k]);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                float wf = w[k];
                asm volatile("" : "+s"(wf)); // converted when it is used, not while the gathers are in flight
                const double wk = (double)wf;
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[v] = fma(wk, (double)x[k][v], acc[v]);
                *reinterpret_cast<float4 *>(dt + k * GRAD4_LD + 4 * lane) = make_float4(x[k][0], x[k][1], x[k][2], x[k][3]);
            }
            reduce_parked(g, 8);
            c = cn;
            w = wn;
        }
        if (g < m.end) { // the row's last entries, fewer than eight: same order, every entry guarded (wave-uniform)
            const int n = m.end - g;
            float x[8][4];
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (k < n) gatherv<4>(rin, so, (unsigned)sidx[g + k] * ldb, x[k]);
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (k < n) {
                    const double wk = (double)svals[g + k];
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[v] = fma(wk, (double)x[k][v], acc[v]);
                    *reinterpret_cast<float4 *>(dt + k * GRAD4_LD + 4 * lane) = make_float4(x[k][0], x[k][1], x[k][2], x[k][3]);
                }
            reduce_parked(g, n);
        }
        if (a.store_out && live) {
            float o[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) o[v] = act_backprop(a.act, acc[v], xp[v], a.cap);
            stv<4>(a.out + (size_t)m.row * ld + s, o);
        }
    }
}

// ---------------------------------------------------------------------------
// K3: output delta (Eq. 6):  D = dLoss * [0 < X_L < cap]
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_output_delta(const float *__restrict__ dloss,
                                                      const float *__restrict__ xl,
                                                      float *__restrict__ d, size_t n, float cap, int act)
{
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n;
         e += (size_t)gridDim.x * blockDim.x)
        d[e] = act_backprop(act, (double)dloss[e], xl[e], cap);
}

// ---------------------------------------------------------------------------
// One sample per step (B = 1, the paper's own training experiments: one input
// vector per SGD step, Section 6.1).  Lanes over samples would idle 63 of 64
// lanes, so there are three products of their own, all taking each row's sum in
// storage order (same result as everywhere else):
//   k_spmv_stage  wide layers with short rows: lanes over a contiguous stretch of entries,
//                 products parked in LDS, then a lane per row adds them up;
//   k_spmv_wave   narrow layers, or long rows up to 16384 rows: a wavefront per row;
//   k_spmv        the rest (wide layers with long rows): a lane per row.
// ---------------------------------------------------------------------------
template <int MODE>
__global__ void __launch_bounds__(256) k_spmv(const SpmmArgs a)
{
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= a.n_rows) return;
    const int beg = a.row_ptr[row], end = a.row_ptr[row + 1];
    double acc = 0.0;
    constexpr int U = 16; // entries requested together; the additions stay in storage order
    for (int p0 = beg; p0 < end; p0 += U) {
        int c[U];
        float w[U], x[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int p = min(p0 + k, end - 1);
            c[k] = a.idx[p];
            w[k] = MODE == 1 ? a.vals[a.perm[p]] : a.vals[p];
        }
#pragma unroll
        for (int k = 0; k < U; ++k) x[k] = a.in[c[k]];
#pragma unroll
        for (int k = 0; k < U; ++k)
            if (p0 + k < end) acc = fma((double)w[k], (double)x[k], acc);
    }
    if (MODE == 0) a.out[row] = act_apply(a.act, acc + (a.aux ? (double)a.aux[row] : 0.0), a.cap);
    else a.out[row] = act_backprop(a.act, acc, a.aux[row], a.cap);
}

// Same product for narrow layers, where a lane per row leaves most of the chip idle: a wavefront
// per row.  The row's entries and the activations they point at are fetched by two wave-wide loads
// (entry k in lane k); the sum itself is still taken in storage order, every lane redoing it from
// the broadcast operands.
template <int MODE>
__global__ void __launch_bounds__(BLOCK_THREADS) k_spmv_wave(const SpmmArgs a)
{
    const int lane = threadIdx.x & 63;
    const int row = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6)));
    if (row >= a.n_rows) return;
    const int beg = a.row_ptr[row], end = a.row_ptr[row + 1];
    double acc = 0.0;
    for (int base = beg; base < end; base += 64) {
        const int n = min(64, end - base);
        float w_l = 0.0f, x_l = 0.0f;
        if (lane < n) {
            const int p = base + lane;
            w_l = MODE == 1 ? a.vals[a.perm[p]] : a.vals[p];
            x_l = a.in[a.idx[p]];
        }
        for (int k = 0; k < n; ++k) {
            const double wk = (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_l), k));
            const double xk = (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(x_l), k));
            acc = fma(wk, xk, acc);
        }
    }
    if (lane == 0) {
        if (MODE == 0) a.out[row] = act_apply(a.act, acc + (a.aux ? (double)a.aux[row] : 0.0), a.cap);
        else a.out[row] = act_backprop(a.act, acc, a.aux[row], a.cap);
    }
}

// Wide layers at B = 1: a 64-lane workgroup owns R consecutive rows, whose entries are one contiguous
// stretch of the index arrays.  All lanes walk that stretch together (coalesced index and value
// loads, one gathered activation per entry) and park the products w*x, which are exact in fp64, in
// LDS; then lane r adds the products of row r in storage order, the same sum as everywhere else.
// The stretch is taken in segments of SPMV_STAGE entries, so rows of any length work.
#define SPMV_STAGE 1024
#define SPMV_STAGE_MIN_ROWS 2048 // below this a wavefront per row is as fast (measured)
template <int MODE, int J>
__global__ void __launch_bounds__(64) k_spmv_stage(const SpmmArgs a, int R)
{
    __shared__ double prod[SPMV_STAGE + SPMV_STAGE / 32]; // one pad per 32 entries: lanes that start 32 apart hit different banks
    const int lane = threadIdx.x;
    const int r0 = blockIdx.x * R;
    const int nr = min(R, a.n_rows - r0); // >= 1 by the grid size
    const int row = r0 + lane;
    int p = 0, end = 0;
    if (lane < nr) { p = a.row_ptr[row]; end = a.row_ptr[row + 1]; }
    const int e0 = a.row_ptr[r0], e1 = a.row_ptr[r0 + nr];
    double acc = 0.0;
    for (int sb = e0; sb < e1; sb += SPMV_STAGE) {
        const int se = min(sb + SPMV_STAGE, e1);
        for (int j0 = 0; j0 * 64 < se - sb; j0 += J) {
            int c[J];
            float w[J], x[J];
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const int e = sb + (j0 + j) * 64 + lane;
                c[j] = -1;
                if (e < se) {
                    c[j] = a.idx[e];
                    w[j] = MODE == 1 ? a.vals[a.perm[e]] : a.vals[e];
                }
            }
#pragma unroll
            for (int j = 0; j < J; ++j)
                if (c[j] >= 0) x[j] = a.in[c[j]];
#pragma unroll
            for (int j = 0; j < J; ++j)
                if (c[j] >= 0) {
                    const int q = (j0 + j) * 64 + lane;
                    prod[q + (q >> 5)] = (double)w[j] * (double)x[j];
                }
        }
        __syncthreads();
        const int pe = min(end, se); // my row's entries inside this segment are [p, pe)
        if (p < pe) {
            for (; p < pe; p += 4) { // four parked products requested together, added one after the other
                double v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int q = min(p + k, pe - 1) - sb;
                    v[k] = prod[q + (q >> 5)];
                }
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (p + k < pe) acc += v[k];
            }
            p = pe;
        }
        __syncthreads();
    }
    if (lane < nr) {
        if (MODE == 0) a.out[row] = act_apply(a.act, acc + (a.aux ? (double)a.aux[row] : 0.0), a.cap);
        else a.out[row] = act_backprop(a.act, acc, a.aux[row], a.cap);
    }
}

// The same kernel as the backward sweep of a one-sample step that also forms the gradient (B = 1 has no sum over
// samples: g(j, i) = Delta_l(j) X_{l-1}(i), one product per entry).  The rows are those of W_l^T, the values are read
// from their copy in that order, and the lane that holds entry (j, i) for the product also has Delta_l(j); it fetches
// X_{l-1}(i) through t_col and stores the gradient at the entry's place in the transposed index, in a stream.
template <int J>
__global__ void __launch_bounds__(64) k_spmv_stage_grad(const SpmmArgs a, int R, const int32_t *__restrict__ t_col)
{
    __shared__ double prod[SPMV_STAGE + SPMV_STAGE / 32];
    const int lane = threadIdx.x;
    const int r0 = blockIdx.x * R;
    const int nr = min(R, a.n_rows - r0); // >= 1 by the grid size
    const int row = r0 + lane;
    int p = 0, end = 0;
    if (lane < nr) { p = a.row_ptr[row]; end = a.row_ptr[row + 1]; }
    const int e0 = a.row_ptr[r0], e1 = a.row_ptr[r0 + nr];
    double acc = 0.0;
    for (int sb = e0; sb < e1; sb += SPMV_STAGE) {
        const int se = min(sb + SPMV_STAGE, e1);
        for (int j0 = 0; j0 * 64 < se - sb; j0 += J) {
            int c[J], ti[J];
            float w[J], x[J], xi[J];
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const int e = sb + (j0 + j) * 64 + lane;
                c[j] = -1;
                if (e < se) {
                    c[j] = a.idx[e];
                    w[j] = a.vals[e];
                    ti[j] = t_col[e];
                }
            }
#pragma unroll
            for (int j = 0; j < J; ++j)
                if (c[j] >= 0) {
                    x[j] = a.in[c[j]];
                    xi[j] = a.aux[ti[j]];
                }
#pragma unroll
            for (int j = 0; j < J; ++j)
                if (c[j] >= 0) {
                    const int q = (j0 + j) * 64 + lane;
                    prod[q + (q >> 5)] = (double)w[j] * (double)x[j];
                    a.g_part[sb + q] = (float)((double)x[j] * (double)xi[j]);
                }
        }
        if (!a.store_out) continue; // first layer: only the gradient (uniform for the workgroup)
        __syncthreads();
        const int pe = min(end, se); // my row's entries inside this segment are [p, pe)
        if (p < pe) {
            for (; p < pe; p += 4) { // four parked products requested together, added one after the other
                double v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int q = min(p + k, pe - 1) - sb;
                    v[k] = prod[q + (q >> 5)];
                }
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (p + k < pe) acc += v[k];
            }
            p = pe;
        }
        __syncthreads();
    }
    if (a.store_out && lane < nr) a.out[row] = act_backprop(a.act, acc, a.aux[row], a.cap);
}

// Update for B = 1: no sum over samples, so the lanes take the entries of the rows:
// vals[p] -= lr * delta(row) * x(col[p]).  A wavefront holds 64 >> lpr_log2 rows of 1 << lpr_log2
// lanes each (chosen from the mean row length, so that short rows do not idle half the lanes);
// the first lane of a row does its bias.
__global__ void __launch_bounds__(BLOCK_THREADS)
k_update_b1(const LayerDev *__restrict__ layers, int layer0, int lpr_log2, float lr, int update_bias, int emit,
            float *__restrict__ g_out, float *__restrict__ gb_out)
{
    const LayerDev &L = layers[layer0 + blockIdx.y];
    const int lane = threadIdx.x & 63;
    const int lpr = 1 << lpr_log2;
    const int l = lane & (lpr - 1);
    const int row = ((blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6)) << (6 - lpr_log2)) + (lane >> lpr_log2);
    if (row >= L.n_out) return;
    const int beg = L.row_ptr[row], end = L.row_ptr[row + 1];
    const float d = L.D[row];
    const double dlr = (double)lr;
    for (int p = beg + l; p < end; p += lpr) {
        const float g = (float)((double)d * (double)L.X_prev[L.col_idx[p]]);
        if (emit) { if (g_out) g_out[p] = g; }
        else L.vals[p] = (float)((double)L.vals[p] - dlr * (double)g);
    }
    if (l == 0) {
        if (emit) { if (gb_out) gb_out[row] = d; }
        else if (update_bias) L.bias[row] = (float)((double)L.bias[row] - dlr * (double)d);
    }
}

// ---------------------------------------------------------------------------
// K4: gradient on the stored pattern (Eq. 4) fused with the update (Eq. 5)
//   blockIdx.y = layer; a wavefront takes rows_per_wave rows one after the other (several when rows
//   are short: fewer, longer-lived wavefronts).  Lane = 16*eg + sg: edge group
//   eg handles 8 consecutive entries of a 32-entry chunk of the row, sample
//   lane sg handles samples sg*V + 16*V*t.  A 16-lane butterfly then leaves
//   the 8 sums of an edge group in 8 different lanes, which write them back.
//   emit == 0: vals -= lr*g, bias -= lr*gb (if update_bias)
//   emit == 1: g_out / gb_out receive the gradient of the single layer
// ---------------------------------------------------------------------------
// HOLD > 0: the batch has at most 16 * V * HOLD samples and the lane keeps its share of the row of Delta in
// registers for the whole row (long rows: otherwise it is read again for every 32-entry chunk).
template <int V, int HOLD>
__global__ void __launch_bounds__(64 * UPD_WAVES)
k_update(const LayerDev *__restrict__ layers, int layer0, int n_layers, int interleave, int rows_per_wave, int B,
         float lr, int update_bias, int emit, float *__restrict__ g_out, float *__restrict__ gb_out)
{
    // interleaved: grid = (8 * row groups, groups of 8 layers), blockIdx.x % 8 is both the XCD and the
    // layer inside the group, so all gathers of one layer go through one L2, which then fetches that
    // layer's activations once instead of once per XCD.  Plain (few layers: the XCDs would not all
    // have one): grid = (row groups, layers).
    const int layer_rel = interleave ? (int)(8u * blockIdx.y + (blockIdx.x & 7u)) : (int)blockIdx.y;
    if (layer_rel >= n_layers) return;
    const LayerDev &L = layers[layer0 + layer_rel];
    const int lane = threadIdx.x & 63;
    const unsigned rgi = interleave ? (blockIdx.x >> 3) : blockIdx.x;
    const int r0 = __builtin_amdgcn_readfirstlane((int)((rgi * UPD_WAVES + (threadIdx.x >> 6)) * rows_per_wave));
  for (int r = r0; r < min(r0 + rows_per_wave, L.n_out); ++r) {
    const int4 task = L.sched[r];
    const int row = task.x, beg = task.y, end = task.z;
    const size_t ld = (size_t)B;
    const float *drow = L.D + (size_t)row * ld;
    const float *xp = L.X_prev;
    const double dlr = (double)lr;

    // bias gradient: sum of the row of Delta over the samples
    if (emit ? gb_out != nullptr : update_bias != 0) {
        double sum = 0.0;
        for (int s = lane * V; s < B; s += 64 * V) {
            float d[V];
            ldv<V>(drow + s, d);
#pragma unroll
            for (int v = 0; v < V; ++v) sum += (double)d[v];
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
        if (lane == 0) {
            const float gb = (float)sum;
            if (emit) gb_out[row] = gb;
            else L.bias[row] = (float)((double)L.bias[row] - dlr * (double)gb);
        }
    }
    if (emit && g_out == nullptr) continue;

    const int sg = lane & 15, eg = lane >> 4;
    float dh[HOLD > 0 ? HOLD : 1][V];
    if constexpr (HOLD > 0) {
#pragma unroll
        for (int t = 0; t < HOLD; ++t) {
            const int s = sg * V + 16 * V * t;
#pragma unroll
            for (int v = 0; v < V; ++v) dh[t][v] = 0.0f;
            if (s < B) ldv<V>(drow + s, dh[t]);
        }
    }
    for (int base = beg; base < end; base += 32) {
        const int p0 = base + eg * 8;
        size_t coff[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int p = p0 + k;
            coff[k] = (size_t)(p < end ? L.col_idx[p] : L.col_idx[beg]) * ld;
        }
        // the weight this lane will rewrite at the end of the chunk, requested now
        const int kw = ((lane >> 3) & 1) * 4 + ((lane >> 2) & 1) * 2 + ((lane >> 1) & 1);
        const bool writer = (lane & 1) == 0 && p0 + kw < end;
        float w_old = 0.0f;
        if (writer && !emit) w_old = L.vals[p0 + kw];
        double a[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) a[k] = 0.0;
        auto pass = [&](int s, const float (&df)[V]) { // the chunk's 8 entries against V samples of this lane
            float x[8][V];
#pragma unroll
            for (int k = 0; k < 8; ++k) ldv<V>(xp + coff[k] + s, x[k]);
            double d[V];
#pragma unroll
            for (int v = 0; v < V; ++v) d[v] = (double)df[v];
#pragma unroll
            for (int k = 0; k < 8; ++k)
#pragma unroll
                for (int v = 0; v < V; ++v) a[k] = fma(d[v], (double)x[k][v], a[k]);
        };
        if constexpr (HOLD > 0) {
#pragma unroll
            for (int t = 0; t < HOLD; ++t) {
                const int s = sg * V + 16 * V * t;
                if (s < B) pass(s, dh[t]);
            }
        } else {
            for (int s = sg * V; s < B; s += 16 * V) {
                float df[V];
                ldv<V>(drow + s, df);
                pass(s, df);
            }
        }
        // 16-lane transpose-reduce: 8 values/lane -> 1 value/lane (register indices are compile-time)
        {
            const bool up8 = (lane & 8) != 0, up4 = (lane & 4) != 0, up2 = (lane & 2) != 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double send = up8 ? a[j] : a[j + 4];
                const double keep = up8 ? a[j + 4] : a[j];
                a[j] = keep + __shfl_xor(send, 8);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const double send = up4 ? a[j] : a[j + 2];
                const double keep = up4 ? a[j + 2] : a[j];
                a[j] = keep + __shfl_xor(send, 4);
            }
            {
                const double send = up2 ? a[0] : a[1];
                const double keep = up2 ? a[1] : a[0];
                a[0] = keep + __shfl_xor(send, 2);
            }
        }
        a[0] += __shfl_xor(a[0], 1);
        if (writer) {
            const float g = (float)a[0];
            if (emit) g_out[p0 + kw] = g;
            else L.vals[p0 + kw] = (float)((double)w_old - dlr * (double)g);
        }
    }
  }
}

// ---------------------------------------------------------------------------
// K4b: the descent step when the fused backward kernels have left the gradient of the stored
// entries in G[0] (and G[1], the other half of the batch): vals -= lr * g, a flat streaming pass
// over the entries of every layer (grid = (chunks of entries, layers)); k_apply_bias forms the bias
// gradient sum_s Delta(row, s).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(TR_THREADS) k_apply(const LayerDev *__restrict__ layers, int n_parts, float lr)
{
    // The gradient and one copy of the values are in the order of the transposed index: this pass is a stream over
    // both.  The new values also go to `mid`, grouped by the chunk of the CSR array they belong to: a workgroup
    // takes a span of TR_SPAN consecutive entries, puts the new values into the order they have in mid in LDS
    // (mid_slot) and stores them from there, neighbouring threads into neighbouring places of a run (mid_dst).
    // k_spread_vals then fills the CSR copy, which the forward pass reads, chunk by chunk.  The workgroups of
    // one XCD take neighbouring spans, so that the pieces of a cache line of mid meet in one L2.
    __shared__ __attribute__((aligned(16))) float stage[TR_SPAN];
    const LayerDev &L = layers[blockIdx.y];
    const int nb = (int)gridDim.x; // a multiple of 8
    const int vb = ((int)blockIdx.x & 7) * (nb >> 3) + ((int)blockIdx.x >> 3);
    const int64_t q0 = (int64_t)vb * TR_SPAN;
    if (q0 >= L.nnz) return;
    const int cnt = (int)min((int64_t)TR_SPAN, (int64_t)L.nnz - q0), cnt4 = cnt >> 2;
    const double dlr = (double)lr;
    const float *__restrict__ g0 = L.G[0] + q0;
    const float *__restrict__ g1 = L.G[1] + q0;
    const uint16_t *__restrict__ slot = L.mid_slot + q0;
    const int32_t *__restrict__ dst = L.mid_dst + q0;
    float *__restrict__ vals_t = L.vals_t + q0;
    float *__restrict__ mid = L.mid;
    const int tid = (int)threadIdx.x;
#define APPLY_ONE(G0, G1, W) (float)((double)(W) - dlr * (double)(float)(n_parts == 2 ? (double)(G0) + (double)(G1) : (double)(G0)))
    for (int k = tid; k < cnt4; k += TR_THREADS) { // q0 is a multiple of 4 and the arrays are 16-byte aligned
        const float4 a = reinterpret_cast<const float4 *>(g0)[k];
        float4 b = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (n_parts == 2) b = reinterpret_cast<const float4 *>(g1)[k];
        float4 w = reinterpret_cast<const float4 *>(vals_t)[k];
        const ushort4 o = reinterpret_cast<const ushort4 *>(slot)[k];
        w.x = APPLY_ONE(a.x, b.x, w.x); w.y = APPLY_ONE(a.y, b.y, w.y);
        w.z = APPLY_ONE(a.z, b.z, w.z); w.w = APPLY_ONE(a.w, b.w, w.w);
        reinterpret_cast<float4 *>(vals_t)[k] = w;
        stage[o.x] = w.x; stage[o.y] = w.y; stage[o.z] = w.z; stage[o.w] = w.w;
    }
    if (tid < (cnt & 3)) {
        const int k = 4 * cnt4 + tid;
        const float w = APPLY_ONE(g0[k], n_parts == 2 ? g1[k] : 0.0f, vals_t[k]);
        vals_t[k] = w;
        stage[slot[k]] = w;
    }
#undef APPLY_ONE
    __syncthreads();
    for (int k = tid; k < cnt; k += TR_THREADS) mid[dst[k]] = stage[k];
}

// Chunk c of the CSR values from entries [c TR_CHUNK, (c+1) TR_CHUNK) of mid: placed in LDS by mid_loc, then
// written out in order.  grid = (chunks, layers).
__global__ void __launch_bounds__(TR_THREADS) k_spread_vals(const LayerDev *__restrict__ layers)
{
    __shared__ __attribute__((aligned(16))) float chunk[TR_CHUNK];
    const LayerDev &L = layers[blockIdx.y];
    const int64_t c0 = (int64_t)blockIdx.x * TR_CHUNK;
    if (c0 >= L.nnz) return;
    const int cnt = (int)min((int64_t)TR_CHUNK, (int64_t)L.nnz - c0), cnt4 = cnt >> 2;
    const float *__restrict__ mid = L.mid + c0;
    const uint16_t *__restrict__ loc = L.mid_loc + c0;
    float *__restrict__ vals = L.vals + c0;
    for (int k = (int)threadIdx.x; k < cnt4; k += TR_THREADS) { // c0 is a multiple of 4 and the arrays are 16-byte aligned
        const float4 v = reinterpret_cast<const float4 *>(mid)[k];
        const ushort4 o = reinterpret_cast<const ushort4 *>(loc)[k];
        chunk[o.x] = v.x; chunk[o.y] = v.y; chunk[o.z] = v.z; chunk[o.w] = v.w;
    }
    if ((int)threadIdx.x < (cnt & 3)) chunk[loc[4 * cnt4 + (int)threadIdx.x]] = mid[4 * cnt4 + (int)threadIdx.x];
    __syncthreads();
    for (int k = (int)threadIdx.x; k < cnt4; k += TR_THREADS)
        reinterpret_cast<float4 *>(vals)[k] = reinterpret_cast<const float4 *>(chunk)[k];
    if ((int)threadIdx.x < (cnt & 3)) vals[4 * cnt4 + (int)threadIdx.x] = chunk[4 * cnt4 + (int)threadIdx.x];
}

// The gradient that k_apply applies, for inspection, in CSR order: out[t_perm[q]] = g0[q] (+ g1[q]), the same
// rounding as in k_apply.
__global__ void __launch_bounds__(256) k_sum_parts(const float *__restrict__ g0, const float *__restrict__ g1,
                                                   const int32_t *__restrict__ perm, float *__restrict__ out, int n)
{
    for (int q = blockIdx.x * 256 + threadIdx.x; q < n; q += gridDim.x * 256) {
        double g = (double)g0[q];
        if (g1) g += (double)g1[q];
        out[perm[q]] = (float)g;
    }
}

// vals_t[q] = vals[t_perm[q]]: brings the transposed-order copy of the values up to date after the CSR copy
// was changed by something other than k_apply (sdnn_set_weights, the separate update kernel).
__global__ void __launch_bounds__(256) k_refresh_vals_t(const LayerDev *__restrict__ layers)
{
    const LayerDev &L = layers[blockIdx.y];
    if (!L.vals_t) return;
    for (int q = blockIdx.x * 256 + threadIdx.x; q < L.nnz; q += gridDim.x * 256) L.vals_t[q] = L.vals[L.t_perm[q]];
}

// 16 lanes per row, four rows per wavefront at a time, 16 consecutive rows per wavefront.
// gb_out == NULL: bias -= lr * gb; otherwise the bias gradient of the one layer is stored there instead.
__global__ void __launch_bounds__(BLOCK_THREADS) k_apply_bias(const LayerDev *__restrict__ layers, int B, float lr,
                                                              float *__restrict__ gb_out)
{
    const LayerDev &L = layers[blockIdx.y];
    const int lane = threadIdx.x & 63, l = lane & 15;
    const int row0 = (blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6)) * 16 + (lane >> 4);
    const bool vec = (B & 3) == 0; // rows of Delta are 16-byte aligned
    for (int k = 0; k < 4; ++k) {
        const int row = row0 + 4 * k;
        double sum = 0.0;
        if (row < L.n_out) {
            const float *drow = L.D + (size_t)row * B;
            if (vec) {
                for (int s = 4 * l; s < B; s += 64) {
                    const float4 d = *reinterpret_cast<const float4 *>(drow + s);
                    sum += (double)d.x; sum += (double)d.y; sum += (double)d.z; sum += (double)d.w;
                }
            } else {
                for (int s = l; s < B; s += 16) sum += (double)drow[s];
            }
        }
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
        if (l == 0 && row < L.n_out) {
            if (gb_out) gb_out[row] = (float)sum;
            else L.bias[row] = (float)((double)L.bias[row] - (double)lr * (double)(float)sum);
        }
    }
}

// ---------------------------------------------------------------------------
// Inference that drops dead samples.  With ReLU and biases <= 0 a sample whose activations are all
// zero after some layer stays all zero in every later layer, so its column need not be computed any
// more.  Every few layers the live columns of the activation block are moved to the front (in
// order) and the product kernels are told how many columns still matter; the count lives in device
// memory, so nothing waits for the host.  map[c] remembers which sample sits in column c.
// ---------------------------------------------------------------------------
#define LIVE_ROWS 64  // rows per workgroup of the final scatter
#define PACK_ROWS 16  // rows per workgroup of k_pack
#define PACK_MAX_B 8192

// map = identity, both flag arrays cleared, n_live = B
__global__ void __launch_bounds__(256) k_skip_init(int32_t *__restrict__ map, int32_t *__restrict__ flags0,
                                                   int32_t *__restrict__ flags1, int32_t *__restrict__ n_live, int B)
{
    for (int s = blockIdx.x * 256 + threadIdx.x; s < B; s += gridDim.x * 256) { map[s] = s; flags0[s] = 0; flags1[s] = 0; }
    if (blockIdx.x == 0 && threadIdx.x == 0) *n_live = B;
}

// Packs the flagged columns of X [n_rows][ld] to the front, in order and in place.  Every workgroup
// derives the new position of each column from the flags by itself (a prefix sum over at most
// PACK_MAX_B flags) and then moves its own rows: a wavefront walks a row in chunks of 64 columns,
// front to back; a chunk is read completely before any of it is written and lands at or before its
// own place, so nothing unread is overwritten.  Workgroup 0 also writes the state of the next
// round, which nobody reads during this launch: the sample ids of the packed columns, the new
// count, and a cleared flag array.  If no column died nothing moves.
__global__ void __launch_bounds__(256) k_pack(float *X, int n_rows, int ld, const int32_t *__restrict__ flags,
                                              const int32_t *__restrict__ n_live_in, const int32_t *__restrict__ map_in,
                                              int32_t *__restrict__ n_live_out, int32_t *__restrict__ map_out,
                                              int32_t *__restrict__ flags_next)
{
    __shared__ int32_t newpos[PACK_MAX_B];
    __shared__ int wave_sum[4];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int nl = *n_live_in;
    const int per = (nl + 255) / 256;
    const int c0 = min(t * per, nl), c1 = min(c0 + per, nl);
    int cnt = 0;
    for (int c = c0; c < c1; ++c) cnt += flags[c] != 0;
    int x = cnt; // inclusive prefix sum over the 256 threads
    for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(x, off);
        if (lane >= off) x += y;
    }
    if (lane == 63) wave_sum[wave] = x;
    __syncthreads();
    int before = 0, nl_new = 0;
    for (int w = 0; w < 4; ++w) {
        const int v = wave_sum[w];
        if (w < wave) before += v;
        nl_new += v;
    }
    int pos = before + x - cnt;
    for (int c = c0; c < c1; ++c) newpos[c] = flags[c] != 0 ? pos++ : -1;
    __syncthreads();
    if (blockIdx.x == 0) {
        for (int c = c0; c < c1; ++c)
            if (newpos[c] >= 0) map_out[newpos[c]] = map_in[c];
        for (int c = t; c < ld; c += 256) flags_next[c] = 0;
        if (t == 0) *n_live_out = nl_new;
    }
    if (nl_new == nl) return;
    const int r_end = min(n_rows, ((int)blockIdx.x + 1) * PACK_ROWS);
    for (int r = (int)blockIdx.x * PACK_ROWS + wave; r < r_end; r += 4) {
        float *row = X + (size_t)r * ld;
        for (int cb = 0; cb < nl; cb += 64) {
            const int c = cb + lane;
            int np = -1;
            float v = 0.0f;
            if (c < nl) { np = newpos[c]; v = row[c]; }
            wave_lds_sync(); // every lane has read its column before any lane overwrites one
            if (np >= 0) row[np] = v;
        }
    }
}

// XL[r][map[c]] = X[r][c] for c < n_live (the other columns of XL were zeroed before)
__global__ void __launch_bounds__(256) k_scatter_cols(const float *__restrict__ X, float *__restrict__ XL, int n,
                                                      int ld, const int32_t *__restrict__ map,
                                                      const int32_t *__restrict__ n_live)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= *n_live) return;
    const int dc = map[c];
    const int r0 = blockIdx.y * LIVE_ROWS, r1 = min(n, r0 + LIVE_ROWS);
    for (int r = r0; r < r1; ++r) XL[(size_t)r * ld + dc] = X[(size_t)r * ld + c];
}

__global__ void __launch_bounds__(256) k_fill_f32(float *__restrict__ p, size_t n, float v)
{
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (size_t)gridDim.x * blockDim.x) p[e] = v;
}

// ---------------------------------------------------------------------------
// Measurement aid: the ceiling of the gather path.  Every wavefront streams per_wave gathers of
// random rows (64 * V floats, one V-float piece per lane, through the same buffer loads as the
// product kernels) from a table, 8 in flight, and does nothing else with them.  What this reaches for
// a table of a given size is what the product kernels can reach at best for an operand of that size.
// ---------------------------------------------------------------------------
template <int V>
__global__ void __launch_bounds__(BLOCK_THREADS) k_gather_probe(const int32_t *__restrict__ idx, const float *__restrict__ table,
                                                                size_t table_bytes, int per_wave, float *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    const int32_t *my = idx + wave * (size_t)per_wave;
    const __amdgpu_buffer_rsrc_t r = make_rsrc(table, table_bytes);
    const unsigned so = 4u * (unsigned)(lane * V), ldb = 4u * 64u * V;
    float sum = 0.0f;
    for (int base = 0; base < per_wave; base += 64) {
        const int c_l = base + lane < per_wave ? my[base + lane] : 0;
        const int n = min(64, per_wave - base);
        for (int g = 0; g + 8 <= n; g += 8) {
            float x[8][V];
#pragma unroll
            for (int k = 0; k < 8; ++k) gatherv<V>(r, so, (unsigned)__builtin_amdgcn_readlane(c_l, g + k) * ldb, x[k]);
#pragma unroll
            for (int k = 0; k < 8; ++k)
#pragma unroll
                for (int v = 0; v < V; ++v) sum += x[k][v];
        }
    }
    out[wave * 64 + lane] = sum;
}

// ---------------------------------------------------------------------------
// loss-gradient helpers
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_mse_dloss(const float *__restrict__ x,
                                                   const float *__restrict__ y,
                                                   float *__restrict__ out, size_t n, double B)
{
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n;
         e += (size_t)gridDim.x * blockDim.x)
        out[e] = (float)(((double)x[e] - (double)y[e]) / B);
}

__global__ void __launch_bounds__(256) k_softmax_ce_dloss(const float *__restrict__ x,
                                                          const int32_t *__restrict__ labels,
                                                          float *__restrict__ out, int n, int B,
                                                          int n_classes)
{
    const int first = n - n_classes;
    // zero the rows that carry no logit
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < (size_t)first * B;
         e += (size_t)gridDim.x * blockDim.x)
        out[e] = 0.0f;
    for (int s = blockIdx.x * blockDim.x + threadIdx.x; s < B; s += gridDim.x * blockDim.x) {
        double m = -INFINITY;
        for (int c = 0; c < n_classes; ++c) m = fmax(m, (double)x[(size_t)(first + c) * B + s]);
        double z = 0.0;
        for (int c = 0; c < n_classes; ++c) z += exp((double)x[(size_t)(first + c) * B + s] - m);
        const int lab = labels[s];
        for (int c = 0; c < n_classes; ++c) {
            double pr = exp((double)x[(size_t)(first + c) * B + s] - m) / z;
            if (c == lab) pr -= 1.0;
            out[(size_t)(first + c) * B + s] = (float)(pr / (double)B);
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
enum { ST_IDLE = 0, ST_FORWARD = 1, ST_BACKWARD = 2 };

struct sdnn_net {
    int32_t n_layers = 0;
    sdnn_config cfg{};
    std::vector<LayerDev> layers; // host copy of the descriptors (device pointers inside)
    LayerDev *d_layers = nullptr; // device copy
    float *d_x0 = nullptr;        // training: X_0 [n_in(1)][max_batch]
    float *d_ping = nullptr, *d_pong = nullptr; // inference: two activation buffers
    int n_cu = 0;                 // compute units of the device
    int occ_spmm[2][3][2][2] = {}; // resident workgroups per CU of k_spmm<V,MODE,U,tiles inner>, U = 8, 16
    int occ_grad = 0;             // the same for k_bwd_grad
    int grad_v = 1;               // samples per lane of the fused sweep of the last backward pass (1: k_bwd_grad, 4: k_bwd_grad4,
                                  // 0: one sample per step, k_spmv_stage_grad)
    int occ_panel[2][4] = {};     // the same for k_spmm_panel<R,MODE>, R = 1, 2, 4, 8
    std::vector<int32_t> max_len[2]; // per layer: longest row of W (0) and of W^T (1)
    std::vector<char> clustered[2];  // per layer: reorder_rows found clusters in W (0), in W^T (1)
    bool lds_ready = false;          // every layer has its lane-major copy (k_fwd_lds can run)
    bool lds_attr_set = false;       // the kernels' dynamic LDS limit has been raised
    int grad_parts = 0;           // > 0: the last backward pass left the entries' gradient in G[0..grad_parts)
    bool vals_t_stale = false;    // the CSR values were changed by something that does not maintain vals_t
    hipStream_t side = nullptr;   // second stream for the other half of the batch (small layers)
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    int32_t *d_flags[2] = {nullptr, nullptr}, *d_map[2] = {nullptr, nullptr}, *d_n_live[2] = {nullptr, nullptr}; // inference: dead-sample skipping, two rounds' state
    bool bias_nonpos = false;     // every bias of layers 2..L is <= 0 (as uploaded; cleared when a bias is replaced)
    int state = ST_IDLE;
    int32_t B = 0;
    int32_t max_n = 0;
    char err[512] = "";
};

static int fail(sdnn_net *net, int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (net) snprintf(net->err, sizeof net->err, "%s", buf);
    sdnn_set_global_error("%s", buf);
    return code;
}

#define HIP_TRY(net, expr)                                                                   \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess)                                                                \
            return fail(net, SDNN_EHIP, "%s: %s", #expr, hipGetErrorString(e_));              \
    } while (0)

extern "C" const char *sdnn_last_error(const sdnn_net *net)
{
    return net ? net->err : sdnn_global_error();
}

// Fixed staging array of sdnn_forward_noalloc (the variant of sdnn_forward for callers that cannot
// allocate): it lives in the library's device image, one copy per GPU, until the process ends.
static __device__ __align__(256) unsigned char scratch[SDNN_NOALLOC_SCRATCH_BYTES];
#define MAX_DEVICES 64
static void *g_scratch_ptr[MAX_DEVICES]; // device address of `scratch` on each GPU, looked up once per GPU
static std::mutex g_scratch_mutex;

// Address of this GPU's copy of the array (the array's name is only a host-side handle of the
// symbol: kernels and copies must be given the address that the runtime reports).
static int scratch_address(sdnn_net *net, void **ptr)
{
    int devid = -1;
    HIP_TRY(net, hipGetDevice(&devid));
    if (devid < 0 || devid >= MAX_DEVICES) return fail(net, SDNN_EINVAL, "device %d: more GPUs than supported", devid);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[devid]) {
        void *p = nullptr;
        HIP_TRY(net, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(net, SDNN_EHIP, "hipGetSymbolAddress returned NULL");
        g_scratch_ptr[devid] = p;
    }
    *ptr = g_scratch_ptr[devid];
    return SDNN_OK;
}

static inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

// Workspace plan: offsets of every array, in one pass (also used to size it).
struct Plan {
    struct PerLayer {
        size_t row_ptr, col_idx, vals, bias, t_row_ptr, t_row_idx, t_perm, sched, t_sched, X, D, G[2], vals_t, mid_slot, mid_dst, mid_loc, mid, t_col;
        size_t lm, lm_off, lm_row, lm_bias, lm_entries, lm_blocks;
    };
    std::vector<PerLayer> pl;
    size_t table = 0, x0 = 0, ping = 0, pong = 0, flags[2] = {0, 0}, map[2] = {0, 0}, n_live[2] = {0, 0}, total = 0;
};

static int check_config(const sdnn_layer *layers, int32_t n_layers, const sdnn_config *cfg)
{
    if (!layers || !cfg) return fail(nullptr, SDNN_EINVAL, "layers or cfg is NULL");
    if (n_layers < 1) return fail(nullptr, SDNN_EINVAL, "n_layers must be >= 1");
    if (cfg->max_batch < 1) return fail(nullptr, SDNN_EINVAL, "max_batch must be >= 1");
    if (cfg->activation != SDNN_ACT_RELU_CAP && cfg->activation != SDNN_ACT_SIGMOID)
        return fail(nullptr, SDNN_EINVAL, "unknown activation %d", cfg->activation);
    if (cfg->activation == SDNN_ACT_RELU_CAP && !(cfg->act_cap > 0.0f))
        return fail(nullptr, SDNN_EINVAL, "act_cap must be > 0 (or +inf)");
    if (cfg->fuse_gradient < SDNN_FUSE_OFF || cfg->fuse_gradient > SDNN_FUSE_ON)
        return fail(nullptr, SDNN_EINVAL, "unknown fuse_gradient %d", cfg->fuse_gradient);
    if (cfg->panel_cols < SDNN_PANEL_OFF) return fail(nullptr, SDNN_EINVAL, "panel_cols must be >= -1");
    if (cfg->reorder_rows != 0 && cfg->reorder_rows != 1) return fail(nullptr, SDNN_EINVAL, "reorder_rows must be 0 or 1");
    if (cfg->lds_forward < SDNN_LDS_OFF || cfg->lds_forward > SDNN_LDS_ON)
        return fail(nullptr, SDNN_EINVAL, "unknown lds_forward %d", cfg->lds_forward);
    for (int32_t l = 0; l < n_layers; ++l) {
        const sdnn_layer &y = layers[l];
        if (y.n_out < 0 || y.n_in < 0 || !y.row_ptr)
            return fail(nullptr, SDNN_EINVAL, "layer %d: bad size or NULL row_ptr", l + 1);
        if (l > 0 && y.n_in != layers[l - 1].n_out)
            return fail(nullptr, SDNN_EINVAL, "layer %d: n_in %d != n_out %d of layer %d", l + 1,
                        y.n_in, layers[l - 1].n_out, l);
        if ((int64_t)y.n_out * cfg->max_batch >= ((int64_t)1 << 40))
            return fail(nullptr, SDNN_EINVAL, "layer %d: activation block too large", l + 1);
    }
    return SDNN_OK;
}

// The fused backward + gradient kernels pay from layers of 4096 rows on, whose launches are bound by gather
// throughput; below that, where the latency of a launch binds, the separate update is faster (measured step
// time against the separate kernels: 1024 rows +10 %, 4096 rows -5 %, 16384 rows -20 %, 65536 rows -30 %).
// Nets with long rows take the fused sweep for batches of up to 256 samples (grad_fusable): AUTO sets it up for
// them when max_batch allows it.
static bool grad_buffers_wanted(const sdnn_layer *layers, int32_t n_layers, const sdnn_config *cfg)
{
    if (!cfg->training || cfg->fuse_gradient == SDNN_FUSE_OFF) return false;
    if (cfg->fuse_gradient == SDNN_FUSE_ON) return true;
    int64_t rows = 0, nnz = 0;
    for (int32_t l = 0; l < n_layers; ++l) {
        rows += layers[l].n_out;
        nnz += layers[l].row_ptr ? layers[l].row_ptr[layers[l].n_out] : 0;
    }
    // long rows: fused where the whole batch fits one launch of the four-samples-per-lane sweep
    return rows >= (int64_t)4096 * n_layers && (nnz < 128 * rows || cfg->max_batch <= 256);
}

// The LDS-resident forward (k_fwd_lds) carries LDS_T samples through all layers with two activation
// buffers of (widest layer) x LDS_T floats in LDS; it is set up for inference nets whose widest
// layer fits.
static bool lds_forward_wanted(const sdnn_layer *layers, int32_t n_layers, const sdnn_config *cfg)
{
    if (cfg->training || cfg->lds_forward == SDNN_LDS_OFF) return false;
    for (int32_t l = 0; l < n_layers; ++l)
        if (layers[l].n_out > LDS_MAX_N || layers[l].n_in > LDS_MAX_N) return false;
    return true;
}

// Row lengths, longest first: block b of the lane-major copy is as deep as its first row.
static size_t lm_padded_entries(const sdnn_layer &y, std::vector<int32_t> &lens)
{
    lens.resize((size_t)y.n_out);
    for (int32_t r = 0; r < y.n_out; ++r) lens[r] = y.row_ptr[r + 1] - y.row_ptr[r];
    std::sort(lens.begin(), lens.end(), std::greater<int32_t>());
    size_t total = 0;
    for (int32_t r = 0; r < y.n_out; r += 64) total += 64 * (size_t)lens[r];
    return total;
}

static void make_plan(const sdnn_layer *layers, int32_t n_layers, const sdnn_config *cfg, Plan &pl)
{
    // Arrays of 1 MiB and more start on a multiple of their size rounded down to a power of two, at most
    // 2 MiB: where the gathered activation blocks lie relative to the 2 MiB granules of the address
    // translation is worth 9 % of the inference time on 16384-neuron layers (measured: 452 vs 414 ms).
    // The arrays are laid out kind by kind, all layers of a kind in a row, so that arrays of equal
    // size follow each other without padding.
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t align = 256;
        if (bytes >= ((size_t)1 << 20)) {
            align = (size_t)1 << 20;
            while (align < ((size_t)2 << 20) && 2 * align <= bytes) align *= 2;
        }
        off = (off + align - 1) & ~(align - 1);
        const size_t o = off;
        off += align_up(bytes);
        return o;
    };
    pl.pl.resize(n_layers);
    pl.table = take(sizeof(LayerDev) * (size_t)n_layers);
    const size_t mb = (size_t)cfg->max_batch;
    const bool gw = grad_buffers_wanted(layers, n_layers, cfg);
    const bool lm = lds_forward_wanted(layers, n_layers, cfg);
    size_t max_n = 0;
    std::vector<size_t> nnz((size_t)n_layers);
    for (int32_t l = 0; l < n_layers; ++l) {
        const sdnn_layer &y = layers[l];
        nnz[l] = (size_t)y.row_ptr[y.n_out];
        Plan::PerLayer &q = pl.pl[l];
        q.X = q.D = q.G[0] = q.G[1] = q.vals_t = q.mid_slot = q.mid_dst = q.mid_loc = q.mid = q.t_col = 0;
        q.lm = q.lm_off = q.lm_row = q.lm_bias = q.lm_entries = q.lm_blocks = 0;
        if (lm) {
            std::vector<int32_t> lens;
            q.lm_entries = lm_padded_entries(y, lens);
            q.lm_blocks = ((size_t)y.n_out + 63) / 64;
        }
        max_n = std::max(max_n, (size_t)std::max(y.n_out, y.n_in));
    }
#define PLAN_KIND(field, bytes_expr)                                   \
    for (int32_t l = 0; l < n_layers; ++l) {                           \
        const sdnn_layer &y = layers[l];                               \
        Plan::PerLayer &q = pl.pl[l];                                  \
        (void)y;                                                       \
        q.field = take(bytes_expr);                                    \
    }
    PLAN_KIND(row_ptr, 4 * ((size_t)y.n_out + 1))
    PLAN_KIND(col_idx, 4 * nnz[l])
    PLAN_KIND(vals, 4 * nnz[l])
    PLAN_KIND(bias, 4 * (size_t)y.n_out)
    PLAN_KIND(t_row_ptr, 4 * ((size_t)y.n_in + 1))
    PLAN_KIND(t_row_idx, 4 * nnz[l])
    PLAN_KIND(t_perm, 4 * nnz[l])
    PLAN_KIND(sched, 16 * (size_t)y.n_out)
    PLAN_KIND(t_sched, 16 * (size_t)y.n_in)
    if (lm) {
        PLAN_KIND(lm, 8 * q.lm_entries)
        PLAN_KIND(lm_off, 4 * (q.lm_blocks + 1))
        PLAN_KIND(lm_row, 4 * 64 * q.lm_blocks)
        PLAN_KIND(lm_bias, 4 * 64 * q.lm_blocks)
    }
    if (cfg->training) {
        pl.x0 = take(4 * (size_t)layers[0].n_in * mb);
        PLAN_KIND(X, 4 * (size_t)y.n_out * mb)
        PLAN_KIND(D, 4 * (size_t)y.n_out * mb)
        if (gw) {
            PLAN_KIND(G[0], 4 * nnz[l])
            PLAN_KIND(G[1], 4 * nnz[l])
            PLAN_KIND(vals_t, 4 * nnz[l])
            PLAN_KIND(mid_slot, 2 * nnz[l])
            PLAN_KIND(mid_dst, 4 * nnz[l])
            PLAN_KIND(mid_loc, 2 * nnz[l])
            PLAN_KIND(mid, 4 * nnz[l])
            if (cfg->max_batch == 1) PLAN_KIND(t_col, 4 * nnz[l])
        }
    } else {
        pl.ping = take(4 * max_n * mb);
        pl.pong = take(4 * max_n * mb);
        for (int k = 0; k < 2; ++k) {
            pl.flags[k] = take(4 * mb);
            pl.map[k] = take(4 * mb);
            pl.n_live[k] = take(4);
        }
    }
#undef PLAN_KIND
    pl.total = off;
}

extern "C" int sdnn_workspace_bytes(const sdnn_layer *layers, int32_t n_layers,
                                    const sdnn_config *cfg, size_t *bytes)
{
    if (!bytes) return fail(nullptr, SDNN_EINVAL, "bytes is NULL");
    int rc = check_config(layers, n_layers, cfg);
    if (rc) return rc;
    for (int32_t l = 0; l < n_layers; ++l)
        if (layers[l].row_ptr[0] != 0 || layers[l].row_ptr[layers[l].n_out] < 0)
            return fail(nullptr, SDNN_EINVAL, "layer %d: malformed row_ptr", l + 1);
    Plan pl;
    try {
        make_plan(layers, n_layers, cfg, pl);
    } catch (...) {
        return fail(nullptr, SDNN_ENOMEM, "host allocation failed");
    }
    *bytes = pl.total;
    return SDNN_OK;
}

extern "C" int sdnn_create(const sdnn_layer *layers, int32_t n_layers, const sdnn_config *cfg,
                           void *d_workspace, size_t workspace_bytes, void *stream_,
                           sdnn_net **out)
{
    if (!out) return fail(nullptr, SDNN_EINVAL, "out is NULL");
    *out = nullptr;
    int rc = check_config(layers, n_layers, cfg);
    if (rc) return rc;
    for (int32_t l = 0; l < n_layers; ++l) {
        rc = sdnn_check_csr(layers[l].n_out, layers[l].n_in, layers[l].row_ptr, layers[l].col_idx);
        if (rc) return fail(nullptr, rc, "layer %d: %s", l + 1, sdnn_global_error());
        if (layers[l].row_ptr[layers[l].n_out] > 0 && !layers[l].values)
            return fail(nullptr, SDNN_EINVAL, "layer %d: values is NULL", l + 1);
    }
    if (!d_workspace) return fail(nullptr, SDNN_EINVAL, "d_workspace is NULL");
    if (((uintptr_t)d_workspace & 255) != 0)
        return fail(nullptr, SDNN_EINVAL, "d_workspace must be 256-byte aligned");
    Plan pl;
    try {
        make_plan(layers, n_layers, cfg, pl);
    } catch (...) {
        return fail(nullptr, SDNN_ENOMEM, "host allocation failed");
    }
    if (workspace_bytes < pl.total)
        return fail(nullptr, SDNN_ENOMEM, "workspace too small: %zu < %zu", workspace_bytes, pl.total);

    hipStream_t stream = (hipStream_t)stream_;
    sdnn_net *net = new (std::nothrow) sdnn_net;
    if (!net) return fail(nullptr, SDNN_ENOMEM, "host allocation failed");
    net->n_layers = n_layers;
    net->cfg = *cfg;
    try {
        net->layers.resize(n_layers);
        net->max_len[0].resize(n_layers);
        net->max_len[1].resize(n_layers);
        net->clustered[0].resize(n_layers);
        net->clustered[1].resize(n_layers);
    } catch (...) {
        delete net;
        return fail(nullptr, SDNN_ENOMEM, "host allocation failed");
    }
    char *base = (char *)d_workspace;
    auto fail_free = [&](int code) { sdnn_destroy(net); return code; };

    // Host part of the setup (transposed index, row schedules): independent per layer, so a group of layers is
    // prepared by one host thread each, then uploaded with one synchronisation for the whole group.
    struct HostIdx {
        std::vector<int32_t> t_row_ptr, t_row_idx, t_perm, order, t_order;
        std::vector<int4> sched, t_sched;
        std::vector<float> vals_t;
        std::vector<int32_t> mid_dst;
        std::vector<uint16_t> mid_slot, mid_loc;
        std::vector<int32_t> t_col;
        std::vector<int2> lm;
        std::vector<int32_t> lm_off, lm_row;
        std::vector<float> lm_bias;
        int32_t max_len = 0, t_max_len = 0;
        bool clustered = false, t_clustered = false; // reorder_rows found rows that share columns
        int rc = SDNN_OK;
    };
    const bool want_lm = lds_forward_wanted(layers, n_layers, cfg);
    const bool gw_ = grad_buffers_wanted(layers, n_layers, cfg);
    auto prepare = [&](int32_t l, HostIdx &h) {
        try {
            const sdnn_layer &y = layers[l];
            const size_t nnz = (size_t)y.row_ptr[y.n_out];
            h.t_row_ptr.resize((size_t)y.n_in + 1);
            h.t_row_idx.resize(nnz);
            h.t_perm.resize(nnz);
            h.order.resize(y.n_out);
            h.t_order.resize(y.n_in);
            h.sched.resize(y.n_out);
            h.t_sched.resize(y.n_in);
            h.rc = sdnn_transpose_pattern(y.n_out, y.n_in, y.row_ptr, y.col_idx, h.t_row_ptr.data(),
                                          h.t_row_idx.data(), h.t_perm.data());
            if (h.rc) return;
            if (cfg->reorder_rows) {
                // rows that share columns become neighbours and are dealt to one XCD
                const size_t n_max = (size_t)std::max(y.n_out, y.n_in);
                std::vector<int32_t> clustered(n_max), cluster_of(n_max);
                // "found something": on average at least two rows per cluster
                auto found = [&](int32_t n) {
                    int32_t n_clusters = 0;
                    for (int32_t r = 0; r < n; ++r) n_clusters = std::max(n_clusters, cluster_of[r] + 1);
                    return 2 * (int64_t)n_clusters <= n;
                };
                h.rc = sdnn_cluster_rows(y.n_out, y.n_in, y.row_ptr, y.col_idx, SDNN_CLUSTER_ROWS, clustered.data(),
                                         cluster_of.data());
                if (!h.rc) h.clustered = found(y.n_out);
                if (!h.rc) h.rc = sdnn_deal_rows_to_xcds(y.n_out, y.row_ptr, clustered.data(), h.order.data());
                if (!h.rc) h.rc = sdnn_cluster_rows(y.n_in, y.n_out, h.t_row_ptr.data(), h.t_row_idx.data(), SDNN_CLUSTER_ROWS,
                                                    clustered.data(), cluster_of.data());
                if (!h.rc) h.t_clustered = found(y.n_in);
                if (!h.rc) h.rc = sdnn_deal_rows_to_xcds(y.n_in, h.t_row_ptr.data(), clustered.data(), h.t_order.data());
                if (h.rc) return;
            } else {
                sdnn_row_schedule(y.n_out, y.row_ptr, h.order.data());
                sdnn_row_schedule(y.n_in, h.t_row_ptr.data(), h.t_order.data());
            }
            for (int32_t r = 0; r < y.n_out; ++r)
                h.sched[r] = make_int4(h.order[r], y.row_ptr[h.order[r]], y.row_ptr[h.order[r] + 1], 0);
            for (int32_t r = 0; r < y.n_in; ++r)
                h.t_sched[r] = make_int4(h.t_order[r], h.t_row_ptr[h.t_order[r]], h.t_row_ptr[h.t_order[r] + 1], 0);
            if (gw_ && cfg->max_batch == 1) { // one sample per step: the fused sweep looks up each entry's row of W^T
                h.t_col.resize(nnz);
                for (int32_t i = 0; i < y.n_in; ++i)
                    for (int32_t q = h.t_row_ptr[i]; q < h.t_row_ptr[i + 1]; ++q) h.t_col[(size_t)q] = i;
            }
            if (gw_) { // the values in the order of the transposed index, for the fused backward sweep
                h.vals_t.resize(nnz);
                h.mid_slot.resize(nnz);
                h.mid_dst.resize(nnz);
                h.mid_loc.resize(nnz);
                // every chunk of the CSR array but the last holds TR_CHUNK entries, so chunk c's group starts at c TR_CHUNK
                const size_t n_chunks = (nnz + TR_CHUNK - 1) / TR_CHUNK;
                std::vector<int32_t> filled(n_chunks, 0), in_span(n_chunks, 0), touched;
                for (size_t s0 = 0; s0 < nnz; s0 += TR_SPAN) {
                    const size_t s1 = std::min(nnz, s0 + (size_t)TR_SPAN);
                    touched.clear();
                    for (size_t q = s0; q < s1; ++q) {
                        const size_t c = (size_t)h.t_perm[q] / TR_CHUNK;
                        if (in_span[c]++ == 0) touched.push_back((int32_t)c);
                    }
                    std::sort(touched.begin(), touched.end());
                    int32_t run = 0; // in_span[c]: from the span's count for chunk c to the rank of its next entry
                    for (int32_t c : touched) { const int32_t n = in_span[c]; in_span[c] = run; run += n; }
                    for (size_t q = s0; q < s1; ++q) {
                        const size_t p = (size_t)h.t_perm[q], c = p / TR_CHUNK;
                        const size_t m = c * TR_CHUNK + (size_t)filled[c]++;
                        const int32_t k = in_span[c]++;
                        h.vals_t[q] = y.values[p];
                        h.mid_slot[q] = (uint16_t)k;
                        h.mid_dst[s0 + (size_t)k] = (int32_t)m;
                        h.mid_loc[m] = (uint16_t)(p - c * TR_CHUNK);
                    }
                    for (int32_t c : touched) in_span[c] = 0;
                }
            }
            if (want_lm) {
                // lane-major copy: always in longest-first order, whatever the row schedule is
                std::vector<int32_t> by_len((size_t)y.n_out);
                sdnn_row_schedule(y.n_out, y.row_ptr, by_len.data());
                const int32_t nb = (y.n_out + 63) / 64;
                h.lm_off.assign((size_t)nb + 1, 0);
                h.lm_row.assign((size_t)nb * 64, -1);
                h.lm_bias.assign((size_t)nb * 64, 0.0f);
                for (int32_t b = 0; b < nb; ++b) {
                    const int32_t first = by_len[(size_t)b * 64];
                    h.lm_off[b + 1] = h.lm_off[b] + 64 * (y.row_ptr[first + 1] - y.row_ptr[first]);
                }
                h.lm.assign((size_t)h.lm_off[nb], make_int2(0, 0)); // padding: column 0, weight +0.0
                for (int32_t b = 0; b < nb; ++b)
                    for (int32_t lane = 0; lane < 64 && b * 64 + lane < y.n_out; ++lane) {
                        const int32_t row = by_len[(size_t)b * 64 + lane];
                        h.lm_row[(size_t)b * 64 + lane] = row;
                        if (y.bias) h.lm_bias[(size_t)b * 64 + lane] = y.bias[row];
                        for (int32_t p = y.row_ptr[row]; p < y.row_ptr[row + 1]; ++p) {
                            int32_t bits;
                            memcpy(&bits, &y.values[p], 4);
                            h.lm[(size_t)h.lm_off[b] + 64 * (size_t)(p - y.row_ptr[row]) + lane] = make_int2(y.col_idx[p], bits);
                        }
                    }
            }
            h.max_len = h.t_max_len = 0;
            for (int32_t r = 0; r < y.n_out; ++r) h.max_len = std::max(h.max_len, y.row_ptr[r + 1] - y.row_ptr[r]);
            for (int32_t r = 0; r < y.n_in; ++r) h.t_max_len = std::max(h.t_max_len, h.t_row_ptr[r + 1] - h.t_row_ptr[r]);
        } catch (...) {
            h.rc = SDNN_ENOMEM;
        }
    };
#define UP(dst, src, bytes)                                                                   \
    do {                                                                                      \
        if ((bytes) > 0) {                                                                    \
            hipError_t e_ = hipMemcpyAsync((void *)(dst), (src), (bytes), hipMemcpyHostToDevice, stream); \
            if (e_ != hipSuccess)                                                             \
                return fail_free(fail(nullptr, SDNN_EHIP, "upload: %s", hipGetErrorString(e_))); \
        }                                                                                     \
    } while (0)
#define SYNC()                                                                                \
    do {                                                                                      \
        hipError_t e_ = hipStreamSynchronize(stream);                                         \
        if (e_ != hipSuccess)                                                                 \
            return fail_free(fail(nullptr, SDNN_EHIP, "upload: %s", hipGetErrorString(e_)));  \
    } while (0)
    try {
        const bool gw = grad_buffers_wanted(layers, n_layers, cfg);
        int32_t max_out = 0;
        for (int32_t l = 0; l < n_layers; ++l) max_out = std::max(max_out, layers[l].n_out);
        const std::vector<float> zeros((size_t)max_out, 0.0f); // stands in for a NULL bias
        unsigned hw = std::thread::hardware_concurrency();
        const int32_t group = (int32_t)std::max(1u, std::min({hw ? hw : 1u, 16u, (unsigned)n_layers}));
        std::vector<HostIdx> idx((size_t)group);
        for (int32_t l0 = 0; l0 < n_layers; l0 += group) {
            const int32_t ng = std::min(group, n_layers - l0);
            {
                std::vector<std::thread> workers;
                for (int32_t k = 1; k < ng; ++k) {
                    try {
                        workers.emplace_back(prepare, l0 + k, std::ref(idx[k]));
                    } catch (...) { // no more threads: do it here
                        prepare(l0 + k, idx[k]);
                    }
                }
                prepare(l0, idx[0]);
                for (std::thread &w : workers) w.join();
            }
            for (int32_t k = 0; k < ng; ++k) {
                const int32_t l = l0 + k;
                const HostIdx &h = idx[k];
                if (h.rc) return fail_free(fail(nullptr, h.rc, "layer %d: host setup failed (out of memory?)", l + 1));
                const sdnn_layer &y = layers[l];
                const Plan::PerLayer &q = pl.pl[l];
                const size_t nnz = (size_t)y.row_ptr[y.n_out];
                LayerDev &d = net->layers[l];
                d.n_out = y.n_out; d.n_in = y.n_in; d.nnz = (int32_t)nnz; d.pad_ = 0;
                d.row_ptr = (const int32_t *)(base + q.row_ptr);
                d.col_idx = (const int32_t *)(base + q.col_idx);
                d.vals = (float *)(base + q.vals);
                d.bias = (float *)(base + q.bias);
                d.t_row_ptr = (const int32_t *)(base + q.t_row_ptr);
                d.t_row_idx = (const int32_t *)(base + q.t_row_idx);
                d.t_perm = (const int32_t *)(base + q.t_perm);
                d.sched = (const int4 *)(base + q.sched);
                d.t_sched = (const int4 *)(base + q.t_sched);
                d.X = cfg->training ? (float *)(base + q.X) : nullptr;
                d.D = cfg->training ? (float *)(base + q.D) : nullptr;
                d.G[0] = gw ? (float *)(base + q.G[0]) : nullptr;
                d.G[1] = gw ? (float *)(base + q.G[1]) : nullptr;
                d.vals_t = gw ? (float *)(base + q.vals_t) : nullptr;
                d.mid_slot = gw ? (const uint16_t *)(base + q.mid_slot) : nullptr;
                d.mid_dst = gw ? (const int32_t *)(base + q.mid_dst) : nullptr;
                d.mid_loc = gw ? (const uint16_t *)(base + q.mid_loc) : nullptr;
                d.mid = gw ? (float *)(base + q.mid) : nullptr;
                d.t_col = gw && cfg->max_batch == 1 ? (const int32_t *)(base + q.t_col) : nullptr;
                d.lm = want_lm ? (int2 *)(base + q.lm) : nullptr;
                d.lm_off = want_lm ? (const int32_t *)(base + q.lm_off) : nullptr;
                d.lm_row = want_lm ? (const int32_t *)(base + q.lm_row) : nullptr;
                d.lm_bias = want_lm ? (float *)(base + q.lm_bias) : nullptr;
                d.n_blocks = want_lm ? (int32_t)q.lm_blocks : 0;
                d.pad2_ = 0;
                d.X_prev = !cfg->training ? nullptr
                           : l == 0       ? (float *)(base + pl.x0)
                                          : net->layers[l - 1].X;
                net->max_n = std::max(net->max_n, std::max(y.n_out, y.n_in));
                net->max_len[0][l] = h.max_len;
                net->max_len[1][l] = h.t_max_len;
                net->clustered[0][l] = h.clustered;
                net->clustered[1][l] = h.t_clustered;
                UP(d.row_ptr, y.row_ptr, 4 * ((size_t)y.n_out + 1));
                UP(d.col_idx, y.col_idx, 4 * nnz);
                UP(d.vals, y.values, 4 * nnz);
                UP(d.bias, y.bias ? y.bias : zeros.data(), 4 * (size_t)y.n_out);
                UP(d.t_row_ptr, h.t_row_ptr.data(), 4 * ((size_t)y.n_in + 1));
                UP(d.t_row_idx, h.t_row_idx.data(), 4 * nnz);
                UP(d.t_perm, h.t_perm.data(), 4 * nnz);
                UP(d.sched, h.sched.data(), 16 * (size_t)y.n_out);
                UP(d.t_sched, h.t_sched.data(), 16 * (size_t)y.n_in);
                if (gw) UP(d.vals_t, h.vals_t.data(), 4 * nnz);
                if (gw) UP(d.mid_slot, h.mid_slot.data(), 2 * nnz);
                if (gw) UP(d.mid_dst, h.mid_dst.data(), 4 * nnz);
                if (gw) UP(d.mid_loc, h.mid_loc.data(), 2 * nnz);
                if (d.t_col) UP(d.t_col, h.t_col.data(), 4 * nnz);
                if (want_lm) {
                    if (h.lm.size() != q.lm_entries)
                        return fail_free(fail(nullptr, SDNN_EINVAL, "layer %d: lane-major copy does not match its plan", l + 1));
                    UP(d.lm, h.lm.data(), 8 * h.lm.size());
                    UP(d.lm_off, h.lm_off.data(), 4 * h.lm_off.size());
                    UP(d.lm_row, h.lm_row.data(), 4 * h.lm_row.size());
                    UP(d.lm_bias, h.lm_bias.data(), 4 * h.lm_bias.size());
                }
            }
            SYNC(); // the group's host arrays are reused by the next group
        }
        net->d_layers = (LayerDev *)(base + pl.table);
        UP(net->d_layers, net->layers.data(), sizeof(LayerDev) * (size_t)n_layers);
        SYNC();
    } catch (...) {
        return fail_free(fail(nullptr, SDNN_ENOMEM, "host allocation failed during setup"));
    }
#undef UP
#undef SYNC
    {
        int devid = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&devid) != hipSuccess || hipGetDeviceProperties(&prop, devid) != hipSuccess)
            return fail_free(fail(nullptr, SDNN_EHIP, "cannot query the device"));
        net->n_cu = prop.multiProcessorCount;
        void *scratch_dev = nullptr; // this GPU's copy of the fixed staging array of sdnn_forward_noalloc
        if (scratch_address(nullptr, &scratch_dev) != SDNN_OK) return fail_free(SDNN_EHIP);
        // default priority, like every stream here
        if (hipStreamCreateWithFlags(&net->side, hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&net->ev_fork, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&net->ev_join, hipEventDisableTiming) != hipSuccess)
            return fail_free(fail(nullptr, SDNN_EHIP, "cannot create the side stream"));
    }
    if (cfg->training) {
        net->d_x0 = (float *)(base + pl.x0);
    } else {
        net->d_ping = (float *)(base + pl.ping);
        net->d_pong = (float *)(base + pl.pong);
        for (int k = 0; k < 2; ++k) {
            net->d_flags[k] = (int32_t *)(base + pl.flags[k]);
            net->d_map[k] = (int32_t *)(base + pl.map[k]);
            net->d_n_live[k] = (int32_t *)(base + pl.n_live[k]);
        }
    }
    net->lds_ready = want_lm;
    net->bias_nonpos = true;
    for (int32_t l = 1; l < n_layers; ++l)
        if (layers[l].bias)
            for (int32_t r = 0; r < layers[l].n_out; ++r)
                if (!(layers[l].bias[r] <= 0.0f)) net->bias_nonpos = false;
    *out = net;
    return SDNN_OK;
}

extern "C" void sdnn_destroy(sdnn_net *net)
{
    if (!net) return;
    if (net->side) { (void)hipStreamSynchronize(net->side); (void)hipStreamDestroy(net->side); }
    if (net->ev_fork) (void)hipEventDestroy(net->ev_fork);
    if (net->ev_join) (void)hipEventDestroy(net->ev_join);
    delete net;
}

// Forward and backward treat the samples independently (the batch vectors are columns of X), so a
// pass over small layers is run as two half-batches on two streams: each stream's kernels depend
// only on its own previous kernel, and while one stream sits in the latencies at the head or tail
// of a kernel, the other one computes.  Returns the samples per lane to use (0 = do not split).
static int split_v(const sdnn_net *net, int B)
{
    if (B % 128 != 0 || (int64_t)net->max_n * B > ((int64_t)1 << 21)) return 0;
    // long rows (hundreds of entries) keep a wavefront busy for long: nothing to hide, and wider lanes pay more
    int64_t nnz = 0, rows = 0;
    for (const LayerDev &d : net->layers) { nnz += d.nnz; rows += d.n_out; }
    if (nnz >= 128 * rows) return 0;
    return B % 512 == 0 ? 4 : B % 256 == 0 ? 2 : 1; // two or more tiles of 64*V samples
}

// After a failure between fork and join: bring the helper stream back into the caller's stream, so that the
// caller's stream (or a capture in progress) is not left with a dangling fork.
static void join_side(sdnn_net *net, hipStream_t stream)
{
    if (hipEventRecord(net->ev_join, net->side) == hipSuccess) (void)hipStreamWaitEvent(stream, net->ev_join, 0);
}

static inline bool aligned(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// Samples per lane for the row-per-wavefront product: as wide as the batch
// and the alignment of the operands allow without idling most of the wave.
static int pick_v_spmm(int B, const void *a, const void *b, const void *c)
{
    if (B % 4 == 0 && B > 128 && aligned(a, 16) && aligned(b, 16) && aligned(c, 16)) return 4;
    if (B % 2 == 0 && B > 64 && aligned(a, 8) && aligned(b, 8) && aligned(c, 8)) return 2;
    return 1;
}

// Kernel tables.  The forward kernels are compiled per activation, the backward ones once (ACT = 0).
template <int MODE, int V, int U, bool TI>
static const void *spmm_fn_act(int act)
{
    if (MODE == 0 && act == ACT_SIGMOID) return (const void *)k_spmm<V, MODE, U, TI, (MODE == 0 ? ACT_SIGMOID : 0)>;
    return (const void *)k_spmm<V, MODE, U, TI, 0>;
}
template <int MODE, int V>
static const void *spmm_fn_v(int U, bool ti, int act)
{
    if (ti) return spmm_fn_act<MODE, V, 8, true>(act);
    if (U == 16) return spmm_fn_act<MODE, V, 16, false>(act);
    return spmm_fn_act<MODE, V, 8, false>(act);
}
template <int MODE>
static const void *spmm_fn(int V, int U, bool ti, int act)
{
    return V == 4 ? spmm_fn_v<MODE, 4>(U, ti, act) : V == 2 ? spmm_fn_v<MODE, 2>(U, ti, act) : spmm_fn_v<MODE, 1>(U, ti, act);
}
template <int MODE, int R>
static const void *panel_fn_act(int act)
{
    if (MODE == 0 && act == ACT_SIGMOID) return (const void *)k_spmm_panel<R, MODE, (MODE == 0 ? ACT_SIGMOID : 0)>;
    return (const void *)k_spmm_panel<R, MODE, 0>;
}
template <int MODE>
static const void *panel_fn(int ri, int act)
{
    return ri == 0 ? panel_fn_act<MODE, 1>(act) : ri == 1 ? panel_fn_act<MODE, 2>(act)
           : ri == 2 ? panel_fn_act<MODE, 4>(act) : panel_fn_act<MODE, 8>(act);
}

// The panel sweep (k_spmm_panel) over all 64-sample tiles of the batch; a's operand fields are filled in.
template <int MODE>
static int launch_spmm_panel(sdnn_net *net, const LayerDev &d, SpmmArgs a, int B, int panel, hipStream_t stream,
                             int sub_begin, int sub_end)
{
    a.tile_base = (uint32_t)(sub_begin / 64);
    a.n_tiles = (uint32_t)((sub_end - sub_begin + 63) / 64);
    const int n_cols = MODE == 0 ? d.n_in : d.n_out;
    // rows per wavefront: enough for the wavefronts resident on an XCD to hold all the rows that the XCD
    // has of one tile, so that the whole tile is swept panel by panel in one go (at most 8)
    const int xcds = 8;
    const int64_t rows_per_xcd = a.n_tiles >= 8 ? a.n_rows : (a.n_rows + xcds - 1) / xcds;
    int ri = 0;
    for (;; ++ri) {
        const void *fn_r = panel_fn<MODE>(ri, net->cfg.activation);
        int &occ = net->occ_panel[MODE][ri];
        if (occ == 0) {
            HIP_TRY(net, hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, fn_r, BLOCK_THREADS, 0));
            if (occ < 1) occ = 1;
        }
        const int64_t resident = (int64_t)occ * WAVES_PER_BLOCK * (net->n_cu / xcds);
        if ((resident << ri) >= rows_per_xcd) break;
        if (ri == 3) break;
    }
    const int R = 1 << ri;
    const void *fn = panel_fn<MODE>(ri, net->cfg.activation);
    a.n_rg = (uint32_t)((a.n_rows + WAVES_PER_BLOCK * R - 1) / (WAVES_PER_BLOCK * R));
    const uint64_t blocks = (uint64_t)a.n_tiles * a.n_rg;
    if (blocks > 0x7fffffffull) return fail(net, SDNN_EINVAL, "grid too large");
    a.n_vblocks = (uint32_t)blocks;
    uint64_t g = std::min<uint64_t>(blocks, (uint64_t)net->occ_panel[MODE][ri] * (uint64_t)net->n_cu);
    if (g >= 8) g &= ~(uint64_t)7;
    int n_cols_arg = n_cols;
    void *args[] = {(void *)&a, (void *)&n_cols_arg, (void *)&panel};
    HIP_TRY(net, hipLaunchKernel(fn, dim3((unsigned)g), dim3(BLOCK_THREADS), args, 0, stream));
    HIP_TRY(net, hipGetLastError());
    return SDNN_OK;
}

// part/n_parts: the batch tiles of the launch are the part-th of n_parts equal shares (n_parts = 2
// when a pass is run as two independent half-batches on two streams); force_v: samples per lane, 0 = choose.
template <int MODE>
static int launch_spmm(sdnn_net *net, const LayerDev &d, const float *in, float *out,
                       const float *aux, int B, hipStream_t stream, int part = 0, int n_parts = 1, int force_v = 0,
                       const int32_t *n_live = nullptr, int32_t *flags = nullptr, int sub_begin = 0, int sub_end = 0)
{
    // sub_begin .. sub_end: the launch covers these samples only (sub_begin a multiple of SUB_ALIGN, or of 64 where
    // every layer takes the panel sweep; sub_end == 0: all of them, split by part / n_parts)
    const bool sub = sub_end > 0;
    if (!sub) sub_end = B;
    SpmmArgs a;
    a.n_live = n_live;
    a.flags = flags;
    a.g_part = nullptr; a.store_out = 1;
    if (MODE == 0) {
        a.row_ptr = d.row_ptr; a.idx = d.col_idx; a.perm = nullptr; a.sched = d.sched;
        a.n_rows = d.n_out;
    } else {
        a.row_ptr = d.t_row_ptr; a.idx = d.t_row_idx; a.perm = d.t_perm; a.sched = d.t_sched;
        a.n_rows = d.n_in;
    }
    a.vals = d.vals; a.in = in; a.out = out; a.aux = aux; a.B = B; a.cap = net->cfg.act_cap; a.act = net->cfg.activation;
    if (a.n_rows == 0) return SDNN_OK;
    a.in_bytes = 4 * (size_t)(MODE == 0 ? d.n_in : d.n_out) * (size_t)B;
    if (a.in_bytes >= ((size_t)1 << 32))
        return fail(net, SDNN_EINVAL, "activation block of %zu bytes exceeds 4 GiB: use a smaller B", a.in_bytes);
    if (B == 1) {
        const int64_t nnz = d.nnz;
        if (a.n_rows >= SPMV_STAGE_MIN_ROWS && nnz < 128 * (int64_t)a.n_rows) {
            // short rows, wide layer: R consecutive rows per 64-lane workgroup (measured: 8, and 16 from 32768 rows)
            const int R = a.n_rows >= 32768 ? 16 : 8;
            hipLaunchKernelGGL((k_spmv_stage<MODE, 8>), dim3((unsigned)((a.n_rows + R - 1) / R)), dim3(64), 0, stream, a, R);
        } else if (a.n_rows <= 16384) // a wavefront per row while that still fits the chip a few times over
            hipLaunchKernelGGL(k_spmv_wave<MODE>, dim3((unsigned)((a.n_rows + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK)),
                               dim3(BLOCK_THREADS), 0, stream, a);
        else
            hipLaunchKernelGGL(k_spmv<MODE>, dim3((unsigned)((a.n_rows + 255) / 256)), dim3(256), 0, stream, a);
        HIP_TRY(net, hipGetLastError());
        return SDNN_OK;
    }
    // Wide layers with short rows: when a 64-sample tile of the operand (n_cols x 256 B) is at least twice
    // the chip's eight L2s, the panel sweep is faster (measured, 65536 columns: forward of a 64-sample
    // minibatch 64.8 -> 53.6 us per layer, inference in blocks of 1024 samples 217 -> 179 ms per 24 layers;
    // 16384 columns and fewer: slower than the kernels below).  sdnn_config.panel_cols overrides.
    if (!n_live && !flags && n_parts == 1 && force_v == 0 && net->cfg.panel_cols >= 0) {
        const int l = (int)(&d - net->layers.data());
        const int n_cols = MODE == 0 ? d.n_in : d.n_out;
        int panel = net->cfg.panel_cols;
        // (not where reorder_rows has found clusters: their locality comes from the row order, which the
        // panel kernel's larger workgroups would deal to the XCDs differently: 9.8 vs 6.8 ms on a structured net)
        if (panel == 0 && (int64_t)n_cols * 256 >= ((int64_t)8 << 20) && d.nnz > 0 && !net->clustered[MODE][l])
            panel = sub_end - sub_begin > 448 ? 6144 : 8192; // eight or more tiles: every XCD sweeps tiles of its own
        if (panel > 0 && net->max_len[MODE][l] <= 64)
            return launch_spmm_panel<MODE>(net, d, a, B, panel, stream, sub_begin, sub_end);
    }
    const int V = force_v ? force_v : pick_v_spmm(B, in, out, MODE == 1 ? aux : nullptr);
    const uint32_t all_tiles = (uint32_t)((B + 64 * V - 1) / (64 * V));
    a.tile_base = all_tiles * (uint32_t)part / (uint32_t)n_parts;
    a.n_tiles = all_tiles * (uint32_t)(part + 1) / (uint32_t)n_parts - a.tile_base;
    if (sub) {
        if (sub_begin % (64 * V) != 0) return fail(net, SDNN_EHIP, "internal: sub-block at sample %d, tiles of %d", sub_begin, 64 * V);
        a.tile_base = (uint32_t)(sub_begin / (64 * V));
        a.n_tiles = (uint32_t)((sub_end - sub_begin + 64 * V - 1) / (64 * V));
    }
    if (a.n_tiles == 0) return SDNN_OK;
    a.n_rg = (uint32_t)((a.n_rows + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    const uint64_t blocks = (uint64_t)a.n_tiles * a.n_rg;
    if (blocks > 0x7fffffffull) return fail(net, SDNN_EINVAL, "grid too large");
    a.n_vblocks = (uint32_t)blocks;
    // Measured policy.  Short rows (a few tens of entries): 8 gathers in flight per lane (16 costs a
    // third of the occupancy) and a grid of what the chip holds at once, whose workgroups walk the
    // virtual blocks.  Long, uneven rows (hundreds of entries): 16 in flight and one workgroup per
    // virtual block, so that the hardware hands out the rows, longest first, as wavefronts retire.
    const bool long_rows = (int64_t)d.nnz >= 128 * (int64_t)a.n_rows;
    uint64_t g = blocks;
    // short rows and a few batch tiles (shared by all XCDs): workgroups are dealt row groups and walk the tiles
    const bool tiles_inner = !long_rows && a.n_tiles >= 2 && a.n_tiles < 8;
    if (tiles_inner) g = a.n_rg;
    const int U = long_rows ? 16 : 8;
    const void *fn = spmm_fn<MODE>(V, U, tiles_inner, net->cfg.activation);
    if (!long_rows) {
        int &per_cu = net->occ_spmm[MODE][V == 4 ? 2 : V == 2 ? 1 : 0][tiles_inner ? 1 : 0][U == 16 ? 1 : 0];
        if (per_cu == 0) {
            HIP_TRY(net, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, BLOCK_THREADS, 0));
            if (per_cu < 1) per_cu = 1;
        }
        g = std::min(g, (uint64_t)per_cu * (uint64_t)net->n_cu);
    }
    if (g >= 8) g &= ~(uint64_t)7; // keeps virtual block id % 8 == workgroup id % 8 (XCD-wise tiles)
    void *args[] = {(void *)&a};
    HIP_TRY(net, hipLaunchKernel(fn, dim3((unsigned)g), dim3(BLOCK_THREADS), args, 0, stream));
    HIP_TRY(net, hipGetLastError());
    return SDNN_OK;
}

// Whether the single-launch LDS-resident forward is the faster way to run this block of B samples.
static bool lds_forward_pays(const sdnn_net *net, int B)
{
    if (!net->lds_ready || net->cfg.lds_forward == SDNN_LDS_OFF) return false;
    for (const LayerDev &d : net->layers)
        if (d.n_out == 0) return false; // an empty layer: leave it to the general path
    if (net->cfg.lds_forward == SDNN_LDS_ON) return true;
    // Measured on nets of 32-entry rows (N = 1024 and 4096, 120 layers): the single launch takes about
    // 2 us + 0.13 ns per stored entry per layer for every round of workgroups (one workgroup of LDS_T samples
    // per CU), the per-layer kernels about 4.5 us + 0.21 ps per entry and sample per layer.
    int64_t nnz = 0;
    for (const LayerDev &d : net->layers) nnz += d.nnz;
    const double nnz_layer = (double)nnz / (double)net->n_layers;
    const int wgs = (B + LDS_T - 1) / LDS_T;
    const int rounds = (wgs + net->n_cu - 1) / std::max(net->n_cu, 1);
    const double t_fused = rounds * (2.0e-6 + 0.13e-9 * nnz_layer);
    const double t_layers = 4.5e-6 + 0.21e-12 * nnz_layer * (double)B;
    return t_fused < t_layers;
}

// Eq. 3 for l = 1..L.  Inference nets stage the activations between the layers in ping / pong
// (each at least 4 * max_n * B bytes); training nets keep every X_l in the workspace and ignore them.
// Width in samples of the sub-blocks that an inference pass is cut into, 0 = one piece.  A sub-block's share of an
// activation buffer is held to SUB_BYTES; the width is a multiple of SUB_ALIGN (the widest tile of the product
// kernels), or of 64 where every layer takes the panel sweep (64-sample tiles throughout).
#define SUB_BYTES ((int64_t)16 << 20)
#define SUB_ALIGN 256
static int sub_block_width(const sdnn_net *net, int B)
{
    if ((int64_t)net->max_n * B * 4 <= 2 * SUB_BYTES || B == 1) return 0;
    int64_t nnz = 0, rows = 0; // long rows: bound by the L1 and the VALU, not by where the operand comes from (slower: 61 -> 67 ms)
    for (const LayerDev &d : net->layers) { nnz += d.nnz; rows += d.n_out; }
    if (nnz >= 128 * rows) return 0;
    bool all_panel = net->cfg.panel_cols >= 0;
    for (int l = 0; l < net->n_layers && all_panel; ++l) {
        const LayerDev &d = net->layers[l];
        const bool wide = net->cfg.panel_cols > 0 || ((int64_t)d.n_in * 256 >= ((int64_t)8 << 20) && d.nnz > 0 && !net->clustered[0][l]);
        all_panel = wide && net->max_len[0][l] <= 64;
    }
    const int align = all_panel ? 64 : SUB_ALIGN;
    int64_t w = SUB_BYTES / (4 * (int64_t)net->max_n) / align * align;
    if (w < align) w = align;
    return w >= B ? 0 : (int)w;
}

static int forward_impl(sdnn_net *net, const float *d_X0, int32_t B, float *d_XL, void *stream_, float *ping,
                        float *pong)
{
    const bool training = net->cfg.training != 0;
    hipStream_t stream = (hipStream_t)stream_;
    net->state = ST_IDLE;
    const int L = net->n_layers;
    if (lds_forward_pays(net, B)) {
        const void *fn = net->cfg.activation == ACT_SIGMOID ? (const void *)k_fwd_lds<ACT_SIGMOID> : (const void *)k_fwd_lds<ACT_RELU_CAP>;
        int buf_floats = LDS_T * ((net->max_n + 3) & ~3);
        const size_t lds_bytes = 2 * sizeof(float) * (size_t)buf_floats;
        if (!net->lds_attr_set) { // more than the default 64 KiB of dynamic LDS per workgroup
            HIP_TRY(net, hipFuncSetAttribute((const void *)k_fwd_lds<ACT_SIGMOID>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * 4 * LDS_T * LDS_MAX_N));
            HIP_TRY(net, hipFuncSetAttribute((const void *)k_fwd_lds<ACT_RELU_CAP>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * 4 * LDS_T * LDS_MAX_N));
            net->lds_attr_set = true;
        }
        const LayerDev *layers = net->d_layers;
        int n_layers = L, b = B, vec_io = (B % 4 == 0 && aligned(d_X0, 16) && aligned(d_XL, 16)) ? 1 : 0;
        float cap = net->cfg.act_cap;
        void *args[] = {(void *)&layers, (void *)&n_layers, (void *)&d_X0, (void *)&d_XL, (void *)&b, (void *)&buf_floats,
                        (void *)&cap, (void *)&vec_io};
        HIP_TRY(net, hipLaunchKernel(fn, dim3((unsigned)((B + LDS_T - 1) / LDS_T)), dim3(64 * LDS_WAVES), args, lds_bytes, stream));
        HIP_TRY(net, hipGetLastError());
        net->B = B;
        net->state = ST_FORWARD;
        return SDNN_OK;
    }
    const float *in = d_X0;
    if (training) {
        const size_t bytes = 4 * (size_t)net->layers[0].n_in * B;
        if (bytes) HIP_TRY(net, hipMemcpyAsync(net->d_x0, d_X0, bytes, hipMemcpyDeviceToDevice, stream));
        in = net->d_x0;
    }
    int sv = split_v(net, B);
    if (sv > 1 && (!aligned(d_X0, 4 * sv) || (d_XL && !aligned(d_XL, 4 * sv)))) sv = 0;
    if (sv) {
        HIP_TRY(net, hipEventRecord(net->ev_fork, stream));
        HIP_TRY(net, hipStreamWaitEvent(net->side, net->ev_fork, 0));
    }
    // Inference on large activation blocks: the samples are independent (the columns of X, Section 5.1), so the
    // block is taken through all layers in sub-blocks whose two activation buffers stay in the memory-side
    // cache (what a layer wrote is what the next one gathers): measured on 65536-neuron layers, blocks of 1024
    // samples: 179 ms per 24 layers in one piece, 161 ms in sub-blocks of 64; 16384 neurons, 4096 samples: 41.5 ms
    // per 48 layers in one piece, 39.1 in sub-blocks of 256.
    const int sub_w = training || sv ? 0 : sub_block_width(net, B);
    if (sub_w > 0) {
        for (int s0 = 0; s0 < B; s0 += sub_w) {
            const int s1 = std::min(B, s0 + sub_w);
            const float *sin = d_X0;
            for (int l = 0; l < L; ++l) {
                const LayerDev &d = net->layers[l];
                float *out = l == L - 1 ? d_XL : ((l & 1) ? pong : ping);
                const int rc = launch_spmm<0>(net, d, sin, out, d.bias, B, stream, 0, 1, 0, nullptr, nullptr, s0, s1);
                if (rc) return rc;
                sin = out;
            }
        }
        net->B = B;
        net->state = ST_FORWARD;
        return SDNN_OK;
    }
    for (int l = 0; l < L; ++l) {
        const LayerDev &d = net->layers[l];
        float *out = training ? d.X : (l == L - 1 ? d_XL : ((l & 1) ? pong : ping));
        int rc = sv ? launch_spmm<0>(net, d, in, out, d.bias, B, stream, 0, 2, sv)
                    : launch_spmm<0>(net, d, in, out, d.bias, B, stream);
        if (!rc && sv) rc = launch_spmm<0>(net, d, in, out, d.bias, B, net->side, 1, 2, sv);
        if (rc) {
            if (sv) join_side(net, stream);
            return rc;
        }
        in = out;
    }
    if (sv) {
        HIP_TRY(net, hipEventRecord(net->ev_join, net->side));
        HIP_TRY(net, hipStreamWaitEvent(stream, net->ev_join, 0));
    }
    if (training && d_XL) {
        const size_t bytes = 4 * (size_t)net->layers[L - 1].n_out * B;
        if (bytes) HIP_TRY(net, hipMemcpyAsync(d_XL, net->layers[L - 1].X, bytes, hipMemcpyDeviceToDevice, stream));
    }
    net->B = B;
    net->state = ST_FORWARD;
    return SDNN_OK;
}

static int check_forward_args(sdnn_net *net, const float *d_X0, int32_t B, const float *d_XL)
{
    if (!net) return fail(nullptr, SDNN_EINVAL, "net is NULL");
    if (!d_X0) return fail(net, SDNN_EINVAL, "d_X0 is NULL");
    if (B < 1 || B > net->cfg.max_batch)
        return fail(net, SDNN_EINVAL, "B = %d outside 1..max_batch = %d", B, net->cfg.max_batch);
    if (!net->cfg.training && !d_XL) return fail(net, SDNN_EINVAL, "d_XL is NULL");
    return SDNN_OK;
}

extern "C" int sdnn_forward(sdnn_net *net, const float *d_X0, int32_t B, float *d_XL, void *stream_)
{
    const int rc = check_forward_args(net, d_X0, B, d_XL);
    if (rc) return rc;
    return forward_impl(net, d_X0, B, d_XL, stream_, net->d_ping, net->d_pong);
}

// ---------------------------------------------------------------------------
// sdnn_forward for callers that cannot allocate: the activations between the layers are staged in
// a fixed array that lives in the library's device image, one copy per GPU, instead of in two
// buffers of a caller-allocated workspace.
// ---------------------------------------------------------------------------
extern "C" int sdnn_forward_noalloc(sdnn_net *net, const float *d_X0, int32_t B, float *d_XL, void *stream_)
{
    int rc = check_forward_args(net, d_X0, B, d_XL);
    if (rc) return rc;
    if (net->cfg.training)
        return fail(net, SDNN_ESTATE, "sdnn_forward_noalloc is for inference nets (training = 0): a training net "
                                      "keeps every X_l in its workspace");
    const size_t half = (size_t)SDNN_NOALLOC_SCRATCH_BYTES / 2;
    const size_t need = 4 * (size_t)net->max_n * (size_t)B; // one activation buffer, 256-byte aligned by `half`
    if (need > half)
        return fail(net, SDNN_EINVAL, "sdnn_forward_noalloc: an activation block of %d neurons x %d samples needs "
                                      "%zu bytes, the fixed staging array holds %zu per buffer: use a smaller B",
                    net->max_n, B, need, half);
    void *base = nullptr;
    rc = scratch_address(net, &base);
    if (rc) return rc;
    return forward_impl(net, d_X0, B, d_XL, stream_, (float *)base, (float *)((char *)base + half));
}


static unsigned ew_blocks(size_t n)
{
    size_t b = (n + 255) / 256;
    return (unsigned)std::min<size_t>(std::max<size_t>(b, 1), 8192);
}

extern "C" int sdnn_forward_skip_dead(sdnn_net *net, const float *d_X0, int32_t B, float *d_XL,
                                      int32_t check_every, int32_t *d_n_live, void *stream_)
{
    if (!net) return fail(nullptr, SDNN_EINVAL, "net is NULL");
    if (!d_X0 || !d_XL) return fail(net, SDNN_EINVAL, "d_X0 or d_XL is NULL");
    if (B < 1 || B > net->cfg.max_batch)
        return fail(net, SDNN_EINVAL, "B = %d outside 1..max_batch = %d", B, net->cfg.max_batch);
    if (check_every < 1) return fail(net, SDNN_EINVAL, "check_every must be >= 1");
    if (net->cfg.training) return fail(net, SDNN_ESTATE, "dead-sample skipping is for inference nets (training = 0)");
    if (net->cfg.activation != SDNN_ACT_RELU_CAP)
        return fail(net, SDNN_ESTATE, "dead-sample skipping needs the ReLU activation (f(0) = 0)");
    if (!net->bias_nonpos)
        return fail(net, SDNN_ESTATE, "dead-sample skipping needs every bias of layers 2..L to be <= 0 "
                                      "(a positive bias revives a dead sample; replaced biases are not inspected)");
    if (B > PACK_MAX_B) return fail(net, SDNN_EINVAL, "B = %d: dead-sample skipping packs blocks of at most %d samples", B, PACK_MAX_B);
    hipStream_t stream = (hipStream_t)stream_;
    net->state = ST_IDLE;
    const int L = net->n_layers;
    hipLaunchKernelGGL(k_skip_init, dim3(ew_blocks((size_t)B)), dim3(256), 0, stream, net->d_map[0], net->d_flags[0],
                       net->d_flags[1], net->d_n_live[0], B);
    HIP_TRY(net, hipGetLastError());
    const float *in = d_X0;
    int k = 0; // packing round: its state is in slot k & 1, the next round's in the other slot
    for (int l = 0; l < L; ++l) {
        const LayerDev &d = net->layers[l];
        float *out = (l & 1) ? net->d_pong : net->d_ping;
        // one sample: nothing to pack, this is the plain pass
        const bool check = (l + 1) % check_every == 0 && l + 1 < L && B > 1 && d.n_out > 0;
        const int rc = launch_spmm<0>(net, d, in, out, d.bias, B, stream, 0, 1, 0, net->d_n_live[k & 1],
                                      check ? net->d_flags[k & 1] : nullptr);
        if (rc) return rc;
        if (check) {
            hipLaunchKernelGGL(k_pack, dim3((unsigned)((d.n_out + PACK_ROWS - 1) / PACK_ROWS)), dim3(256), 0, stream, out,
                               d.n_out, B, net->d_flags[k & 1], net->d_n_live[k & 1], net->d_map[k & 1],
                               net->d_n_live[(k + 1) & 1], net->d_map[(k + 1) & 1], net->d_flags[(k + 1) & 1]);
            HIP_TRY(net, hipGetLastError());
            ++k;
        }
        in = out;
    }
    const int n_last = net->layers[L - 1].n_out;
    if (n_last > 0) {
        hipLaunchKernelGGL(k_fill_f32, dim3(ew_blocks((size_t)n_last * B)), dim3(256), 0, stream, d_XL,
                           (size_t)n_last * B, 0.0f);
        hipLaunchKernelGGL(k_scatter_cols, dim3((unsigned)((B + 255) / 256), (unsigned)((n_last + LIVE_ROWS - 1) / LIVE_ROWS)),
                           dim3(256), 0, stream, in, d_XL, n_last, B, net->d_map[k & 1], net->d_n_live[k & 1]);
        HIP_TRY(net, hipGetLastError());
    }
    if (d_n_live) HIP_TRY(net, hipMemcpyAsync(d_n_live, net->d_n_live[k & 1], 4, hipMemcpyDeviceToDevice, stream));
    net->B = B;
    return SDNN_OK;
}

// Fused back-propagation + entry gradient of one layer for the part-th of n_parts 64-sample windows.
// store_out = 0 for the first layer (gradient only: there is no Delta_0, out may be NULL).
static int launch_bwd_grad(sdnn_net *net, const LayerDev &d, float *out, int B, hipStream_t stream, int part,
                           int store_out)
{
    SpmmArgs a;
    a.row_ptr = d.t_row_ptr; a.idx = d.t_row_idx; a.perm = nullptr; a.sched = d.t_sched; a.n_rows = d.n_in;
    a.vals = d.vals_t; a.in = d.D; a.out = out; a.aux = d.X_prev; a.B = B; a.cap = net->cfg.act_cap;
    a.act = net->cfg.activation; a.n_live = nullptr; a.flags = nullptr;
    a.g_part = d.G[part]; a.store_out = store_out;
    if (a.n_rows == 0 || d.nnz == 0) {
        if (d.nnz == 0 && store_out && a.n_rows > 0) // no entries: Delta_{l-1} = 0, nothing to differentiate
            return launch_spmm<1>(net, d, d.D, out, d.X_prev, B, stream, part, part == 0 && B <= 64 ? 1 : 2, 1);
        return SDNN_OK;
    }
    a.in_bytes = 4 * (size_t)d.n_out * (size_t)B;
    if (a.in_bytes >= ((size_t)1 << 32))
        return fail(net, SDNN_EINVAL, "activation block of %zu bytes exceeds 4 GiB: use a smaller B", a.in_bytes);
    a.tile_base = (uint32_t)part; // windows of 64 samples
    a.n_tiles = 1;
    a.n_rg = (uint32_t)((a.n_rows + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    a.n_vblocks = a.n_rg;
    if (net->grad_v == 0) { // B = 1
        const int R = a.n_rows >= 32768 ? 16 : 8;
        a.row_ptr = d.t_row_ptr;
        const int32_t *t_col = d.t_col;
        hipLaunchKernelGGL((k_spmv_stage_grad<8>), dim3((unsigned)((a.n_rows + R - 1) / R)), dim3(64), 0, stream, a, R, t_col);
        HIP_TRY(net, hipGetLastError());
        return SDNN_OK;
    }
    if (net->grad_v == 4) {
        // long, uneven rows: one workgroup per four rows, so that the hardware hands out the rows, longest first, as
        // wavefronts retire
        a.tile_base = 0;
        void *args4[] = {(void *)&a};
        HIP_TRY(net, hipLaunchKernel((const void *)k_bwd_grad4<8>, dim3(a.n_vblocks), dim3(BLOCK_THREADS), args4, 0, stream));
        HIP_TRY(net, hipGetLastError());
        return SDNN_OK;
    }
    const void *fn = (const void *)k_bwd_grad<8>;
    if (net->occ_grad == 0) {
        HIP_TRY(net, hipOccupancyMaxActiveBlocksPerMultiprocessor(&net->occ_grad, fn, BLOCK_THREADS, 0));
        if (net->occ_grad < 1) net->occ_grad = 1;
    }
    uint64_t g = std::min<uint64_t>(a.n_vblocks, (uint64_t)net->occ_grad * (uint64_t)net->n_cu);
    if (g >= 8) g &= ~(uint64_t)7;
    void *args[] = {(void *)&a};
    HIP_TRY(net, hipLaunchKernel(fn, dim3((unsigned)g), dim3(BLOCK_THREADS), args, 0, stream));
    HIP_TRY(net, hipGetLastError());
    return SDNN_OK;
}

// The fused kernels take launches of at most 64 samples with one sample per lane: the whole batch
// (B <= 64) or its two halves on two streams (B = 128 on small layers); rows must be short.
static int grad_fusable(const sdnn_net *net, int B, int sv, int *v)
{
    *v = 1;
    if (net->layers[0].G[0] == nullptr) return 0;
    if (B == 1) { // one sample per step: wide layers with short rows only (among those that k_spmv_stage takes)
        // measured step of the 120-layer sigmoid nets, fused vs separate: 65536 rows 6.39 vs 7.80 ms, 16384 rows 2.27
        // vs 2.59, 4096 rows 1.57 vs 1.51 (launch-bound: one more launch per step than it saves)
        if (net->layers[0].t_col == nullptr) return 0;
        for (const LayerDev &d : net->layers)
            if (d.n_in < 8192 || (int64_t)d.nnz >= 128 * (int64_t)d.n_in) return 0;
        *v = 0;
        return 1;
    }
    int64_t nnz = 0, rows = 0;
    for (const LayerDev &d : net->layers) { nnz += d.nnz; rows += d.n_out; }
    if (nnz >= 128 * rows) { // long rows: the whole batch in one launch, four samples per lane (k_bwd_grad4)
        if (B > 256 || B % 4 != 0) return 0;
        *v = 4;
        return 1;
    }
    if (sv == 1 && B == 128) return 2;
    if (sv == 0 && B <= 64) return 1;
    return 0;
}

extern "C" int sdnn_backward(sdnn_net *net, const float *d_dLoss, void *stream_)
{
    if (!net) return fail(nullptr, SDNN_EINVAL, "net is NULL");
    if (!net->cfg.training) return fail(net, SDNN_ESTATE, "net was not created for training");
    if (net->state != ST_FORWARD)
        return fail(net, SDNN_ESTATE, "sdnn_backward needs a directly preceding sdnn_forward");
    if (!d_dLoss) return fail(net, SDNN_EINVAL, "d_dLoss is NULL");
    hipStream_t stream = (hipStream_t)stream_;
    const int L = net->n_layers, B = net->B;
    const LayerDev &last = net->layers[L - 1];
    const size_t n = (size_t)last.n_out * B;
    if (n) {
        hipLaunchKernelGGL(k_output_delta, dim3(ew_blocks(n)), dim3(256), 0, stream, d_dLoss, last.X,
                           last.D, n, net->cfg.act_cap, net->cfg.activation);
        HIP_TRY(net, hipGetLastError());
    }
    const int sv = split_v(net, B);
    const int gp = grad_fusable(net, B, sv, &net->grad_v);
    net->grad_parts = gp;
    if (gp && net->vals_t_stale) { // the CSR values were replaced or stepped by the separate update since the last sweep
        int max_nnz = 0;
        for (const LayerDev &d : net->layers) max_nnz = std::max(max_nnz, d.nnz);
        for (int l0 = 0; l0 < L && max_nnz > 0; l0 += 65535) {
            const int nl = std::min(65535, L - l0);
            hipLaunchKernelGGL(k_refresh_vals_t, dim3((unsigned)std::min(4096, (max_nnz + 2047) / 2048), (unsigned)nl), dim3(256), 0,
                               stream, net->d_layers + l0);
            HIP_TRY(net, hipGetLastError());
        }
        net->vals_t_stale = false;
    }
    if (sv) {
        HIP_TRY(net, hipEventRecord(net->ev_fork, stream));
        HIP_TRY(net, hipStreamWaitEvent(net->side, net->ev_fork, 0));
    }
    for (int l = L - 1; l >= (gp ? 0 : 1); --l) {
        const LayerDev &d = net->layers[l];
        // Delta_{l} (0-based l-1) = (W^T Delta_{l+1}) masked by X_{l}
        float *dprev = l >= 1 ? net->layers[l - 1].D : nullptr;
        int rc;
        if (gp) {
            rc = launch_bwd_grad(net, d, dprev, B, stream, 0, l >= 1);
            if (!rc && gp == 2) rc = launch_bwd_grad(net, d, dprev, B, net->side, 1, l >= 1);
        } else {
            rc = sv ? launch_spmm<1>(net, d, d.D, dprev, d.X_prev, B, stream, 0, 2, sv)
                    : launch_spmm<1>(net, d, d.D, dprev, d.X_prev, B, stream);
            if (!rc && sv) rc = launch_spmm<1>(net, d, d.D, dprev, d.X_prev, B, net->side, 1, 2, sv);
        }
        if (rc) {
            if (sv) join_side(net, stream);
            return rc;
        }
    }
    if (sv) {
        HIP_TRY(net, hipEventRecord(net->ev_join, net->side));
        HIP_TRY(net, hipStreamWaitEvent(stream, net->ev_join, 0));
    }
    net->state = ST_BACKWARD;
    return SDNN_OK;
}

static int pick_v_update(int B, const void *a, const void *b)
{
    return (B % 4 == 0 && aligned(a, 16) && aligned(b, 16)) ? 4 : 1;
}

static int launch_update(sdnn_net *net, int layer0, int n_layers, float lr, int emit, float *g,
                         float *gb, hipStream_t stream)
{
    int max_rows = 0;
    for (int l = layer0; l < layer0 + n_layers; ++l) max_rows = std::max(max_rows, net->layers[l].n_out);
    if (max_rows == 0) return SDNN_OK;
    const int B = net->B;
    if (B == 1) {
        // lanes per row: the power of two that covers the mean row length, 8..64
        int64_t nnz = 0, rows = 0;
        for (int l = layer0; l < layer0 + n_layers; ++l) { nnz += net->layers[l].nnz; rows += net->layers[l].n_out; }
        int lpr_log2 = 3;
        while (lpr_log2 < 6 && ((int64_t)rows << lpr_log2) < nnz) ++lpr_log2;
        const int rows_per_block = WAVES_PER_BLOCK << (6 - lpr_log2);
        for (int l0 = 0; l0 < n_layers; l0 += 65535) {
            const int nl = std::min(65535, n_layers - l0);
            dim3 grid((unsigned)((max_rows + rows_per_block - 1) / rows_per_block), (unsigned)nl);
            hipLaunchKernelGGL(k_update_b1, grid, dim3(BLOCK_THREADS), 0, stream, net->d_layers, layer0 + l0, lpr_log2,
                               lr, net->cfg.update_bias, emit, g, gb);
            HIP_TRY(net, hipGetLastError());
        }
        return SDNN_OK;
    }
    // all activation / delta buffers are 256-byte aligned; rows are aligned iff B % 4 == 0
    const int V = pick_v_update(B, net->layers[layer0].D, net->layers[layer0].X_prev);
    // short rows: a wavefront takes several rows one after the other (fewer, longer-lived wavefronts); long rows: one
    int64_t nnz = 0, rows = 0;
    for (int l = layer0; l < layer0 + n_layers; ++l) { nnz += net->layers[l].nnz; rows += net->layers[l].n_out; }
    const int rpw = nnz < 128 * rows ? 4 : 1; // measured on config 2: 2.49 / 2.37 / 2.32 / 2.33 ms for 1 / 2 / 4 / 8
    const unsigned n_rg = (unsigned)((max_rows + UPD_WAVES * rpw - 1) / (UPD_WAVES * rpw));
    // with many layers, interleave them over the XCDs (one L2 per layer); with few, keep all XCDs on each layer
    const int interleave = n_layers >= 64;
    for (int l0 = 0; l0 < n_layers; l0 += 65535) {
        const int nl = std::min(65535, n_layers - l0);
        dim3 grid(interleave ? 8u * n_rg : n_rg, (unsigned)(interleave ? (nl + 7) / 8 : nl));
        if (V == 4 && rpw == 1 && B <= 256) // long rows: the row of Delta stays in registers
            hipLaunchKernelGGL((k_update<4, 4>), grid, dim3(64 * UPD_WAVES), 0, stream, net->d_layers,
                               layer0 + l0, nl, interleave, rpw, B, lr, net->cfg.update_bias, emit, g, gb);
        else if (V == 4)
            hipLaunchKernelGGL((k_update<4, 0>), grid, dim3(64 * UPD_WAVES), 0, stream, net->d_layers,
                               layer0 + l0, nl, interleave, rpw, B, lr, net->cfg.update_bias, emit, g, gb);
        else
            hipLaunchKernelGGL((k_update<1, 0>), grid, dim3(64 * UPD_WAVES), 0, stream, net->d_layers,
                               layer0 + l0, nl, interleave, rpw, B, lr, net->cfg.update_bias, emit, g, gb);
        HIP_TRY(net, hipGetLastError());
    }
    return SDNN_OK;
}

extern "C" int sdnn_sgd_step(sdnn_net *net, float lr, void *stream_)
{
    if (!net) return fail(nullptr, SDNN_EINVAL, "net is NULL");
    if (!net->cfg.training) return fail(net, SDNN_ESTATE, "net was not created for training");
    if (net->state != ST_BACKWARD)
        return fail(net, SDNN_ESTATE, "sdnn_sgd_step needs a preceding sdnn_backward");
    int rc = SDNN_OK;
    if (net->grad_parts > 0) { // the gradient of the entries is already there
        int max_rows = 0, max_nnz = 0;
        for (const LayerDev &d : net->layers) { max_rows = std::max(max_rows, d.n_out); max_nnz = std::max(max_nnz, d.nnz); }
        for (int l0 = 0; l0 < net->n_layers; l0 += 65535) {
            const int nl = std::min(65535, net->n_layers - l0);
            if (max_nnz > 0) { // a span per workgroup, a multiple of 8 workgroups per layer
                const unsigned gx = (unsigned)((((int64_t)max_nnz + TR_SPAN - 1) / TR_SPAN + 7) & ~(int64_t)7);
                hipLaunchKernelGGL(k_apply, dim3(gx, (unsigned)nl), dim3(TR_THREADS), 0, (hipStream_t)stream_,
                                   net->d_layers + l0, net->grad_parts, lr);
                hipLaunchKernelGGL(k_spread_vals, dim3((unsigned)((max_nnz + TR_CHUNK - 1) / TR_CHUNK), (unsigned)nl),
                                   dim3(TR_THREADS), 0, (hipStream_t)stream_, net->d_layers + l0);
            }
            if (max_rows > 0 && net->cfg.update_bias)
                hipLaunchKernelGGL(k_apply_bias, dim3((unsigned)((max_rows + 16 * WAVES_PER_BLOCK - 1) / (16 * WAVES_PER_BLOCK)), (unsigned)nl),
                                   dim3(BLOCK_THREADS), 0, (hipStream_t)stream_, net->d_layers + l0, net->B, lr, (float *)nullptr);
            HIP_TRY(net, hipGetLastError());
        }
    } else {
        rc = launch_update(net, 0, net->n_layers, lr, 0, nullptr, nullptr, (hipStream_t)stream_);
        if (net->layers[0].vals_t) net->vals_t_stale = true; // this kernel steps the CSR copy only
    }
    if (rc) return rc;
    net->state = ST_IDLE;
    return SDNN_OK;
}

extern "C" int sdnn_weight_grad(sdnn_net *net, int32_t layer, float *d_g, float *d_gb, void *stream_)
{
    if (!net) return fail(nullptr, SDNN_EINVAL, "net is NULL");
    if (!net->cfg.training) return fail(net, SDNN_ESTATE, "net was not created for training");
    if (net->state != ST_BACKWARD)
        return fail(net, SDNN_ESTATE, "sdnn_weight_grad needs a preceding sdnn_backward");
    if (layer < 1 || layer > net->n_layers) return fail(net, SDNN_EINVAL, "layer out of range");
    if (!d_g && !d_gb) return SDNN_OK;
    if (net->grad_parts > 0) {
        // the backward sweep has already formed the gradient that sdnn_sgd_step will apply: hand out that one
        const LayerDev &d = net->layers[layer - 1];
        hipStream_t stream = (hipStream_t)stream_;
        if (d_g && d.nnz > 0)
            hipLaunchKernelGGL(k_sum_parts, dim3((unsigned)std::min(4096, (d.nnz + 2047) / 2048)), dim3(256), 0, stream,
                               (const float *)d.G[0], net->grad_parts == 2 ? (const float *)d.G[1] : (const float *)nullptr,
                               d.t_perm, d_g, d.nnz);
        if (d_gb && d.n_out > 0)
            hipLaunchKernelGGL(k_apply_bias, dim3((unsigned)((d.n_out + 16 * WAVES_PER_BLOCK - 1) / (16 * WAVES_PER_BLOCK)), 1u),
                               dim3(BLOCK_THREADS), 0, stream, net->d_layers + (layer - 1), net->B, 0.0f, d_gb);
        HIP_TRY(net, hipGetLastError());
        return SDNN_OK;
    }
    return launch_update(net, layer - 1, 1, 0.0f, 1, d_g, d_gb, (hipStream_t)stream_);
}

static int copy_dd(sdnn_net *net, void *dst, const void *src, size_t bytes, void *stream_)
{
    if (bytes) HIP_TRY(net, hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, (hipStream_t)stream_));
    return SDNN_OK;
}

extern "C" int sdnn_get_activation(sdnn_net *net, int32_t layer, float *d_dst, void *stream_)
{
    if (!net) return fail(nullptr, SDNN_EINVAL, "net is NULL");
    if (!net->cfg.training) return fail(net, SDNN_ESTATE, "activations are kept in training mode only");
    if (net->state == ST_IDLE && net->B == 0) return fail(net, SDNN_ESTATE, "no forward pass yet");
    if (layer < 0 || layer > net->n_layers) return fail(net, SDNN_EINVAL, "layer out of range");
    if (!d_dst) return fail(net, SDNN_EINVAL, "d_dst is NULL");
    const float *src = layer == 0 ? net->d_x0 : net->layers[layer - 1].X;
    const size_t n = layer == 0 ? net->layers[0].n_in : net->layers[layer - 1].n_out;
    return copy_dd(net, d_dst, src, 4 * n * net->B, stream_);
}

extern "C" int sdnn_get_delta(sdnn_net *net, int32_t layer, float *d_dst, void *stream_)
{
    if (!net) return fail(nullptr, SDNN_EINVAL, "net is NULL");
    if (!net->cfg.training) return fail(net, SDNN_ESTATE, "deltas are kept in training mode only");
    if (net->state != ST_BACKWARD) return fail(net, SDNN_ESTATE, "no backward pass to read");
    if (layer < 1 || layer > net->n_layers) return fail(net, SDNN_EINVAL, "layer out of range");
    if (!d_dst) return fail(net, SDNN_EINVAL, "d_dst is NULL");
    return copy_dd(net, d_dst, net->layers[layer - 1].D, 4 * (size_t)net->layers[layer - 1].n_out * net->B, stream_);
}

extern "C" int sdnn_get_weights(sdnn_net *net, int32_t layer, float *d_values, float *d_bias, void *stream_)
{
    if (!net) return fail(nullptr, SDNN_EINVAL, "net is NULL");
    if (layer < 1 || layer > net->n_layers) return fail(net, SDNN_EINVAL, "layer out of range");
    const LayerDev &d = net->layers[layer - 1];
    int rc = SDNN_OK;
    if (d_values) rc = copy_dd(net, d_values, d.vals, 4 * (size_t)d.nnz, stream_);
    if (!rc && d_bias) rc = copy_dd(net, d_bias, d.bias, 4 * (size_t)d.n_out, stream_);
    return rc;
}

extern "C" int sdnn_set_weights(sdnn_net *net, int32_t layer, const float *d_values,
                                const float *d_bias, void *stream_)
{
    if (!net) return fail(nullptr, SDNN_EINVAL, "net is NULL");
    if (layer < 1 || layer > net->n_layers) return fail(net, SDNN_EINVAL, "layer out of range");
    const LayerDev &d = net->layers[layer - 1];
    int rc = SDNN_OK;
    if (d_values) {
        rc = copy_dd(net, d.vals, d_values, 4 * (size_t)d.nnz, stream_);
        if (!rc && d.vals_t && d.nnz > 0) { // the transposed-order copy follows at once
            hipLaunchKernelGGL(k_refresh_vals_t, dim3((unsigned)std::min(4096, (d.nnz + 2047) / 2048), 1u), dim3(256), 0,
                               (hipStream_t)stream_, net->d_layers + (layer - 1));
            HIP_TRY(net, hipGetLastError());
        }
    }
    if (!rc && d_bias) {
        rc = copy_dd(net, d.bias, d_bias, 4 * (size_t)d.n_out, stream_);
        if (layer > 1) net->bias_nonpos = false; // device data: its signs are not inspected
    }
    if (!rc && (d_values || d_bias) && d.lm && d.n_blocks > 0) { // keep the lane-major copy current
        hipLaunchKernelGGL(k_lm_refresh, dim3((unsigned)d.n_blocks), dim3(64), 0, (hipStream_t)stream_, net->d_layers + (layer - 1));
        HIP_TRY(net, hipGetLastError());
    }
    return rc;
}

extern "C" int sdnn_layer_shape(const sdnn_net *net, int32_t layer, int32_t *n_out, int32_t *n_in,
                                int64_t *nnz)
{
    if (!net) return fail(nullptr, SDNN_EINVAL, "net is NULL");
    if (layer < 1 || layer > net->n_layers) return fail(nullptr, SDNN_EINVAL, "layer out of range");
    const LayerDev &d = net->layers[layer - 1];
    if (n_out) *n_out = d.n_out;
    if (n_in) *n_in = d.n_in;
    if (nnz) *nnz = d.nnz;
    return SDNN_OK;
}

extern "C" int sdnn_mse_dloss(const float *d_XL, const float *d_Y, int32_t n, int32_t B,
                              float *d_out, void *stream_)
{
    if (!d_XL || !d_Y || !d_out) return fail(nullptr, SDNN_EINVAL, "NULL pointer");
    if (n < 0 || B < 1) return fail(nullptr, SDNN_EINVAL, "bad size");
    const size_t cnt = (size_t)n * B;
    if (!cnt) return SDNN_OK;
    hipLaunchKernelGGL(k_mse_dloss, dim3(ew_blocks(cnt)), dim3(256), 0, (hipStream_t)stream_, d_XL,
                       d_Y, d_out, cnt, (double)B);
    HIP_TRY(nullptr, hipGetLastError());
    return SDNN_OK;
}

extern "C" int sdnn_softmax_ce_dloss(const float *d_XL, const int32_t *d_labels, int32_t n,
                                     int32_t B, int32_t n_classes, float *d_out, void *stream_)
{
    if (!d_XL || !d_labels || !d_out) return fail(nullptr, SDNN_EINVAL, "NULL pointer");
    if (n < 1 || B < 1 || n_classes < 1 || n_classes > n) return fail(nullptr, SDNN_EINVAL, "bad size");
    const size_t cnt = std::max((size_t)(n - n_classes) * B, (size_t)B);
    hipLaunchKernelGGL(k_softmax_ce_dloss, dim3(ew_blocks(cnt)), dim3(256), 0, (hipStream_t)stream_,
                       d_XL, d_labels, d_out, n, B, n_classes);
    HIP_TRY(nullptr, hipGetLastError());
    return SDNN_OK;
}

extern "C" int sdnn_gather_probe(const float *d_table, int32_t table_rows, int32_t v, const int32_t *d_idx,
                                 int32_t n_waves, int32_t per_wave, float *d_out, void *stream_)
{
    if (!d_table || !d_idx || !d_out) return fail(nullptr, SDNN_EINVAL, "NULL pointer");
    if (v != 1 && v != 2 && v != 4) return fail(nullptr, SDNN_EINVAL, "v must be 1, 2 or 4");
    if (table_rows < 1 || n_waves < WAVES_PER_BLOCK || n_waves % WAVES_PER_BLOCK || per_wave < 8 || per_wave % 8)
        return fail(nullptr, SDNN_EINVAL, "table_rows >= 1, n_waves a positive multiple of %d, per_wave a positive multiple of 8",
                    WAVES_PER_BLOCK);
    const size_t bytes = (size_t)table_rows * 256 * (size_t)v;
    if (bytes >= ((size_t)1 << 32)) return fail(nullptr, SDNN_EINVAL, "table of %zu bytes exceeds 4 GiB", bytes);
    const dim3 grid((unsigned)(n_waves / WAVES_PER_BLOCK)), block(BLOCK_THREADS);
    hipStream_t stream = (hipStream_t)stream_;
    if (v == 4) hipLaunchKernelGGL(k_gather_probe<4>, grid, block, 0, stream, d_idx, d_table, bytes, per_wave, d_out);
    else if (v == 2) hipLaunchKernelGGL(k_gather_probe<2>, grid, block, 0, stream, d_idx, d_table, bytes, per_wave, d_out);
    else hipLaunchKernelGGL(k_gather_probe<1>, grid, block, 0, stream, d_idx, d_table, bytes, per_wave, d_out);
    HIP_TRY(nullptr, hipGetLastError());
    return SDNN_OK;
}
