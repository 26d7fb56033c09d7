/*
 * CPU oracle for sparse-DNN SGD: TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow transcription of the sequential method (Section 3.2, Eqs. 3-7,
 * Algorithm 1) in the minibatch form of Section 5.1 (batch vectors are the
 * columns of X).  It is what the HIP library is checked against and shares no
 * code with it.  Only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it.
 *
 * Storage type REAL is chosen at compile time: float (the precision of the GPU
 * path) or double (used only to check the gradients by finite differences).
 * Every sum is accumulated in double, in the order the definition states, and
 * rounded once when stored.
 *
 * Matrices: W is n_out x n_in CSR (row_ptr, col_idx, vals); W(j,i) links neuron
 * i of the previous layer to neuron j of this layer.  Activations and deltas
 * are dense [neurons][B], row-major (one row per neuron, B samples in a row).
 *
 * The OpenMP loops below split independent output elements between threads;
 * the order of the additions inside every sum does not depend on the thread
 * count.
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>

#ifndef REAL
#define REAL float
#endif
#ifndef SUFFIX
#define SUFFIX f32
#endif
#define CAT2(a, b) a##_##b
#define CAT(a, b) CAT2(a, b)
#define FN(name) CAT(name, SUFFIX)

#ifdef _OPENMP
#include <omp.h>
int FN(oracle_threads)(void) { return omp_get_max_threads(); }
/* Thread count of the following calls (timing only; results do not depend on it). */
void FN(oracle_set_threads)(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int FN(oracle_threads)(void) { return 1; }
void FN(oracle_set_threads)(int n) { (void)n; }
#endif

#include <math.h>

/* Two activations (Section 4.1 leaves f open and lists ReLU and the sigmoid among the choices;
 * the paper's training experiments use the sigmoid, Section 6.1):
 *   kind 0: f(z) = min(max(z, 0), cap); cap = +inf gives plain ReLU.  f' is 1
 *           strictly inside (0, cap) and 0 elsewhere, evaluated from the stored
 *           output x = f(z): 0 < x < cap  <=>  0 < z < cap.
 *   kind 1: f(z) = 1 / (1 + exp(-z));  f'(z) = x (1 - x) from the stored x. */
static inline double act(int kind, double z, double cap) {
    if (kind == 1) return 1.0 / (1.0 + exp(-z));
    if (z < 0.0) z = 0.0;
    if (z > cap) z = cap;
    return z;
}
static inline double act_deriv_from_output(int kind, double x, double cap) {
    if (kind == 1) return x * (1.0 - x);
    return (x > 0.0 && x < cap) ? 1.0 : 0.0;
}

/* Eq. 3 / Algorithm 1 (feed-forward step), batch form:  Xout = f(W Xin + b 1^T).
 * z(j,s) = sum over the stored entries of row j, in storage order. */
void FN(oracle_forward_layer)(int32_t n_out, const int32_t *row_ptr, const int32_t *col_idx,
                              const REAL *vals, const REAL *bias, const REAL *Xin, int32_t B,
                              int kind, double cap, REAL *Xout)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int32_t j = 0; j < n_out; ++j) {
        for (int32_t s = 0; s < B; ++s) {
            double z = 0.0;
            for (int32_t p = row_ptr[j]; p < row_ptr[j + 1]; ++p)
                z += (double)vals[p] * (double)Xin[(size_t)col_idx[p] * B + s];
            if (bias) z += (double)bias[j];
            Xout[(size_t)j * B + s] = (REAL)act(kind, z, cap);
        }
    }
}

/* Eq. 6 / Algorithm 1 (output-layer delta):  delta^L = grad_{x^L} J  (.)  f'(z^L). */
void FN(oracle_output_delta)(int32_t n, int32_t B, const REAL *dLoss, const REAL *XL, int kind,
                             double cap, REAL *DL)
{
    for (size_t e = 0; e < (size_t)n * B; ++e)
        DL[e] = (REAL)((double)dLoss[e] * act_deriv_from_output(kind, (double)XL[e], cap));
}

/* Eq. 7 / Algorithm 1 (delta propagation):  Dprev = (W^T D) (.) f'(z_prev).
 * Written as the sparse AXPY form of Section 5 (s(i) += W(j,i) delta(j) for
 * every stored entry), rows j visited in ascending order, so that each s(i)
 * adds its terms by ascending j.  No transposed copy of W is built.
 * If Xprev is NULL no derivative is applied (plain transposed product). */
void FN(oracle_backward_layer)(int32_t n_out, int32_t n_in, const int32_t *row_ptr,
                               const int32_t *col_idx, const REAL *vals, const REAL *D,
                               const REAL *Xprev, int32_t B, int kind, double cap, REAL *Dprev)
{
    double *S = (double *)calloc((size_t)n_in * B, sizeof(double));
#pragma omp parallel for schedule(static)
    for (int32_t s = 0; s < B; ++s) {
        for (int32_t j = 0; j < n_out; ++j) {
            double dj = (double)D[(size_t)j * B + s];
            for (int32_t p = row_ptr[j]; p < row_ptr[j + 1]; ++p)
                S[(size_t)col_idx[p] * B + s] += (double)vals[p] * dj;
        }
    }
    for (size_t e = 0; e < (size_t)n_in * B; ++e) {
        double m = Xprev ? act_deriv_from_output(kind, (double)Xprev[e], cap) : 1.0;
        Dprev[e] = (REAL)(S[e] * m);
    }
    free(S);
}

/* Eq. 4 / Algorithm 1 (weight gradient), confined to the stored entries of W and summed
 * over the samples of the batch:  g(p) = sum_s delta(j,s) x_prev(i,s) for the
 * p-th stored entry (j,i);  bias gradient gb(j) = sum_s delta(j,s) (the bias
 * is the weight of a link from a constant-1 neuron, Section 3.2). */
void FN(oracle_weight_grad)(int32_t n_out, const int32_t *row_ptr, const int32_t *col_idx,
                            const REAL *D, const REAL *Xprev, int32_t B, REAL *g, REAL *gb)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int32_t j = 0; j < n_out; ++j) {
        for (int32_t p = row_ptr[j]; p < row_ptr[j + 1]; ++p) {
            double acc = 0.0;
            for (int32_t s = 0; s < B; ++s)
                acc += (double)D[(size_t)j * B + s] * (double)Xprev[(size_t)col_idx[p] * B + s];
            g[p] = (REAL)acc;
        }
        if (gb) {
            double acc = 0.0;
            for (int32_t s = 0; s < B; ++s) acc += (double)D[(size_t)j * B + s];
            gb[j] = (REAL)acc;
        }
    }
}

/* Eq. 5 / Algorithm 1 (descent step) on an array of parameters:  w <- w - eta * g. */
void FN(oracle_sgd_apply)(size_t n, REAL *w, const REAL *g, double lr)
{
    for (size_t e = 0; e < n; ++e)
        w[e] = (REAL)((double)w[e] - lr * (double)g[e]);
}
