/*
 * sdnn: sparse-DNN feed-forward / back-propagation / SGD update on one AMD
 * MI355X (gfx950).  C ABI; plain pointers and sizes only.
 *
 * The library computes the sequential SGD method for sparse layered networks
 * (Section 3.2, Eqs. 3-7, Algorithm 1) in its minibatch form (Section 5.1:
 * the B sample vectors are the columns of a matrix X and every per-layer
 * product becomes W X):
 *
 *   forward   X_l = f(W_l X_{l-1} + b_l 1^T),  l = 1..L          (Eq. 3)
 *             f(z) = min(max(z, 0), act_cap)   or   1/(1+exp(-z))
 *   backward  Delta_L = dLoss (.) f'(Z_L)                        (Eq. 6)
 *             Delta_{l-1} = (W_l^T Delta_l) (.) f'(Z_{l-1})      (Eq. 7)
 *   update    W_l(j,i) -= lr * sum_s Delta_l(j,s) X_{l-1}(i,s)   (Eqs. 4-5)
 *             for the stored entries (j,i) of W_l only; the sparsity pattern
 *             never changes.  b_l(j) -= lr * sum_s Delta_l(j,s) (the bias is
 *             the weight of a link from a constant-one neuron, Section 3.2).
 *
 * f'(z) is 1 for 0 < z < act_cap and 0 elsewhere (sigmoid: x(1-x)); it is
 * evaluated from the stored output x = f(z).  Back-propagation uses the weights of the forward
 * pass (Algorithm 1 forms delta^{k-1} before it updates W^k); every update is
 * applied by sdnn_sgd_step.  Delta_0 is not formed.
 *
 * Arithmetic: fp32 storage, every sum accumulated in fp64 and rounded once
 * when stored.  No atomics: results are bit-reproducible from run to run.
 *
 * Layouts
 *   W_l        n_out x n_in, CSR: row_ptr int32[n_out+1], col_idx int32[nnz]
 *              (strictly ascending inside a row), values fp32[nnz];
 *              W_l(j,i) links neuron i of layer l-1 to neuron j of layer l.
 *   X, Delta   dense fp32 [neurons][B], row-major: the B samples of one neuron
 *              are contiguous (leading dimension B).
 *
 * Pointers named d_* are DEVICE pointers, all others are HOST pointers.
 * `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 * device work is ordered on that stream and is asynchronous; argument and
 * state errors are reported synchronously.  (For small layers a pass runs its two
 * half-batches concurrently: the second half goes to a helper stream of the net,
 * forked from and joined back into `stream` with events, so the caller sees
 * ordinary stream order.)  The library never allocates device
 * memory: the caller hands in one workspace at sdnn_create and keeps it alive
 * until sdnn_destroy.
 *
 * The three passes allocate nothing and never synchronise, so a caller may
 * capture them in a HIP graph.  A net is not thread-safe: calls on one net must
 * not overlap (different nets are independent).
 *
 * Every function that returns int returns SDNN_OK or a negative code and never
 * throws or aborts; sdnn_last_error gives the message of the last failure.
 */
#ifndef SDNN_H
#define SDNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SDNN_OK 0
#define SDNN_EINVAL (-1) /* null pointer, malformed CSR, size out of range   */
#define SDNN_ESTATE (-2) /* call order violated, or net is not in training mode */
#define SDNN_ENOMEM (-3) /* workspace too small / host allocation failed     */
#define SDNN_EHIP (-4)   /* the HIP runtime reported an error                 */

typedef struct sdnn_net sdnn_net; /* opaque */

/* One layer, HOST arrays, copied by sdnn_create (the caller may free them). */
typedef struct {
    int32_t n_out, n_in;
    const int32_t *row_ptr; /* [n_out+1], row_ptr[0] == 0, non-decreasing      */
    const int32_t *col_idx; /* [nnz], in [0, n_in), strictly ascending per row */
    const float *values;    /* [nnz]                                           */
    const float *bias;      /* [n_out] or NULL (= zeros)                       */
} sdnn_layer;

#define SDNN_ACT_RELU_CAP 0 /* f(z) = min(max(z,0),act_cap); f' = [0 < x < act_cap]                 */
#define SDNN_ACT_SIGMOID 1  /* f(z) = 1/(1+exp(-z)); f' = x(1-x): the paper's training setup (Sec. 6.1) */

typedef struct {
    float act_cap;       /* activation cap; +INFINITY = plain ReLU; must be > 0  */
    int32_t max_batch;   /* largest B a forward call may use (sizes the workspace) */
    int32_t training;    /* 1: keep X_0..X_L and Delta_1..Delta_L; 0: inference only */
    int32_t update_bias; /* 1: sdnn_sgd_step also updates the biases             */
    int32_t activation;  /* SDNN_ACT_RELU_CAP or SDNN_ACT_SIGMOID (act_cap ignored) */
    int32_t fuse_gradient; /* SDNN_FUSE_AUTO / _ON / _OFF, see below               */
    int32_t panel_cols;  /* SDNN_PANEL_AUTO, SDNN_PANEL_OFF, or a panel width > 0, see below */
    int32_t reorder_rows; /* 1: order the rows for gather locality at sdnn_create, see below; 0: longest first */
    int32_t lds_forward; /* SDNN_LDS_AUTO / _ON / _OFF, see below                  */
} sdnn_config;

/* Where the batch allows it, sdnn_backward can form the gradient of the stored entries (Eq. 4) in
 * the same sweep that back-propagates through W_l (Eq. 7): both need the rows of Delta_l that an
 * entry points at.  Short rows (fewer than 128 entries on average): launches of at most 64 samples,
 * i.e. B <= 64, or B = 128 as two halves; long rows: B <= 256 and a multiple of 4 (four samples per
 * lane); one sample per step (B = 1) on a net created with max_batch == 1 whose layers all have 8192
 * inputs or more and short rows (4 more bytes per entry then); other batch sizes take the separate
 * kernels on the same net.  The net then keeps the values
 * a second time, in the order of the transposed index, which that sweep reads in a stream; the
 * gradient is left in the same order, sdnn_sgd_step is a streaming pass over both and rebuilds the
 * CSR copy in a second pass that moves whole runs of entries.  Same results within the rounding of
 * the sum over samples; costs 24 more bytes of workspace per stored entry.  AUTO turns it on for
 * nets whose layers have 4096 rows or more on average (long rows: if max_batch <= 256), where it is
 * faster. */
#define SDNN_FUSE_AUTO 0
#define SDNN_FUSE_ON 1
#define SDNN_FUSE_OFF (-1)

/* Wide layers with short rows (at most 64 entries): the products of Eqs. 3 and 7 can sweep their
 * operand in panels of panel_cols rows, every wavefront carrying several matrix rows through the
 * panels, so that an L2 holds one panel at a time.  Column indices ascend inside a row, so every sum
 * keeps its order: same bits.  AUTO (0) uses it where it is faster (operand tiles of 8 MiB and more,
 * i.e. layers of 32768 neurons and wider); a positive value forces that panel width wherever the
 * rows are short enough; OFF never uses it. */
#define SDNN_PANEL_AUTO 0
#define SDNN_PANEL_OFF (-1)

/* reorder_rows = 1: the order in which the rows of W_l (and of W_l^T) are handed to the wavefronts is chosen
 * for locality of the gathered operand rows instead of by row length alone: rows that share columns
 * are clustered (sdnn_cluster_rows) and every cluster is dealt to one XCD, four neighbours to a
 * workgroup (sdnn_deal_rows_to_xcds), so that an operand row is pulled into one L2 once and reused
 * there.  This is the single-GPU counterpart of the locality that the paper's partitioned runs gain
 * (Section 6.3, the discussion of the time breakdown): only the schedule changes, every sum keeps
 * its order, the results are the same bits.  It pays on structured topologies; on patterns without
 * shared columns (uniformly random links) nothing is gained. */
#define SDNN_CLUSTER_ROWS 256 /* largest cluster */

/* Inference nets (training = 0) whose widest layer has at most 4096 neurons can run sdnn_forward as ONE
 * launch in which a workgroup carries 4 samples through all layers with their activations held in
 * LDS (the samples are independent, Section 5.1, so nothing is exchanged between workgroups); the
 * weights are streamed from a second, lane-major copy that sdnn_create builds (8 more bytes of
 * workspace per stored entry; sdnn_set_weights keeps it current).  Every row still adds its terms
 * in storage order: same bits as the per-layer kernels.  AUTO builds the copy and uses the launch
 * where it is faster (enough samples to fill the chip, or layers so small that per-layer launches
 * are bound by their latency); ON uses it whenever the copy exists; OFF never builds it. */
#define SDNN_LDS_AUTO 0
#define SDNN_LDS_ON 1
#define SDNN_LDS_OFF (-1)

/* ---- setup (Algorithm 1's inputs {W^k}; the paper likewise precomputes its
 *      per-layer index maps once, outside the timed iterations) ------------- */

/* Number of workspace bytes sdnn_create needs for these layers and config. */
int sdnn_workspace_bytes(const sdnn_layer *layers, int32_t n_layers, const sdnn_config *cfg,
                         size_t *bytes);

/* Validates the layers (consecutive layers must agree: n_in(l+1) == n_out(l)),
 * builds the transposed index of every W_l and the row schedules, and copies
 * everything into d_workspace (device, >= workspace bytes; 256-byte aligned at least, a 2 MiB
 * boundary for full speed: the large arrays are placed on multiples of up to 2 MiB from its start).
 * Synchronises `stream` before returning.  On failure *out is NULL. */
int sdnn_create(const sdnn_layer *layers, int32_t n_layers, const sdnn_config *cfg,
                void *d_workspace, size_t workspace_bytes, void *stream, sdnn_net **out);

/* Frees the host-side handle only (the workspace belongs to the caller). */
void sdnn_destroy(sdnn_net *net);

/* ---- the three passes --------------------------------------------------- */

/* Eq. 3 for l = 1..L on a block of B samples (1 <= B <= max_batch).
 * d_X0 [n_in(1)][B] in; d_XL [n_out(L)][B] out (may be NULL in training mode).
 * In training mode X_0..X_L are kept in the workspace (X_0 is copied). */
int sdnn_forward(sdnn_net *net, const float *d_X0, int32_t B, float *d_XL, void *stream);

/* For callers that cannot allocate device memory at all: code running under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc, and so cannot provide the activation buffers that
 * sdnn_forward finds in a freshly allocated workspace.  Same computation and same bits as sdnn_forward on
 * an inference net (training = 0; SDNN_ESTATE otherwise), but the activations between the layers are
 * staged in a fixed array of SDNN_NOALLOC_SCRATCH_BYTES inside the library's device image (every GPU the
 * library runs on holds its own copy until the process ends) instead of the workspace's two buffers.
 * The call allocates nothing (no hipMalloc / hipFree, no allocating library routine).  Limit: one
 * activation block must fit half of the array, 4 * (widest layer) * B <= SDNN_NOALLOC_SCRATCH_BYTES / 2,
 * else SDNN_EINVAL and nothing is launched.  The array keeps the previous call's contents; every element
 * that a call reads it has written before, so nothing needs clearing.  All calls on one GPU share the
 * array: calls that overlap on one GPU (different nets, streams or threads) race; order them. */
#define SDNN_NOALLOC_SCRATCH_BYTES (16u << 20)
int sdnn_forward_noalloc(sdnn_net *net, const float *d_X0, int32_t B, float *d_XL, void *stream);

/* The same result as sdnn_forward on an inference net (training = 0), computed without the samples
 * that have died: with the clamped ReLU and biases <= 0, a sample whose activations are all zero
 * after some layer stays zero in every later layer (Eq. 3 with x = 0 gives f(b) = 0), so its column
 * is dropped.  After every check_every-th layer (>= 1) the live columns are packed to the front of
 * the block on the device; no host synchronisation.  Needs SDNN_ACT_RELU_CAP and every bias of
 * layers 2..L <= 0 as passed to sdnn_create (SDNN_ESTATE otherwise, also after sdnn_set_weights
 * replaced such a bias); B <= 8192 (SDNN_EINVAL otherwise); with B = 1 nothing is packed.
 * d_n_live: NULL, or device int32[1] that receives the number of samples still live after the
 * last check.  The throughput of this call counts edges that were never visited and is reported
 * apart from that of sdnn_forward. */
int sdnn_forward_skip_dead(sdnn_net *net, const float *d_X0, int32_t B, float *d_XL,
                           int32_t check_every, int32_t *d_n_live, void *stream);

/* Eqs. 6-7.  d_dLoss [n_out(L)][B] = dJ/dX_L of the caller's loss, B as in the
 * forward call that must directly precede it.  Training mode only. */
int sdnn_backward(sdnn_net *net, const float *d_dLoss, void *stream);

/* Eqs. 4-5 on every layer, confined to the stored pattern.  Needs a preceding
 * sdnn_backward and consumes it (a second step is SDNN_ESTATE). */
int sdnn_sgd_step(sdnn_net *net, float lr, void *stream);

/* ---- inspection (parity tests, checkpoints) ------------------------------
 * All copy into caller-provided DEVICE buffers on `stream`. */
int sdnn_get_activation(sdnn_net *net, int32_t layer /*0..L*/, float *d_dst, void *stream);
int sdnn_get_delta(sdnn_net *net, int32_t layer /*1..L*/, float *d_dst, void *stream);
/* Eq. 4 without applying it: d_g [nnz(layer)] in CSR order, d_gb [n_out] (either may be NULL).
 * layer in 1..L; needs a preceding sdnn_backward (does not consume it). */
int sdnn_weight_grad(sdnn_net *net, int32_t layer, float *d_g, float *d_gb, void *stream);
int sdnn_get_weights(sdnn_net *net, int32_t layer /*1..L*/, float *d_values, float *d_bias,
                     void *stream);
int sdnn_set_weights(sdnn_net *net, int32_t layer /*1..L*/, const float *d_values,
                     const float *d_bias, void *stream);
/* Sizes of layer 1..L: any output pointer may be NULL. */
int sdnn_layer_shape(const sdnn_net *net, int32_t layer, int32_t *n_out, int32_t *n_in,
                     int64_t *nnz);

/* ---- loss gradients of the two benchmark losses (the library itself is
 *      loss-agnostic: only dJ/dX_L enters, Eq. 6) --------------------------- */

/* J = 1/(2B) sum ||x_s - y_s||^2  =>  d_out = (X_L - Y)/B, all [n][B]. */
int sdnn_mse_dloss(const float *d_XL, const float *d_Y, int32_t n, int32_t B, float *d_out,
                   void *stream);
/* J = -1/B sum_s log softmax(last n_classes rows of X_L)[label_s]
 *  =>  d_out = (softmax - onehot)/B on those rows, 0 elsewhere.  d_labels int32[B]. */
int sdnn_softmax_ce_dloss(const float *d_XL, const int32_t *d_labels, int32_t n, int32_t B,
                          int32_t n_classes, float *d_out, void *stream);

/* ---- measurement aid ---------------------------------------------------------
 * The ceiling of the gather path that the products of Eqs. 3 and 7 depend on: n_waves wavefronts
 * (a multiple of 4) each stream per_wave (a multiple of 8) gathers of rows of 64*v floats (v = 1, 2, 4:
 * one v-float piece per lane) from d_table [table_rows][64*v], the rows given by d_idx
 * [n_waves * per_wave] (each in [0, table_rows): out-of-range rows read as zeros), 8 gathers in flight
 * per wavefront, no arithmetic beyond a running sum stored to d_out [n_waves * 64].  Timed by the caller;
 * bench.py --gather-ceiling tabulates it by table size. */
int sdnn_gather_probe(const float *d_table, int32_t table_rows, int32_t v, const int32_t *d_idx, int32_t n_waves,
                      int32_t per_wave, float *d_out, void *stream);

/* ---- host-only pieces of the setup, exported so they can be checked
 *      without a GPU (all pointers HOST) ------------------------------------ */

/* SDNN_OK or SDNN_EINVAL (message via sdnn_last_error(NULL)). */
int sdnn_check_csr(int32_t n_out, int32_t n_in, const int32_t *row_ptr, const int32_t *col_idx);
/* Transposed index of a pattern: for column i of W, t_row_ptr[i]..t_row_ptr[i+1]
 * lists the rows j (ascending) holding an entry (j,i) in t_row_idx, and in
 * t_perm the position of that entry in the CSR arrays (so W^T needs no second
 * copy of the values).  t_row_ptr [n_in+1], t_row_idx/t_perm [nnz]. */
int sdnn_transpose_pattern(int32_t n_out, int32_t n_in, const int32_t *row_ptr,
                           const int32_t *col_idx, int32_t *t_row_ptr, int32_t *t_row_idx,
                           int32_t *t_perm);
/* Row schedule: the rows ordered by decreasing number of stored entries (the
 * paper's per-row cost, Section 5), ties by ascending row.  order [n_rows]. */
int sdnn_row_schedule(int32_t n_rows, const int32_t *row_ptr, int32_t *order);

/* Greedy clustering of the rows of a pattern by shared columns (one pass; a row joins the open cluster
 * that most of its columns were last used by, if at least a quarter of them were, else it opens a new
 * one; clusters close at max_cluster_rows).  order [n_rows]: the rows cluster by cluster, clusters by
 * decreasing longest row, rows inside a cluster by decreasing length.  cluster_of [n_rows] or NULL:
 * the rank of each row's cluster in that order. */
int sdnn_cluster_rows(int32_t n_rows, int32_t n_cols, const int32_t *row_ptr, const int32_t *col_idx,
                      int32_t max_cluster_rows, int32_t *order, int32_t *cluster_of);
/* Deals a row order out to the 8 XCDs: `order` is cut into 8 contiguous stretches of about equal
 * numbers of entries and stretch x fills the schedule places 32q + 4x .. 32q + 4x + 3, the rows that
 * run on XCD x (workgroups take 4 consecutive rows; workgroup ids go round the XCDs).  dealt [n_rows]. */
int sdnn_deal_rows_to_xcds(int32_t n_rows, const int32_t *row_ptr, const int32_t *order, int32_t *dealt);

/* Message of the last failure on this net, or (net == NULL) of the last
 * failure of a call that had no net, on the calling thread. */
const char *sdnn_last_error(const sdnn_net *net);
const char *sdnn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SDNN_H */
