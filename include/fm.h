/*
 * fm.h -- C ABI of the MI355X factorization-machine (FM) pass of DS-FACTO.
 *
 * One GPU, gfx950.  Plain pointers and sizes only.  "HOST" marks host memory,
 * "DEVICE" marks device memory owned by the caller (fp32, contiguous; the arrays
 * with K floats per row -- V, G, grad_V -- 16-byte aligned, FM_EINVAL otherwise).  The
 * library owns only what hangs off an fm_matrix handle.
 *
 * Notation (paper symbol in quotes where it differs):
 *   X        N x D sparse data matrix, rows are examples        (Section 3)
 *   w0,w,V   bias, linear weights [D], latent factors [D x K] row-major (Section 3.2)
 *   a = X w                  linear aggregate                    (2nd term of eq. fm_model2)
 *   G = X V  [N x K]         latent aggregate, the paper's "a_ik" (eq. compute_a_jk)
 *   q_i = sum_j x_ij^2 |v_j|^2   the subtracted square term      (eq. fm_model2)
 *   r [N]                    loss multiplier, the paper's "G_i"  (cases after eq. updates_v)
 *
 * Every function returns FM_OK (0) or a negative fm_status; none throws, aborts
 * or prints.  fm_last_error() gives a message for the last failure on a handle.
 * Work is enqueued on the given hipStream_t (passed as void*; NULL = default
 * stream); only functions with HOST outputs wait for the stream.  One handle
 * must be used by one thread at a time.
 */
#ifndef FM_MI355X_H
#define FM_MI355X_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FM_OK = 0,
    FM_EINVAL = -1,    /* bad argument (null pointer, K out of range, ...) */
    FM_ENOMEM = -2,    /* device or host allocation failed */
    FM_EUNSORTED = -3, /* rowptr not monotone, or columns not strictly ascending in a row */
    FM_ERANGE = -4,    /* index outside [0,D), sizes outside the supported range */
    FM_ESTATE = -5,    /* call needs a structure that was not built yet */
    FM_EHIP = -6       /* a HIP runtime call failed */
} fm_status;

typedef enum { FM_LOSS_SQUARED = 0, FM_LOSS_LOGISTIC = 1 } fm_loss;

typedef struct fm_matrix fm_matrix; /* opaque: device CSR, CSC, stratum index, aggregates, workspace */

/* Hyper-parameters of Table "Notations" (K, lambda_w, lambda_v, eta) and the loss.
 *   loss_scale s multiplies every r_i and the data term of the objective:
 *     s = 1   gives the update equations as printed (eqs. updates_w, updates_v),
 *     s = 1/N gives the normalised objective (eq. fm_obj).
 *   K must be 1..64, or a multiple of 4 up to 256. */
typedef struct {
    int32_t K;
    int32_t loss;              /* fm_loss */
    float lambda_w, lambda_v;  /* regularisers of w and V */
    float eta;                 /* step size */
    float loss_scale;          /* s */
    int32_t update_w0;         /* 0/1: take the bias step w0 -= eta * sum_i r_i */
    int32_t reg_full_per_cell; /* stratified epoch: 0 = a cell step applies the share |I|/N of
                                  lambda (one epoch's worth per epoch); 1 = full lambda each step */
    int32_t refresh_all_rows;  /* stratified epoch: 0 = a cell refreshes only its own rows' aggregates
                                  (Section 4.2: other row blocks stay stale until the re-computation);
                                  1 = every stratum ends with an exact refresh of all rows */
    int32_t stale_aux;         /* stratified epoch: 1 = the two phases of Algorithm 1: every cell step of
                                  the epoch reads the aggregates computed at its start (no refresh between
                                  strata; Section 4.2, staleness), and the next fm_stratified_begin
                                  recomputes them.  Overrides refresh_all_rows. */
    int32_t half_gather;       /* 1 = the passes that gather rows of V (fm_forward, fm_evaluate, the forward of
                                  fm_sgd_epoch and of every batch of fm_minibatch_epoch) read them from a
                                  half-precision copy (IEEE binary16, round to nearest even) that the call
                                  refreshes from V first: the score is that of the model with rounded factors,
                                  sums in fp32; gradient and step use the fp32 V.  Halves the bytes of every
                                  gathered row.  K % 4 == 0.  Beyond the paper (it fixes no precision); the
                                  stratified calls and fm_forward_noalloc return FM_EINVAL with it. */
} fm_params;

/* ---- building the data structures (Section 3: X is read by rows for the score,
 *      by columns for the update of w_j, v_j; Section 4.3: double partition) ---- */

/* Validate a HOST CSR matrix and copy it to the device.  rowptr[0]=0, rowptr[N]=nnz,
 * monotone; inside a row columns strictly ascending and in [0,D).  Stored zeros are
 * legal.  N, D < 2^31, nnz < 2^32.  *out receives a new handle (free with fm_destroy). */
int fm_build_csr(int64_t N, int64_t D, int64_t nnz, const int64_t* rowptr /*HOST N+1*/,
                 const int32_t* col /*HOST nnz*/, const float* val /*HOST nnz*/,
                 void* hip_stream, fm_matrix** out);

/* Device transpose into CSC: rows ascending inside each column (stable). */
int fm_build_csc(fm_matrix* m, void* hip_stream);

/* Double partition into P contiguous row blocks and P contiguous column blocks,
 * block b of n items = [floor(b n/P), floor((b+1) n/P)) in 64-bit arithmetic, and the
 * ring schedule: stratum s holds the P disjoint cells (p, (p+s) mod P), stratum 0 on
 * the diagonal (Section 4.2, figure of the communication pattern).  Builds, for every
 * stratum, the CSR and the CSC of the matrix restricted to that stratum's cells: two re-ordered copies of the
 * entries plus, per stratum, the list of the rows and of the columns that have an entry there (memory
 * proportional to the entries, not to P (N + D)).
 * Needs fm_build_csc.  1 <= P <= 2^20; the table of entries per cell is kept for P <= 4096. */
int fm_partition(fm_matrix* m, int32_t P, void* hip_stream);

/* The same with every column handed from worker to worker on its own (Algorithm 1; Section 4.3: the
 * parameter tuples circulate one by one, initial placement at random).  Rows are split into P floor-split
 * row blocks as above; column j starts at worker place[j] in [0,P) (HOST, D entries, e.g. drawn from a
 * seeded generator) and is handed on after every round against the numbering of the workers: in round
 * s it is at worker (place[j] - s) mod P, and after P rounds it has met every row block once.  Round s
 * takes the place of stratum s in every stratified call (fm_stratified_epoch with stale_aux = 1 is
 * Algorithm 1's update phase followed, at the next epoch's start, by its re-computation loop; without
 * stale_aux a worker refreshes its own rows after every round).  place[j] = column block of j gives
 * fm_partition.  In fm_get_block_index cell_nnz[p*P + c] then counts the entries of row block p in the
 * columns placed at worker c, and col_bounds must be NULL. */
int fm_partition_placed(fm_matrix* m, int32_t P, const int32_t* place /*HOST D*/, void* hip_stream);

/* Copies for bit-exact checks (HOST outputs, sized by the caller). */
int fm_get_csc(const fm_matrix* m, int64_t* colptr /*D+1*/, int32_t* row /*nnz*/, float* val /*nnz*/);
int fm_get_block_index(const fm_matrix* m, int64_t* row_bounds /*P+1*/, int64_t* col_bounds /*P+1*/,
                       int64_t* cell_nnz /*P*P, [p*P+q]; FM_ESTATE for P > 4096*/);
int fm_get_stratum_nnz(const fm_matrix* m, int32_t s, int64_t* nnz_out /*HOST 1*/);
int fm_get_stratum_csr(const fm_matrix* m, int32_t s, int64_t* rowptr /*N+1, starts at 0*/,
                       int32_t* col, float* val);
int fm_get_stratum_csc(const fm_matrix* m, int32_t s, int64_t* colptr /*D+1, starts at 0*/,
                       int32_t* row, float* val);

/* Row batches for fm_minibatch_epoch: B contiguous floor-split row blocks, and for every batch
 * the CSC of the matrix restricted to its rows (rows keep their global numbers, ascending per
 * column).  Needs fm_build_csc.  1 <= B <= 2^20 (B = N is one example per step).  Independent of fm_partition. */
int fm_partition_batches(fm_matrix* m, int32_t B, void* hip_stream);
int fm_get_batch_csc(const fm_matrix* m, int32_t b, int64_t* colptr /*HOST D+1, starts at 0*/,
                     int32_t* row /*HOST*/, float* val /*HOST*/);

/* ---- the pass ---- */

/* Steps 1-3: aggregates, predictions (eq. fm_model2), loss and multipliers.
 *   yhat_i = w0 + a_i + 1/2 (sum_k G_ik^2 - q_i)
 *   squared : l = 1/2 (yhat-y)^2,        r = s (yhat - y)
 *   logistic: l = log(1+exp(-y yhat)),   r = -s y / (1+exp(y yhat)),  y in {-1,+1} (not checked)
 * Any DEVICE output may be NULL.  r and loss_sum need y.  loss_sum (HOST, 1 double)
 * receives sum_i l_i (unscaled) and makes the call wait for the stream. */
int fm_forward(fm_matrix* m, const fm_params* p, const float* y /*DEVICE N, nullable*/,
               const float* w0 /*DEVICE 1*/, const float* w /*DEVICE D*/, const float* V /*DEVICE D*K*/,
               float* yhat /*DEVICE N*/, float* a /*DEVICE N*/, float* G /*DEVICE N*K*/,
               float* q /*DEVICE N*/, float* r /*DEVICE N*/, double* loss_sum /*HOST*/,
               void* hip_stream);

/* fm_forward for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same computation and same DEVICE outputs as
 * fm_forward, from the same kernels; what differs:
 *   - the call allocates and frees nothing and never waits for the stream;
 *   - sums (DEVICE, 2 doubles, nullable; needs y) receives sum_i l_i (unscaled) and sum_i r_i;
 *   - the per-workgroup partial sums live in a static device array of 2 MiB + 16 KiB that every
 *     GPU the library runs on holds until the process ends (its address is resolved when a handle
 *     is created on that GPU).  With sums the row kernel may have at most 262,144 workgroups
 *     (N <= 16,777,216 at K = 16; 64 / lanes-per-row rows per wavefront, 4 wavefronts per
 *     workgroup): larger N return FM_ERANGE.  Nothing in the array has to start at zero;
 *   - all calls on one GPU share that array: calls that overlap in time on one GPU (two streams, two
 *     handles, two threads) race on it when both ask for sums;
 *   - FM_ESTATE while fm_profile_enable is on (the timers create events), or when the current
 *     device is not the one the handle was created on. */
int fm_forward_noalloc(fm_matrix* m, const fm_params* p, const float* y /*DEVICE N, nullable*/,
                       const float* w0 /*DEVICE 1*/, const float* w /*DEVICE D*/, const float* V /*DEVICE D*K*/,
                       float* yhat /*DEVICE N*/, float* a /*DEVICE N*/, float* G /*DEVICE N*K*/,
                       float* q /*DEVICE N*/, float* r /*DEVICE N*/, double* sums /*DEVICE 2*/,
                       void* hip_stream);

/* Predictive performance of (w0, w, V) on this matrix and labels y, as the paper's figures report
 * it (Section 5, test RMSE for regression and test accuracy for classification):
 *   metrics[0] = mean loss (1/N) sum_i l_i   (p->loss; loss_scale is not applied)
 *   metrics[1] = sqrt((1/N) sum_i (yhat_i - y_i)^2)
 *   metrics[2] = fraction of i with sign(yhat_i) == y_i, y in {-1,+1}, yhat_i == 0 counted as +1
 * metrics is HOST 3; the call waits for the stream.  The scores are staged in the handle's aggregate
 * storage: aggregates of an earlier pass are gone afterwards (fm_get_aux then fails with FM_ESTATE). */
int fm_evaluate(fm_matrix* m, const fm_params* p, const float* y /*DEVICE N*/, const float* w0 /*DEVICE 1*/,
                const float* w /*DEVICE D*/, const float* V /*DEVICE D*K*/, double* metrics /*HOST 3*/,
                void* hip_stream);

/* Step 4: gradients of  s sum_i l_i + lambda_w/2 |w|^2 + lambda_v/2 |V|^2  from given r, G
 * (eqs. updates_w0/updates_w/updates_v, regulariser with the sign of gradient descent):
 *   grad_w0 = sum_i r_i
 *   grad_w  = X^T r + lambda_w w
 *   grad_V  = X^T (r . G) - diag((X o X)^T r) V + lambda_v V
 * Atomic-free pass over the CSC copy; needs fm_build_csc.  Outputs may be NULL.  For K that the
 * handle keeps as packed aggregate rows (K % 4 == 0, K <= 28) r and G are first copied into them. */
int fm_gradient(fm_matrix* m, const fm_params* p, const float* r /*DEVICE N*/, const float* G /*DEVICE N*K*/,
                const float* w /*DEVICE D*/, const float* V /*DEVICE D*K*/,
                float* grad_w0 /*DEVICE 1*/, float* grad_w /*DEVICE D*/, float* grad_V /*DEVICE D*K*/,
                void* hip_stream);

/* One full-gradient step (steps 1-5): forward, multipliers, gradient, and
 * (w0, w, V) -= eta * gradient in place, the gradient never being stored.
 * objective (HOST, 2 doubles, nullable): data term s sum_i l_i and regulariser
 * lambda_w/2 |w|^2 + lambda_v/2 |V|^2, both at the parameters the call STARTED from;
 * a non-NULL objective makes the call wait for the stream. */
int fm_sgd_epoch(fm_matrix* m, const fm_params* p, const float* y /*DEVICE N*/,
                 float* w0 /*DEVICE 1*/, float* w /*DEVICE D*/, float* V /*DEVICE D*K*/,
                 double* objective /*HOST 2*/, void* hip_stream);

/* One doubly-separable stratified epoch (Sections 4.2-4.3, synchronous ring):
 *   aggregates a, G, q and multipliers r recomputed from scratch (the re-computation pass);
 *   for s = 0..P-1, all P cells (I_p, J_(p+s) mod P) of the stratum concurrently:
 *       block gradient of the cell's columns over the cell's rows, from r and G as they stand,
 *       step on w_J, V_J (regulariser share per fm_params), deltas kept,
 *       incremental refresh a_I += X_IJ dw_J, G_I += X_IJ dV_J, q_I likewise, r_I recomputed;
 *   bias step from the multipliers as they stand (if update_w0).
 * A column with no entry in its cell only takes the regulariser's step there, as one multiplication
 * by 1 - eta rho lambda; this call may take such steps later (before the column's next step with
 * data, or at the end of the epoch) as one multiplication by their product, formed in fp64: equal to
 * taking them one by one up to the rounding of those fp32 multiplications.
 * With stale_aux the refresh line is skipped (Algorithm 1's update phase).
 * objective (HOST 2, nullable): data term and regulariser from a fresh forward at the
 * FINAL parameters (costs one more pass).  Needs fm_partition. */
int fm_stratified_epoch(fm_matrix* m, const fm_params* p, const float* y, float* w0, float* w, float* V,
                        double* objective /*HOST 2*/, void* hip_stream);

/* One pass of mini-batch gradient descent over the B row batches, in order (Section 4.1: the
 * stochastic updates of w_j and v_jk, taken a batch of examples at a time).  For batch b, rows I_b:
 *   steps 1-3 on the rows of I_b at the parameters as they stand;
 *   gradient of  s sum_{i in I_b} l_i + rho_b (lambda_w/2 |w|^2 + lambda_v/2 |V|^2)  and the step on
 *   w0 (if update_w0), w, V;  rho_b = |I_b|/N, or 1 with reg_full_per_cell.
 * With B = 1 this is fm_sgd_epoch.  objective (HOST 2, nullable): from a fresh forward at the FINAL
 * parameters (costs one more pass).  Needs fm_partition_batches. */
int fm_minibatch_epoch(fm_matrix* m, const fm_params* p, const float* y, float* w0, float* w, float* V,
                       double* objective /*HOST 2*/, void* hip_stream);

/* The three parts of fm_stratified_epoch, for callers that interleave their own work
 * (or inspect the aggregates) between strata: begin = re-computation pass, step = one
 * stratum s, end = bias step. */
int fm_stratified_begin(fm_matrix* m, const fm_params* p, const float* y, const float* w0, const float* w,
                        const float* V, void* hip_stream);
int fm_stratified_step(fm_matrix* m, const fm_params* p, int32_t s, const float* y, const float* w0,
                       float* w, float* V, void* hip_stream);
int fm_stratified_end(fm_matrix* m, const fm_params* p, float* w0, void* hip_stream);

/* Copy the aggregates the handle holds (after fm_sgd_epoch, fm_minibatch_epoch or any stratified
 * call; a and q only after a stratified call; nothing after fm_evaluate: FM_ESTATE) into caller
 * DEVICE arrays; any may be NULL. */
int fm_get_aux(const fm_matrix* m, float* a /*N*/, float* G /*N*K*/, float* q /*N*/, float* r /*N*/,
               void* hip_stream);

/* Per-kernel timing with HIP events on the launch stream.  While enabled, every kernel
 * launch of this handle is bracketed by two events, and kernels that normally overlap on
 * internal side streams run back to back on the launch stream, so that each is timed alone.
 * fm_profile_read waits for the stream, then reports for kernel id k (0 <= k < fm_profile_kernels()) the number of
 * launches and their total time in milliseconds since the last reset, and resets. */
int fm_profile_enable(fm_matrix* m, int32_t on);
int fm_profile_kernels(void);
const char* fm_profile_kernel_name(int32_t k);
int fm_profile_read(fm_matrix* m, int64_t* launches /*HOST nk*/, double* total_ms /*HOST nk*/);

/* Switches between code paths that compute the same thing, per handle; tests run every one of them
 * against the oracle.  Results do not depend on them beyond fp32 rounding.
 *   FM_OPT_AUX_PLANAR    1: the handle keeps the aggregates planar (G [N x K], then r, a, q) for every
 *                        K; 0 (default): as packed rows [G | r | a | q | pad] when [G | r] fits one
 *                        128-byte line (K % 4 == 0, K <= 28).  Changing it drops the aggregates held.
 *   FM_OPT_SIDE_STREAMS  1 (default): column kernels that touch disjoint columns overlap on two
 *                        internal streams; 0: everything on the caller's stream.
 *   FM_OPT_LAZY_REG      1 (default): fm_stratified_epoch and fm_minibatch_epoch postpone the
 *                        regulariser-only steps of columns without entries in a cell or batch; 0: every
 *                        column takes its step in every stratum or batch.
 *   FM_OPT_GRAPH         fm_stratified_epoch replayed from a captured HIP graph: 0 never, 1 (default)
 *                        when there are 32 strata or more, or 16 and strata small enough for the launches
 *                        to dominate, 2 always.
 *   FM_OPT_DENSE_ROWS    1 (default): a matrix in which every row stores all D columns (D and K in
 *                        {32, 64}) takes dense kernels on the matrix cores for fm_forward, fm_gradient and
 *                        fm_sgd_epoch (G = XV and X^T(r.G) as fp32 contractions; the column indices are not
 *                        read); 0: the sparse kernels, as for every other matrix. */
typedef enum {
    FM_OPT_AUX_PLANAR = 0,
    FM_OPT_SIDE_STREAMS = 1,
    FM_OPT_LAZY_REG = 2,
    FM_OPT_GRAPH = 3,
    FM_OPT_DENSE_ROWS = 4
} fm_option;
int fm_set_option(fm_matrix* m, int32_t option /*fm_option*/, int32_t value);

/* Work-decomposition knobs of the column side, per handle, for callers that tune or test them; they
 * must be set before fm_build_csc (FM_ESTATE afterwards).  A value <= 0 keeps the current one.
 *   seg              entries per work item of a long column                      (default 256; the
 *                    per-stratum and per-batch matrices use 256 or 128, chosen per matrix, unless set here)
 *   panel            rows per panel of the L2-blocked traversal of heavy columns (default 32768)
 *   heavy_per_panel  a column is heavy if it averages this many entries per panel (default 16)
 *   vlong            columns with more items are summed by a whole workgroup      (default 512)
 *   min_panels       matrices with fewer panels use plain segments only           (default 64)
 * Results do not depend on these values beyond fp32 rounding. */
int fm_set_tuning(fm_matrix* m, int32_t seg, int32_t panel, int32_t heavy_per_panel, int32_t vlong,
                  int32_t min_panels);
/*   tile_rows     rows of aggregates staged in LDS by the kernel for dense-ish columns
 *   min_per_tile  a column is dense-ish if it averages this many entries per tile; 0 = none
 *   tile_seg      entries per work item inside a tile
 * Defaults follow the shape of the matrix and the latent size of the pass: 1024 / 12 / 512 for tall
 * matrices (N >= 2^21) while two tiles of 1024 rows fit the LDS of a compute unit (K a multiple of
 * 4, K <= 16); 128 / 2 / 128 and 256 / 4 / 256 for matrices of fewer than 2^17 and 2^18 rows; else
 * 512 / 8 / 256.
 * min_per_tile < 0 keeps the current value. */
int fm_set_tile_tuning(fm_matrix* m, int32_t tile_rows, int32_t min_per_tile, int32_t tile_seg);

int fm_destroy(fm_matrix* m);
const char* fm_last_error(const fm_matrix* m); /* m may be NULL: last build error of this thread */

#ifdef __cplusplus
}
#endif
#endif /* FM_MI355X_H */
