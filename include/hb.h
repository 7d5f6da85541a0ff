/*
 * hb.h -- C ABI of the MI355X (gfx950) Hogbatch GPU-worker mini-batch step.
 *
 * The library implements the body of the GPU worker's ExecuteWork handler of the paper
 * "Heterogeneous CPU+GPU Stochastic Gradient Descent Algorithms" (Ma & Rusu, 2020):
 * Algorithm 1 / Algorithm 2, worker side -- "Gradient" then "Update model" -- for a
 * fully-connected network, on a device-resident deep copy of the model (Section 5.1, GPU
 * workers; Section 6.2), at whatever batch size the coordinator assigns (Algorithm 2
 * rescales it by a user-set factor on every request, so B is arbitrary and changes from
 * call to call), plus the replica <-> global-model exchange of Section 6.2.
 *
 * Conventions
 *   layer_dims = [d_0, d_1, ..., d_L], n_dims = L + 1 >= 2.
 *   W_l is d_l x d_{l-1}, row-major (out x in: the orientation of Section 3, W^l in
 *   R^{d_{l+1} x d_l}); b_l has d_l entries.
 *   Flat parameter / gradient layout, fp32, P = sum_l (d_l d_{l-1} + d_l) elements:
 *       [W_1, b_1, W_2, b_2, ..., W_L, b_L].
 *   X is B x d_0 row-major (one example per row, Section 3), a DEVICE pointer: fp32 in
 *   HB_F32 mode, bfloat16 in HB_BF16_F32MASTER mode.
 *   y is a DEVICE pointer to B int32 labels: class index in [0, d_L) for
 *   HB_LOSS_SOFTMAX_CE; -1 / +1 for HB_LOSS_LOGISTIC (d_L = 1: loss on the margin
 *   y * z; d_L = 2: two-way softmax with class (y + 1) / 2).  Labels are not range-checked;
 *   an out-of-range label cannot cause an out-of-bounds access, only a wrong loss.  With
 *   HB_CHECK_LABELS=1 in the environment every batch call first counts them on the device
 *   (one more pass over y and a synchronisation) and fails with HB_ERR_INVALID if there are any.
 *   The batch gradient is the MEAN over the batch of the per-example gradients; the
 *   loss a step returns is the mean batch loss at the weights before the update.
 *
 * Ownership: the handle owns every device buffer it uses (replica, gradient partials,
 * activations sized for max_B).  The caller owns X, y, the CSR arrays, gradient output
 * buffers and the host model; nothing of the caller's is retained after a call returns,
 * except that *_async calls read their inputs until the stream reaches that point.
 *
 * Threading: one handle is driven by one thread at a time (the GPU worker is the
 * exclusive interface of its device, Section 5.1).  hb_model_merge reads and writes the
 * host model without any atomicity with respect to other host threads (Hogbatch updates
 * the shared model without synchronisation, Section 6.1).
 *
 * Errors: int-returning calls give HB_OK or a negative code; float-returning calls give
 * a quiet NaN on error; hb_mlp_create gives NULL.  hb_last_error() then describes the
 * failure.  Every argument check happens before any device call.
 */
#ifndef HB_H
#define HB_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hb_model hb_model;

enum { HB_ACT_SIGMOID = 0, HB_ACT_RELU = 1 };
enum { HB_LOSS_SOFTMAX_CE = 0, HB_LOSS_LOGISTIC = 1 };
enum { HB_F32 = 0, HB_BF16_F32MASTER = 1 };
enum {
    HB_OK = 0,
    HB_ERR_INVALID = -1,     /* bad argument */
    HB_ERR_ALLOC = -2,       /* host or device allocation failed */
    HB_ERR_DEVICE = -3,      /* a HIP call failed */
    HB_ERR_UNSUPPORTED = -4, /* valid request this build does not implement */
    HB_ERR_STATE = -5        /* call made in the wrong state (e.g. step before configure) */
};

/*
 * Describe the network (Section 5.2, initialisation: the model configuration is passed to
 * the GPU worker).  Host-only: touches no device.  activation applies to the hidden layers
 * (sigmoid per Section 7.1, or ReLU); loss is softmax cross-entropy (Section 7.1) or
 * logistic (needs d_L <= 2).  layer_dims is a HOST pointer, copied.  NULL on error.
 */
hb_model *hb_mlp_create(const int32_t *layer_dims, int32_t n_dims, int activation, int loss);

/*
 * Allocate the device replica and the workspace for batches of up to max_B rows (Section
 * 5.2, initialisation: a GPU worker allocates its device memory up front).  dtype: HB_F32 or
 * HB_BF16_F32MASTER (bf16 weights/activations, fp32 master weights and accumulation).
 * sparse_first_layer != 0 selects CSR input for layer 1 (then only the *_csr step calls
 * are valid, and only HB_F32).  hip_stream is a hipStream_t (NULL = the default stream)
 * on which every kernel and copy of this handle is issued; the device current at this
 * call is the handle's device.  Parameters start as zeros.  May be called once.
 */
int hb_mlp_configure(hb_model *m, int dtype, int64_t max_B, int sparse_first_layer,
                     void *hip_stream);

/* Free everything the handle owns.  NULL is allowed. */
void hb_model_destroy(hb_model *m);

/* P, the length of the flat parameter vector.  -1 if m is NULL. */
int64_t hb_model_num_params(const hb_model *m);

/* Replica <- host_flat (HOST pointer, P floats).  Synchronises the stream. */
int hb_model_set_params(hb_model *m, const float *host_flat);

/* host_flat <- replica (fp32 master weights).  Synchronises the stream. */
int hb_model_get_params(hb_model *m, float *host_flat);

/*
 * host_out <- the hidden activations A_layer (Section 3, Eq. (1)) that the most recent batch call
 * of this handle computed for its first B rows: B x d_layer fp32, row-major, HOST pointer;
 * 1 <= layer < L.  In the bf16 mode the stored bf16 values are widened (exactly).  For
 * inspection and tests: it shows which hidden units a ReLU network switched on.  Synchronises the
 * stream.  The contents are those of whichever call ran last (step, gradient or loss).
 */
int hb_model_get_activations(hb_model *m, int32_t layer, int64_t B, float *host_out);

/*
 * One GPU-worker step (Algorithm 1, worker lines "Gradient" and "Update model"; Section 3,
 * Eq. (1) forward, Eq. (2) backward, Eq. (3) W <- W - lr * g) on the replica, for the
 * B rows at dX / dy (DEVICE pointers), 1 <= B <= max_B.  Returns the pre-update mean
 * loss after synchronising the stream; NaN on error.
 */
float hb_batch_step(hb_model *m, const void *dX, const int32_t *dy, int64_t B, float lr);

/*
 * Same step without any host synchronisation: the mean loss is written to *d_loss (DEVICE
 * pointer, one float, may be NULL) when the stream reaches that point.  For dense input the
 * call enqueues kernels only (no memset or copy, no allocation), so it may be recorded by a
 * stream capture on the handle's stream once one ordinary call has been made; a replay does
 * what the call did (same pointers, B and lr).  Replay is no faster than calling: the host
 * already runs ahead of the device.
 */
int hb_batch_step_async(hb_model *m, const void *dX, const int32_t *dy, int64_t B, float lr,
                        float *d_loss);

/*
 * The step for a CSR batch (sparse first layer; the paper processes its data densely and
 * names sparse input as future work in Section 8 -- this is the benchmark's
 * real-sim-shaped configuration).  d_row_ptr: B + 1 int32 starting at 0; d_col_idx /
 * d_vals: nnz entries, column indices in [0, d_0), any order within a row (DEVICE
 * pointers).  nnz must equal d_row_ptr[B]; it is passed so that no device read is needed
 * to size the launch.  A column may occur more than once in a row (the products add).
 * Column indices and the row pointer are trusted: an index outside [0, d_0) is an
 * out-of-bounds access.  With HB_CHECK_INDICES=1 in the environment every CSR call first
 * checks them on the device (one more pass over the arrays and a synchronisation) and fails
 * with HB_ERR_INVALID before any kernel dereferences them.  Only the weight columns that occur
 * in the batch are touched.
 * The CSR arrays are also read by a stream the handle owns (the per-batch column sort runs
 * beside the forward pass); that work is joined into the handle's stream before the step ends
 * there, so "until the stream reaches the end of the step" still bounds every read.
 */
float hb_batch_step_csr(hb_model *m, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                        const float *d_vals, int64_t nnz, const int32_t *dy, int64_t B,
                        float lr);
int hb_batch_step_csr_async(hb_model *m, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                            const float *d_vals, int64_t nnz, const int32_t *dy, int64_t B,
                            float lr, float *d_loss);

/*
 * Gradient only (Section 6.2: the stale-replica alternative computes the gradient on the
 * replica and lets the caller apply it to the current global model).  The replica is
 * left untouched; d_grad_flat (DEVICE pointer, P floats, flat layout) receives the mean
 * gradient.  Returns the mean loss after synchronising; NaN on error.
 */
float hb_batch_grad(hb_model *m, const void *dX, const int32_t *dy, int64_t B,
                    float *d_grad_flat);
float hb_batch_grad_csr(hb_model *m, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                        const float *d_vals, int64_t nnz, const int32_t *dy, int64_t B,
                        float *d_grad_flat);

/*
 * Forward pass and mean loss only, no gradient, no update (Section 5.2: the loss is
 * evaluated with a forward pass over batches that fit the worker's memory).
 */
float hb_batch_loss(hb_model *m, const void *dX, const int32_t *dy, int64_t B);

/*
 * The same forward pass without host synchronisation: the mean loss of the B rows is written
 * to *d_loss (DEVICE pointer, one float, may be NULL) in stream order.  Dense input.
 */
int hb_batch_loss_async(hb_model *m, const void *dX, const int32_t *dy, int64_t B, float *d_loss);

/*
 * hb_batch_loss_async for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  No handle is needed: the
 * network is described as for hb_mlp_create (HOST pointer layer_dims), d_params is the flat
 * fp32 parameter vector on the DEVICE (P floats, 16-byte aligned, only read), dX is B x d_0 fp32
 * row-major and dy B int32 labels (DEVICE pointers), d_loss (DEVICE pointer, one float, required)
 * receives the mean loss of the B rows in stream order on hip_stream (a hipStream_t, NULL = the
 * default stream).  Dense fp32 input only.  The call allocates and frees nothing on the device
 * and does not synchronise: the activations and the per-block loss sums live in a workspace of
 * HB_STATIC_SCRATCH_BYTES that is part of the library's device image (every device the library
 * is loaded on holds one copy until the process ends).  A batch whose activations
 * (sum over l >= 1 of B x d_l floats, rows padded to 4 floats) and loss sums do not fit is
 * HB_ERR_UNSUPPORTED; nothing has been launched then.  Every call on a device shares that
 * device's workspace, which keeps the previous call's contents (each call overwrites all it
 * reads): calls on one device whose execution may overlap -- different streams, or host threads
 * whose streams are not ordered -- race; calls on one stream are safe.  The result is the one
 * hb_batch_loss_async gives for a replica holding d_params (the same kernels run).
 */
#define HB_STATIC_SCRATCH_BYTES (64u << 20)
int hb_batch_loss_static(const int32_t *layer_dims, int32_t n_dims, int activation, int loss,
                         const float *d_params, const float *dX, const int32_t *dy, int64_t B, float *d_loss,
                         void *hip_stream);

/* Forward pass and mean loss of a CSR batch (arguments as hb_batch_step_csr), with and without
 * host synchronisation. */
float hb_batch_loss_csr(hb_model *m, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                        const float *d_vals, int64_t nnz, const int32_t *dy, int64_t B);
int hb_batch_loss_csr_async(hb_model *m, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                            const float *d_vals, int64_t nnz, const int32_t *dy, int64_t B,
                            float *d_loss);

/*
 * Replica <-> global model exchange (Section 6.2: the replica is a deep copy of the
 * global model, pushed back to it after the update; a stale replica's contribution can be
 * damped).  With H = host_model (HOST pointer, P floats, flat layout; pinned memory makes
 * the copies asynchronous) and D = the device replica:
 *     M = (1 - weight) * H + weight * D,   then   H <- M and D <- M.
 * weight = 0: replica <- global (the deep copy on ExecuteWork); weight = 1: global <-
 * replica (the push); 0 < weight < 1: damped push.  weight outside [0, 1] or NaN is
 * HB_ERR_INVALID.  Synchronises the stream before returning.
 */
int hb_model_merge(hb_model *device_replica, float *host_model, float weight);

/* Message and code of the last failing call on this thread ("" / HB_OK if none). */
const char *hb_last_error(void);
int hb_last_error_code(void);

/*
 * Per-kernel timing, for measurement only (the benchmark's roofline figures).  While
 * enabled, every kernel of a step is launched with a pair of events attached to its own
 * dispatch, so that the recorded time is the kernel's execution time and nothing else.
 * hb_profile_read synchronises the stream, adds up what was recorded since the last read
 * into one entry per (kind, layer), writes at most cap entries to out (HOST pointer),
 * stores the number of entries in *n_out and clears the record.
 */
enum {
    HB_K_FWD_GEMM = 0,   /* Z_l = A_{l-1} W_l^T + b_l, activation          (Eq. (1)) */
    HB_K_DA_GEMM = 1,    /* delta_{l-1} = (delta_l W_l) * f'                (Eq. (2)) */
    HB_K_DW_GEMM = 2,    /* dW_l = delta_l^T A_{l-1}, db_l (split-K partials) (Eq. (2)) */
    HB_K_LOSS = 3,       /* loss and output delta                           (Section 7.1) */
    HB_K_UPDATE = 4,     /* W <- W - lr * sum of partials, all tensors      (Eq. (3)) */
    HB_K_SPMM_FWD = 5,   /* CSR first layer, forward */
    HB_K_SPARSE_DW = 6,  /* CSR first layer, gradient + update of the touched columns */
    HB_K_OTHER = 7,
    HB_K_OUT_LAYER = 8,  /* narrow output layer: forward + loss + delta + its gradients, fused */
    HB_K_BWD_PAIR = 9    /* backward-data and weight-gradient product of one layer in one launch;
                            M, N, K are the backward-data shape, flops / bytes cover both */
};
typedef struct hb_kernel_stat {
    int32_t kind;            /* HB_K_* */
    int32_t layer;           /* 1..L, or 0 when the kernel is not per layer */
    int64_t M, N, K;         /* product shape C[M x N] += A[M x K] B[K x N]; 0 if not a product */
    int64_t launches;
    double total_ms;         /* sum of the kernel execution times */
    double flops_per_launch; /* algorithmic: 2 M N K for a product */
    double bytes_per_launch; /* algorithmic HBM bytes: each operand read once, result written once */
    double cache_bytes_per_launch; /* CSR kernels: bytes of the row gathers (one weight / delta row per
                                      stored entry), served by the caches; 0 elsewhere */
} hb_kernel_stat;
int hb_profile_enable(hb_model *m, int on);
int hb_profile_read(hb_model *m, hb_kernel_stat *out, int32_t cap, int32_t *n_out);

/*
 * Planning aid, host only (no device call): the number of slices of the batch in which the bf16
 * mode computes the weight gradient dW_l = D_l^T A_{l-1} (Eq. (2)) of a d_out x d_in layer at batch
 * size B -- products with too few output tiles to fill the device are split over the batch and
 * their partial sums added in a fixed order; 1 = not split.  With capacity != 0: the largest
 * count any batch size up to B can get, which is what hb_mlp_configure(max_B = B) reserves room
 * for.  0 on invalid arguments.
 */
int32_t hb_plan_bf16_dw_slices(int32_t d_out, int32_t d_in, int64_t B, int32_t capacity);

/* Library version string, e.g. for logs. */
const char *hb_version(void);

/*
 * ---- Adaptive Hogbatch scheduling and the GPU worker's loop --------------------------------
 *
 * hb_sched is the coordinator's ScheduleWork handler of Algorithm 2 (Section 6.3): host-only
 * state, no device calls.  It keeps, for each of n_workers workers E, the number of model
 * updates u^E last reported and the batch size b^E with thresholds min_b^E <= b^E <=
 * max_b^E, the factor alpha (> 1; the paper's default is 2) and the examples of the current
 * epoch not yet handed out, a contiguous range [cursor, n_examples).
 *
 * hb_sched_request(s, E, u, &begin, &count) is one ScheduleWork message: it records u^E = u;
 * if u^E is below the smallest update count of all OTHER workers, b^E <- max(b^E / alpha,
 * min_b^E); else if it is above their largest, b^E <- min(b^E * alpha, max_b^E) (b^E / alpha
 * and b^E * alpha rounded to the nearest integer, at least 1; a single worker is never
 * rescaled); then, if b^E examples are left, *begin / *count name the next b^E of them
 * (they are removed from the epoch), else *count = 0: nothing is sent and the worker is
 * done for this epoch.  Requests are served one at a time (internally locked), as the
 * coordinator serves them serially.  u is a double because a CPU worker reports
 * t * beta updates per batch (Algorithm 2, CPU worker).
 * hb_sched_new_epoch makes the whole training set available again (Section 6.1: the process
 * is restarted with the full dataset); update counts and batch sizes carry over.
 * The arrays min_b, max_b, init_b have n_workers entries (HOST pointers, copied).
 */
typedef struct hb_sched hb_sched;
hb_sched *hb_sched_create(int64_t n_examples, int32_t n_workers, const int64_t *min_b, const int64_t *max_b,
                          const int64_t *init_b, double alpha);
void hb_sched_destroy(hb_sched *s);
int hb_sched_request(hb_sched *s, int32_t worker, double updates, int64_t *begin, int64_t *count);
int hb_sched_new_epoch(hb_sched *s);
int64_t hb_sched_batch_size(const hb_sched *s, int32_t worker); /* current b^E; -1 on error */
int64_t hb_sched_remaining(const hb_sched *s);                  /* examples left in the epoch; -1 on error */

/*
 * The GPU worker's share of one epoch (Section 5.1, GPU workers; Section 6.2): until the
 * coordinator sends nothing more, ask for a batch (reporting one model update per step taken),
 * copy its rows from the HOST-resident training data to the device on a copy stream while the
 * previous batch is still computing, and run the step on the replica with
 * lr = lr_per_example * b (learning rate proportional to the batch size, Section 6.2).
 * Every merge_every steps (and once at the end if any step is unmerged) the replica is merged
 * with host_model as hb_model_merge(m, host_model, merge_weight) does; merge_every = 0 or
 * host_model = NULL: never.  No merge waits for the device.  merge_weight = 1 (the push of
 * Section 6.2): the replica is snapshot in stream order and travels to host_model on a third
 * stream while the next steps run (the copy is issued once the next step has been enqueued;
 * directly if host_model is page-locked, else through a page-locked buffer and a host copy).  merge_weight < 1: host_model is first copied to the
 * device on that stream (read at the merge point of the host's program order, which runs ahead
 * of the device by at most one exchange), blended with the replica in stream order, and the
 * blend travels back like a push (not for weight 0).  Every transfer has landed when the call
 * returns.  While the call runs, host_model may be read and written at any time; what other
 * workers write to it between the read and the landing of the blend is overwritten.
 *   host_X  n_examples x d_0 row-major in HOST memory (fp32, or bfloat16 in the bf16 mode),
 *           page-locked memory makes the copies asynchronous;  host_y  n_examples int32.
 *   *updates (in/out, may be NULL -> starts at 0): the worker's update count u^E, carried
 *   from epoch to epoch;  *steps_out, *loss_sum_out (may be NULL): steps taken in this call and
 *   the sum of their pre-update mean losses.
 * The request for batch k+1 is made while batch k computes, with the update count batch k
 * will have produced.  The host waits for a batch's copy to land before it enqueues the step
 * (it runs one step ahead of the device); HB_WORKER_STREAMWAIT=1 in the environment makes the
 * device wait instead.  Dense input only (HB_ERR_UNSUPPORTED for a CSR model, which
 * hb_worker_run_epoch_csr serves); the scheduler's max_b of this worker must not exceed the
 * model's max_B.  Synchronises the model's stream before returning.
 */
int hb_worker_run_epoch(hb_model *m, hb_sched *s, int32_t worker, const void *host_X, const int32_t *host_y,
                        float lr_per_example, float *host_model, int32_t merge_every, float merge_weight,
                        double *updates, int64_t *steps_out, double *loss_sum_out);

/*
 * The same loop for a model configured with sparse_first_layer, over HOST-resident CSR training
 * data (sparse input is the future work of Section 8; the loop is that of Section 5.1 / 6.2
 * unchanged): host_row_ptr has n_examples + 1 non-decreasing int64 entries, host_col_idx /
 * host_vals the stored entries (column indices in [0, d_0): every batch's indices are checked on
 * the host before the batch is sent, and one outside the range is HB_ERR_INVALID).
 * For each batch the slice of the row pointer is rebased to start at 0 on the host (into a
 * page-locked array of the handle) and travels with the batch's column indices, values and
 * labels on the copy stream while the previous batch computes; the step is
 * hb_batch_step_csr_async.  The device buffers for indices and values grow on demand (with a
 * stream synchronisation when they do).  A batch with more than 2^31 - 1 stored entries, or a
 * row pointer that decreases, is HB_ERR_INVALID (the steps taken until then stay applied).
 * Merging, update counts and outputs are those of hb_worker_run_epoch; HB_ERR_UNSUPPORTED for a
 * dense model.
 */
int hb_worker_run_epoch_csr(hb_model *m, hb_sched *s, int32_t worker, const int64_t *host_row_ptr,
                            const int32_t *host_col_idx, const float *host_vals, const int32_t *host_y,
                            float lr_per_example, float *host_model, int32_t merge_every, float merge_weight,
                            double *updates, int64_t *steps_out, double *loss_sum_out);

/*
 * Loss of the replica over a HOST-resident dataset (the evaluation stage of Section 5.2: the
 * loss is computed at the end of an epoch, by a forward pass over all examples in sub-batches
 * that fit the device): rows [0, n_examples) are sent in pieces of at most `batch` rows
 * (<= max_B) through the same double-buffered transfer as the worker loop, hb_batch_loss's
 * forward pass runs on each (asynchronously: the piece means are collected on the device and
 * fetched 256 at a time), and *mean_loss receives the mean over all n_examples (the piece
 * means weighted by their sizes, accumulated in double).  The replica is not modified.
 */
int hb_worker_eval_loss(hb_model *m, const void *host_X, const int32_t *host_y, int64_t n_examples, int64_t batch,
                        double *mean_loss);
/* The same evaluation over HOST-resident CSR data (arrays as for hb_worker_run_epoch_csr) for a
 * model configured with sparse_first_layer; the pieces run through hb_batch_loss_csr_async. */
int hb_worker_eval_loss_csr(hb_model *m, const int64_t *host_row_ptr, const int32_t *host_col_idx,
                            const float *host_vals, const int32_t *host_y, int64_t n_examples, int64_t batch,
                            double *mean_loss);

/*
 * The CPU worker's share of one epoch (Algorithm 2, CPU worker; Sections 6.1-6.3), host code
 * only: until the coordinator sends nothing more, ask for a batch, split it into `threads`
 * contiguous sub-batches (sizes differ by at most one), let one thread per sub-batch compute
 * the mean gradient of its sub-batch on the SHARED fp32 host model (Eq. (1)-(2)) and apply it
 * with lr = lr_per_example * (sub-batch size) (Eq. (3)) without locks or atomics, then count
 * threads * beta model updates (beta in (0, 1]: the fraction of conflicting updates assumed to
 * survive).  With a batch of `threads` examples this is Hogwild.  The network is described as
 * for hb_mlp_create; host_model uses the flat layout; host_X is fp32.  *updates is in/out as
 * for the GPU worker; *batches_out, *loss_sum_out (may be NULL): batches taken and the sum
 * over batches and threads of the sub-batch mean losses.  With threads = 1 the result is
 * deterministic: plain sequential mini-batch SGD in fp32.
 */
int hb_cpu_worker_run_epoch(hb_sched *s, int32_t worker, const int32_t *layer_dims, int32_t n_dims, int activation,
                            int loss, const float *host_X, const int32_t *host_y, float *host_model,
                            float lr_per_example, int32_t threads, double beta, double *updates,
                            int64_t *batches_out, double *loss_sum_out);

/*
 * One epoch of CPU+GPU Hogbatch / Adaptive Hogbatch (Sections 6.2-6.3, Algorithm 2) with one CPU
 * worker and one GPU worker: hb_cpu_worker_run_epoch runs as worker `cpu_worker` of the
 * scheduler on a thread started for it, hb_worker_run_epoch as worker `gpu_worker` on the
 * calling thread, both over the same fp32 rows host_X / host_y and the same host_model (the
 * global model, P floats): the CPU threads update it in place without locks, the GPU replica
 * `gpu` (HB_F32, dense; its network is also the CPU worker's) is merged with it every
 * merge_every (>= 1) steps with merge_weight as in hb_worker_run_epoch.  Fixed batch sizes
 * (min_b = max_b in the scheduler) give CPU+GPU Hogbatch, a range gives Adaptive Hogbatch.
 * The call returns when neither worker is sent anything more.  *gpu_updates / *cpu_updates
 * (in/out, may be NULL -> start at 0) carry the workers' update counts from epoch to epoch;
 * *stats (may be NULL) receives the steps / batches taken and the sums of their pre-update mean
 * losses.  The replica should hold the global model when the first epoch starts
 * (hb_model_set_params or hb_model_merge with weight 0).  If a worker fails, the other one still
 * finishes the epoch and the first error (the GPU worker's, if both) is returned.
 */
typedef struct hb_epoch_stats {
    int64_t gpu_steps, cpu_batches;
    double gpu_loss_sum, cpu_loss_sum;
} hb_epoch_stats;
int hb_hogbatch_run_epoch(hb_sched *s, hb_model *gpu, int32_t gpu_worker, int32_t cpu_worker, const float *host_X,
                          const int32_t *host_y, float *host_model, float lr_per_example, int32_t cpu_threads,
                          double beta, int32_t merge_every, float merge_weight, double *gpu_updates,
                          double *cpu_updates, hb_epoch_stats *stats);

#ifdef __cplusplus
}
#endif
#endif /* HB_H */
