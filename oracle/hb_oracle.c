/*
 * hb_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 CPU statement of what one Hogbatch GPU-worker mini-batch step
 * computes.  It exists to check the HIP library; it shares no code with it, and only
 * the tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * What it follows in the paper ("Heterogeneous CPU+GPU Stochastic Gradient Descent
 * Algorithms", Ma & Rusu, 2020):
 *   - forward pass, Section 3, Eq. (1): L^{l+1} = F_l(W^l . L^l), W^l in R^{d_{l+1} x d_l};
 *     on a batch the matrix-vector products become matrix-matrix products;
 *   - backward pass, Section 3, Eq. (2): the chain rule from the loss back through the
 *     layers (the equation is schematic; the standard backpropagation recurrences are
 *     written out below);
 *   - update, Section 3, Eq. (3) and Algorithm 1 (worker, "Update model"):
 *     W <- W - eta * g;
 *   - sigmoid hidden units, softmax output and cross-entropy loss, Section 7.1
 *     (Methodology);
 *   - the deep-copied GPU replica and its push to the global model, Section 6.2.
 * Readings where the paper is silent (all listed in the design notes of this repository):
 *   bias vectors b_l are included; the batch gradient is the MEAN over the batch; ReLU
 *   (derivative 0 at 0) and logistic loss are additional choices; the loss returned by a
 *   step is the mean batch loss at the pre-update weights.
 *
 * Conventions: layer_dims = [d_0 .. d_L]; W_l is d_l x d_{l-1} row-major (out x in, the
 * paper's orientation); flat parameter/gradient layout [W_1, b_1, W_2, b_2, ..., W_L, b_L];
 * X is B x d_0 row-major.  Labels: class index in [0, d_L) for softmax cross-entropy;
 * -1/+1 for logistic loss (d_L = 1: margin form; d_L = 2: two-way softmax with class
 * (y+1)/2).
 *
 * Every loop below is the definition itself: no blocking, no fusion, no reordering.  The
 * only concession to run time is an OpenMP "parallel for" over independent output rows.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { HBO_ACT_SIGMOID = 0, HBO_ACT_RELU = 1 };
enum { HBO_LOSS_SOFTMAX_CE = 0, HBO_LOSS_LOGISTIC = 1 };

int hbo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void hbo_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int64_t hbo_num_params(const int32_t *dims, int32_t n_dims)
{
    int64_t p = 0;
    for (int l = 1; l < n_dims; ++l) p += (int64_t)dims[l] * dims[l - 1] + dims[l];
    return p;
}

/* offset of W_l (l = 1..L) in the flat layout; b_l follows it directly */
static int64_t w_offset(const int32_t *dims, int l)
{
    int64_t p = 0;
    for (int j = 1; j < l; ++j) p += (int64_t)dims[j] * dims[j - 1] + dims[j];
    return p;
}

static int check_args(const int32_t *dims, int32_t n_dims, int act, int loss, int64_t B)
{
    if (!dims || n_dims < 2 || B < 1) return -1;
    for (int l = 0; l < n_dims; ++l) if (dims[l] < 1) return -1;
    if (act != HBO_ACT_SIGMOID && act != HBO_ACT_RELU) return -1;
    if (loss != HBO_LOSS_SOFTMAX_CE && loss != HBO_LOSS_LOGISTIC) return -1;
    if (loss == HBO_LOSS_LOGISTIC && dims[n_dims - 1] > 2) return -1;
    return 0;
}

/* nearest bfloat16 (ties to even) of a finite fp32 value */
static float bf16_rne_f32(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) != 0x7f800000u) {
        const uint32_t lower = u & 0xffffu;
        u &= 0xffff0000u;
        if (lower > 0x8000u || (lower == 0x8000u && (u & 0x10000u))) u += 0x10000u;
    } else {
        u &= 0xffff0000u; /* inf/nan: keep the top half */
    }
    memcpy(&f, &u, 4);
    return f;
}

/*
 * Storage rounding of the mixed-precision policy "bf16 activations and weights, fp32
 * master weights and accumulation": a value that the policy keeps in bf16 between two
 * products (a hidden activation, a delta) is the fp32 result rounded to bf16.  With
 * store_bf16 == 0 nothing is rounded.
 */
static double stored(double v, int store_bf16)
{
    return store_bf16 ? (double)bf16_rne_f32((float)v) : v;
}

/* Section 7.1: sigmoid hidden activation; ReLU is the additional choice. */
static double act_fn(int act, double z)
{
    if (act == HBO_ACT_SIGMOID) return 1.0 / (1.0 + exp(-z));
    return z > 0.0 ? z : 0.0;
}

/* derivative of the activation, written in terms of the stored output a = f(z) */
static double act_deriv_from_output(int act, double a)
{
    if (act == HBO_ACT_SIGMOID) return a * (1.0 - a);
    return a > 0.0 ? 1.0 : 0.0; /* relu: z > 0 <=> a > 0; derivative at 0 is 0 */
}

/*
 * Eq. (1) for layers 2..L on a batch, given A_1 (or A_0 when first = 1).
 * acts[l] is B x d_l; acts[L] holds the raw output scores Z_L (the output function is
 * part of the loss below).
 */
static void forward_from(const int32_t *dims, int L, int act, const double *params,
                         double **acts, int64_t B, int first, int store_bf16)
{
    for (int l = first; l <= L; ++l) {
        const int din = dims[l - 1], dout = dims[l];
        const double *W = params + w_offset(dims, l);
        const double *b = W + (int64_t)dout * din;
        const double *Ain = acts[l - 1];
        double *Aout = acts[l];
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < B; ++i) {
            for (int j = 0; j < dout; ++j) {
                double z = b[j];
                for (int k = 0; k < din; ++k) z += Ain[i * din + k] * W[(int64_t)j * din + k];
                Aout[i * dout + j] = (l < L) ? stored(act_fn(act, z), store_bf16) : z;
            }
        }
    }
}

/* first layer on a CSR batch: the sums run over the stored non-zeros only */
static void forward_first_csr(const int32_t *dims, int L, int act, const double *params,
                              const int32_t *row_ptr, const int32_t *col_idx,
                              const double *vals, double *A1, int64_t B)
{
    const int din = dims[0], dout = dims[1];
    const double *W = params;
    const double *b = W + (int64_t)dout * din;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < B; ++i) {
        for (int j = 0; j < dout; ++j) {
            double z = b[j];
            for (int32_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p)
                z += vals[p] * W[(int64_t)j * din + col_idx[p]];
            A1[i * dout + j] = (1 < L) ? act_fn(act, z) : z;
        }
    }
}

/*
 * Loss and output delta (Section 7.1: softmax output, cross-entropy loss; mean over the
 * batch).  Z is B x K; delta (B x K) receives d(mean loss)/dZ.  Returns the mean loss.
 */
static double loss_and_delta(int loss, int K, const double *Z, const int32_t *y, int64_t B,
                             double *delta, int store_bf16)
{
    double total = 0.0;
    for (int64_t i = 0; i < B; ++i) {
        const double *z = Z + i * K;
        if (loss == HBO_LOSS_LOGISTIC && K == 1) {
            /* l = log(1 + exp(-y z)), stable form */
            const double m = (double)y[i] * z[0];
            const double li = (m < 0.0 ? -m : 0.0) + log1p(exp(-fabs(m)));
            /* dl/dz = -y * sigma(-m) */
            const double s = (m >= 0.0) ? exp(-m) / (1.0 + exp(-m)) : 1.0 / (1.0 + exp(m));
            total += li;
            if (delta) delta[i] = stored(-(double)y[i] * s / (double)B, store_bf16);
        } else {
            const int c = (loss == HBO_LOSS_LOGISTIC) ? (y[i] + 1) / 2 : y[i];
            double mx = z[0];
            for (int k = 1; k < K; ++k) if (z[k] > mx) mx = z[k];
            double se = 0.0;
            for (int k = 0; k < K; ++k) se += exp(z[k] - mx);
            const double lse = mx + log(se);
            total += lse - z[c];
            if (delta)
                for (int k = 0; k < K; ++k)
                    delta[i * K + k] =
                        stored((exp(z[k] - lse) - (k == c ? 1.0 : 0.0)) / (double)B, store_bf16);
        }
    }
    return total / (double)B;
}

static double **alloc_acts(const int32_t *dims, int L, int64_t B, int from)
{
    double **a = (double **)calloc((size_t)L + 1, sizeof(double *));
    if (!a) return NULL;
    for (int l = from; l <= L; ++l) {
        a[l] = (double *)malloc(sizeof(double) * (size_t)B * dims[l]);
        if (!a[l]) return NULL;
    }
    return a;
}

static void free_acts(double **a, int L, int from)
{
    if (!a) return;
    for (int l = from; l <= L; ++l) free(a[l]);
    free(a);
}

/*
 * Eq. (2) written out: for l = L..1
 *   dW_l[j,k] = sum_i delta_l[i,j] * A_{l-1}[i,k],  db_l[j] = sum_i delta_l[i,j],
 *   delta_{l-1}[i,k] = (sum_j delta_l[i,j] * W_l[j,k]) * f'(.)          (l > 1)
 * all with the weights the forward pass used.  The first layer's input is either the
 * dense X (csr == 0) or the CSR arrays.
 */
static void backward(const int32_t *dims, int L, int act, const double *params, double **acts,
                     double *delta_L, int64_t B, const double *X, const int32_t *row_ptr,
                     const int32_t *col_idx, const double *vals, double *grad, int store_bf16)
{
    double *delta = delta_L;
    for (int l = L; l >= 1; --l) {
        const int din = dims[l - 1], dout = dims[l];
        const int64_t woff = w_offset(dims, l);
        const double *W = params + woff;
        double *dW = grad + woff;
        double *db = dW + (int64_t)dout * din;
        if (l > 1 || X) {
            const double *Ain = (l > 1) ? acts[l - 1] : X;
#pragma omp parallel for schedule(static)
            for (int j = 0; j < dout; ++j) {
                for (int k = 0; k < din; ++k) {
                    double s = 0.0;
                    for (int64_t i = 0; i < B; ++i) s += delta[i * dout + j] * Ain[i * din + k];
                    dW[(int64_t)j * din + k] = s;
                }
            }
        } else {
            /* sparse first layer: only columns that occur in the batch receive anything */
            memset(dW, 0, sizeof(double) * (size_t)dout * din);
#pragma omp parallel for schedule(static)
            for (int j = 0; j < dout; ++j)
                for (int64_t i = 0; i < B; ++i)
                    for (int32_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p)
                        dW[(int64_t)j * din + col_idx[p]] += delta[i * dout + j] * vals[p];
        }
        for (int j = 0; j < dout; ++j) {
            double s = 0.0;
            for (int64_t i = 0; i < B; ++i) s += delta[i * dout + j];
            db[j] = s;
        }
        if (l > 1) {
            double *prev = (double *)malloc(sizeof(double) * (size_t)B * din);
            const double *Aprev = acts[l - 1];
#pragma omp parallel for schedule(static)
            for (int64_t i = 0; i < B; ++i) {
                for (int k = 0; k < din; ++k) {
                    double s = 0.0;
                    for (int j = 0; j < dout; ++j) s += delta[i * dout + j] * W[(int64_t)j * din + k];
                    prev[i * din + k] =
                        stored(s * act_deriv_from_output(act, Aprev[i * din + k]), store_bf16);
                }
            }
            if (delta != delta_L) free(delta);
            delta = prev;
        }
    }
    if (delta != delta_L) free(delta);
}

/*
 * Mean batch loss and, when grad != NULL, the flat batch gradient [dW_1, db_1, ...].
 * Dense input when X != NULL, else CSR.  Returns NaN on invalid arguments.
 */
static double loss_grad(const int32_t *dims, int32_t n_dims, int act, int loss,
                        const double *params, const double *X, const int32_t *row_ptr,
                        const int32_t *col_idx, const double *vals, const int32_t *y,
                        int64_t B, double *grad, int store_bf16)
{
    if (check_args(dims, n_dims, act, loss, B) != 0 || !params || !y) return NAN;
    const int L = n_dims - 1;
    double **acts = alloc_acts(dims, L, B, 1);
    if (!acts) return NAN;
    if (X) {
        acts[0] = (double *)X;
        forward_from(dims, L, act, params, acts, B, 1, store_bf16);
    } else {
        forward_first_csr(dims, L, act, params, row_ptr, col_idx, vals, acts[1], B);
        forward_from(dims, L, act, params, acts, B, 2, store_bf16);
    }
    const int K = dims[L];
    double *delta = grad ? (double *)malloc(sizeof(double) * (size_t)B * K) : NULL;
    const double mean_loss = loss_and_delta(loss, K, acts[L], y, B, delta, store_bf16);
    if (grad) {
        backward(dims, L, act, params, acts, delta, B, X, row_ptr, col_idx, vals, grad, store_bf16);
        free(delta);
    }
    acts[0] = NULL;
    free_acts(acts, L, 1);
    return mean_loss;
}

/* ---- exported entry points (all arrays fp64 unless stated) ---- */

double hbo_batch_loss(const int32_t *dims, int32_t n_dims, int act, int loss,
                      const double *params, const double *X, const int32_t *y, int64_t B)
{
    if (!X) return NAN;
    return loss_grad(dims, n_dims, act, loss, params, X, NULL, NULL, NULL, y, B, NULL, 0);
}

double hbo_batch_grad(const int32_t *dims, int32_t n_dims, int act, int loss,
                      const double *params, const double *X, const int32_t *y, int64_t B,
                      double *grad)
{
    if (!X || !grad) return NAN;
    return loss_grad(dims, n_dims, act, loss, params, X, NULL, NULL, NULL, y, B, grad, 0);
}

double hbo_batch_grad_csr(const int32_t *dims, int32_t n_dims, int act, int loss,
                          const double *params, const int32_t *row_ptr, const int32_t *col_idx,
                          const double *vals, const int32_t *y, int64_t B, double *grad)
{
    if (!row_ptr || !col_idx || !vals || !grad) return NAN;
    return loss_grad(dims, n_dims, act, loss, params, NULL, row_ptr, col_idx, vals, y, B, grad, 0);
}

/*
 * The same gradient under the mixed-precision storage policy (bf16 activations / deltas,
 * fp32 accumulation): the caller passes X and the weight matrices already rounded to bf16
 * (biases and all sums stay unrounded); hidden activations and deltas are rounded to bf16
 * where the policy stores them.  The update itself is applied by the caller to the fp32
 * master weights with hbo_sgd_update.
 */
double hbo_batch_grad_bf16_storage(const int32_t *dims, int32_t n_dims, int act, int loss,
                                   const double *params, const double *X, const int32_t *y,
                                   int64_t B, double *grad)
{
    if (!X || !grad) return NAN;
    return loss_grad(dims, n_dims, act, loss, params, X, NULL, NULL, NULL, y, B, grad, 1);
}

/* Eq. (3): W <- W - eta * g, over the flat vector */
void hbo_sgd_update(double *params, const double *grad, int64_t P, double lr)
{
    for (int64_t i = 0; i < P; ++i) params[i] = params[i] - lr * grad[i];
}

/* one whole step: gradient at the current weights, then the update; returns the
 * pre-update mean loss */
double hbo_batch_step(const int32_t *dims, int32_t n_dims, int act, int loss, double *params,
                      const double *X, const int32_t *y, int64_t B, double lr)
{
    const int64_t P = hbo_num_params(dims, n_dims);
    double *g = (double *)malloc(sizeof(double) * (size_t)P);
    if (!g) return NAN;
    const double l = hbo_batch_grad(dims, n_dims, act, loss, params, X, y, B, g);
    if (l == l) hbo_sgd_update(params, g, P, lr);
    free(g);
    return l;
}

double hbo_batch_step_csr(const int32_t *dims, int32_t n_dims, int act, int loss,
                          double *params, const int32_t *row_ptr, const int32_t *col_idx,
                          const double *vals, const int32_t *y, int64_t B, double lr)
{
    const int64_t P = hbo_num_params(dims, n_dims);
    double *g = (double *)malloc(sizeof(double) * (size_t)P);
    if (!g) return NAN;
    const double l = hbo_batch_grad_csr(dims, n_dims, act, loss, params, row_ptr, col_idx,
                                        vals, y, B, g);
    if (l == l) hbo_sgd_update(params, g, P, lr);
    free(g);
    return l;
}

/*
 * Replica exchange (Section 6.2: the GPU replica is a deep copy of the global model and
 * is pushed back to it; a stale replica's contribution may be damped).  One reading that
 * covers all three: M = (1-w) H + w D, and afterwards both H and D hold M.
 */
void hbo_model_merge(double *D, double *H, int64_t P, double w)
{
    for (int64_t i = 0; i < P; ++i) {
        const double m = (1.0 - w) * H[i] + w * D[i];
        H[i] = m;
        D[i] = m;
    }
}

/* float32 -> bfloat16 value (returned as float32), round to nearest, ties to even */
void hbo_bf16_round(const float *in, float *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        uint32_t u;
        memcpy(&u, &in[i], 4);
        if ((u & 0x7f800000u) != 0x7f800000u) { /* finite */
            const uint32_t lower = u & 0xffffu;
            u &= 0xffff0000u;
            if (lower > 0x8000u || (lower == 0x8000u && (u & 0x10000u))) u += 0x10000u;
        } else {
            u &= 0xffff0000u; /* inf/nan: keep the top half */
        }
        memcpy(&out[i], &u, 4);
    }
}
