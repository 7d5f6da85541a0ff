// Internal declarations shared by the HIP translation units of libhb (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

struct hb_model;

namespace hb {

// Optional pair of events attached to one kernel dispatch: their elapsed time is that
// kernel's own execution time (used by the per-kernel profile the benchmark reads).
struct LaunchEvents {
    hipEvent_t start = nullptr;
    hipEvent_t stop = nullptr;
};

template <typename F, typename... Args>
inline hipError_t launch_kernel(F kernel, dim3 grid, dim3 block, hipStream_t stream,
                                const LaunchEvents &ev, Args... args)
{
    if (ev.start != nullptr)
        hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, ev.start, ev.stop, 0, args...);
    else
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, args...);
    return hipGetLastError();
}

// ---------------------------------------------------------------- fp32 MFMA GEMM
// C[M x N] (+)= sum_k A(m,k) * B(n,k), fp32 operands, fp32 MFMA accumulation.
//   A K-major: A(m,k) = A[m*lda + k];  A M-major: A(m,k) = A[k*lda + m]  (same for B).
// The three layer products of the step map onto it as
//   forward   Z_l       = A_{l-1} . W_l^T      (A K-major, B K-major, epilogue FWD)
//   backward  D_{l-1}   = (D_l . W_l) * f'     (A K-major, B M-major, epilogue DA)
//   gradient  dW_l      = D_l^T . A_{l-1}      (A M-major, B M-major, epilogue DW, split over K = batch)
enum GemmKind { GEMM_FWD = 0, GEMM_DA = 1, GEMM_DW = 2 };
enum { ACT_NONE = -1, ACT_SIGMOID = 0, ACT_RELU = 1 };

struct GemmArgs {
    const void *A;
    const void *B;
    void *C;
    int M, N, K;
    int lda, ldb, ldc;
    int a_vec, b_vec;          // 16-byte vector loads are legal for this operand
    int splits;                // gridDim.y; slice s covers k in [s*k_chunk, min(K,(s+1)*k_chunk))
    int k_chunk;               // multiple of the kernel's BK
    long long c_split_stride;  // elements between the C slices of successive splits
    const float *bias;         // FWD: bias[N] (may be null)
    const void *aux;           // DA: stored output of the layer whose derivative is applied
    int ldaux;
    float *colsum;             // DW: column sums of A (= bias gradient partials) [splits][M], may be null
    int act;                   // ACT_*
    int tiles_m, tiles_n;
    int no_fast_loop;          // tuning aid (HB_GEMM_NOFAST): always take the guarded main loop
};

// Chooses the tile shape for (kind, M, N, K), fills tiles/splits (splits <= max_splits)
// and launches.  Returns the number of K-splits used through *splits_out.
hipError_t launch_gemm_f32(GemmKind kind, GemmArgs a, int max_splits, int *splits_out,
                           hipStream_t stream, const LaunchEvents &ev = LaunchEvents());

// The backward-data and the weight-gradient product of one hidden layer in a single launch
// (both read the same D_l and are independent).  gemm_f32_pair_ok: the shapes suit the fixed
// tile shapes of that kernel; otherwise launch the two products separately.
bool gemm_f32_pair_ok(const GemmArgs &da, const GemmArgs &dw);
hipError_t launch_gemm_f32_bwd_pair(GemmArgs da, GemmArgs dw, int max_splits, int *splits_out,
                                    hipStream_t stream, const LaunchEvents &ev = LaunchEvents());

// Number of split-K slices launch_gemm_f32 will use for a DW product of this shape
// (so that the caller can size the partial buffers).
int gemm_f32_dw_splits(int M, int N, int K, int max_splits);

// ---------------------------------------------------------------- bf16 MFMA GEMM
// C[M x N] = sum_k A[m*lda + k] * B[n*ldb + k] (bmaj: A[k*lda + m] * B[k*ldb + n]), bf16 operands,
// fp32 accumulation.  Outputs
// (each optional): fp32 C, bf16 C, and a transposed bf16 copy Ct[n*ldct + m].
//   FWD: C = act(acc + bias)                    DA: C = acc * f'(aux)
//   DW : C_f32 is the fp32 master weight: C_f32 -= lr * acc, and C / Ct are its bf16 copies
//        (write_grad: C_f32 = acc, nothing else is written)
struct GemmBf16Args {
    const void *A;
    const void *B;
    int M, N, K;
    long long lda, ldb;
    int a_vec, b_vec;      // 16-byte vector loads are legal (ld % 8 == 0, base 16-byte aligned)
    void *C_f32;
    long long ldc;
    void *C_bf16;
    long long ldcb;
    void *Ct_bf16;
    long long ldct;
    const float *bias;
    const void *aux;       // backward-data: the layer's bf16 activations [M x ldaux] ...
    long long ldaux;
    const void *aux_t;     // ... and, optional, their transposed copy [N x ldauxt]: four rows per 8-byte load
    long long ldauxt;
    // ReLU decisions of a hidden layer as bits, one 16-bit word per lane and 32 x 32 block of the
    // layer's activations, word ((m / 32) * mask_nb + n / 32) * 64 + lane in the MFMA accumulator
    // layout (lane = 32 h + r owns rows 8 q + 4 h + e of column r: bit 8 (e & 1) + 2 q + (e >> 1)
    // is set when the stored bf16 activation is positive).  The forward product writes them
    // (mask_out), the backward-data product of the layer above reads them (mask_in) instead of
    // the activations themselves: 128 bytes per block instead of 2 KB.
    unsigned short *mask_out;
    const unsigned short *mask_in;
    int mask_nb;           // 32-column blocks per block row: ceil(N / 32)
    // backward-data product, optional: column sums of the stored (bf16) result over slices of its
    // rows, colsum_partial[slice * N + n] -- the bias gradient of the layer below, which then
    // needs no pass of its own over D.  Only the LDS-direct kernel produces them (slice =
    // 128 rows: the two row halves of each tile row); launch_gemm_bf16 reports the number of
    // slices written, 0 if the product went to another kernel or colsum_cap slices are too few.
    float *colsum_partial;
    int colsum_cap;
    int act;
    int write_grad;
    float lr;
    // weight gradient with batch-major operands: A[k * lda + m], B[k * ldb + n] (the row-major
    // deltas and activations themselves; LDS-direct kernel only, see gemm_bf16_dw_bmaj_ok)
    int bmaj;
    int tiles_m, tiles_n;
    // weight gradient split over the contraction (the batch): slice s covers k in
    // [s k_chunk, (s+1) k_chunk) and writes its plain fp32 partial product at
    // C_f32 + s c_split_stride (write_grad form, no bf16 outputs).  0: no split.
    int k_chunk;
    long long c_split_stride;
};
hipError_t launch_gemm_bf16(GemmKind kind, GemmBf16Args a, hipStream_t stream,
                            const LaunchEvents &ev = LaunchEvents(), int *colsum_slices_out = nullptr);
// Slices for a weight-gradient product whose 256 x 256 tiles would leave half of the CUs (or
// more) idle; 1 = do not split.  gemm_bf16_dw_splits_cap(M, N, max_K) is the largest count
// gemm_bf16_dw_splits returns for any K <= max_K and any leading dimensions (it is
// non-decreasing in K): the figure to size the slice buffer with.
int gemm_bf16_dw_splits(int M, int N, int K, long long lda, long long ldb);
// The weight gradient M x N over K batch rows can take its operands batch-major (bmaj).
bool gemm_bf16_dw_bmaj_ok(int M, int N, int K, long long lda, long long ldb, const void *A, const void *B);
int gemm_bf16_dw_splits_cap(int M, int N, int K);
// out[i] = sum_s partial[s * stride + i]  (grad != null: written there)  or  master[i] -= lr * sum
hipError_t launch_dw_reduce(const float *partial, int splits, long long stride, long long count, float *master,
                            float *grad, float lr, hipStream_t stream, const LaunchEvents &ev = LaunchEvents());
hipError_t launch_transpose_bf16(const void *in, long long ldi, void *out, long long ldo, int R, int C,
                                 hipStream_t stream, const LaunchEvents &ev = LaunchEvents());
// bf16 copies (row-major and transposed) of an fp32 matrix W [R x C]
hipError_t launch_shadow(const float *W, int R, int C, void *shadow, long long lds_, void *shadow_t,
                         long long ldt, hipStream_t stream);
// g[j] = sum_b Dt[j*ld + b];  bias[j] -= lr g[j]  (grad == null)  or  grad[j] = g[j]
hipError_t launch_rowsum_bias(const void *Dt, long long ld, int d, long long B, float *bias, float *grad,
                              float lr, hipStream_t stream, const LaunchEvents &ev = LaunchEvents());

// the same from the row-major delta D [B x ld] (ld % 8 == 0, 16-byte aligned): column sums in
// colsum_bias_slices(B) slices of the batch (partial: slices x d floats), added in index order
int colsum_bias_slices(long long B);
// the second step alone, on `slices` x d partial sums that are already there
hipError_t launch_colsum_bias_finalize(const float *partial, int slices, int d, float *bias, float *grad, float lr,
                                       hipStream_t stream, const LaunchEvents &ev = LaunchEvents());
hipError_t launch_colsum_bias(const void *D, long long ld, int d, long long B, float *partial, float *bias,
                              float *grad, float lr, hipStream_t stream, const LaunchEvents &ev = LaunchEvents());

// ---------------------------------------------------------------- loss / delta
struct LossArgs {
    const float *Z;   // B x ldz logits (fp32)
    int ldz;
    const int32_t *y;
    long long B;
    int K;            // d_L
    int loss;         // HB_LOSS_*
    void *delta;      // B x ldd, receives d(mean loss)/dZ (fp32, or bf16 when delta_bf16); may be null
    int ldd;
    int delta_bf16;
    int zero_pad;            // bf16 delta: columns K .. ldd-1 of every row are written as zeros
    float *block_partials;   // one loss sum per block (>= loss_grid_blocks entries)
    int vec4;                // set by launch_loss: rows of Z and delta allow 16-byte / 8-byte accesses
};
// The mean loss is finished by the next consumer on the stream: sum of n block partials / B.
struct LossFinalize {
    const float *partials;
    int n;                   // 0: nothing to do
    long long B;
    float *out;              // 1 float: mean loss
    float *out2;             // optional second destination (the caller's d_loss), may be null
};
hipError_t launch_loss_finalize(const LossFinalize &f, hipStream_t stream,
                                const LaunchEvents &ev = LaunchEvents());
int loss_grid_blocks(long long B, int K);
hipError_t launch_loss(const LossArgs &a, hipStream_t stream, const LaunchEvents &ev = LaunchEvents());

// ---------------------------------------------------------------- fused narrow output layer
struct OutLayerArgs {
    const float *A;      // B x lda : A_{L-1}
    int lda;
    const float *W;      // K x d   : W_L (row-major, 16-byte aligned)
    const float *bias;   // K
    const int32_t *y;
    long long B;
    int d, K;            // d = d_{L-1} (multiple of 4), K = d_L <= 16
    int loss, act;       // HB_LOSS_*, ACT_* of the hidden layers
    int backward;        // 0: loss only
    float *Dprev;        // B x ldp : D_{L-1} (may be null when L == 1 ... not used then)
    int ldp;
    float *dW_partial;   // [blocks][K x d]
    float *db_partial;   // [blocks][K]
    float *Z, *DL;       // optional copies of the logits / D_L (B x ldz), may be null
    int ldz;
    float *block_partials;   // one loss sum per block
    int R;               // rows per block (set by the launcher)
};
// Largest rows-per-block for (d, K), or 0 when the fused kernel does not apply; the rows per
// block actually used for a batch of B rows; the smallest value that can be.
int out_layer_rows(int d, int K);
int out_layer_rows_for_batch(int d, int K, long long B);
int out_layer_min_rows();
hipError_t launch_out_layer(OutLayerArgs a, hipStream_t stream, const LaunchEvents &ev = LaunchEvents());

// ---------------------------------------------------------------- update
// One segment = one parameter tensor: value[i] -= lr * sum_s partial[s*stride + i]   (STEP)
//                                 or  grad[i]  =       sum_s partial[s*stride + i]   (GRAD)
struct UpdateSeg {
    float *param;
    float *grad_out;
    const float *partial;
    long long count;
    long long stride;
    int splits;
};
constexpr int HB_MAX_SEGS = 40;
struct UpdateArgs {
    UpdateSeg seg[HB_MAX_SEGS];
    int n_seg;
    float lr;
    int write_grad;   // 0: update params; 1: write grad_out
    LossFinalize fin; // fin.n > 0: one extra block row of the grid finishes the mean loss
};
hipError_t launch_update(const UpdateArgs &a, hipStream_t stream, const LaunchEvents &ev = LaunchEvents());

// D[i] = H[i] = (1-w) H[i] + w D[i]   (H is a device staging copy of the host model)
hipError_t launch_merge(float *D, float *H, long long n, float w, hipStream_t stream);
hipError_t launch_fill_u32(unsigned int *p, long long n, unsigned int v, hipStream_t stream);
// adds the number of out-of-domain labels to *bad (device counter); debug aid
hipError_t launch_label_check(const int32_t *y, long long B, int K, int loss, unsigned int *bad, hipStream_t stream);
// adds the number of defects of a CSR batch to *bad: column indices outside [0, d0), row pointer
// not starting at 0 / decreasing / not ending at nnz; debug aid
hipError_t launch_csr_check(const int32_t *row_ptr, const int32_t *col_idx, long long nnz, long long B, int d0,
                            unsigned int *bad, hipStream_t stream);


// ---------------------------------------------------------------- CSR first layer
struct SpmmArgs {
    const int32_t *row_ptr;
    const int32_t *col_idx;
    const float *vals;
    const float *W1t;   // d_0 x ldw: row c holds the d_1 weights of input column c
    int ldw;
    const float *bias;  // d_1
    float *out;         // B x ldo
    int ldo;
    int d1;
    int act;
    int vec;            // d_1 % 4 == 0 and all rows 16-byte aligned
};
hipError_t launch_spmm_fwd(const SpmmArgs &a, long long B, hipStream_t stream,
                           const LaunchEvents &ev = LaunchEvents());

struct SparseDwArgs {
    const int32_t *col_start;    // d_0 + 1: segment of each column in csc_ent
    const int32_t *chunk_start;  // d_0 + 3: descriptor of each column; [d_0] = number of descriptors, [d_0 + 1] = of class 0, [d_0 + 2] = of classes 0 and 1
    const int4 *chunk_desc;      // per column of the batch (per part of a very long one), by size class: {column, first entry, end entry, parts of the column}
    const int2 *csc_ent;         // the batch's non-zeros by column: {row, value bits}
    const float *delta;          // B x ldd
    int ldd;
    float *W1t;
    int ldw;
    float *grad_out;             // null: update W1t; else dW_1 in the flat d_1 x d_0 layout (pre-zeroed)
    int d0, d1;
    float lr;
    int vec;
};
// Per-batch CSC (column-segmented copy of the batch's non-zeros) by a multi-block counting
// sort; hist is scratch of csc_hist_elems(max_B, d0) int32, cnt of csc_cnt_elems(d0) int32.
// Needs csc_supported(d0, max_B):
// the column histogram of one block and its slice of row_ptr live in LDS.
bool csc_supported(int d0, long long max_B);
size_t sparse_desc_capacity(int d0, long long nnz_cap);  // descriptors of a batch of at most nnz_cap non-zeros
size_t csc_hist_elems(long long max_B, int d0);
size_t csc_cnt_elems(int d0);
hipError_t launch_csc_build(const int32_t *row_ptr, const int32_t *col_idx, const float *vals,
                            long long nnz, long long B, int d0, int32_t *hist, int32_t *cnt,
                            int32_t *col_start, int32_t *chunk_start, int4 *chunk_desc, int2 *csc_ent,
                            hipStream_t stream, const LaunchEvents &ev_hist = LaunchEvents(),
                            const LaunchEvents &ev_colsum = LaunchEvents(),
                            const LaunchEvents &ev_scan = LaunchEvents(),
                            const LaunchEvents &ev_place = LaunchEvents());
hipError_t launch_sparse_dw(const SparseDwArgs &a, long long nnz, hipStream_t stream,
                            const LaunchEvents &ev = LaunchEvents());
hipError_t launch_colsum(const float *delta, int ldd, long long B, int d, int splits, float *partial,
                         hipStream_t stream, const LaunchEvents &ev = LaunchEvents());
hipError_t launch_transpose(const float *in, float *out, int R, int C, hipStream_t stream);

// ---------------------------------------------------------------- for the worker loop (worker.hip)
struct ModelInfo {
    int d0, d_out;
    int dtype;          // HB_F32 / HB_BF16_F32MASTER
    int sparse;
    long long max_B, P;
    hipStream_t stream;
};
// false (and the thread's error text set) if m is null or not configured
bool model_info(const hb_model *m, ModelInfo *out);
// the replica's flat fp32 parameters on the device (dense models: always current)
const float *model_params_device(const hb_model *m);
// the network behind a handle: layer widths d_0 .. d_L (n entries), activation, loss
bool model_arch(const hb_model *m, const int **dims, int *n, int *act, int *loss);
// brings the flat buffer up to date in stream order (a sparse first layer's weights live
// transposed beside it); nothing to do for dense models
int model_flat_refresh(hb_model *m);
// M = (1 - w) G + w D in stream order, written to the replica D AND to d_global (P floats on
// the device), followed by whatever keeps the replica's derived copies current (bf16 shadows)
int model_blend_with_device(hb_model *m, float *d_global, float w);
// slot in the handle where the worker loop keeps its staging buffers between calls; the
// deleter runs in hb_model_destroy
void **model_worker_slot(hb_model *m, void (*deleter)(void *));
// records the calling thread's error text and code; returns code
int set_error(int code, const char *fmt, ...);

}  // namespace hb
