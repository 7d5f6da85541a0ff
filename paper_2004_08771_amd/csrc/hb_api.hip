// C ABI of libhb (see include/hb.h): handle, argument validation, and the order in which
// the kernels of one GPU-worker mini-batch step are issued on the handle's stream
// (Algorithm 1 / Algorithm 2 of the paper, worker side: "Gradient", then "Update model").
#include "../../include/hb.h"
#include "hb_internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <mutex>
#include <new>
#include <vector>

using namespace hb;

namespace {

thread_local char g_err[512] = "";
thread_local int g_err_code = HB_OK;

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    g_err_code = code;
    return code;
}

float fail_nan(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    g_err_code = HB_ERR_INVALID;
    return std::numeric_limits<float>::quiet_NaN();
}

void clear_error()
{
    g_err[0] = 0;
    g_err_code = HB_OK;
}

#define HB_HIP(call)                                                                        \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess)                                                               \
            return fail(HB_ERR_DEVICE, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), \
                        __FILE__, __LINE__);                                                \
    } while (0)

constexpr int MAX_LAYERS = 16;       // weight layers; 2 * MAX_LAYERS <= HB_MAX_SEGS
constexpr int MAX_SPLITS = 64;
constexpr int64_t MAX_BATCH = 1 << 22;
constexpr int64_t MAX_DIM = 1 << 24;

int round_up(int x, int m) { return (x + m - 1) / m * m; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

enum StepMode { MODE_STEP = 0, MODE_GRAD = 1, MODE_LOSS = 2 };

// Workspace of hb_batch_loss_static (the entry point for callers that cannot allocate): the
// activations of the forward pass and the per-block loss partials live in this file-scope
// device array instead of buffers from hipMalloc.  Every device the library runs on holds
// its own copy until the process ends.
constexpr size_t STATIC_SCRATCH_BYTES = HB_STATIC_SCRATCH_BYTES;
constexpr int STATIC_MAX_DEVICES = 64;
}  // namespace

static __device__ __align__(256) unsigned char hb_static_scratch[HB_STATIC_SCRATCH_BYTES];

namespace {
// In host code the array's name is only a stand-in: the address each device holds it at comes
// from hipGetSymbolAddress, asked once per device with that device current.
std::mutex g_scratch_mu;
unsigned char *g_scratch_ptr[STATIC_MAX_DEVICES] = {};

int static_scratch_for_current_device(unsigned char **out)
{
    int dev = -1;
    HB_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= STATIC_MAX_DEVICES)
        return fail(HB_ERR_UNSUPPORTED, "device %d is outside the %d devices the static workspace serves", dev,
                    STATIC_MAX_DEVICES);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HB_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(hb_static_scratch)));
        if (!p) return fail(HB_ERR_DEVICE, "hipGetSymbolAddress returned a null address for the static workspace");
        g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
    }
    *out = g_scratch_ptr[dev];
    return HB_OK;
}

}  // namespace

struct hb_model {
    std::vector<int> dims;  // d_0 .. d_L
    int L = 0;
    int act = 0, loss = 0;
    int64_t P = 0;
    std::vector<int64_t> w_off, b_off;  // [1..L] offsets in the flat layout

    bool configured = false;
    int dtype = HB_F32;
    int64_t max_B = 0;
    bool sparse = false;
    hipStream_t stream = nullptr;
    int device = -1;

    float *d_params = nullptr;           // flat layout, fp32 (master) weights
    std::vector<int> ld;                 // leading dimension of the activation of layer l
    std::vector<float *> acts;           // [1..L]: max_B x ld[l]
    std::vector<float *> delta;          // [1..L]: d(loss)/dZ_l, max_B x ld[l] (one buffer per layer)
    std::vector<float *> partial_w, partial_b;  // [1..L] split-K gradient partials
    std::vector<int> cap_splits;
    int out_rows = 0;                    // rows per block of the fused output-layer kernel (0: not used)
    float *d_loss_partials = nullptr;
    float *d_loss = nullptr;
    float *h_loss = nullptr;             // pinned
    float *d_stage = nullptr;            // P floats: staging copy of the host model

    // bf16 mode: bf16 copies of every weight matrix (row-major and transposed), bf16
    // activations / deltas in both layouts; acts[L] holds the fp32 logits
    std::vector<int> ld8;                       // row length of the bf16 tensors of layer l: d_l rounded up to 8 (output layer: see configure)
    std::vector<void *> shadow, shadow_t;       // [1..L]
    std::vector<void *> act_bf, act_t;          // [1..L-1] / [0..L-1]
    float *bias_partial[2] = {nullptr, nullptr};  // slices x max d_l each: column sums of a row-major delta
    int bias_partial_slices = 0;                  // rows of each
    std::vector<unsigned short *> relu_mask;    // [1..L-1], ReLU nets: decision bits of the hidden activations
    void *delta_bf[2] = {nullptr, nullptr};
    void *delta_t[2] = {nullptr, nullptr};

    // sparse first layer: W_1 lives transposed (d_0 x d_1); the W_1 region of d_params is
    // only a staging area for set/get/merge
    float *d_w1t = nullptr;
    int32_t *d_col_cnt = nullptr, *d_col_start = nullptr, *d_chunk_start = nullptr;
    int32_t *d_cursor = nullptr;  // per-block column histograms / cursors of the CSC build
    int2 *d_csc_ent = nullptr;           // the batch's non-zeros by column: {row, value bits}
    float *dw_partial = nullptr;         // bf16 mode: slices of a split weight gradient (largest layer that splits)
    size_t dw_partial_cap = 0;           // its capacity in floats
    void *worker_state = nullptr;        // staging buffers of the worker loop (worker.hip), kept between epochs
    void (*worker_state_free)(void *) = nullptr;
    int4 *d_chunk_desc = nullptr;        // descriptors of the batch's columns (capacity follows the CSC arrays)
    int64_t csc_cap = 0;
    // the per-batch CSC build depends on the batch only: it runs on a stream of its own beside
    // the forward pass and is joined before the sparse weight gradient
    hipStream_t csc_stream = nullptr;
    hipEvent_t csc_fork = nullptr, csc_join = nullptr;
    int b1_splits = 1;
    std::vector<void *> owned;           // every device allocation, for destroy

    // per-kernel profile (measurement only)
    struct ProfRec {
        hb_kernel_stat info;
        hipEvent_t start, stop;
    };
    bool prof_on = false;
    std::vector<ProfRec> prof;
    std::vector<hipEvent_t> free_events;
};

namespace {

template <typename T>
int dev_alloc(hb_model *m, T **out, size_t count)
{
    void *p = nullptr;
    const size_t bytes = (count ? count : 1) * sizeof(T);
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess)
        return fail(HB_ERR_ALLOC, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
    m->owned.push_back(p);
    *out = static_cast<T *>(p);
    return HB_OK;
}

void release_device(hb_model *m)
{

    for (auto &r : m->prof) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    m->prof.clear();
    for (hipEvent_t e : m->free_events) (void)hipEventDestroy(e);
    m->free_events.clear();
    if (m->csc_stream) {
        (void)hipStreamSynchronize(m->csc_stream);
        (void)hipStreamDestroy(m->csc_stream);
    }
    if (m->csc_fork) (void)hipEventDestroy(m->csc_fork);
    if (m->csc_join) (void)hipEventDestroy(m->csc_join);
    m->csc_stream = nullptr;
    m->csc_fork = m->csc_join = nullptr;
    if (m->d_csc_ent) (void)hipFree(m->d_csc_ent);
    if (m->d_chunk_desc) (void)hipFree(m->d_chunk_desc);
    m->d_csc_ent = nullptr;
    m->d_chunk_desc = nullptr;
    m->csc_cap = 0;
    for (void *p : m->owned) (void)hipFree(p);
    m->owned.clear();
    if (m->h_loss) (void)hipHostFree(m->h_loss);
    m->h_loss = nullptr;
}

// Events for one profiled dispatch (empty when profiling is off or events run out).
LaunchEvents prof_begin(hb_model *m, int kind, int layer, int64_t M, int64_t N, int64_t K, double flops,
                        double bytes, double cache_bytes = 0.0)
{
    LaunchEvents ev;
    if (!m->prof_on) return ev;
    hipEvent_t e[2] = {nullptr, nullptr};
    for (int i = 0; i < 2; ++i) {
        if (!m->free_events.empty()) {
            e[i] = m->free_events.back();
            m->free_events.pop_back();
        } else if (hipEventCreate(&e[i]) != hipSuccess) {
            if (i == 1) m->free_events.push_back(e[0]);
            return ev;
        }
    }
    hb_model::ProfRec r;
    r.info = hb_kernel_stat{kind, layer, M, N, K, 1, 0.0, flops, bytes, cache_bytes};
    r.start = e[0];
    r.stop = e[1];
    m->prof.push_back(r);
    ev.start = e[0];
    ev.stop = e[1];
    return ev;
}

double gemm_bytes(int64_t M, int64_t N, int64_t K, int64_t extra)
{
    return 4.0 * ((double)M * K + (double)N * K + (double)M * N + (double)extra);
}

int check_handle(const hb_model *m, bool need_configured)
{
    if (!m) return fail(HB_ERR_INVALID, "model handle is NULL");
    if (need_configured && !m->configured)
        return fail(HB_ERR_STATE, "hb_mlp_configure has not been called on this model");
    return HB_OK;
}

struct Input {
    const float *X = nullptr;  // dense B x d_0, or
    const int32_t *row_ptr = nullptr, *col_idx = nullptr;
    const float *vals = nullptr;
    int64_t nnz = 0;
};

// W1t <-> the W_1 region of the flat buffer (sparse mode only)
int sync_w1t_from_flat(hb_model *m)
{
    if (!m->sparse) return HB_OK;
    HB_HIP(launch_transpose(m->d_params + m->w_off[1], m->d_w1t, m->dims[1], m->dims[0], m->stream));
    return HB_OK;
}

int sync_flat_from_w1t(hb_model *m)
{
    if (!m->sparse) return HB_OK;
    HB_HIP(launch_transpose(m->d_w1t, m->d_params + m->w_off[1], m->dims[0], m->dims[1], m->stream));
    return HB_OK;
}

// The per-batch CSC arrays grow on demand (nnz is only known per call).
int ensure_csc_capacity(hb_model *m, int64_t nnz)
{
    if (nnz <= m->csc_cap) return HB_OK;
    HB_HIP(hipStreamSynchronize(m->stream));
    if (m->csc_stream) HB_HIP(hipStreamSynchronize(m->csc_stream));
    int64_t cap = m->csc_cap > 0 ? m->csc_cap : 1024;
    while (cap < nnz) cap *= 2;
    if (m->d_csc_ent) (void)hipFree(m->d_csc_ent);
    if (m->d_chunk_desc) (void)hipFree(m->d_chunk_desc);
    m->d_csc_ent = nullptr;
    m->d_chunk_desc = nullptr;
    m->csc_cap = 0;
    const size_t max_desc = sparse_desc_capacity(m->dims[0], cap);
    if (hipMalloc(reinterpret_cast<void **>(&m->d_csc_ent), sizeof(int2) * (size_t)cap) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&m->d_chunk_desc), sizeof(int4) * max_desc) != hipSuccess)
        return fail(HB_ERR_ALLOC, "could not allocate the per-batch CSC workspace for %lld non-zeros",
                    (long long)nnz);
    m->csc_cap = cap;
    return HB_OK;
}

// Issues the kernels of one step.
int run_step(hb_model *m, const Input &in, const int32_t *y, int64_t B, float lr, StepMode mode,
             float *d_grad_flat, float *d_loss_user)
{
    const int L = m->L;
    const int Bi = (int)B;
    hipStream_t st = m->stream;
    const float *X = in.X;

    // narrow output layers (d_L <= 16) are handled by one fused kernel: forward, loss, D_L,
    // D_{L-1} and the dW_L / db_L partials from a single read of A_{L-1}
    const bool fused_out = m->out_rows > 0 && aligned16(m->d_params + m->w_off[L]);
    const int L_gemm = fused_out ? L - 1 : L;

    // ---- sparse first layer: the batch's CSC arrays (needed by the weight gradient only) are
    // built beside the forward pass.  The fork event also orders the build behind the previous
    // step's weight gradient, which read the same arrays.
    auto csc_build = [&](hipStream_t s) -> int {
        HB_HIP(launch_csc_build(in.row_ptr, in.col_idx, in.vals, in.nnz, B, m->dims[0], m->d_cursor,
                                m->d_col_cnt, m->d_col_start, m->d_chunk_start, m->d_chunk_desc,
                                m->d_csc_ent, s,
                                prof_begin(m, HB_K_OTHER, 2, 0, 0, 0, 0.0, 4.0 * in.nnz),
                                prof_begin(m, HB_K_OTHER, 3, 0, 0, 0, 0.0,
                                           8.0 * (double)csc_hist_elems(B, m->dims[0])),
                                prof_begin(m, HB_K_OTHER, 4, 0, 0, 0, 0.0, 16.0 * m->dims[0]),
                                prof_begin(m, HB_K_OTHER, 5, 0, 0, 0, 0.0, 16.0 * in.nnz)));
        return HB_OK;
    };
    const bool csc_beside = m->sparse && mode != MODE_LOSS && m->csc_stream != nullptr;
    if (csc_beside) {
        // forked at the start of the step: later fork points (behind the first or second forward
        // product) measured the same
        HB_HIP(hipEventRecord(m->csc_fork, st));
        HB_HIP(hipStreamWaitEvent(m->csc_stream, m->csc_fork, 0));
        const int rc_b = csc_build(m->csc_stream);
        if (rc_b != HB_OK) return rc_b;
        HB_HIP(hipEventRecord(m->csc_join, m->csc_stream));
    }

    // ---- forward, Eq. (1): A_l = f(A_{l-1} W_l^T + b_l); the last layer keeps raw scores
    for (int l = 1; l <= L_gemm; ++l) {
        if (l == 1 && m->sparse) {
            SpmmArgs sp = {};
            sp.row_ptr = in.row_ptr;
            sp.col_idx = in.col_idx;
            sp.vals = in.vals;
            sp.W1t = m->d_w1t;
            sp.ldw = m->dims[1];
            sp.bias = m->d_params + m->b_off[1];
            sp.out = m->acts[1];
            sp.ldo = m->ld[1];
            sp.d1 = m->dims[1];
            sp.act = (L > 1) ? m->act : ACT_NONE;
            sp.vec = (m->dims[1] % 4 == 0) && aligned16(sp.bias);
            // algorithmic HBM bytes: the CSR arrays, each touched weight row once (at most
            // min(nnz, d_0) rows), the output; the row gathers themselves (one weight row per stored
            // entry) are cache traffic and reported apart
            const double touched_rows = (double)(in.nnz < m->dims[0] ? in.nnz : m->dims[0]);
            const double gather = (double)in.nnz * 4.0 * m->dims[1];
            HB_HIP(launch_spmm_fwd(sp, B, st,
                                   prof_begin(m, HB_K_SPMM_FWD, 1, B, m->dims[1], in.nnz,
                                              2.0 * in.nnz * m->dims[1],
                                              8.0 * in.nnz + 4.0 * (B + 1.0) + 4.0 * touched_rows * m->dims[1] +
                                                  4.0 * B * (m->dims[1] + 1.0),
                                              gather)));
            continue;
        }
        GemmArgs g = {};
        g.A = (l == 1) ? X : m->acts[l - 1];
        g.lda = (l == 1) ? m->dims[0] : m->ld[l - 1];
        g.B = m->d_params + m->w_off[l];
        g.ldb = m->dims[l - 1];
        g.C = m->acts[l];
        g.ldc = m->ld[l];
        g.M = Bi;
        g.N = m->dims[l];
        g.K = m->dims[l - 1];
        g.a_vec = aligned16(g.A) && (g.lda % 4 == 0);
        g.b_vec = aligned16(g.B) && (g.ldb % 4 == 0);
        g.bias = m->d_params + m->b_off[l];
        g.act = (l < L) ? m->act : ACT_NONE;
        HB_HIP(launch_gemm_f32(GEMM_FWD, g, 1, nullptr, st,
                               prof_begin(m, HB_K_FWD_GEMM, l, g.M, g.N, g.K, 2.0 * g.M * g.N * g.K,
                                          gemm_bytes(g.M, g.N, g.K, g.N))));
    }

    // the kernel that computes the loss leaves one partial sum per block; the update kernel
    // (or, when there is none, a one-block kernel) turns them into the mean
    LossFinalize fin = {};
    fin.partials = m->d_loss_partials;
    fin.B = B;
    fin.out = m->d_loss;
    fin.out2 = d_loss_user;
    int out_blocks = 0;
    if (fused_out) {
        OutLayerArgs o = {};
        o.A = m->acts[L - 1];
        o.lda = m->ld[L - 1];
        o.W = m->d_params + m->w_off[L];
        o.bias = m->d_params + m->b_off[L];
        o.y = y;
        o.B = B;
        o.d = m->dims[L - 1];
        o.K = m->dims[L];
        o.loss = m->loss;
        o.act = m->act;
        o.backward = (mode != MODE_LOSS) ? 1 : 0;
        o.Dprev = m->delta[L - 1];
        o.ldp = m->ld[L - 1];
        o.dW_partial = m->partial_w[L];
        o.db_partial = m->partial_b[L];
        o.block_partials = m->d_loss_partials;
        const int rows = out_layer_rows_for_batch(o.d, o.K, B);
        out_blocks = (int)((B + rows - 1) / rows);
        const double flops = (o.backward ? 6.0 : 2.0) * B * o.d * o.K;
        const double bytes = 4.0 * B * o.d * (o.backward ? 2.0 : 1.0) + 4.0 * B;
        HB_HIP(launch_out_layer(o, st, prof_begin(m, HB_K_OUT_LAYER, L, B, o.K, o.d, flops, bytes)));
        fin.n = out_blocks;
        if (mode == MODE_LOSS) {
            HB_HIP(launch_loss_finalize(fin, st));
            return HB_OK;
        }
    }

    // ---- loss and output delta (Section 7.1)
    LossArgs la = {};
    la.Z = m->acts[L];
    la.ldz = m->ld[L];
    la.y = y;
    la.B = B;
    la.K = m->dims[L];
    la.loss = m->loss;
    la.delta = (mode == MODE_LOSS) ? nullptr : m->delta[L];
    la.ldd = m->ld[L];
    la.delta_bf16 = 0;
    la.block_partials = m->d_loss_partials;
    if (!fused_out) {
        HB_HIP(launch_loss(la, st, prof_begin(m, HB_K_LOSS, 0, 0, 0, 0, 0.0,
                                              4.0 * B * (la.K * (la.delta ? 2.0 : 1.0) + 1.0))));
        fin.n = loss_grid_blocks(B, la.K);
        if (mode == MODE_LOSS) {
            HB_HIP(launch_loss_finalize(fin, st));
            return HB_OK;
        }
    }

    // ---- backward, Eq. (2), with the weights the forward pass used.  (Running the
    // weight-gradient products on a second stream next to the backward-data chain was
    // measured and dropped: the two kernels slow each other down by as much as they overlap.)
    UpdateArgs ua = {};
    ua.lr = lr;
    ua.write_grad = (mode == MODE_GRAD) ? 1 : 0;
    ua.fin = fin;
    hipStream_t sw_stream = st;
    if (fused_out) {  // layer L's gradient partials came out of the fused kernel, one per row block
        UpdateSeg &sw = ua.seg[ua.n_seg++];
        sw.param = m->d_params + m->w_off[L];
        sw.grad_out = d_grad_flat ? d_grad_flat + m->w_off[L] : nullptr;
        sw.partial = m->partial_w[L];
        sw.count = (long long)m->dims[L] * m->dims[L - 1];
        sw.stride = sw.count;
        sw.splits = out_blocks;
        UpdateSeg &sb = ua.seg[ua.n_seg++];
        sb.param = m->d_params + m->b_off[L];
        sb.grad_out = d_grad_flat ? d_grad_flat + m->b_off[L] : nullptr;
        sb.partial = m->partial_b[L];
        sb.count = m->dims[L];
        sb.stride = m->dims[L];
        sb.splits = out_blocks;
    }
    for (int l = L_gemm; l >= 1; --l) {
        const float *delta_l = m->delta[l];
        GemmArgs gda = {};  // D_{l-1} = (D_l W_l) * f'(A_{l-1})
        if (l > 1) {
            gda.A = delta_l;
            gda.lda = m->ld[l];
            gda.B = m->d_params + m->w_off[l];
            gda.ldb = m->dims[l - 1];
            gda.C = m->delta[l - 1];
            gda.ldc = m->ld[l - 1];
            gda.M = Bi;
            gda.N = m->dims[l - 1];
            gda.K = m->dims[l];
            gda.a_vec = aligned16(gda.A) && (gda.lda % 4 == 0);
            gda.b_vec = aligned16(gda.B) && (gda.ldb % 4 == 0);
            gda.aux = m->acts[l - 1];
            gda.ldaux = m->ld[l - 1];
            gda.act = m->act;
        }
        GemmArgs gdw = {};  // dW_l = D_l^T A_{l-1} (split-K partials), db_l = column sums of D_l
        gdw.A = delta_l;
        gdw.lda = m->ld[l];
        gdw.B = (l == 1) ? X : m->acts[l - 1];
        gdw.ldb = (l == 1) ? m->dims[0] : m->ld[l - 1];
        gdw.C = m->partial_w[l];
        gdw.ldc = m->dims[l - 1];
        gdw.c_split_stride = (long long)m->dims[l] * m->dims[l - 1];
        gdw.M = m->dims[l];
        gdw.N = m->dims[l - 1];
        gdw.K = Bi;
        gdw.a_vec = aligned16(gdw.A) && (gdw.lda % 4 == 0);
        gdw.b_vec = aligned16(gdw.B) && (gdw.ldb % 4 == 0);
        gdw.colsum = m->partial_b[l];
        gdw.act = ACT_NONE;
        const bool dense_dw = !(l == 1 && m->sparse);
        int splits = 1;
        bool dw_done = false;
        if (l > 1 && dense_dw && gemm_f32_pair_ok(gda, gdw)) {
            HB_HIP(launch_gemm_f32_bwd_pair(
                gda, gdw, m->cap_splits[l], &splits, st,
                prof_begin(m, HB_K_BWD_PAIR, l, gda.M, gda.N, gda.K,
                           2.0 * gda.M * gda.N * gda.K + 2.0 * gdw.M * gdw.N * gdw.K,
                           gemm_bytes(gda.M, gda.N, gda.K, (int64_t)gda.M * gda.N) +
                               gemm_bytes(gdw.M, gdw.N, gdw.K, gdw.M))));
            dw_done = true;
        } else if (l > 1) {
            HB_HIP(launch_gemm_f32(GEMM_DA, gda, 1, nullptr, st,
                                   prof_begin(m, HB_K_DA_GEMM, l, gda.M, gda.N, gda.K,
                                              2.0 * gda.M * gda.N * gda.K,
                                              gemm_bytes(gda.M, gda.N, gda.K, (int64_t)gda.M * gda.N))));
        }
        if (l == 1 && m->sparse) {
            // db_1: column sums of delta_1; dW_1: column-segmented sums over the non-zeros,
            // applied to W1t directly (only columns that occur in the batch are touched)
            HB_HIP(launch_colsum(delta_l, m->ld[1], B, m->dims[1], m->b1_splits, m->partial_b[1], sw_stream,
                                 prof_begin(m, HB_K_OTHER, 1, 0, 0, 0, (double)B * m->dims[1],
                                            4.0 * B * m->dims[1])));
            UpdateSeg &sb = ua.seg[ua.n_seg++];
            sb.param = m->d_params + m->b_off[1];
            sb.grad_out = d_grad_flat ? d_grad_flat + m->b_off[1] : nullptr;
            sb.partial = m->partial_b[1];
            sb.count = m->dims[1];
            sb.stride = m->dims[1];
            sb.splits = m->b1_splits;
            if (csc_beside) {
                HB_HIP(hipStreamWaitEvent(sw_stream, m->csc_join, 0));
            } else {
                const int rc_b = csc_build(sw_stream);
                if (rc_b != HB_OK) return rc_b;
            }
            SparseDwArgs sd = {};
            sd.col_start = m->d_col_start;
            sd.chunk_start = m->d_chunk_start;
            sd.chunk_desc = m->d_chunk_desc;
            sd.csc_ent = m->d_csc_ent;
            sd.delta = delta_l;
            sd.ldd = m->ld[1];
            sd.W1t = m->d_w1t;
            sd.ldw = m->dims[1];
            sd.d0 = m->dims[0];
            sd.d1 = m->dims[1];
            sd.lr = lr;
            sd.vec = (m->dims[1] % 4 == 0);
            if (mode == MODE_GRAD) {
                sd.grad_out = d_grad_flat + m->w_off[1];
                HB_HIP(hipMemsetAsync(sd.grad_out, 0, sizeof(float) * (size_t)m->dims[1] * m->dims[0], sw_stream));
            }
            // algorithmic bytes: delta_1 rows gathered once per non-zero is cache traffic; HBM sees
            // delta_1 once, the CSC arrays, and a read + write of each touched weight row (bounded
            // by min(nnz, d_0) rows)
            const double touched = (double)(in.nnz < m->dims[0] ? in.nnz : m->dims[0]);
            HB_HIP(launch_sparse_dw(sd, in.nnz, sw_stream,
                                    prof_begin(m, HB_K_SPARSE_DW, 1, m->dims[1], m->dims[0], in.nnz,
                                               2.0 * in.nnz * m->dims[1],
                                               4.0 * B * m->dims[1] + 8.0 * in.nnz +
                                                   8.0 * touched * m->dims[1],
                                               (double)in.nnz * 4.0 * m->dims[1])));
            continue;
        }
        if (!dw_done)
            HB_HIP(launch_gemm_f32(GEMM_DW, gdw, m->cap_splits[l], &splits, sw_stream,
                                   prof_begin(m, HB_K_DW_GEMM, l, gdw.M, gdw.N, gdw.K,
                                              2.0 * gdw.M * gdw.N * gdw.K,
                                              gemm_bytes(gdw.M, gdw.N, gdw.K, gdw.M))));

        UpdateSeg &sw = ua.seg[ua.n_seg++];
        sw.param = m->d_params + m->w_off[l];
        sw.grad_out = d_grad_flat ? d_grad_flat + m->w_off[l] : nullptr;
        sw.partial = m->partial_w[l];
        sw.count = (long long)m->dims[l] * m->dims[l - 1];
        sw.stride = sw.count;
        sw.splits = splits;
        UpdateSeg &sb = ua.seg[ua.n_seg++];
        sb.param = m->d_params + m->b_off[l];
        sb.grad_out = d_grad_flat ? d_grad_flat + m->b_off[l] : nullptr;
        sb.partial = m->partial_b[l];
        sb.count = m->dims[l];
        sb.stride = m->dims[l];
        sb.splits = splits;
    }

    // ---- Eq. (3): W <- W - lr g for every tensor in one launch (or the gradient itself)
    double upd_bytes = 0.0;  // read W, read one gradient, write W
    for (int i = 0; i < ua.n_seg; ++i) upd_bytes += 12.0 * (double)ua.seg[i].count;
    HB_HIP(launch_update(ua, st, prof_begin(m, HB_K_UPDATE, 0, 0, 0, 0, 2.0 * (double)m->P, upd_bytes)));
    return HB_OK;
}

int refresh_shadows(hb_model *m)
{
    if (m->dtype != HB_BF16_F32MASTER) return HB_OK;
    for (int l = 1; l <= m->L; ++l)
        HB_HIP(launch_shadow(m->d_params + m->w_off[l], m->dims[l], m->dims[l - 1], m->shadow[l],
                             m->ld8[l - 1], m->shadow_t[l], m->ld8[l], m->stream));
    return HB_OK;
}

// The step in bf16 mode.  X is dense B x d_0 bf16.
int run_step_bf16(hb_model *m, const void *X, const int32_t *y, int64_t B, float lr, StepMode mode,
                  float *d_grad_flat, float *d_loss_user)
{
    const int L = m->L;
    const int Bi = (int)B;
    const long long ldB = round_up(Bi, 8);
    hipStream_t st = m->stream;
    const bool back = (mode != MODE_LOSS);

    // bmaj[l]: the weight gradient of layer l reads the row-major D_l and A_{l-1} themselves
    // (batch-major operands); then neither D_l^T nor A_{l-1}^T is needed for it.  Transposed
    // activations are still written for a sigmoid layer, whose backward-data epilogue reads them.
    std::vector<char> bmaj((size_t)L + 2, 0);
    static const bool bmaj_off = getenv("HB_BF16_BMAJ") && atoi(getenv("HB_BF16_BMAJ")) == 0;  // tuning aid
    if (back && !bmaj_off)
        for (int l = 1; l <= L; ++l)
            bmaj[l] = gemm_bf16_dw_bmaj_ok(m->dims[l], m->dims[l - 1], Bi, m->ld8[l],
                                           (l == 1) ? (long long)m->dims[0] : (long long)m->ld8[l - 1],
                                           m->delta_bf[l & 1], (l == 1) ? X : m->act_bf[l - 1]);
    if (back && !bmaj[1])  // X^T for dW_1 = D_1^T X
        HB_HIP(launch_transpose_bf16(X, m->dims[0], m->act_t[0], ldB, Bi, m->dims[0], st,
                                     prof_begin(m, HB_K_OTHER, 1, 0, 0, 0, 0.0, 4.0 * B * m->dims[0])));
    for (int l = 1; l <= L; ++l) {
        GemmBf16Args g = {};
        g.A = (l == 1) ? X : m->act_bf[l - 1];
        g.lda = (l == 1) ? m->dims[0] : m->ld8[l - 1];
        g.B = m->shadow[l];
        g.ldb = m->ld8[l - 1];
        g.M = Bi;
        g.N = m->dims[l];
        g.K = m->dims[l - 1];
        g.a_vec = aligned16(g.A) && (g.lda % 8 == 0);
        g.b_vec = 1;
        g.bias = m->d_params + m->b_off[l];
        if (l < L) {
            g.act = m->act;
            g.C_bf16 = m->act_bf[l];
            g.ldcb = m->ld8[l];
            if (back) {
                if (!bmaj[l + 1] || m->act == ACT_SIGMOID) {
                    g.Ct_bf16 = m->act_t[l];
                    g.ldct = ldB;
                }
                if (m->act == ACT_RELU) {  // the decisions the backward-data product of layer l+1 applies
                    g.mask_out = m->relu_mask[l];
                    g.mask_nb = (m->dims[l] + 31) / 32;
                }
            }
        } else {
            g.act = ACT_NONE;
            g.C_f32 = m->acts[L];
            g.ldc = m->ld[L];
        }
        HB_HIP(launch_gemm_bf16(GEMM_FWD, g, st,
                                prof_begin(m, HB_K_FWD_GEMM, l, g.M, g.N, g.K, 2.0 * g.M * g.N * g.K,
                                           2.0 * ((double)g.M * g.K + (double)g.N * g.K + 2.0 * g.M * g.N))));
    }

    LossArgs la = {};
    la.Z = m->acts[L];
    la.ldz = m->ld[L];
    la.y = y;
    la.B = B;
    la.K = m->dims[L];
    la.loss = m->loss;
    la.delta = back ? m->delta_bf[L & 1] : nullptr;
    la.ldd = m->ld8[L];
    la.delta_bf16 = 1;
    la.zero_pad = 1;
    la.block_partials = m->d_loss_partials;
    HB_HIP(launch_loss(la, st, prof_begin(m, HB_K_LOSS, 0, 0, 0, 0, 0.0, B * (4.0 * la.K + 2.0 * la.K + 4.0))));
    LossFinalize fin = {m->d_loss_partials, loss_grid_blocks(B, la.K), B, m->d_loss, d_loss_user};
    HB_HIP(launch_loss_finalize(fin, st));
    if (!back) return HB_OK;
    if (!bmaj[L])
        HB_HIP(launch_transpose_bf16(m->delta_bf[L & 1], m->ld8[L], m->delta_t[L & 1], ldB, Bi, m->dims[L], st,
                                     prof_begin(m, HB_K_OTHER, 2, 0, 0, 0, 0.0, 4.0 * B * m->dims[L])));

    const bool grad_mode = (mode == MODE_GRAD);
    std::vector<int> colsum_slices((size_t)L + 2, 0);  // [l] > 0: slices of column sums of D_l already written
    for (int l = L; l >= 1; --l) {
        if (l > 1) {
            GemmBf16Args g = {};
            g.A = m->delta_bf[l & 1];
            g.lda = m->ld8[l];
            g.B = m->shadow_t[l];
            g.ldb = m->ld8[l];
            g.M = Bi;
            g.N = m->dims[l - 1];
            g.K = (l == L) ? m->ld8[l] : m->dims[l];  // output layer: zero padding included (see ld8)
            g.a_vec = 1;
            g.b_vec = 1;
            g.aux = m->act_bf[l - 1];
            g.ldaux = m->ld8[l - 1];
            g.aux_t = m->act_t[l - 1];  // written by the forward pass of layer l-1
            g.ldauxt = ldB;
            if (m->act == ACT_RELU) {
                g.mask_in = m->relu_mask[l - 1];
                g.mask_nb = (m->dims[l - 1] + 31) / 32;
            }
            g.act = m->act;
            g.C_bf16 = m->delta_bf[(l - 1) & 1];
            g.ldcb = m->ld8[l - 1];
            if (!bmaj[l - 1]) {
                g.Ct_bf16 = m->delta_t[(l - 1) & 1];
                g.ldct = ldB;
            }
            g.colsum_partial = m->bias_partial[(l - 1) & 1];  // the bias gradient of layer l-1, if this kernel can
            g.colsum_cap = m->bias_partial_slices;
            const double Kd = m->dims[l];  // priced without the padding
            HB_HIP(launch_gemm_bf16(GEMM_DA, g, st,
                                    prof_begin(m, HB_K_DA_GEMM, l, g.M, g.N, m->dims[l], 2.0 * g.M * g.N * Kd,
                                               2.0 * ((double)g.M * Kd + (double)g.N * Kd + 3.0 * g.M * g.N)),
                                    &colsum_slices[l - 1]));
        }
        GemmBf16Args g = {};
        if (bmaj[l]) {
            g.bmaj = 1;
            g.A = m->delta_bf[l & 1];
            g.lda = m->ld8[l];
            g.B = (l == 1) ? X : m->act_bf[l - 1];
            g.ldb = (l == 1) ? m->dims[0] : m->ld8[l - 1];
        } else {
            g.A = m->delta_t[l & 1];
            g.lda = ldB;
            g.B = m->act_t[l - 1];
            g.ldb = ldB;
        }
        g.M = m->dims[l];
        g.N = m->dims[l - 1];
        g.K = Bi;
        g.a_vec = 1;
        g.b_vec = 1;
        g.act = ACT_NONE;
        g.lr = lr;
        g.ldc = m->dims[l - 1];
        if (grad_mode) {
            g.write_grad = 1;
            g.C_f32 = d_grad_flat + m->w_off[l];
        } else {
            g.C_f32 = m->d_params + m->w_off[l];
            g.C_bf16 = m->shadow[l];
            g.ldcb = m->ld8[l - 1];
            g.Ct_bf16 = m->shadow_t[l];
            g.ldct = m->ld8[l];
        }
        int sp = m->dw_partial ? (g.bmaj ? gemm_bf16_dw_splits_cap(g.M, g.N, g.K)
                                         : gemm_bf16_dw_splits(g.M, g.N, g.K, g.lda, g.ldb))
                               : 1;
        // never more slices than the buffer allocated at configure time holds
        if (sp > 1 && (size_t)sp * (size_t)g.M * (size_t)g.N > m->dw_partial_cap)
            sp = (int)(m->dw_partial_cap / ((size_t)g.M * (size_t)g.N));
        if (sp > 1) {
            // too few tiles for the chip: slices of the batch give partial products, summed (and
            // applied to the master weights) by a second kernel; the bf16 copies are refreshed after
            GemmBf16Args gs = g;
            gs.write_grad = 1;
            gs.C_f32 = m->dw_partial;
            gs.C_bf16 = nullptr;
            gs.Ct_bf16 = nullptr;
            gs.k_chunk = (int)round_up((g.K + sp - 1) / sp, 64);
            gs.c_split_stride = (long long)g.M * g.N;
            const int slices = (g.K + gs.k_chunk - 1) / gs.k_chunk;
            HB_HIP(launch_gemm_bf16(GEMM_DW, gs, st,
                                    prof_begin(m, HB_K_DW_GEMM, l, g.M, g.N, g.K, 2.0 * g.M * g.N * g.K,
                                               2.0 * ((double)g.M * g.K + (double)g.N * g.K) +
                                                   4.0 * slices * g.M * g.N)));
            HB_HIP(launch_dw_reduce(m->dw_partial, slices, gs.c_split_stride, gs.c_split_stride,
                                    m->d_params + m->w_off[l], grad_mode ? d_grad_flat + m->w_off[l] : nullptr, lr,
                                    st, prof_begin(m, HB_K_UPDATE, l, 0, 0, 0, (double)slices * g.M * g.N,
                                                   4.0 * (slices + 2) * g.M * g.N)));
            if (!grad_mode)
                HB_HIP(launch_shadow(m->d_params + m->w_off[l], m->dims[l], m->dims[l - 1], m->shadow[l],
                                     m->ld8[l - 1], m->shadow_t[l], m->ld8[l], st));
        } else {
            HB_HIP(launch_gemm_bf16(GEMM_DW, g, st,
                                    prof_begin(m, HB_K_DW_GEMM, l, g.M, g.N, g.K, 2.0 * g.M * g.N * g.K,
                                               2.0 * ((double)g.M * g.K + (double)g.N * g.K) +
                                                   (grad_mode ? 4.0 : 12.0) * g.M * g.N)));
        }
        if (colsum_slices[l] > 0)  // the backward-data epilogue that wrote D_l left its column sums
            HB_HIP(launch_colsum_bias_finalize(m->bias_partial[l & 1], colsum_slices[l], m->dims[l],
                                               m->d_params + m->b_off[l],
                                               grad_mode ? d_grad_flat + m->b_off[l] : nullptr, lr, st,
                                               prof_begin(m, HB_K_OTHER, 3, 0, 0, 0,
                                                          (double)colsum_slices[l] * m->dims[l],
                                                          4.0 * colsum_slices[l] * m->dims[l])));
        else if (bmaj[l])
            HB_HIP(launch_colsum_bias(m->delta_bf[l & 1], m->ld8[l], m->dims[l], B, m->bias_partial[l & 1],
                                      m->d_params + m->b_off[l], grad_mode ? d_grad_flat + m->b_off[l] : nullptr,
                                      lr, st,
                                      prof_begin(m, HB_K_UPDATE, l, 0, 0, 0, (double)B * m->dims[l],
                                                 2.0 * B * m->dims[l])));
        else
            HB_HIP(launch_rowsum_bias(m->delta_t[l & 1], ldB, m->dims[l], B, m->d_params + m->b_off[l],
                                      grad_mode ? d_grad_flat + m->b_off[l] : nullptr, lr, st,
                                      prof_begin(m, HB_K_UPDATE, l, 0, 0, 0, (double)B * m->dims[l],
                                                 2.0 * B * m->dims[l])));
    }
    return HB_OK;
}

int validate_batch_call(hb_model *m, const void *a, const int32_t *dy, int64_t B, bool want_sparse)
{
    int rc = check_handle(m, true);
    if (rc != HB_OK) return rc;
    if (m->sparse != want_sparse)
        return fail(HB_ERR_INVALID, want_sparse
                                        ? "CSR call on a model configured for dense input"
                                        : "dense call on a model configured with sparse_first_layer");
    if (!a) return fail(HB_ERR_INVALID, "input pointer is NULL");
    if (!dy) return fail(HB_ERR_INVALID, "label pointer dy is NULL");
    if (B < 1 || B > m->max_B)
        return fail(HB_ERR_INVALID, "B = %lld is outside [1, max_B = %lld]", (long long)B,
                    (long long)m->max_B);
    // HB_CHECK_LABELS=1 (debug aid, costs a pass over y and a synchronisation per call): labels
    // outside their domain are an error instead of a silently wrong loss
    static const bool check_labels = getenv("HB_CHECK_LABELS") && atoi(getenv("HB_CHECK_LABELS")) != 0;
    if (check_labels) {
        unsigned int *d_bad = reinterpret_cast<unsigned int *>(m->d_loss + 3);
        unsigned int bad = 0;
        HB_HIP(launch_fill_u32(d_bad, 1, 0u, m->stream));
        HB_HIP(launch_label_check(dy, B, m->dims[m->L], m->loss, d_bad, m->stream));
        HB_HIP(hipMemcpyAsync(&bad, d_bad, sizeof(bad), hipMemcpyDeviceToHost, m->stream));
        HB_HIP(hipStreamSynchronize(m->stream));
        if (bad)
            return fail(HB_ERR_INVALID, "%u of the %lld labels are outside their domain (%s)", bad, (long long)B,
                        m->loss == HB_LOSS_LOGISTIC ? "+1 / -1" : "class index in [0, d_L)");
    }
    return HB_OK;
}

int validate_csr_call(hb_model *m, const int32_t *rp, const int32_t *ci, const float *va, int64_t nnz,
                      const int32_t *dy, int64_t B, Input *in)
{
    int rc = validate_batch_call(m, rp, dy, B, true);
    if (rc != HB_OK) return rc;
    if (nnz < 0 || nnz > 0x7fffffffLL || nnz > B * (int64_t)m->dims[0])
        return fail(HB_ERR_INVALID, "nnz = %lld is outside [0, min(2^31 - 1, B * d_0)]", (long long)nnz);
    if (nnz > 0 && (!ci || !va)) return fail(HB_ERR_INVALID, "d_col_idx / d_vals is NULL");
    // HB_CHECK_INDICES=1 (debug aid, costs a pass over the CSR arrays and a synchronisation per
    // call): a column index outside [0, d_0) or a malformed row pointer is an error here, before
    // any kernel dereferences them, instead of an out-of-bounds access
    static const bool check_indices = getenv("HB_CHECK_INDICES") && atoi(getenv("HB_CHECK_INDICES")) != 0;
    if (check_indices) {
        unsigned int *d_bad = reinterpret_cast<unsigned int *>(m->d_loss + 3);
        unsigned int bad = 0;
        HB_HIP(launch_fill_u32(d_bad, 1, 0u, m->stream));
        HB_HIP(launch_csr_check(rp, ci, nnz, B, m->dims[0], d_bad, m->stream));
        HB_HIP(hipMemcpyAsync(&bad, d_bad, sizeof(bad), hipMemcpyDeviceToHost, m->stream));
        HB_HIP(hipStreamSynchronize(m->stream));
        if (bad)
            return fail(HB_ERR_INVALID,
                        "the CSR batch has %u defects (column index outside [0, %d), or a row pointer that does not "
                        "start at 0, decreases, or does not end at nnz = %lld)", bad, m->dims[0], (long long)nnz);
    }
    in->row_ptr = rp;
    in->col_idx = ci;
    in->vals = va;
    in->nnz = nnz;
    return HB_OK;
}

int fetch_loss(hb_model *m, float *out)
{
    HB_HIP(hipMemcpyAsync(m->h_loss, m->d_loss, sizeof(float), hipMemcpyDeviceToHost, m->stream));
    HB_HIP(hipStreamSynchronize(m->stream));
    *out = *m->h_loss;
    return HB_OK;
}

}  // namespace

namespace hb {

bool model_info(const hb_model *m, ModelInfo *out)
{
    if (check_handle(m, true) != HB_OK) return false;
    out->d0 = m->dims[0];
    out->d_out = m->dims[m->L];
    out->dtype = m->dtype;
    out->sparse = m->sparse ? 1 : 0;
    out->max_B = m->max_B;
    out->P = m->P;
    out->stream = m->stream;
    return true;
}

bool model_arch(const hb_model *m, const int **dims, int *n, int *act, int *loss)
{
    if (check_handle(m, false) != HB_OK) return false;
    *dims = m->dims.data();
    *n = (int)m->dims.size();
    *act = m->act;
    *loss = m->loss;
    return true;
}

const float *model_params_device(const hb_model *m) { return m->d_params; }

int model_flat_refresh(hb_model *m) { return sync_flat_from_w1t(m); }

int model_blend_with_device(hb_model *m, float *d_global, float w)
{
    int rc = sync_flat_from_w1t(m);
    if (rc != HB_OK) return rc;
    HB_HIP(launch_merge(m->d_params, d_global, m->P, w, m->stream));
    rc = sync_w1t_from_flat(m);
    if (rc == HB_OK) rc = refresh_shadows(m);
    return rc;
}

void **model_worker_slot(hb_model *m, void (*deleter)(void *))
{
    m->worker_state_free = deleter;
    return &m->worker_state;
}

int set_error(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    g_err_code = code;
    return code;
}

}  // namespace hb

extern "C" {

const char *hb_last_error(void) { return g_err; }
int hb_last_error_code(void) { return g_err_code; }

int hb_profile_enable(hb_model *m, int on)
{
    int rc = check_handle(m, true);
    if (rc != HB_OK) return rc;
    m->prof_on = on != 0;
    return HB_OK;
}

int hb_profile_read(hb_model *m, hb_kernel_stat *out, int32_t cap, int32_t *n_out)
{
    int rc = check_handle(m, true);
    if (rc != HB_OK) return rc;
    if (!out || !n_out || cap < 1) return fail(HB_ERR_INVALID, "out / n_out is NULL or cap < 1");
    HB_HIP(hipStreamSynchronize(m->stream));
    std::vector<hb_kernel_stat> acc;
    for (auto &r : m->prof) {
        float ms = 0.f;
        HB_HIP(hipEventElapsedTime(&ms, r.start, r.stop));
        m->free_events.push_back(r.start);
        m->free_events.push_back(r.stop);
        bool found = false;
        for (auto &a : acc)
            if (a.kind == r.info.kind && a.layer == r.info.layer && a.M == r.info.M && a.N == r.info.N &&
                a.K == r.info.K) {
                a.launches += 1;
                a.total_ms += ms;
                found = true;
                break;
            }
        if (!found) {
            hb_kernel_stat s = r.info;
            s.total_ms = ms;
            acc.push_back(s);
        }
    }
    m->prof.clear();
    const int32_t n = (int32_t)acc.size() < cap ? (int32_t)acc.size() : cap;
    for (int32_t i = 0; i < n; ++i) out[i] = acc[i];
    *n_out = n;
    return HB_OK;
}
const char *hb_version(void) { return "hb-mlp 0.2 (gfx950)"; }

int32_t hb_plan_bf16_dw_slices(int32_t d_out, int32_t d_in, int64_t B, int32_t capacity)
{
    if (d_out < 1 || d_in < 1 || B < 1 || B > MAX_BATCH) return 0;
    if (capacity) return gemm_bf16_dw_splits_cap(d_out, d_in, (int)B);
    const long long ldB = round_up((int)B, 8);
    return gemm_bf16_dw_splits(d_out, d_in, (int)B, ldB, ldB);
}

hb_model *hb_mlp_create(const int32_t *layer_dims, int32_t n_dims, int activation, int loss)
{
    if (!layer_dims) { fail(HB_ERR_INVALID, "layer_dims is NULL"); return nullptr; }
    if (n_dims < 2 || n_dims > MAX_LAYERS + 1) {
        fail(HB_ERR_INVALID, "n_dims = %d is outside [2, %d]", n_dims, MAX_LAYERS + 1);
        return nullptr;
    }
    for (int i = 0; i < n_dims; ++i)
        if (layer_dims[i] < 1 || layer_dims[i] > MAX_DIM) {
            fail(HB_ERR_INVALID, "layer_dims[%d] = %d is outside [1, %lld]", i, layer_dims[i],
                 (long long)MAX_DIM);
            return nullptr;
        }
    if (activation != HB_ACT_SIGMOID && activation != HB_ACT_RELU) {
        fail(HB_ERR_INVALID, "unknown activation %d", activation);
        return nullptr;
    }
    if (loss != HB_LOSS_SOFTMAX_CE && loss != HB_LOSS_LOGISTIC) {
        fail(HB_ERR_INVALID, "unknown loss %d", loss);
        return nullptr;
    }
    if (loss == HB_LOSS_LOGISTIC && layer_dims[n_dims - 1] > 2) {
        fail(HB_ERR_INVALID, "logistic loss needs d_L <= 2, got %d", layer_dims[n_dims - 1]);
        return nullptr;
    }
    hb_model *m = new (std::nothrow) hb_model();
    if (!m) { fail(HB_ERR_ALLOC, "out of host memory"); return nullptr; }
    m->dims.assign(layer_dims, layer_dims + n_dims);
    m->L = n_dims - 1;
    m->act = activation;
    m->loss = loss;
    m->w_off.assign(n_dims, 0);
    m->b_off.assign(n_dims, 0);
    int64_t off = 0;
    for (int l = 1; l <= m->L; ++l) {
        m->w_off[l] = off;
        off += (int64_t)m->dims[l] * m->dims[l - 1];
        m->b_off[l] = off;
        off += m->dims[l];
    }
    m->P = off;
    clear_error();
    return m;
}

int64_t hb_model_num_params(const hb_model *m) { return m ? m->P : -1; }

int hb_mlp_configure(hb_model *m, int dtype, int64_t max_B, int sparse_first_layer, void *hip_stream)
{
    int rc = check_handle(m, false);
    if (rc != HB_OK) return rc;
    if (m->configured) return fail(HB_ERR_STATE, "model is already configured");
    if (dtype != HB_F32 && dtype != HB_BF16_F32MASTER)
        return fail(HB_ERR_INVALID, "unknown dtype %d", dtype);
    if (max_B < 1 || max_B > MAX_BATCH)
        return fail(HB_ERR_INVALID, "max_B = %lld is outside [1, %lld]", (long long)max_B,
                    (long long)MAX_BATCH);
    if (sparse_first_layer && dtype != HB_F32)
        return fail(HB_ERR_INVALID, "sparse_first_layer needs dtype HB_F32");
    if (sparse_first_layer && !csc_supported(m->dims[0], max_B))
        return fail(HB_ERR_UNSUPPORTED,
                    "sparse_first_layer: d_0 = %d columns with max_B = %lld does not fit the per-batch "
                    "column sort (d_0 <= 36864 and 4 (d_0 + max_B / 64) <= 150 KB)",
                    m->dims[0], (long long)max_B);

    int dev = -1;
    HB_HIP(hipGetDevice(&dev));
    m->device = dev;
    m->dtype = dtype;
    m->max_B = max_B;
    m->sparse = sparse_first_layer != 0;
    m->stream = static_cast<hipStream_t>(hip_stream);

    const int L = m->L;
    m->ld.assign(L + 1, 0);
    m->acts.assign(L + 1, nullptr);
    m->partial_w.assign(L + 1, nullptr);
    m->partial_b.assign(L + 1, nullptr);
    m->cap_splits.assign(L + 1, 1);
    for (int l = 0; l <= L; ++l) {
        m->ld[l] = round_up(m->dims[l], 4);
    }
    m->ld[0] = m->dims[0];  // X is the caller's, unpadded

    rc = dev_alloc(m, &m->d_params, (size_t)m->P);
    if (rc == HB_OK) rc = dev_alloc(m, &m->d_stage, (size_t)m->P);
    if (dtype == HB_F32) {
        for (int l = 1; l <= L && rc == HB_OK; ++l) {
            rc = dev_alloc(m, &m->acts[l], (size_t)max_B * m->ld[l]);
            if (rc != HB_OK) break;
            if (l == 1 && m->sparse) {
                m->b1_splits = (int)((max_B + 127) / 128 < MAX_SPLITS ? (max_B + 127) / 128 : MAX_SPLITS);
                m->cap_splits[l] = m->b1_splits;
                rc = dev_alloc(m, &m->partial_b[l], (size_t)m->cap_splits[l] * m->dims[l]);
                continue;
            }
            m->cap_splits[l] = gemm_f32_dw_splits(m->dims[l], m->dims[l - 1], (int)max_B, MAX_SPLITS);
            if (l == L && L >= 2) {
                m->out_rows = out_layer_rows(m->dims[L - 1], m->dims[L]);
                if (m->out_rows > 0) {  // one partial per row block of the fused kernel
                    const int rmin = out_layer_min_rows();
                    const int blocks = (int)((max_B + rmin - 1) / rmin);
                    if (blocks > m->cap_splits[l]) m->cap_splits[l] = blocks;
                }
            }
            rc = dev_alloc(m, &m->partial_w[l], (size_t)m->cap_splits[l] * m->dims[l] * m->dims[l - 1]);
            if (rc == HB_OK) rc = dev_alloc(m, &m->partial_b[l], (size_t)m->cap_splits[l] * m->dims[l]);
        }
        m->delta.assign(L + 1, nullptr);
        for (int l = 1; l <= L && rc == HB_OK; ++l) rc = dev_alloc(m, &m->delta[l], (size_t)max_B * m->ld[l]);
    } else {
        // bf16 mode: 2-byte buffers in both layouts; only the logits stay fp32
        const size_t ldB = (size_t)round_up((int)max_B, 8);
        m->ld8.assign(L + 1, 0);
        m->shadow.assign(L + 1, nullptr);
        m->shadow_t.assign(L + 1, nullptr);
        m->act_bf.assign(L + 1, nullptr);
        m->act_t.assign(L + 1, nullptr);
        m->relu_mask.assign(L + 1, nullptr);
        int max_ld8 = 8, max_d = 1;
        for (int l = 0; l <= L; ++l) {
            // rows of 8 elements (16 bytes); the output layer's rows are padded to a whole k-tile
            // of 64 when that adds less than half a tile: its delta is the left operand of the
            // last layer's backward-data product, which then needs no masked tail (the padding
            // is zero on both sides: the loss kernel writes it, the weight copies keep it)
            m->ld8[l] = (l == L && m->dims[l] % 64 >= 32) ? round_up(m->dims[l], 64) : round_up(m->dims[l], 8);
            if (l >= 1 && m->ld8[l] > max_ld8) max_ld8 = m->ld8[l];
            if (l >= 1 && m->dims[l] > max_d) max_d = m->dims[l];
        }
        rc = dev_alloc(m, &m->acts[L], (size_t)max_B * m->ld[L]);
        for (int l = 1; l <= L && rc == HB_OK; ++l) {
            unsigned short *p = nullptr;
            rc = dev_alloc(m, &p, (size_t)m->dims[l] * m->ld8[l - 1]);
            m->shadow[l] = p;
            if (rc == HB_OK) rc = dev_alloc(m, &p, (size_t)m->dims[l - 1] * m->ld8[l]);
            m->shadow_t[l] = p;
        }
        for (int l = 0; l < L && rc == HB_OK; ++l) {
            unsigned short *p = nullptr;
            if (l >= 1) {
                rc = dev_alloc(m, &p, (size_t)max_B * m->ld8[l]);
                m->act_bf[l] = p;
            }
            if (rc == HB_OK) rc = dev_alloc(m, &p, (size_t)m->dims[l] * ldB);
            m->act_t[l] = p;
            if (l >= 1 && m->act == ACT_RELU && rc == HB_OK) {  // 64 words per 32 x 32 block
                rc = dev_alloc(m, &p, (size_t)((max_B + 31) / 32) * (size_t)((m->dims[l] + 31) / 32) * 64);
                m->relu_mask[l] = p;
            }
        }
        for (int i = 0; i < 2 && rc == HB_OK; ++i) {
            unsigned short *p = nullptr;
            rc = dev_alloc(m, &p, (size_t)max_B * max_ld8);
            m->delta_bf[i] = p;
            if (rc == HB_OK) rc = dev_alloc(m, &p, (size_t)max_d * ldB);
            m->delta_t[i] = p;
        }
        {
            // weight gradients with too few 256 x 256 tiles are split over the batch: room for the
            // largest number of slices any batch size up to max_B can ask for, in any layer
            size_t need = 0;
            for (int l = 1; l <= L; ++l) {
                const int sp = gemm_bf16_dw_splits_cap(m->dims[l], m->dims[l - 1], (int)max_B);
                const size_t n = (sp > 1) ? (size_t)sp * m->dims[l] * m->dims[l - 1] : 0;
                if (n > need) need = n;
            }
            if (need > 0 && rc == HB_OK) rc = dev_alloc(m, &m->dw_partial, need);
            if (rc == HB_OK) m->dw_partial_cap = need;
        }
        {
            // the bias gradient's partial column sums: from a pass over D of its own, or two per
            // 256-row tile from the backward-data epilogue that wrote D (the sums of D_{l-1} are
            // written while those of D_l wait for their turn: two buffers)
            int rows = colsum_bias_slices(max_B);
            const long long fused = 2 * ((max_B + 255) / 256);
            if (fused <= 1024 && fused > rows) rows = (int)fused;
            m->bias_partial_slices = rows;
            for (int i = 0; i < 2 && rc == HB_OK; ++i)
                rc = dev_alloc(m, &m->bias_partial[i], (size_t)rows * (size_t)max_d);
        }
    }
    if (m->sparse && rc == HB_OK) {
        const size_t d0 = (size_t)m->dims[0];
        rc = dev_alloc(m, &m->d_w1t, d0 * m->dims[1]);
        if (rc == HB_OK) rc = dev_alloc(m, &m->d_col_cnt, csc_cnt_elems(d0));
        if (rc == HB_OK) rc = dev_alloc(m, &m->d_col_start, d0 + 1);
        if (rc == HB_OK) rc = dev_alloc(m, &m->d_chunk_start, d0 + 3);
        if (rc == HB_OK) rc = dev_alloc(m, &m->d_cursor, csc_hist_elems(max_B, m->dims[0]));
        // HB_CSC_INLINE=1 (tuning aid) keeps the CSC build on the handle's stream, before the weight gradient
        static const bool csc_inline = getenv("HB_CSC_INLINE") && atoi(getenv("HB_CSC_INLINE")) != 0;
        if (rc == HB_OK && !csc_inline) {
            if (hipStreamCreateWithFlags(&m->csc_stream, hipStreamNonBlocking) != hipSuccess ||  // default priority
                hipEventCreateWithFlags(&m->csc_fork, hipEventDisableTiming) != hipSuccess ||
                hipEventCreateWithFlags(&m->csc_join, hipEventDisableTiming) != hipSuccess)
                rc = fail(HB_ERR_DEVICE, "cannot create the stream and events of the CSC build: %s",
                          hipGetErrorString(hipGetLastError()));
        }
    }
    {
        // one loss partial per block of whichever kernel computes the loss
        size_t nblk = (size_t)loss_grid_blocks(max_B, m->dims[L]);
        if (m->out_rows > 0 && (size_t)((max_B + out_layer_min_rows() - 1) / out_layer_min_rows()) > nblk)
            nblk = (size_t)((max_B + out_layer_min_rows() - 1) / out_layer_min_rows());
        if (rc == HB_OK) rc = dev_alloc(m, &m->d_loss_partials, nblk + 1);
    }
    if (rc == HB_OK) rc = dev_alloc(m, &m->d_loss, 4);
    if (rc != HB_OK) { release_device(m); return rc; }
    hipError_t e = hipHostMalloc(reinterpret_cast<void **>(&m->h_loss), 64, hipHostMallocDefault);
    if (e != hipSuccess) {
        release_device(m);
        return fail(HB_ERR_ALLOC, "hipHostMalloc failed: %s", hipGetErrorString(e));
    }
    e = hipMemsetAsync(m->d_params, 0, sizeof(float) * (size_t)m->P, m->stream);
    if (e == hipSuccess && m->sparse)
        e = hipMemsetAsync(m->d_w1t, 0, sizeof(float) * (size_t)m->dims[0] * m->dims[1], m->stream);
    if (e == hipSuccess && dtype == HB_BF16_F32MASTER) {
        // zero weights -> zero bf16 copies (padding columns included)
        for (int l = 1; l <= L && e == hipSuccess; ++l) {
            e = hipMemsetAsync(m->shadow[l], 0, 2 * (size_t)m->dims[l] * m->ld8[l - 1], m->stream);
            if (e == hipSuccess)
                e = hipMemsetAsync(m->shadow_t[l], 0, 2 * (size_t)m->dims[l - 1] * m->ld8[l], m->stream);
        }
    }
    if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
    if (e != hipSuccess) {
        release_device(m);
        return fail(HB_ERR_DEVICE, "initialising device buffers failed: %s", hipGetErrorString(e));
    }
    m->configured = true;
    clear_error();
    return HB_OK;
}

void hb_model_destroy(hb_model *m)
{
    if (!m) return;
    if (m->configured) (void)hipStreamSynchronize(m->stream);
    if (m->worker_state && m->worker_state_free) m->worker_state_free(m->worker_state);
    release_device(m);
    delete m;
}

int hb_model_set_params(hb_model *m, const float *host_flat)
{
    int rc = check_handle(m, true);
    if (rc != HB_OK) return rc;
    if (!host_flat) return fail(HB_ERR_INVALID, "host_flat is NULL");
    HB_HIP(hipMemcpyAsync(m->d_params, host_flat, sizeof(float) * (size_t)m->P, hipMemcpyHostToDevice,
                          m->stream));
    rc = sync_w1t_from_flat(m);
    if (rc == HB_OK) rc = refresh_shadows(m);
    if (rc != HB_OK) return rc;
    HB_HIP(hipStreamSynchronize(m->stream));
    return HB_OK;
}

int hb_model_get_params(hb_model *m, float *host_flat)
{
    int rc = check_handle(m, true);
    if (rc != HB_OK) return rc;
    if (!host_flat) return fail(HB_ERR_INVALID, "host_flat is NULL");
    rc = sync_flat_from_w1t(m);
    if (rc != HB_OK) return rc;
    HB_HIP(hipMemcpyAsync(host_flat, m->d_params, sizeof(float) * (size_t)m->P, hipMemcpyDeviceToHost,
                          m->stream));
    HB_HIP(hipStreamSynchronize(m->stream));
    return HB_OK;
}

int hb_model_get_activations(hb_model *m, int32_t layer, int64_t B, float *host_out)
{
    int rc = check_handle(m, true);
    if (rc != HB_OK) return rc;
    if (!host_out) return fail(HB_ERR_INVALID, "host_out is NULL");
    if (layer < 1 || layer >= m->L)
        return fail(HB_ERR_INVALID, "layer = %d is not a hidden layer (1 .. %d)", layer, m->L - 1);
    if (B < 1 || B > m->max_B)
        return fail(HB_ERR_INVALID, "B = %lld is outside [1, max_B = %lld]", (long long)B, (long long)m->max_B);
    const size_t d = (size_t)m->dims[layer];
    if (m->dtype == HB_F32) {
        HB_HIP(hipMemcpy2DAsync(host_out, d * sizeof(float), m->acts[layer], (size_t)m->ld[layer] * sizeof(float),
                                d * sizeof(float), (size_t)B, hipMemcpyDeviceToHost, m->stream));
        HB_HIP(hipStreamSynchronize(m->stream));
        return HB_OK;
    }
    // bf16 storage: fetch the two-byte values and widen them on the host (exact)
    std::vector<unsigned short> tmp;
    try {
        tmp.resize((size_t)B * d);
    } catch (const std::bad_alloc &) {
        return fail(HB_ERR_ALLOC, "out of host memory");
    }
    HB_HIP(hipMemcpy2DAsync(tmp.data(), d * 2, m->act_bf[layer], (size_t)m->ld8[layer] * 2, d * 2, (size_t)B,
                            hipMemcpyDeviceToHost, m->stream));
    HB_HIP(hipStreamSynchronize(m->stream));
    for (size_t i = 0; i < tmp.size(); ++i) {
        const uint32_t u = (uint32_t)tmp[i] << 16;
        memcpy(&host_out[i], &u, 4);
    }
    return HB_OK;
}

int hb_batch_step_async(hb_model *m, const void *dX, const int32_t *dy, int64_t B, float lr,
                        float *d_loss)
{
    int rc = validate_batch_call(m, dX, dy, B, false);
    if (rc != HB_OK) return rc;
    if (!std::isfinite(lr)) return fail(HB_ERR_INVALID, "lr is not finite");
    if (m->dtype == HB_BF16_F32MASTER) return run_step_bf16(m, dX, dy, B, lr, MODE_STEP, nullptr, d_loss);
    Input in;
    in.X = static_cast<const float *>(dX);
    return run_step(m, in, dy, B, lr, MODE_STEP, nullptr, d_loss);
}

float hb_batch_step(hb_model *m, const void *dX, const int32_t *dy, int64_t B, float lr)
{
    if (hb_batch_step_async(m, dX, dy, B, lr, nullptr) != HB_OK)
        return std::numeric_limits<float>::quiet_NaN();
    float out;
    if (fetch_loss(m, &out) != HB_OK) return std::numeric_limits<float>::quiet_NaN();
    return out;
}

float hb_batch_grad(hb_model *m, const void *dX, const int32_t *dy, int64_t B, float *d_grad_flat)
{
    if (validate_batch_call(m, dX, dy, B, false) != HB_OK)
        return std::numeric_limits<float>::quiet_NaN();
    if (!d_grad_flat) return fail_nan("d_grad_flat is NULL");
    Input in;
    in.X = static_cast<const float *>(dX);
    if ((m->dtype == HB_BF16_F32MASTER ? run_step_bf16(m, dX, dy, B, 0.f, MODE_GRAD, d_grad_flat, nullptr)
                                       : run_step(m, in, dy, B, 0.f, MODE_GRAD, d_grad_flat, nullptr)) != HB_OK)
        return std::numeric_limits<float>::quiet_NaN();
    float out;
    if (fetch_loss(m, &out) != HB_OK) return std::numeric_limits<float>::quiet_NaN();
    return out;
}

int hb_batch_loss_async(hb_model *m, const void *dX, const int32_t *dy, int64_t B, float *d_loss)
{
    int rc = validate_batch_call(m, dX, dy, B, false);
    if (rc != HB_OK) return rc;
    Input in;
    in.X = static_cast<const float *>(dX);
    return m->dtype == HB_BF16_F32MASTER ? run_step_bf16(m, dX, dy, B, 0.f, MODE_LOSS, nullptr, d_loss)
                                         : run_step(m, in, dy, B, 0.f, MODE_LOSS, nullptr, d_loss);
}

float hb_batch_loss(hb_model *m, const void *dX, const int32_t *dy, int64_t B)
{
    if (hb_batch_loss_async(m, dX, dy, B, nullptr) != HB_OK)
        return std::numeric_limits<float>::quiet_NaN();
    float out;
    if (fetch_loss(m, &out) != HB_OK) return std::numeric_limits<float>::quiet_NaN();
    return out;
}

int hb_batch_loss_static(const int32_t *layer_dims, int32_t n_dims, int activation, int loss,
                         const float *d_params, const float *dX, const int32_t *dy, int64_t B, float *d_loss,
                         void *hip_stream)
{
    if (!d_params) return fail(HB_ERR_INVALID, "d_params is NULL");
    if (!dX) return fail(HB_ERR_INVALID, "input pointer is NULL");
    if (!dy) return fail(HB_ERR_INVALID, "label pointer dy is NULL");
    if (!d_loss) return fail(HB_ERR_INVALID, "d_loss is NULL");
    if (!aligned16(d_params)) return fail(HB_ERR_INVALID, "d_params must be 16-byte aligned");
    if (B < 1 || B > MAX_BATCH)
        return fail(HB_ERR_INVALID, "B = %lld is outside [1, %lld]", (long long)B, (long long)MAX_BATCH);
    // a handle on the host only (validates the network exactly as hb_mlp_create does); its device
    // pointers are set to places inside the static workspace below, nothing is allocated on a device
    hb_model *m = hb_mlp_create(layer_dims, n_dims, activation, loss);
    if (!m) return g_err_code;
    struct Free {
        hb_model *m;
        ~Free() { delete m; }  // owns no device memory: `owned` stays empty
    } guard{m};
    const int L = m->L;
    m->dtype = HB_F32;
    m->max_B = B;
    m->stream = static_cast<hipStream_t>(hip_stream);
    m->ld.assign(L + 1, 0);
    m->acts.assign(L + 1, nullptr);
    m->delta.assign(L + 1, nullptr);
    m->partial_w.assign(L + 1, nullptr);
    m->partial_b.assign(L + 1, nullptr);
    m->cap_splits.assign(L + 1, 1);
    for (int l = 1; l <= L; ++l) m->ld[l] = round_up(m->dims[l], 4);
    m->ld[0] = m->dims[0];
    if (L >= 2) m->out_rows = out_layer_rows(m->dims[L - 1], m->dims[L]);
    size_t nblk = (size_t)loss_grid_blocks(B, m->dims[L]);
    if (m->out_rows > 0) {
        const size_t ob = (size_t)((B + out_layer_min_rows() - 1) / out_layer_min_rows());
        if (ob > nblk) nblk = ob;
    }
    // layout: [activations of layer 1 .. L, each B x ld_l floats][loss partials][mean loss], every
    // part starting on a 256-byte boundary
    auto align256 = [](size_t b) { return (b + 255) / 256 * 256; };
    size_t need = 0;
    std::vector<size_t> act_off(L + 1, 0);
    for (int l = 1; l <= L; ++l) {
        act_off[l] = need;
        need += align256(sizeof(float) * (size_t)B * m->ld[l]);
    }
    const size_t partial_off = need;
    need += align256(sizeof(float) * (nblk + 1));
    const size_t loss_off = need;
    need += 256;
    if (need > STATIC_SCRATCH_BYTES)
        return fail(HB_ERR_UNSUPPORTED,
                    "hb_batch_loss_static: B = %lld rows of this network need %zu bytes of workspace, the static "
                    "workspace holds %zu (use a handle from hb_mlp_configure and hb_batch_loss_async instead)",
                    (long long)B, need, STATIC_SCRATCH_BYTES);
    unsigned char *ws = nullptr;
    int rc = static_scratch_for_current_device(&ws);
    if (rc != HB_OK) return rc;
    for (int l = 1; l <= L; ++l) m->acts[l] = reinterpret_cast<float *>(ws + act_off[l]);
    m->d_loss_partials = reinterpret_cast<float *>(ws + partial_off);
    m->d_loss = reinterpret_cast<float *>(ws + loss_off);
    m->d_params = const_cast<float *>(d_params);  // MODE_LOSS only reads the parameters
    m->configured = true;
    Input in;
    in.X = dX;
    return run_step(m, in, dy, B, 0.f, MODE_LOSS, nullptr, d_loss);
}

int hb_batch_step_csr_async(hb_model *m, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                            const float *d_vals, int64_t nnz, const int32_t *dy, int64_t B, float lr,
                            float *d_loss)
{
    Input in;
    int rc = validate_csr_call(m, d_row_ptr, d_col_idx, d_vals, nnz, dy, B, &in);
    if (rc != HB_OK) return rc;
    if (!std::isfinite(lr)) return fail(HB_ERR_INVALID, "lr is not finite");
    rc = ensure_csc_capacity(m, nnz);
    if (rc != HB_OK) return rc;
    return run_step(m, in, dy, B, lr, MODE_STEP, nullptr, d_loss);
}

int hb_batch_loss_csr_async(hb_model *m, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                            const float *d_vals, int64_t nnz, const int32_t *dy, int64_t B, float *d_loss)
{
    Input in;
    int rc = validate_csr_call(m, d_row_ptr, d_col_idx, d_vals, nnz, dy, B, &in);
    if (rc != HB_OK) return rc;
    return run_step(m, in, dy, B, 0.f, MODE_LOSS, nullptr, d_loss);
}

float hb_batch_loss_csr(hb_model *m, const int32_t *d_row_ptr, const int32_t *d_col_idx, const float *d_vals,
                        int64_t nnz, const int32_t *dy, int64_t B)
{
    if (hb_batch_loss_csr_async(m, d_row_ptr, d_col_idx, d_vals, nnz, dy, B, nullptr) != HB_OK)
        return std::numeric_limits<float>::quiet_NaN();
    float out;
    if (fetch_loss(m, &out) != HB_OK) return std::numeric_limits<float>::quiet_NaN();
    return out;
}

float hb_batch_step_csr(hb_model *m, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                        const float *d_vals, int64_t nnz, const int32_t *dy, int64_t B, float lr)
{
    if (hb_batch_step_csr_async(m, d_row_ptr, d_col_idx, d_vals, nnz, dy, B, lr, nullptr) != HB_OK)
        return std::numeric_limits<float>::quiet_NaN();
    float out;
    if (fetch_loss(m, &out) != HB_OK) return std::numeric_limits<float>::quiet_NaN();
    return out;
}

float hb_batch_grad_csr(hb_model *m, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                        const float *d_vals, int64_t nnz, const int32_t *dy, int64_t B,
                        float *d_grad_flat)
{
    Input in;
    if (validate_csr_call(m, d_row_ptr, d_col_idx, d_vals, nnz, dy, B, &in) != HB_OK)
        return std::numeric_limits<float>::quiet_NaN();
    if (!d_grad_flat) return fail_nan("d_grad_flat is NULL");
    if (ensure_csc_capacity(m, nnz) != HB_OK) return std::numeric_limits<float>::quiet_NaN();
    if (run_step(m, in, dy, B, 0.f, MODE_GRAD, d_grad_flat, nullptr) != HB_OK)
        return std::numeric_limits<float>::quiet_NaN();
    float out;
    if (fetch_loss(m, &out) != HB_OK) return std::numeric_limits<float>::quiet_NaN();
    return out;
}

int hb_model_merge(hb_model *m, float *host_model, float weight)
{
    int rc = check_handle(m, true);
    if (rc != HB_OK) return rc;
    if (!host_model) return fail(HB_ERR_INVALID, "host_model is NULL");
    if (!(weight >= 0.f && weight <= 1.f))
        return fail(HB_ERR_INVALID, "weight = %g is outside [0, 1]", (double)weight);
    const size_t bytes = sizeof(float) * (size_t)m->P;
    if (weight == 0.f) {  // replica <- global: the deep copy of the ExecuteWork handler
        HB_HIP(hipMemcpyAsync(m->d_params, host_model, bytes, hipMemcpyHostToDevice, m->stream));
        rc = sync_w1t_from_flat(m);
        if (rc == HB_OK) rc = refresh_shadows(m);
        if (rc != HB_OK) return rc;
    } else if (weight == 1.f) {  // global <- replica: the push after the update
        rc = sync_flat_from_w1t(m);
        if (rc != HB_OK) return rc;
        HB_HIP(hipMemcpyAsync(host_model, m->d_params, bytes, hipMemcpyDeviceToHost, m->stream));
    } else {
        rc = sync_flat_from_w1t(m);
        if (rc != HB_OK) return rc;
        HB_HIP(hipMemcpyAsync(m->d_stage, host_model, bytes, hipMemcpyHostToDevice, m->stream));
        HB_HIP(launch_merge(m->d_params, m->d_stage, m->P, weight, m->stream));
        HB_HIP(hipMemcpyAsync(host_model, m->d_stage, bytes, hipMemcpyDeviceToHost, m->stream));
        rc = sync_w1t_from_flat(m);
        if (rc == HB_OK) rc = refresh_shadows(m);
        if (rc != HB_OK) return rc;
    }
    HB_HIP(hipStreamSynchronize(m->stream));
    return HB_OK;
}

}  // extern "C"
