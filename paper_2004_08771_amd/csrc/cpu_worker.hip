// CPU worker of Adaptive Hogbatch (Algorithm 2 of the paper, right column; Section 6.1 and 6.2):
// a batch is split into t sub-batches, t threads each compute the gradient of their sub-batch
// on the SHARED host model (Section 3, Eq. (1)-(2)) and apply it (Eq. (3)) without any
// synchronisation, and the worker reports t * beta model updates per batch.  With b = t every
// thread handles one example: Hogwild.  Host code only, fp32, plain loops: this is the slow
// partner whose update counts drive the batch-size adaptation of the GPU worker; it shares
// no code with the GPU kernels and none with the test oracle.
#include "hb_internal.h"

#include <atomic>
#include <cmath>
#include <thread>
#include <vector>

#include "../../include/hb.h"

namespace {

struct Net {
    std::vector<int> dims;
    int L = 0, act = 0, loss = 0;
    std::vector<size_t> w_off, b_off;
    size_t P = 0;
    int max_d = 0;
};

bool make_net(const int32_t *layer_dims, int32_t n_dims, int act, int loss, Net *n)
{
    if (!layer_dims || n_dims < 2 || n_dims > 17) return false;
    if (act != HB_ACT_SIGMOID && act != HB_ACT_RELU) return false;
    if (loss != HB_LOSS_SOFTMAX_CE && loss != HB_LOSS_LOGISTIC) return false;
    n->dims.assign(layer_dims, layer_dims + n_dims);
    n->L = n_dims - 1;
    n->act = act;
    n->loss = loss;
    n->w_off.assign(n->L + 1, 0);
    n->b_off.assign(n->L + 1, 0);
    size_t off = 0;
    for (int l = 0; l <= n->L; ++l) {
        if (layer_dims[l] < 1) return false;
        if (layer_dims[l] > n->max_d) n->max_d = layer_dims[l];
    }
    for (int l = 1; l <= n->L; ++l) {
        n->w_off[l] = off;
        off += (size_t)n->dims[l] * n->dims[l - 1];
        n->b_off[l] = off;
        off += n->dims[l];
    }
    n->P = off;
    if (loss == HB_LOSS_LOGISTIC && n->dims[n->L] > 2) return false;
    return true;
}

// Per-thread scratch: activations of every layer, two delta vectors, the sub-batch gradient.
struct Scratch {
    std::vector<std::vector<float>> a;  // a[l]: d_l
    std::vector<float> d0, d1, g;
    explicit Scratch(const Net &n) : a(n.L + 1), d0(n.max_d), d1(n.max_d), g(n.P)
    {
        for (int l = 0; l <= n.L; ++l) a[l].resize(n.dims[l]);
    }
};

// APPLY = false: adds the gradient of one example's loss (scaled by `scale`) to s.g.
// APPLY = true (a sub-batch of one example, i.e. Hogwild): the update W <- W - lr * scale * g is
// applied to the shared model row by row as the gradient is formed (the row's contribution to
// the layer below is taken before the row is changed), with the same arithmetic as the two-step
// form but without a gradient buffer: a third of the memory traffic.  Returns the loss.
template <bool APPLY>
float example_grad(const Net &n, float *W, const float *x, int y, float scale, float lr, Scratch &s)
{
    const int L = n.L;
    for (int k = 0; k < n.dims[0]; ++k) s.a[0][k] = x[k];
    for (int l = 1; l <= L; ++l) {  // Eq. (1)
        const float *w = W + n.w_off[l], *b = W + n.b_off[l];
        const int din = n.dims[l - 1], dout = n.dims[l];
        const float *__restrict__ ap = s.a[l - 1].data();
        for (int j = 0; j < dout; ++j) {
            const float *__restrict__ wr = w + (size_t)j * din;
            // sixteen partial sums: a single running sum is one dependent add per element
            float acc[16] = {};
            int k = 0;
            for (; k + 16 <= din; k += 16)
                for (int q = 0; q < 16; ++q) acc[q] += ap[k + q] * wr[k + q];
            for (int q = 8; q > 0; q >>= 1)
                for (int i = 0; i < q; ++i) acc[i] += acc[i + q];
            float z = b[j] + acc[0];
            for (; k < din; ++k) z += ap[k] * wr[k];
            if (l < L) z = (n.act == HB_ACT_SIGMOID) ? 1.0f / (1.0f + std::exp(-z)) : (z > 0.f ? z : 0.f);
            s.a[l][j] = z;
        }
    }
    // loss and output delta (Section 7.1)
    const int K = n.dims[L];
    float *d = s.d0.data();
    float lossv;
    const float *z = s.a[L].data();
    if (n.loss == HB_LOSS_LOGISTIC && K == 1) {
        const float mg = (float)y * z[0];
        const float e = std::exp(-std::fabs(mg));
        lossv = (mg < 0.f ? -mg : 0.f) + std::log1p(e);
        const float sg = (mg >= 0.f) ? e / (1.f + e) : 1.f / (1.f + e);
        d[0] = -(float)y * sg;
    } else {
        const int c = (n.loss == HB_LOSS_LOGISTIC) ? (y + 1) / 2 : y;
        float mx = z[0];
        for (int k = 1; k < K; ++k) mx = z[k] > mx ? z[k] : mx;
        float se = 0.f;
        for (int k = 0; k < K; ++k) se += std::exp(z[k] - mx);
        const float lse = mx + std::log(se);
        lossv = lse - z[c];
        for (int k = 0; k < K; ++k) d[k] = std::exp(z[k] - lse) - (k == c ? 1.f : 0.f);
    }
    // Eq. (2), from the last layer down
    float *dn = s.d1.data();
    for (int l = L; l >= 1; --l) {
        float *w = W + n.w_off[l], *bl = W + n.b_off[l];
        float *gw = s.g.data() + n.w_off[l], *gb = s.g.data() + n.b_off[l];
        const int din = n.dims[l - 1], dout = n.dims[l];
        const float *__restrict__ al = s.a[l - 1].data();
        if (l > 1)
            for (int k = 0; k < din; ++k) dn[k] = 0.f;
        float *__restrict__ dnr = dn;
        for (int j = 0; j < dout; ++j) {
            const float dj = d[j];
            float *__restrict__ wr = w + (size_t)j * din;
            if (l > 1)
                for (int k = 0; k < din; ++k) dnr[k] += dj * wr[k];
            if (APPLY) {
                bl[j] -= lr * (scale * dj);
                for (int k = 0; k < din; ++k) wr[k] -= lr * (scale * dj * al[k]);
            } else {
                gb[j] += scale * dj;
                float *__restrict__ gr = gw + (size_t)j * din;
                for (int k = 0; k < din; ++k) gr[k] += scale * dj * al[k];
            }
        }
        if (l > 1) {
            for (int k = 0; k < din; ++k) {
                const float o = s.a[l - 1][k];
                dn[k] *= (n.act == HB_ACT_SIGMOID) ? o * (1.f - o) : (o > 0.f ? 1.f : 0.f);
            }
            float *t = d;
            d = dn;
            dn = t;
        }
    }
    return lossv;
}

int cpu_worker_epoch(hb_sched *s, int32_t worker, const int32_t *layer_dims, int32_t n_dims, int activation, int loss,
                     const float *host_X, const int32_t *host_y, float *host_model, float lr_per_example,
                     int32_t threads, double beta, double *updates, int64_t *batches_out, double *loss_sum_out)
{
    Net net;
    if (!make_net(layer_dims, n_dims, activation, loss, &net))
        return hb::set_error(HB_ERR_INVALID, "hb_cpu_worker_run_epoch: bad network description");
    if (!s || !host_X || !host_y || !host_model) return hb::set_error(HB_ERR_INVALID, "hb_cpu_worker_run_epoch: NULL argument");
    if (threads < 1 || threads > 1024) return hb::set_error(HB_ERR_INVALID, "threads must be in [1, 1024]");
    if (!(beta > 0.0 && beta <= 1.0)) return hb::set_error(HB_ERR_INVALID, "beta must be in (0, 1]");
    if (!(lr_per_example >= 0.f) || !std::isfinite(lr_per_example))
        return hb::set_error(HB_ERR_INVALID, "lr_per_example must be finite and >= 0");
    double u = updates ? *updates : 0.0;
    int64_t batches = 0;
    double loss_sum = 0.0;
    std::vector<Scratch> scratch;
    scratch.reserve(threads);
    for (int t = 0; t < threads; ++t) scratch.emplace_back(net);
    std::vector<double> tl(threads, 0.0);
    const int d0 = net.dims[0];
    for (;;) {
        int64_t begin = 0, count = 0;
        const int rc = hb_sched_request(s, worker, u, &begin, &count);
        if (rc != HB_OK) return rc;
        if (count == 0) break;
        // labels index the output scores: a label outside its domain is an error, not a stray read
        for (int64_t i = begin; i < begin + count; ++i) {
            const int32_t yi = host_y[i];
            const bool ok = (loss == HB_LOSS_LOGISTIC) ? (yi == 1 || yi == -1) : (yi >= 0 && yi < net.dims[net.L]);
            if (!ok)
                return hb::set_error(HB_ERR_INVALID, "hb_cpu_worker_run_epoch: label %d of example %lld is outside its domain (%s)",
                                     (int)yi, (long long)i,
                                     loss == HB_LOSS_LOGISTIC ? "+1 / -1" : "class index in [0, d_L)");
        }
        // sub-batch i: rows [begin + i*count/t, begin + (i+1)*count/t)
        auto work = [&](int t) {
            const int64_t lo = begin + count * t / threads, hi = begin + count * (t + 1) / threads;
            tl[t] = 0.0;
            if (hi <= lo) return;
            Scratch &sc = scratch[t];
            const float lr = lr_per_example * (float)(hi - lo);  // proportional to the (sub-)batch size
            if (hi - lo == 1) {  // Hogwild: one example, applied as it is formed
                tl[t] = example_grad<true>(net, host_model, host_X + (size_t)lo * d0, host_y[lo], 1.0f, lr, sc);
                return;
            }
            std::fill(sc.g.begin(), sc.g.end(), 0.f);
            const float inv = 1.0f / (float)(hi - lo);  // gradient of the sub-batch: mean over its examples
            for (int64_t i = lo; i < hi; ++i)
                tl[t] += example_grad<false>(net, host_model, host_X + (size_t)i * d0, host_y[i], inv, 0.f, sc);
            for (size_t p = 0; p < net.P; ++p) host_model[p] -= lr * sc.g[p];  // no locks, no atomics
            tl[t] /= (double)(hi - lo);
        };
        if (threads == 1) {
            work(0);
        } else {
            // Threads are started per batch on purpose: a pool of sleeping threads woken through
            // a condition variable was measured SLOWER (8 threads, 54-512x4-7: 8.8k against 12.6k
            // rows/s at 8 rows per thread), the woken threads starting on the waker's core.
            std::vector<std::thread> pool;
            bool started_all = true;
            try {
                pool.reserve(threads);
                for (int t = 0; t < threads; ++t) pool.emplace_back(work, t);
            } catch (...) {  // no exception may cross the C boundary
                started_all = false;
            }
            for (auto &th : pool) th.join();
            if (!started_all)
                return hb::set_error(HB_ERR_ALLOC, "hb_cpu_worker_run_epoch: could not start %d threads", (int)threads);
        }
        for (int t = 0; t < threads; ++t) loss_sum += tl[t];
        u += (double)threads * beta;  // Algorithm 2, CPU worker: t * beta surviving updates per batch
        ++batches;
    }
    if (updates) *updates = u;
    if (batches_out) *batches_out = batches;
    if (loss_sum_out) *loss_sum_out = loss_sum;
    return HB_OK;
}

}  // namespace

extern "C" int hb_cpu_worker_run_epoch(hb_sched *s, int32_t worker, const int32_t *layer_dims, int32_t n_dims,
                                       int activation, int loss, const float *host_X, const int32_t *host_y,
                                       float *host_model, float lr_per_example, int32_t threads, double beta,
                                       double *updates, int64_t *batches_out, double *loss_sum_out)
{
    try {
        return cpu_worker_epoch(s, worker, layer_dims, n_dims, activation, loss, host_X, host_y, host_model,
                                lr_per_example, threads, beta, updates, batches_out, loss_sum_out);
    } catch (...) {  // allocation of the per-thread scratch: no exception may cross the C boundary
        return hb::set_error(HB_ERR_ALLOC, "hb_cpu_worker_run_epoch: out of host memory");
    }
}
