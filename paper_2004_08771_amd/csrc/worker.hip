// Coordinator-side batch scheduling of Adaptive Hogbatch (Algorithm 2 of the paper,
// ScheduleWork handler; Section 6.3) and the GPU worker's loop around the mini-batch step
// (Section 5.1: the GPU worker is the exclusive interface of its device and pays the
// host-to-device transfer of every batch; Section 6.2: deep copy of the global model, push
// after updating).  Host code only: the step itself is hb_batch_step_async.
//
// gfx950 / HIP design of the loop: two device staging buffers and a copy stream; the rows of
// batch k+1 travel over PCIe while batch k computes.  Both hand-overs are waited for on the
// HOST, which runs one step ahead of the device: the copy into a buffer is issued once the step
// that last read it has finished (the device has the current step queued meanwhile), and a
// step is enqueued once its buffer's copy has landed (issued a whole step earlier), so that
// neither stream ever waits for the other on the device.  A push of the
// replica (merge weight 1) is asynchronous as in Section 6.2: a device-to-device snapshot in
// stream order, then device -> host on a third stream beside the following steps, straight
// into the host model when that is page-locked; a two-way exchange (weight < 1) first brings
// the global model to the device on that stream and blends in stream order.  Everything stays
// at the default stream priority.  The training and the evaluation loop each exist once, for
// dense rows and for CSR rows (sparse first layer): a CSR batch travels as the rebased slice of
// the row pointer plus its column indices and values.
#include "hb_internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdlib>
#include <cstring>
#include <exception>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "../../include/hb.h"

struct hb_sched {
    int64_t n = 0, cursor = 0;
    double alpha = 2.0;
    std::vector<int64_t> min_b, max_b, b;
    std::vector<double> u;
    std::mutex lock;  // the coordinator serves requests serially
};

namespace {

int64_t round_half_away(double x) { return (int64_t)std::floor(x + 0.5); }

}  // namespace

extern "C" {

hb_sched *hb_sched_create(int64_t n_examples, int32_t n_workers, const int64_t *min_b, const int64_t *max_b,
                          const int64_t *init_b, double alpha)
{
    if (n_examples < 0 || n_workers < 1 || !min_b || !max_b || !init_b || !(alpha > 1.0) || !std::isfinite(alpha)) {
        hb::set_error(HB_ERR_INVALID, "hb_sched_create: need n_examples >= 0, n_workers >= 1, threshold arrays, alpha > 1");
        return nullptr;
    }
    for (int32_t w = 0; w < n_workers; ++w)
        if (min_b[w] < 1 || init_b[w] < min_b[w] || max_b[w] < init_b[w]) {
            hb::set_error(HB_ERR_INVALID, "hb_sched_create: worker %d needs 1 <= min_b <= init_b <= max_b", (int)w);
            return nullptr;
        }
    hb_sched *s = new (std::nothrow) hb_sched;
    if (!s) {
        hb::set_error(HB_ERR_ALLOC, "hb_sched_create: out of host memory");
        return nullptr;
    }
    s->n = n_examples;
    s->alpha = alpha;
    s->min_b.assign(min_b, min_b + n_workers);
    s->max_b.assign(max_b, max_b + n_workers);
    s->b.assign(init_b, init_b + n_workers);
    s->u.assign(n_workers, 0.0);
    return s;
}

void hb_sched_destroy(hb_sched *s) { delete s; }

int hb_sched_request(hb_sched *s, int32_t worker, double updates, int64_t *begin, int64_t *count)
{
    if (!s || !begin || !count) return hb::set_error(HB_ERR_INVALID, "hb_sched_request: NULL argument");
    if (worker < 0 || worker >= (int32_t)s->b.size())
        return hb::set_error(HB_ERR_INVALID, "hb_sched_request: worker %d is outside [0, %d)", (int)worker,
                             (int)s->b.size());
    if (!(updates >= 0.0) || !std::isfinite(updates))
        return hb::set_error(HB_ERR_INVALID, "hb_sched_request: update count must be finite and >= 0");
    std::lock_guard<std::mutex> g(s->lock);
    s->u[worker] = updates;
    // smallest / largest update count of all other workers
    bool any = false;
    double min_u = 0.0, max_u = 0.0;
    for (size_t w = 0; w < s->u.size(); ++w) {
        if ((int32_t)w == worker) continue;
        if (!any || s->u[w] < min_u) min_u = s->u[w];
        if (!any || s->u[w] > max_u) max_u = s->u[w];
        any = true;
    }
    int64_t &b = s->b[worker];
    if (any) {
        if (updates < min_u) {  // lagging: smaller batches, more updates
            int64_t nb = round_half_away((double)b / s->alpha);
            if (nb < 1) nb = 1;
            b = nb > s->min_b[worker] ? nb : s->min_b[worker];
        } else if (updates > max_u) {  // ahead: larger batches, fewer updates
            const int64_t nb = round_half_away((double)b * s->alpha);
            b = nb < s->max_b[worker] ? nb : s->max_b[worker];
        }
    }
    *begin = s->cursor;
    if (b <= s->n - s->cursor) {
        *count = b;
        s->cursor += b;
    } else {
        *count = 0;  // nothing is sent: the worker is done for this epoch
    }
    return HB_OK;
}

int hb_sched_new_epoch(hb_sched *s)
{
    if (!s) return hb::set_error(HB_ERR_INVALID, "hb_sched_new_epoch: NULL scheduler");
    std::lock_guard<std::mutex> g(s->lock);
    s->cursor = 0;
    return HB_OK;
}

int64_t hb_sched_batch_size(const hb_sched *s, int32_t worker)
{
    if (!s || worker < 0 || worker >= (int32_t)s->b.size()) {
        hb::set_error(HB_ERR_INVALID, "hb_sched_batch_size: bad scheduler or worker");
        return -1;
    }
    return s->b[worker];
}

int64_t hb_sched_remaining(const hb_sched *s)
{
    if (!s) {
        hb::set_error(HB_ERR_INVALID, "hb_sched_remaining: NULL scheduler");
        return -1;
    }
    return s->n - s->cursor;
}

}  // extern "C"

namespace {

// Device side of the double buffering.  Lives in the model handle from the first epoch on
// (re-created when a larger capacity is needed), released by hb_model_destroy.
struct Staging {
    int64_t cap = 0;
    size_t row_bytes = 0;
    void *x[2] = {nullptr, nullptr};
    int32_t *y[2] = {nullptr, nullptr};
    float *loss = nullptr;       // one slot per step of a window, device
    float *loss_host = nullptr;  // page-locked mirror
    hipStream_t copy = nullptr;
    hipEvent_t filled[2] = {nullptr, nullptr};    // the copy into buffer i has finished
    hipEvent_t consumed[2] = {nullptr, nullptr};  // the step reading buffer i has finished
    // asynchronous push of the replica (merge weight 1): a device snapshot, a page-locked
    // landing buffer for host models in pageable memory, a third stream
    long long snap_elems = 0;
    float *snap = nullptr;
    float *snap_host = nullptr;
    hipStream_t push = nullptr;
    hipEvent_t snap_taken = nullptr;   // the snapshot is complete (model's stream)
    hipEvent_t snap_landed = nullptr;  // the snapshot has reached host memory (push stream)
    hipEvent_t glob_here = nullptr;    // the global model has reached the device (push stream)
    // CSR batches: the slice of the row pointer is rebased to start at 0 in a page-locked array,
    // column indices and values travel as they are
    int64_t nnz_cap = 0;
    int64_t nnz[2] = {0, 0};  // stored entries of the batch in buffer i
    int32_t *rp[2] = {nullptr, nullptr};
    int32_t *rp_host[2] = {nullptr, nullptr};
    int32_t *ci[2] = {nullptr, nullptr};
    float *va[2] = {nullptr, nullptr};
    void release_csr_values()
    {
        for (int i = 0; i < 2; ++i) {
            if (ci[i]) (void)hipFree(ci[i]);
            if (va[i]) (void)hipFree(va[i]);
            ci[i] = nullptr;
            va[i] = nullptr;
        }
        nnz_cap = 0;
    }
    ~Staging()
    {
        if (push) (void)hipStreamSynchronize(push);
        if (snap) (void)hipFree(snap);
        if (snap_host) (void)hipHostFree(snap_host);
        if (snap_taken) (void)hipEventDestroy(snap_taken);
        if (snap_landed) (void)hipEventDestroy(snap_landed);
        if (glob_here) (void)hipEventDestroy(glob_here);
        if (push) (void)hipStreamDestroy(push);
        if (copy) (void)hipStreamSynchronize(copy);
        for (int i = 0; i < 2; ++i) {
            if (x[i]) (void)hipFree(x[i]);
            if (y[i]) (void)hipFree(y[i]);
            if (filled[i]) (void)hipEventDestroy(filled[i]);
            if (consumed[i]) (void)hipEventDestroy(consumed[i]);
        }
        release_csr_values();
        for (int i = 0; i < 2; ++i) {
            if (rp[i]) (void)hipFree(rp[i]);
            if (rp_host[i]) (void)hipHostFree(rp_host[i]);
        }
        if (loss) (void)hipFree(loss);
        if (loss_host) (void)hipHostFree(loss_host);
        if (copy) (void)hipStreamDestroy(copy);
    }
};

constexpr int LOSS_WINDOW = 256;  // losses are fetched in windows of this many steps

#define WK_HIP(call)                                                                               \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess)                                                                      \
            return hb::set_error(HB_ERR_DEVICE, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), \
                                 __FILE__, __LINE__);                                              \
    } while (0)

// The handle's staging buffers, (re)created for at least `cap` rows of `row_bytes` bytes.
int acquire_staging(hb_model *m, const hb::ModelInfo &mi, int64_t cap, size_t row_bytes, Staging **out)
{
    void **slot = hb::model_worker_slot(m, [](void *p) { delete static_cast<Staging *>(p); });
    Staging *sp = static_cast<Staging *>(*slot);
    if (sp && (sp->cap < cap || sp->row_bytes != row_bytes)) {
        WK_HIP(hipStreamSynchronize(mi.stream));
        delete sp;
        sp = nullptr;
        *slot = nullptr;
    }
    if (!sp) {
        sp = new (std::nothrow) Staging;
        if (!sp) return hb::set_error(HB_ERR_ALLOC, "hb_worker_run_epoch: out of host memory");
        *slot = sp;  // owned by the handle from here on, also if an allocation below fails
        sp->cap = 0;
        sp->row_bytes = row_bytes;
        for (int i = 0; i < 2; ++i) {
            if (row_bytes) WK_HIP(hipMalloc(&sp->x[i], row_bytes * (size_t)cap));  // no dense rows for CSR input
            WK_HIP(hipMalloc(reinterpret_cast<void **>(&sp->y[i]), sizeof(int32_t) * (size_t)cap));
            WK_HIP(hipEventCreateWithFlags(&sp->filled[i], hipEventDisableTiming));
            // "consumed" only orders the copy engine behind a step that READ the buffer: no data
            // has to become visible, so the system-scope fence of the record is switched off
            // (its cache write-back and invalidation cost 3 us per step)
            WK_HIP(hipEventCreateWithFlags(&sp->consumed[i], hipEventDisableTiming | hipEventDisableSystemFence));
        }
        WK_HIP(hipMalloc(reinterpret_cast<void **>(&sp->loss), sizeof(float) * LOSS_WINDOW));
        WK_HIP(hipHostMalloc(reinterpret_cast<void **>(&sp->loss_host), sizeof(float) * LOSS_WINDOW,
                             hipHostMallocDefault));
        WK_HIP(hipStreamCreateWithFlags(&sp->copy, hipStreamNonBlocking));  // default priority
        sp->cap = cap;
    }
    *out = sp;
    return HB_OK;
}

// Resources of the asynchronous push, created at the first epoch that pushes.
int acquire_push(Staging &st, long long P)
{
    if (st.snap_elems >= P && st.push) return HB_OK;
    if (st.push) WK_HIP(hipStreamSynchronize(st.push));
    if (st.snap) WK_HIP(hipFree(st.snap));
    if (st.snap_host) WK_HIP(hipHostFree(st.snap_host));
    st.snap = nullptr;
    st.snap_host = nullptr;
    st.snap_elems = 0;
    WK_HIP(hipMalloc(reinterpret_cast<void **>(&st.snap), sizeof(float) * (size_t)P));
    WK_HIP(hipHostMalloc(reinterpret_cast<void **>(&st.snap_host), sizeof(float) * (size_t)P, hipHostMallocDefault));
    if (!st.push) WK_HIP(hipStreamCreateWithFlags(&st.push, hipStreamNonBlocking));  // default priority
    if (!st.snap_taken) WK_HIP(hipEventCreateWithFlags(&st.snap_taken, hipEventDisableTiming));
    if (!st.snap_landed) WK_HIP(hipEventCreateWithFlags(&st.snap_landed, hipEventDisableTiming));
    if (!st.glob_here) WK_HIP(hipEventCreateWithFlags(&st.glob_here, hipEventDisableTiming));
    st.snap_elems = P;
    return HB_OK;
}

// The kernels of a batch must not start before its copy has landed.  The HOST waits for the copy
// (it runs one step ahead of the device, so the copy, issued a whole step earlier, has normally
// finished) and the kernels are then enqueued without any cross-stream dependency: a
// hipStreamWaitEvent on the model's stream costs 4-8 us of idle device time between two steps
// (config 2, B = 4096: 244 -> 240 us per step; B = 512: 104.5 -> 100.5).  When the transfer takes
// longer than the step the device-side wait would start the step a launch latency earlier:
// HB_WORKER_STREAMWAIT=1 selects it (tuning aid).
int wait_filled(Staging &st, int buf, hipStream_t model_stream)
{
    static const bool stream_wait = getenv("HB_WORKER_STREAMWAIT") && atoi(getenv("HB_WORKER_STREAMWAIT")) != 0;
    if (stream_wait) WK_HIP(hipStreamWaitEvent(model_stream, st.filled[buf], 0));
    else WK_HIP(hipEventSynchronize(st.filled[buf]));
    return HB_OK;
}

// Row-pointer staging for the staging buffers' row capacity (kept for the life of the staging buffers) and room for
// batches of `nnz` stored entries, grown with headroom when a batch needs more.  The caller
// makes sure that nothing reads the old buffers any more before they are replaced.
int acquire_csr(Staging &st, int64_t nnz)
{
    for (int i = 0; i < 2; ++i) {
        if (!st.rp[i]) WK_HIP(hipMalloc(reinterpret_cast<void **>(&st.rp[i]), sizeof(int32_t) * (size_t)(st.cap + 1)));
        if (!st.rp_host[i])
            WK_HIP(hipHostMalloc(reinterpret_cast<void **>(&st.rp_host[i]), sizeof(int32_t) * (size_t)(st.cap + 1),
                                 hipHostMallocDefault));
    }
    if (nnz <= st.nnz_cap) return HB_OK;
    st.release_csr_values();
    const int64_t want = nnz + nnz / 4 + 1024;
    for (int i = 0; i < 2; ++i) {
        WK_HIP(hipMalloc(reinterpret_cast<void **>(&st.ci[i]), sizeof(int32_t) * (size_t)want));
        WK_HIP(hipMalloc(reinterpret_cast<void **>(&st.va[i]), sizeof(float) * (size_t)want));
    }
    st.nnz_cap = want;
    return HB_OK;
}

// One push in flight at most.  finish() waits for it and, when the host model is in pageable
// memory, copies the landed snapshot into it; the destructor does the same on every way out
// of the epoch, so nothing writes to the caller's memory after the call has returned.
struct PushGuard {
    Staging &st;
    float *host_model;
    size_t bytes;
    bool direct;  // the host model is page-locked: the copy engine writes into it
    bool in_flight = false;
    int finish()
    {
        if (!in_flight) return HB_OK;
        in_flight = false;
        WK_HIP(hipEventSynchronize(st.snap_landed));
        if (!direct) std::memcpy(host_model, st.snap_host, bytes);
        return HB_OK;
    }
    ~PushGuard() { (void)finish(); }
};

// On every way out of a loop, the failing ones included, nothing is still reading the caller's
// host arrays or writing the staging buffers: all streams are drained (a no-op after the
// loops' own final synchronisation).
struct DrainGuard {
    Staging &st;
    hipStream_t model;
    ~DrainGuard()
    {
        (void)hipStreamSynchronize(st.copy);
        if (st.push) (void)hipStreamSynchronize(st.push);
        (void)hipStreamSynchronize(model);
    }
};

// Host-resident CSR training data: row pointer of n_examples + 1 entries over col_idx / vals.
struct CsrHost {
    const int64_t *row_ptr;
    const int32_t *col_idx;
    const float *vals;
};

// Sends rows [begin, begin + count) of host-resident CSR data into staging buffer `buf` on the
// copy stream: the row-pointer slice rebased to 0, column indices and values as they are.  The
// caller has seen buffer buf's last reader finish.
int send_csr_rows(const char *who, Staging &st, hipStream_t model_stream, const CsrHost &csr, int d0, int buf,
                  int64_t begin, int64_t count)
{
    const int64_t base = csr.row_ptr[begin];
    const int64_t nnz = csr.row_ptr[begin + count] - base;
    if (nnz < 0 || nnz > INT32_MAX)
        return hb::set_error(HB_ERR_INVALID, "%s: rows [%lld, %lld) hold %lld stored entries", who, (long long)begin,
                             (long long)(begin + count), (long long)nnz);
    if (nnz > st.nnz_cap) {
        // both value buffers are replaced: the kernels still reading the other one have to finish
        WK_HIP(hipStreamSynchronize(st.copy));
        WK_HIP(hipStreamSynchronize(model_stream));
        const int rc_c = acquire_csr(st, nnz);
        if (rc_c != HB_OK) return rc_c;
    }
    // rp_host[buf] was last read by the copy that filled this buffer two batches ago; the
    // kernels that waited for that copy have been seen to finish
    int32_t *rp = st.rp_host[buf];
    for (int64_t i = 0; i <= count; ++i) {
        const int64_t off = csr.row_ptr[begin + i] - base;
        if (off < 0 || off > nnz || (i > 0 && off < rp[i - 1]))
            return hb::set_error(HB_ERR_INVALID, "%s: host_row_ptr is not non-decreasing at row %lld", who,
                                 (long long)(begin + i));
        rp[i] = (int32_t)off;
    }
    // the kernels trust column indices: one pass over the batch's indices on the host (it walks
    // them anyway to copy them) turns an index outside [0, d_0) into an error
    {
        const int32_t *ci = csr.col_idx + base;
        unsigned int bad = 0;
        for (int64_t i = 0; i < nnz; ++i) bad |= (unsigned int)((unsigned int)ci[i] >= (unsigned int)d0);
        if (bad) {
            int64_t i = 0;
            while ((unsigned int)ci[i] < (unsigned int)d0) ++i;
            return hb::set_error(HB_ERR_INVALID, "%s: column index %d of stored entry %lld is outside [0, %d)", who,
                                 (int)ci[i], (long long)(base + i), d0);
        }
    }
    st.nnz[buf] = nnz;
    WK_HIP(hipMemcpyAsync(st.rp[buf], rp, sizeof(int32_t) * (size_t)(count + 1), hipMemcpyHostToDevice, st.copy));
    if (nnz > 0) {
        WK_HIP(hipMemcpyAsync(st.ci[buf], csr.col_idx + base, sizeof(int32_t) * (size_t)nnz, hipMemcpyHostToDevice,
                              st.copy));
        WK_HIP(hipMemcpyAsync(st.va[buf], csr.vals + base, sizeof(float) * (size_t)nnz, hipMemcpyHostToDevice,
                              st.copy));
    }
    return HB_OK;
}

}  // namespace

// The worker's loop for dense rows (csr == nullptr) or CSR rows (host_X == nullptr).
static int run_epoch(const char *who, hb_model *m, hb_sched *s, int32_t worker, const void *host_X,
                     const CsrHost *csr, const int32_t *host_y, float lr_per_example, float *host_model,
                     int32_t merge_every, float merge_weight, double *updates, int64_t *steps_out,
                     double *loss_sum_out)
{
    hb::ModelInfo mi;
    if (!hb::model_info(m, &mi)) return hb_last_error_code();
    if (!s || !host_y || (!csr && !host_X) || (csr && (!csr->row_ptr || !csr->col_idx || !csr->vals)))
        return hb::set_error(HB_ERR_INVALID, "%s: NULL argument", who);
    if (worker < 0 || worker >= (int32_t)s->b.size())
        return hb::set_error(HB_ERR_INVALID, "%s: worker %d is outside [0, %d)", who, (int)worker, (int)s->b.size());
    if ((mi.sparse != 0) != (csr != nullptr))
        return hb::set_error(HB_ERR_UNSUPPORTED, csr ? "%s: the model is not configured with sparse_first_layer"
                                                     : "%s: dense input only (hb_worker_run_epoch_csr takes CSR data)",
                             who);
    if (s->max_b[worker] > mi.max_B)
        return hb::set_error(HB_ERR_INVALID, "the scheduler's max_b (%lld) of this worker exceeds the model's max_B (%lld)",
                             (long long)s->max_b[worker], (long long)mi.max_B);
    if (!(lr_per_example >= 0.f) || !std::isfinite(lr_per_example))
        return hb::set_error(HB_ERR_INVALID, "lr_per_example must be finite and >= 0");
    if (merge_every < 0 || (merge_every > 0 && host_model && !(merge_weight >= 0.f && merge_weight <= 1.f)))
        return hb::set_error(HB_ERR_INVALID, "merge_every must be >= 0 and merge_weight in [0, 1]");
    const bool merging = merge_every > 0 && host_model != nullptr;
    // weight 1 is the paper's push (global <- replica, Section 6.2): it leaves the replica as it
    // is; any other weight also brings the global model to the device and blends there.  Either
    // way the transfers run on a third stream beside the steps.
    const bool pushing = merging && merge_weight == 1.f;

    const size_t elem = (mi.dtype == HB_BF16_F32MASTER) ? 2 : 4;
    const size_t row_bytes = csr ? 0 : elem * (size_t)mi.d0;
    const int64_t cap = s->max_b[worker];
    Staging *sp = nullptr;
    {
        const int rc_st = acquire_staging(m, mi, cap, row_bytes, &sp);
        if (rc_st != HB_OK) return rc_st;
    }
    Staging &st = *sp;
    if (csr) {
        const int rc_c = acquire_csr(st, 0);
        if (rc_c != HB_OK) return rc_c;
    }
    DrainGuard drain{st, mi.stream};
    bool host_model_locked = false;
    if (merging) {
        const int rc_p = acquire_push(st, mi.P);
        if (rc_p != HB_OK) return rc_p;
        hipPointerAttribute_t attr;
        if (hipPointerGetAttributes(&attr, host_model) == hipSuccess)
            host_model_locked = (attr.type == hipMemoryTypeHost);
        else
            (void)hipGetLastError();  // ordinary pageable memory is unknown to the runtime
    }
    PushGuard push{st, host_model, sizeof(float) * (size_t)mi.P, host_model_locked};
    // A snapshot (or a blend) is produced in stream order on the model's stream; its journey to
    // the host is ISSUED later, by issue_d2h(), once the next step has been enqueued: the host
    // waits there for the snapshot event, so that the copy call needs no cross-stream wait (an
    // asynchronous copy behind a hipStreamWaitEvent blocks inside the runtime, see fetch()),
    // and the device has work queued while the host waits.
    bool snap_pending = false;  // st.snap is being written / read on the model's stream (snap_taken covers it)
    bool d2h_wanted = false;    // ... and has to travel to the host afterwards
    auto issue_d2h = [&]() -> int {
        if (!snap_pending) return HB_OK;
        snap_pending = false;
        WK_HIP(hipEventSynchronize(st.snap_taken));
        if (!d2h_wanted) return HB_OK;
        d2h_wanted = false;
        WK_HIP(hipMemcpyAsync(push.direct ? host_model : st.snap_host, st.snap, push.bytes, hipMemcpyDeviceToHost,
                              st.push));
        WK_HIP(hipEventRecord(st.snap_landed, st.push));
        push.in_flight = true;
        return HB_OK;
    };
    // everything of the previous exchange is over: st.snap and the landing buffer are free
    auto settle = [&]() -> int {
        int rc_f = issue_d2h();
        return rc_f != HB_OK ? rc_f : push.finish();
    };
    auto push_async = [&]() -> int {
        int rc_f = settle();
        if (rc_f != HB_OK) return rc_f;
        rc_f = hb::model_flat_refresh(m);  // a sparse first layer is kept transposed beside the flat buffer
        if (rc_f != HB_OK) return rc_f;
        WK_HIP(hipMemcpyAsync(st.snap, hb::model_params_device(m), push.bytes, hipMemcpyDeviceToDevice, mi.stream));
        WK_HIP(hipEventRecord(st.snap_taken, mi.stream));
        snap_pending = d2h_wanted = true;
        return HB_OK;
    };

    // Two-way exchange (0 <= weight < 1): the global model travels to the device while the
    // current step still runs, the blend M = (1 - w) global + w replica follows that step in
    // stream order (both the replica and the staging buffer then hold M), and M travels back
    // like a push.  The global model is read when this is called, i.e. up to one exchange
    // earlier than a synchronous hb_model_merge would read it: updates other workers make in
    // between are overwritten by M, as Section 6.2 accepts for concurrent workers.
    auto exchange_async = [&]() -> int {
        int rc_f = settle();
        if (rc_f != HB_OK) return rc_f;
        WK_HIP(hipMemcpyAsync(st.snap, host_model, push.bytes, hipMemcpyHostToDevice, st.push));
        WK_HIP(hipEventRecord(st.glob_here, st.push));
        WK_HIP(hipStreamWaitEvent(mi.stream, st.glob_here, 0));  // followed by kernel launches only
        rc_f = hb::model_blend_with_device(m, st.snap, merge_weight);
        if (rc_f != HB_OK) return rc_f;
        WK_HIP(hipEventRecord(st.snap_taken, mi.stream));
        snap_pending = true;
        d2h_wanted = merge_weight > 0.f;  // weight 0 is the deep copy alone: the global model is unchanged
        return HB_OK;
    };

    double u = updates ? *updates : 0.0;
    int64_t steps = 0;
    double loss_sum = 0.0;
    int in_window = 0;
    int64_t since_merge = 0;
    auto flush_losses = [&]() -> int {
        if (in_window == 0) return HB_OK;
        WK_HIP(hipMemcpyAsync(st.loss_host, st.loss, sizeof(float) * in_window, hipMemcpyDeviceToHost, mi.stream));
        WK_HIP(hipStreamSynchronize(mi.stream));
        for (int i = 0; i < in_window; ++i) loss_sum += st.loss_host[i];
        in_window = 0;
        return HB_OK;
    };
    // ask for a batch and start its transfer into staging buffer `buf`
    auto fetch = [&](int buf, double u_report, int64_t *count) -> int {
        int64_t begin = 0;
        int rc = hb_sched_request(s, worker, u_report, &begin, count);
        if (rc != HB_OK || *count == 0) return rc;
        if (*count > cap) return hb::set_error(HB_ERR_STATE, "scheduler handed out %lld rows, more than max_b", (long long)*count);
        // The buffer's previous reader must be done before it is overwritten.  The HOST waits
        // for it: a hipStreamWaitEvent on the copy stream makes the asynchronous copy call that
        // follows block inside the runtime for far longer (probe with a 150 us kernel per
        // iteration: 215-490 us per iteration against 148 with this host-side wait).
        WK_HIP(hipEventSynchronize(st.consumed[buf]));
        if (csr) {
            const int rc_s = send_csr_rows(who, st, mi.stream, *csr, mi.d0, buf, begin, *count);
            if (rc_s != HB_OK) return rc_s;
        } else {
            WK_HIP(hipMemcpyAsync(st.x[buf], static_cast<const unsigned char *>(host_X) + row_bytes * (size_t)begin,
                                  row_bytes * (size_t)*count, hipMemcpyHostToDevice, st.copy));
        }
        WK_HIP(hipMemcpyAsync(st.y[buf], host_y + begin, sizeof(int32_t) * (size_t)*count, hipMemcpyHostToDevice,
                              st.copy));
        WK_HIP(hipEventRecord(st.filled[buf], st.copy));
        return HB_OK;
    };

    for (int i = 0; i < 2; ++i) WK_HIP(hipEventRecord(st.consumed[i], mi.stream));  // both buffers start free
    int64_t cur = 0, nxt = 0;
    int rc = fetch(0, u, &cur);
    if (rc != HB_OK) return rc;
    int buf = 0;
    while (cur > 0) {
        rc = wait_filled(st, buf, mi.stream);
        if (rc != HB_OK) return rc;
        rc = csr ? hb_batch_step_csr_async(m, st.rp[buf], st.ci[buf], st.va[buf], st.nnz[buf], st.y[buf], cur,
                                           lr_per_example * (float)cur, st.loss + in_window)
                 : hb_batch_step_async(m, st.x[buf], st.y[buf], cur, lr_per_example * (float)cur,
                                       st.loss + in_window);
        if (rc != HB_OK) return rc;
        WK_HIP(hipEventRecord(st.consumed[buf], mi.stream));
        rc = issue_d2h();  // the snapshot taken after step k-1 leaves now that step k is queued
        if (rc != HB_OK) return rc;
        // Batch k+1 is requested while batch k computes, with the update count batch k will
        // have produced.  The request comes AFTER step k has been enqueued: it waits on the
        // host until the other buffer's last reader (step k-1) has finished, and the device
        // must have step k queued by then or it idles meanwhile.
        rc = fetch(buf ^ 1, u + 1.0, &nxt);
        if (rc != HB_OK) return rc;
        u += 1.0;
        ++steps;
        ++since_merge;
        if (++in_window == LOSS_WINDOW) {
            rc = flush_losses();
            if (rc != HB_OK) return rc;
        }
        if (merging && since_merge >= merge_every) {
            rc = pushing ? push_async() : exchange_async();
            if (rc != HB_OK) return rc;
            since_merge = 0;
        }
        cur = nxt;
        buf ^= 1;
    }
    rc = flush_losses();
    if (rc != HB_OK) return rc;
    if (merging && since_merge > 0) {
        rc = pushing ? push_async() : exchange_async();
        if (rc != HB_OK) return rc;
    }
    rc = settle();
    if (rc != HB_OK) return rc;
    WK_HIP(hipStreamSynchronize(st.copy));
    WK_HIP(hipStreamSynchronize(mi.stream));
    if (updates) *updates = u;
    if (steps_out) *steps_out = steps;
    if (loss_sum_out) *loss_sum_out = loss_sum;
    return HB_OK;
}

extern "C" int hb_worker_run_epoch(hb_model *m, hb_sched *s, int32_t worker, const void *host_X,
                                   const int32_t *host_y, float lr_per_example, float *host_model,
                                   int32_t merge_every, float merge_weight, double *updates, int64_t *steps_out,
                                   double *loss_sum_out)
{
    if (!host_X) return hb::set_error(HB_ERR_INVALID, "hb_worker_run_epoch: NULL argument");
    return run_epoch("hb_worker_run_epoch", m, s, worker, host_X, nullptr, host_y, lr_per_example, host_model,
                     merge_every, merge_weight, updates, steps_out, loss_sum_out);
}

extern "C" int hb_worker_run_epoch_csr(hb_model *m, hb_sched *s, int32_t worker, const int64_t *host_row_ptr,
                                       const int32_t *host_col_idx, const float *host_vals, const int32_t *host_y,
                                       float lr_per_example, float *host_model, int32_t merge_every,
                                       float merge_weight, double *updates, int64_t *steps_out,
                                       double *loss_sum_out)
{
    const CsrHost csr{host_row_ptr, host_col_idx, host_vals};
    return run_epoch("hb_worker_run_epoch_csr", m, s, worker, nullptr, &csr, host_y, lr_per_example, host_model,
                     merge_every, merge_weight, updates, steps_out, loss_sum_out);
}

// One epoch of the heterogeneous algorithms: the CPU worker on a thread of its own, the GPU
// worker on the calling thread, both against the same scheduler and host model.
extern "C" int hb_hogbatch_run_epoch(hb_sched *s, hb_model *gpu, int32_t gpu_worker, int32_t cpu_worker,
                                     const float *host_X, const int32_t *host_y, float *host_model,
                                     float lr_per_example, int32_t cpu_threads, double beta, int32_t merge_every,
                                     float merge_weight, double *gpu_updates, double *cpu_updates,
                                     hb_epoch_stats *stats)
{
    hb::ModelInfo mi;
    if (!hb::model_info(gpu, &mi)) return hb_last_error_code();
    if (!s || !host_X || !host_y || !host_model)
        return hb::set_error(HB_ERR_INVALID, "hb_hogbatch_run_epoch: NULL argument");
    if (mi.sparse || mi.dtype != HB_F32)
        return hb::set_error(HB_ERR_UNSUPPORTED,
                             "hb_hogbatch_run_epoch: both workers read the same fp32 dense rows (HB_F32, no sparse first layer)");
    const int32_t n_workers = (int32_t)s->b.size();
    if (gpu_worker < 0 || gpu_worker >= n_workers || cpu_worker < 0 || cpu_worker >= n_workers || gpu_worker == cpu_worker)
        return hb::set_error(HB_ERR_INVALID, "hb_hogbatch_run_epoch: workers %d and %d must be two different workers in [0, %d)",
                             (int)gpu_worker, (int)cpu_worker, (int)n_workers);
    if (merge_every < 1)
        return hb::set_error(HB_ERR_INVALID,
                             "hb_hogbatch_run_epoch: merge_every must be >= 1 (the replica's updates reach the global model by merging only)");
    const int *dims = nullptr;
    int n_dims = 0, act = 0, loss = 0;
    if (!hb::model_arch(gpu, &dims, &n_dims, &act, &loss)) return hb_last_error_code();
    const std::vector<int32_t> dims32(dims, dims + n_dims);

    struct {
        int rc = HB_OK;
        std::string err;
        int64_t batches = 0;
        double loss_sum = 0.0;
    } cpu;
    double cu = cpu_updates ? *cpu_updates : 0.0;
    std::thread cpu_thread;
    try {
        cpu_thread = std::thread([&] {
            cpu.rc = hb_cpu_worker_run_epoch(s, cpu_worker, dims32.data(), n_dims, act, loss, host_X, host_y, host_model,
                                             lr_per_example, cpu_threads, beta, &cu, &cpu.batches, &cpu.loss_sum);
            if (cpu.rc != HB_OK) cpu.err = hb_last_error();  // the error text is per thread
        });
    } catch (const std::exception &e) {
        return hb::set_error(HB_ERR_ALLOC, "hb_hogbatch_run_epoch: cannot start the CPU worker's thread: %s", e.what());
    }
    int64_t gpu_steps = 0;
    double gpu_loss = 0.0;
    const int grc = hb_worker_run_epoch(gpu, s, gpu_worker, host_X, host_y, lr_per_example, host_model, merge_every,
                                        merge_weight, gpu_updates, &gpu_steps, &gpu_loss);
    const std::string gerr = (grc != HB_OK) ? hb_last_error() : "";
    cpu_thread.join();  // whatever happened to the GPU worker, the CPU worker finishes what is left of the epoch
    if (cpu_updates) *cpu_updates = cu;
    if (stats) {
        stats->gpu_steps = gpu_steps;
        stats->cpu_batches = cpu.batches;
        stats->gpu_loss_sum = gpu_loss;
        stats->cpu_loss_sum = cpu.loss_sum;
    }
    if (grc != HB_OK) return hb::set_error(grc, "GPU worker: %s", gerr.c_str());
    if (cpu.rc != HB_OK) return hb::set_error(cpu.rc, "CPU worker: %s", cpu.err.c_str());
    return HB_OK;
}

// The evaluation loop for dense rows (csr == nullptr) or CSR rows (host_X == nullptr).
static int eval_loss(const char *who, hb_model *m, const void *host_X, const CsrHost *csr, const int32_t *host_y,
                     int64_t n_examples, int64_t batch, double *mean_loss)
{
    hb::ModelInfo mi;
    if (!hb::model_info(m, &mi)) return hb_last_error_code();
    if (!host_y || !mean_loss || (!csr && !host_X) || (csr && (!csr->row_ptr || !csr->col_idx || !csr->vals)))
        return hb::set_error(HB_ERR_INVALID, "%s: NULL argument", who);
    if ((mi.sparse != 0) != (csr != nullptr))
        return hb::set_error(HB_ERR_UNSUPPORTED, csr ? "%s: the model is not configured with sparse_first_layer"
                                                     : "%s: dense input only (hb_worker_eval_loss_csr takes CSR data)",
                             who);
    if (n_examples < 1) return hb::set_error(HB_ERR_INVALID, "%s: n_examples must be >= 1", who);
    if (batch < 1 || batch > mi.max_B)
        return hb::set_error(HB_ERR_INVALID, "%s: batch = %lld is outside [1, max_B = %lld]", who, (long long)batch,
                             (long long)mi.max_B);
    const size_t elem = (mi.dtype == HB_BF16_F32MASTER) ? 2 : 4;
    const size_t row_bytes = csr ? 0 : elem * (size_t)mi.d0;
    Staging *sp = nullptr;
    int rc = acquire_staging(m, mi, batch, row_bytes, &sp);
    if (rc != HB_OK) return rc;
    Staging &st = *sp;
    if (csr) {
        rc = acquire_csr(st, 0);
        if (rc != HB_OK) return rc;
    }
    DrainGuard drain{st, mi.stream};
    auto send = [&](int buf, int64_t begin, int64_t count) -> int {
        WK_HIP(hipEventSynchronize(st.consumed[buf]));  // host-side, see the worker loop
        if (csr) {
            const int rc_s = send_csr_rows(who, st, mi.stream, *csr, mi.d0, buf, begin, count);
            if (rc_s != HB_OK) return rc_s;
        } else {
            WK_HIP(hipMemcpyAsync(st.x[buf], static_cast<const unsigned char *>(host_X) + row_bytes * (size_t)begin,
                                  row_bytes * (size_t)count, hipMemcpyHostToDevice, st.copy));
        }
        WK_HIP(hipMemcpyAsync(st.y[buf], host_y + begin, sizeof(int32_t) * (size_t)count, hipMemcpyHostToDevice,
                              st.copy));
        WK_HIP(hipEventRecord(st.filled[buf], st.copy));
        return HB_OK;
    };
    for (int i = 0; i < 2; ++i) WK_HIP(hipEventRecord(st.consumed[i], mi.stream));
    // the pieces' mean losses are collected on the device and fetched a window at a time, so
    // that the host never waits for a single piece
    double sum = 0.0;
    int64_t rows_in_window[LOSS_WINDOW];
    int in_window = 0;
    auto flush = [&]() -> int {
        if (in_window == 0) return HB_OK;
        WK_HIP(hipMemcpyAsync(st.loss_host, st.loss, sizeof(float) * in_window, hipMemcpyDeviceToHost, mi.stream));
        WK_HIP(hipStreamSynchronize(mi.stream));
        for (int i = 0; i < in_window; ++i) sum += (double)st.loss_host[i] * (double)rows_in_window[i];
        in_window = 0;
        return HB_OK;
    };
    int buf = 0;
    int64_t begin = 0, count = n_examples < batch ? n_examples : batch;
    rc = send(0, begin, count);
    if (rc != HB_OK) return rc;
    while (count > 0) {
        const int64_t nbegin = begin + count;
        const int64_t ncount = (n_examples - nbegin) < batch ? (n_examples - nbegin) : batch;
        rc = wait_filled(st, buf, mi.stream);
        if (rc != HB_OK) return rc;
        rc = csr ? hb_batch_loss_csr_async(m, st.rp[buf], st.ci[buf], st.va[buf], st.nnz[buf], st.y[buf], count,
                                           st.loss + in_window)
                 : hb_batch_loss_async(m, st.x[buf], st.y[buf], count, st.loss + in_window);
        if (rc != HB_OK) return rc;
        WK_HIP(hipEventRecord(st.consumed[buf], mi.stream));
        if (ncount > 0) {  // the next piece travels while this one is evaluated (enqueued first, see the worker loop)
            rc = send(buf ^ 1, nbegin, ncount);
            if (rc != HB_OK) return rc;
        }
        rows_in_window[in_window] = count;
        if (++in_window == LOSS_WINDOW) {
            rc = flush();
            if (rc != HB_OK) return rc;
        }
        begin = nbegin;
        count = ncount;
        buf ^= 1;
    }
    rc = flush();
    if (rc != HB_OK) return rc;
    WK_HIP(hipStreamSynchronize(st.copy));
    *mean_loss = sum / (double)n_examples;
    return HB_OK;
}

extern "C" int hb_worker_eval_loss(hb_model *m, const void *host_X, const int32_t *host_y, int64_t n_examples,
                                   int64_t batch, double *mean_loss)
{
    if (!host_X) return hb::set_error(HB_ERR_INVALID, "hb_worker_eval_loss: NULL argument");
    return eval_loss("hb_worker_eval_loss", m, host_X, nullptr, host_y, n_examples, batch, mean_loss);
}

extern "C" int hb_worker_eval_loss_csr(hb_model *m, const int64_t *host_row_ptr, const int32_t *host_col_idx,
                                       const float *host_vals, const int32_t *host_y, int64_t n_examples,
                                       int64_t batch, double *mean_loss)
{
    const CsrHost csr{host_row_ptr, host_col_idx, host_vals};
    return eval_loss("hb_worker_eval_loss_csr", m, nullptr, &csr, host_y, n_examples, batch, mean_loss);
}
