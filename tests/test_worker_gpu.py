"""GPU worker loop (hb_worker_run_epoch) against the fp64 oracle: the sequence of batches the
scheduler hands out is replayed with oracle.batch_step (lr proportional to the batch size,
Section 6.2) and, where merging is on, oracle.model_merge.  The loop prefetches: the request
for batch k+1 is made while batch k computes, reporting the update count batch k will have
produced.  hb_worker_run_epoch_csr is replayed the same way with oracle.batch_step_csr."""
import numpy as np
import pytest

import hb_inputs as hi
from parity_checks import assert_close
import oracle
from oracle.sched import AdaptiveSchedule

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _data(n, dims, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    y = rng.integers(0, dims[-1], size=n).astype(np.int32)
    params = hi.xavier_uniform_params(dims, rng, bias_scale=0.1)
    return X, y, params


def _replay(sched, worker, u0, dims, act, loss, params, X, y, lr_pe, host_model=None, merge_every=0, w=1.0):
    """What the worker loop must do, step by step, on the oracle."""
    p = params.astype(np.float64)
    H = None if host_model is None else host_model.astype(np.float64)
    u, steps, loss_sum, since = float(u0), 0, 0.0, 0
    begin, count = sched.request(worker, u)
    while count > 0:
        nb, nc = sched.request(worker, u + 1.0)
        l, p = oracle.batch_step(dims, act, loss, p, X[begin:begin + count], y[begin:begin + count],
                                 float(np.float32(lr_pe) * np.float32(count)))
        loss_sum += l
        u += 1.0
        steps += 1
        since += 1
        if H is not None and merge_every > 0 and since >= merge_every:
            p, H = oracle.model_merge(p, H, w)
            since = 0
        begin, count = nb, nc
    if H is not None and merge_every > 0 and since > 0:
        p, H = oracle.model_merge(p, H, w)
    return p, H, u, steps, loss_sum


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30)


def _close(dims, got, ref, tol, what="parameters"):
    """Per tensor: relative L2 and the element-wise bound of tests/parity_checks.py."""
    assert_close(dims, np.asarray(got), np.asarray(ref), tol, what)


def test_single_worker_epoch_matches_sequential_oracle_steps():
    import paper_2004_08771_amd as hb
    import torch
    dims, act, loss = (54, 32, 7), hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE
    n = 4096 + 40                                  # 64 full batches and a tail that is dropped
    X, y, params = _data(n, dims, 7)
    lr_pe = 0.1 / 64
    ref_p, _, ref_u, ref_steps, ref_loss = _replay(AdaptiveSchedule(n, [16], [64], [64]), 0, 0, dims, act, loss,
                                                   params, X, y, lr_pe)
    m = hb.Model(dims, act, loss).configure(hb.HB_F32, 64)
    m.set_params(params)
    s = hb.Sched(n, [16], [64], [64])
    hX = torch.from_numpy(X).pin_memory()
    hy = torch.from_numpy(y).pin_memory()
    u, steps, loss_sum = m.worker_run_epoch(s, 0, hX, hy, lr_pe)
    got = np.empty_like(params)
    m.get_params(got)
    assert (u, steps) == (ref_u, ref_steps) == (64.0, 64)
    assert s.remaining() == 40
    assert abs(loss_sum - ref_loss) <= TOL * abs(ref_loss)
    _close(dims, got, ref_p, TOL)
    # second epoch: the update count carries over, the data starts again
    s.new_epoch()
    u2, steps2, _ = m.worker_run_epoch(s, 0, hX, hy, lr_pe, updates=u)
    assert (u2, steps2) == (128.0, 64)
    m.destroy()


def test_worker_epoch_at_the_benchmark_shape():
    """Config 2 (54-512x4-7) at the batch size the benchmark times: two steps of 4096 rows from
    page-locked host memory with a push after every step, replayed on the oracle."""
    import paper_2004_08771_amd as hb
    import torch
    cfg = hi.CONFIGS[2]
    B = 4096
    n = 2 * B + 40
    X, y = hi.make_dense_dataset(2, n)
    params = hi.make_params(2, bias_scale=0.1)
    lr_pe = 0.1 / 256
    host0 = np.zeros_like(params)
    ref_p, ref_H, ref_u, ref_steps, ref_loss = _replay(AdaptiveSchedule(n, [B], [B], [B]), 0, 0, cfg.dims,
                                                       cfg.activation, cfg.loss, params, X, y, lr_pe,
                                                       host_model=host0, merge_every=1, w=1.0)
    m = hb.Model(cfg.dims, cfg.activation, cfg.loss).configure(hb.HB_F32, B)
    m.set_params(params)
    s = hb.Sched(n, [B], [B], [B])
    H = torch.zeros(params.size).pin_memory()
    u, steps, loss_sum = m.worker_run_epoch(s, 0, torch.from_numpy(X).pin_memory(), torch.from_numpy(y).pin_memory(),
                                            lr_pe, host_model=H, merge_every=1, merge_weight=1.0)
    got = np.empty_like(params)
    m.get_params(got)
    m.destroy()
    assert (u, steps) == (ref_u, ref_steps) == (2.0, 2) and s.remaining() == 40
    assert abs(loss_sum - ref_loss) <= TOL * abs(ref_loss)
    _close(cfg.dims, got, ref_p, TOL)
    assert _rel(got - params, ref_p - params) <= 1e-3   # the two updates themselves
    assert np.array_equal(H.numpy(), got)               # the last push carried the final replica


def test_adaptive_batch_sizes_pageable_memory_and_merging():
    """Two workers at the coordinator; the other (CPU) worker has taken its share and reported
    many updates, so the GPU worker's batch shrinks from request to request (alpha = 1.5, ragged
    sizes).  Data in ordinary pageable memory; replica and host model blended every 3 steps."""
    import paper_2004_08771_amd as hb
    dims, act, loss = (40, 96, 48, 5), hi.ACT_RELU, hi.LOSS_SOFTMAX_CE
    n = 6000
    X, y, params = _data(n, dims, 9)
    host0 = (params + np.random.default_rng(3).standard_normal(params.size).astype(np.float32) * 0.01).astype(np.float32)
    lr_pe = 0.05 / 512
    mk = lambda make: make(n, [1, 50], [8, 700], [1, 700], 1.5)

    def cpu_share(s):                 # the CPU worker: 40 batches, 8 updates each
        uc = 0.0
        for _ in range(40):
            s.request(0, uc)
            uc += 8.0

    so = mk(AdaptiveSchedule)
    cpu_share(so)
    ref_p, ref_H, ref_u, ref_steps, ref_loss = _replay(so, 1, 0, dims, act, loss, params, X, y, lr_pe,
                                                       host_model=host0, merge_every=3, w=0.25)
    assert ref_steps > 8 and so.b[1] == 50          # the batch size went all the way down

    sl = mk(hb.Sched)
    cpu_share(sl)
    m = hb.Model(dims, act, loss).configure(hb.HB_F32, 700)
    m.set_params(params)
    H = host0.copy()
    u, steps, loss_sum = m.worker_run_epoch(sl, 1, X, y, lr_pe, host_model=H, merge_every=3, merge_weight=0.25)
    got = np.empty_like(params)
    m.get_params(got)
    m.destroy()
    assert (u, steps) == (ref_u, ref_steps)
    assert sl.batch_size(1) == 50 and sl.remaining() == so.remaining()
    assert abs(loss_sum - ref_loss) <= TOL * abs(ref_loss)
    _close(dims, got, ref_p, TOL)
    _close(dims, H, ref_H, TOL)


@pytest.mark.parametrize("locked", [True, False])
def test_asynchronous_push_of_the_replica(locked):
    """merge_weight = 1 is the push of Section 6.2: the replica is snapshot in stream order and
    travels to the host model beside the following steps, into page-locked memory directly and
    into pageable memory through a landing buffer.  A push leaves the replica alone, so the
    replica must equal plain sequential steps, and the host model must be the replica as it was
    at the last merge point: with merge_every = 4 and 10 steps the pushes follow steps 4 and 8
    and the closing one step 10.  A second epoch pushes after every step, so that each push
    meets the one before it still in flight."""
    import paper_2004_08771_amd as hb
    import torch
    dims, act, loss = (40, 96, 48, 5), hi.ACT_RELU, hi.LOSS_SOFTMAX_CE
    n = 10 * 96
    X, y, params = _data(n, dims, 21)
    lr_pe = 0.05 / 96
    ref_p, ref_H, ref_u, ref_steps, ref_loss = _replay(AdaptiveSchedule(n, [96], [96], [96]), 0, 0, dims, act, loss,
                                                       params, X, y, lr_pe, host_model=np.zeros_like(params),
                                                       merge_every=4, w=1.0)
    m = hb.Model(dims, act, loss).configure(hb.HB_F32, 96)
    m.set_params(params)
    s = hb.Sched(n, [96], [96], [96])
    H = torch.zeros(params.size, dtype=torch.float32)
    if locked:
        H = H.pin_memory()
    u, steps, loss_sum = m.worker_run_epoch(s, 0, X, y, lr_pe, host_model=H, merge_every=4, merge_weight=1.0)
    got = np.empty_like(params)
    m.get_params(got)
    assert (u, steps) == (ref_u, ref_steps) == (10.0, 10)
    assert abs(loss_sum - ref_loss) <= TOL * abs(ref_loss)
    _close(dims, got, ref_p, TOL)
    _close(dims, H.numpy(), ref_H, TOL)
    assert np.array_equal(H.numpy(), got)           # the closing push carried the final replica, bit for bit
    # every push of a longer run lands in order: push after every step, host model = final replica
    s.new_epoch()
    H.zero_()
    m.worker_run_epoch(s, 0, X, y, lr_pe, host_model=H, merge_every=1, merge_weight=1.0, updates=u)
    m.get_params(got)
    m.destroy()
    assert np.array_equal(H.numpy(), got)


def test_deep_copy_of_the_global_model_every_other_step():
    """merge_weight = 0 is the deep copy of the ExecuteWork handler (Section 6.2): the replica is
    overwritten by the global model, which stays as it is.  Every second step throws the
    replica's progress away, so the epoch ends on the global model itself when the number of
    steps is even, and one step away from it when it is odd."""
    import paper_2004_08771_amd as hb
    dims, act, loss = (30, 40, 4), hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE
    X, y, params = _data(7 * 50, dims, 33)
    host0 = (params * 0.5).astype(np.float32)
    lr_pe = 0.1 / 50
    ref_p, ref_H, ref_u, ref_steps, ref_loss = _replay(AdaptiveSchedule(350, [50], [50], [50]), 0, 0, dims, act, loss,
                                                       params, X, y, lr_pe, host_model=host0, merge_every=2, w=0.0)
    m = hb.Model(dims, act, loss).configure(hb.HB_F32, 50)
    m.set_params(params)
    s = hb.Sched(350, [50], [50], [50])
    H = host0.copy()
    u, steps, loss_sum = m.worker_run_epoch(s, 0, X, y, lr_pe, host_model=H, merge_every=2, merge_weight=0.0)
    got = np.empty_like(params)
    m.get_params(got)
    m.destroy()
    assert steps == ref_steps == 7
    assert np.array_equal(H, host0)                 # the global model is only read
    assert np.array_equal(got, host0)               # 7 steps: the closing merge copies it once more
    assert abs(loss_sum - ref_loss) <= TOL * abs(ref_loss)
    _close(dims, got, ref_p, TOL)


def _replay_csr(sched, worker, dims, act, loss, params, rp, ci, va, y, lr_pe, host_model=None, merge_every=0, w=1.0):
    """The CSR loop, step by step, on the oracle (same order of requests as _replay)."""
    p = params.astype(np.float64)
    H = None if host_model is None else host_model.astype(np.float64)
    u, steps, loss_sum, since = 0.0, 0, 0.0, 0
    begin, count = sched.request(worker, u)
    while count > 0:
        nb, nc = sched.request(worker, u + 1.0)
        brp, bci, bva = hi.csr_slice(rp, ci, va, begin, begin + count)
        l, p = oracle.batch_step_csr(dims, act, loss, p, brp, bci, bva, y[begin:begin + count],
                                     float(np.float32(lr_pe) * np.float32(count)))
        loss_sum += l
        u += 1.0
        steps += 1
        since += 1
        if H is not None and merge_every > 0 and since >= merge_every:
            p, H = oracle.model_merge(p, H, w)
            since = 0
        begin, count = nb, nc
    if H is not None and merge_every > 0 and since > 0:
        p, H = oracle.model_merge(p, H, w)
    return p, H, u, steps, loss_sum


def _csr_data(n, dims, seed, mean_nnz):
    rng = np.random.default_rng(seed)
    rp, ci, va = hi.zipf_csr(n, dims[0], rng, mean_nnz=mean_nnz, max_nnz=64)
    y = hi.csr_pm1_labels(rp, ci, va, dims[0], rng)
    params = hi.xavier_uniform_params(dims, rng, bias_scale=0.1)
    return rp.astype(np.int64), ci, va, y, params


@pytest.mark.parametrize("merge", [None, (1, 1.0), (2, 0.5)])
def test_csr_worker_epoch_matches_sequential_oracle_steps(merge):
    """hb_worker_run_epoch_csr: the batches' row-pointer slices are rebased on the host, index and
    value buffers grow on demand (the second epoch's batches are larger than the first's), with
    no merge, a push after every step and a blend every other step."""
    import paper_2004_08771_amd as hb
    import torch
    dims, act, loss = (500, 48, 24, 1), hi.ACT_SIGMOID, hi.LOSS_LOGISTIC
    n = 2000
    rp, ci, va, y, params = _csr_data(n, dims, 21, mean_nnz=12)
    lr_pe = 0.2 / 128
    kw = {} if merge is None else dict(merge_every=merge[0], w=merge[1])
    host0 = None
    if merge is not None:
        host0 = (params + np.random.default_rng(5).standard_normal(params.size).astype(np.float32) * 0.01).astype(np.float32)
    mk = lambda make: make(n, [1, 16], [8, 300], [1, 300], 1.5)

    def cpu_share(s):                 # the other worker took 20 batches and reports many updates
        uc = 0.0
        for _ in range(20):
            s.request(0, uc)
            uc += 8.0

    so = mk(AdaptiveSchedule)
    cpu_share(so)
    ref_p, ref_H, ref_u, ref_steps, ref_loss = _replay_csr(so, 1, dims, act, loss, params, rp, ci, va, y, lr_pe,
                                                           host_model=host0, **kw)
    assert ref_steps > 8

    sl = mk(hb.Sched)
    cpu_share(sl)
    m = hb.Model(dims, act, loss).configure(hb.HB_F32, 300, sparse_first_layer=True)
    m.set_params(params)
    H = None if host0 is None else host0.copy()
    h_ci, h_va = torch.from_numpy(ci).pin_memory(), torch.from_numpy(va).pin_memory()
    gkw = {} if merge is None else dict(host_model=H, merge_every=merge[0], merge_weight=merge[1])
    u, steps, loss_sum = m.worker_run_epoch_csr(sl, 1, rp, h_ci, h_va, y, lr_pe, **gkw)
    got = np.empty_like(params)
    m.get_params(got)
    assert (u, steps) == (ref_u, ref_steps)
    assert sl.remaining() == so.remaining()
    assert abs(loss_sum - ref_loss) <= TOL * abs(ref_loss)
    _close(dims, got, ref_p, TOL)
    if H is not None:
        _close(dims, H, ref_H, TOL)
    m.destroy()


def test_csr_worker_epoch_at_the_benchmark_shape():
    """Config 4 (20958-512x3-2, CSR rows of the real-sim shape) at the batch size the benchmark
    times: two steps of 8192 rows from host memory, replayed on the oracle."""
    import paper_2004_08771_amd as hb
    cfg = hi.CONFIGS[4]
    B = 8192
    n = 2 * B + 50
    rp, ci, va, y = hi.make_csr_dataset(4, n)
    rp = rp.astype(np.int64)
    params = hi.make_params(4, bias_scale=0.1)
    lr_pe = cfg.lr / B
    ref_p, _, ref_u, ref_steps, ref_loss = _replay_csr(AdaptiveSchedule(n, [B], [B], [B]), 0, cfg.dims, cfg.activation,
                                                       cfg.loss, params, rp, ci, va, y, lr_pe)
    m = hb.Model(cfg.dims, cfg.activation, cfg.loss).configure(hb.HB_F32, B, sparse_first_layer=True)
    m.set_params(params)
    s = hb.Sched(n, [B], [B], [B])
    u, steps, loss_sum = m.worker_run_epoch_csr(s, 0, rp, ci, va, y, lr_pe)
    got = np.empty_like(params)
    m.get_params(got)
    m.destroy()
    assert (u, steps) == (ref_u, ref_steps) == (2.0, 2) and s.remaining() == 50
    assert abs(loss_sum - ref_loss) <= TOL * abs(ref_loss)
    _close(cfg.dims, got, ref_p, TOL)
    assert _rel(got - params, ref_p - params) <= 1e-3   # the two updates themselves


def test_csr_worker_buffers_grow_and_errors():
    import paper_2004_08771_amd as hb
    dims, act, loss = (300, 16, 1), hi.ACT_SIGMOID, hi.LOSS_LOGISTIC
    n = 1024
    rp, ci, va, y, params = _csr_data(n, dims, 22, mean_nnz=6)
    m = hb.Model(dims, act, loss).configure(hb.HB_F32, 256, sparse_first_layer=True)
    m.set_params(params)
    # first epoch: small batches size the value buffers; second epoch: 8 times the rows per batch
    s1 = hb.Sched(n, [32], [32], [32])
    u, steps, _ = m.worker_run_epoch_csr(s1, 0, rp, ci, va, y, 1e-3)
    assert steps == 32
    s2 = hb.Sched(n, [256], [256], [256])
    u, steps, loss_sum = m.worker_run_epoch_csr(s2, 0, rp, ci, va, y, 1e-3, updates=u)
    assert (u, steps) == (36.0, 4)
    got = np.empty_like(params)
    m.get_params(got)
    p = params.astype(np.float64)
    ref_loss = 0.0
    for b, cnt, reps in ((32, 32, False), (256, 4, True)):
        for k in range(cnt):
            brp, bci, bva = hi.csr_slice(rp, ci, va, k * b, (k + 1) * b)
            l, p = oracle.batch_step_csr(dims, act, loss, p, brp, bci, bva, y[k * b:(k + 1) * b],
                                         float(np.float32(1e-3) * np.float32(b)))
            ref_loss += l if reps else 0.0
    _close(dims, got, p, TOL)
    assert abs(loss_sum - ref_loss) <= TOL * abs(ref_loss)
    # a row pointer that decreases is refused before anything is copied
    bad = rp.copy()
    bad[10] = bad[9] - 1
    s3 = hb.Sched(n, [32], [32], [32])
    with pytest.raises(hb.HbError):
        m.worker_run_epoch_csr(s3, 0, bad, ci, va, y, 1e-3)
    with pytest.raises(hb.HbError):
        m.worker_run_epoch_csr(hb.Sched(n, [32], [32], [32]), 0, None, ci, va, y, 1e-3)
    # a column index outside [0, d_0) is refused on the host, before the batch that holds it is sent
    # (the kernels trust indices); the batches before it have been applied
    for bad_value in (dims[0], -1):
        bad_ci = ci.copy()
        bad_ci[int(rp[40]) + 1] = bad_value             # row 40 = second batch of 32
        s4 = hb.Sched(n, [32], [32], [32])
        with pytest.raises(hb.HbError) as e:
            m.worker_run_epoch_csr(s4, 0, rp, bad_ci, va, y, 1e-3)
        assert e.value.code == hb.HB_ERR_INVALID and "column index" in str(e.value)
        with pytest.raises(hb.HbError) as e:
            m.worker_eval_loss_csr(rp, bad_ci, va, y, n, 256)
        assert e.value.code == hb.HB_ERR_INVALID
    # dense and CSR loops are not interchangeable
    X = np.zeros((n, dims[0]), dtype=np.float32)
    with pytest.raises(hb.HbError):
        m.worker_run_epoch(hb.Sched(n, [32], [32], [32]), 0, X, y, 1e-3)
    m.destroy()
    d = hb.Model(dims, act, loss).configure(hb.HB_F32, 256)
    d.set_params(params)
    with pytest.raises(hb.HbError):
        d.worker_run_epoch_csr(hb.Sched(n, [32], [32], [32]), 0, rp, ci, va, y, 1e-3)
    d.destroy()


def test_bf16_worker_epoch_follows_the_oracle_with_rounded_operands():
    """The loop in bf16 mode (host rows are bfloat16, 2 bytes each through the staging buffers):
    every step is replayed on the oracle with the weights and the rows rounded to bf16 and fp64
    master weights, to the bf16 tolerance."""
    import paper_2004_08771_amd as hb
    import torch
    dims, act, loss = (64, 128, 64, 10), hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE
    n, b = 2048 + 100, 256
    X, y, params = _data(n, dims, 31)
    lr_pe = 0.1 / 256
    Xr = oracle.bf16_round(X)
    p = params.astype(np.float64)
    ref_loss = 0.0
    for k in range(n // b):
        l, g = oracle.batch_grad(dims, act, loss, oracle.round_weights_bf16(dims, p.astype(np.float32)),
                                 Xr[k * b:(k + 1) * b], y[k * b:(k + 1) * b])
        p = p - float(np.float32(lr_pe) * np.float32(b)) * g
        ref_loss += l
    m = hb.Model(dims, act, loss).configure(hb.HB_BF16_F32MASTER, b)
    m.set_params(params)
    hX = torch.from_numpy(X).to(torch.bfloat16).pin_memory()
    s = hb.Sched(n, [b], [b], [b])
    u, steps, loss_sum = m.worker_run_epoch(s, 0, hX, y, lr_pe)
    got = np.empty_like(params)
    m.get_params(got)
    m.destroy()
    assert (u, steps) == (8.0, 8) and s.remaining() == 100
    assert abs(loss_sum - ref_loss) <= 2e-2 * abs(ref_loss)
    _close(dims, got, p, 2e-2)
    assert _rel(got - params, p - params) <= 5e-2      # the updates themselves, not only the weights they barely move


def test_worker_argument_errors():
    import paper_2004_08771_amd as hb
    dims = (8, 4, 3)
    X, y, params = _data(64, dims, 1)
    m = hb.Model(dims, hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE).configure(hb.HB_F32, 16)
    m.set_params(params)
    s = hb.Sched(64, [4], [32], [32])               # max_b above the model's max_B
    with pytest.raises(hb.HbError):
        m.worker_run_epoch(s, 0, X, y, 0.01)
    s2 = hb.Sched(64, [4], [16], [16])
    with pytest.raises(hb.HbError):
        m.worker_run_epoch(s2, 3, X, y, 0.01)       # no such worker
    with pytest.raises(hb.HbError):
        m.worker_run_epoch(s2, 0, None, y, 0.01)
    assert m.worker_run_epoch(s2, 0, X, y, 0.01)[1] == 4
    m.destroy()


def test_epoch_loss_evaluation_matches_oracle_mean_loss():
    """Section 5.2's evaluation stage: forward-only mean loss over host-resident data in pieces
    (a ragged last piece), fp32 and bf16."""
    import paper_2004_08771_amd as hb
    import torch
    dims, act, loss = (54, 64, 32, 7), hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE
    n = 3000
    X, y, params = _data(n, dims, 21)
    ref = oracle.batch_loss(dims, act, loss, params.astype(np.float64), X, y)
    m = hb.Model(dims, act, loss).configure(hb.HB_F32, 512)
    m.set_params(params)
    before = np.empty_like(params); m.get_params(before)
    got = m.worker_eval_loss(X, y, n, 512)             # 5 pieces of 512 and one of 440
    after = np.empty_like(params); m.get_params(after)
    assert abs(got - ref) <= TOL * abs(ref)
    assert abs(m.worker_eval_loss(X, y, n, 7) - ref) <= TOL * abs(ref)
    np.testing.assert_array_equal(before, after)
    with pytest.raises(hb.HbError):
        m.worker_eval_loss(X, y, n, 513)               # above max_B
    m.destroy()
    Xb = torch.from_numpy(X).to(torch.bfloat16)
    refb = oracle.batch_loss(dims, act, loss, oracle.round_weights_bf16(dims, params), oracle.bf16_round(X), y)
    mb = hb.Model(dims, act, loss).configure(hb.HB_BF16_F32MASTER, 1024)
    mb.set_params(params)
    gotb = mb.worker_eval_loss(Xb, y, n, 1024)
    mb.destroy()
    assert abs(gotb - refb) <= 2e-2 * abs(refb)


def test_csr_epoch_loss_evaluation_matches_oracle_mean_loss():
    """The evaluation stage over CSR data: the oracle's dense forward pass over the expanded rows
    is the reference; pieces of 300 rows with a ragged last one, then pieces of 7."""
    import paper_2004_08771_amd as hb
    dims, act, loss = (400, 40, 1), hi.ACT_RELU, hi.LOSS_LOGISTIC
    n = 1000
    rp, ci, va, y, params = _csr_data(n, dims, 23, mean_nnz=9)
    ref = oracle.batch_loss(dims, act, loss, params.astype(np.float64), hi.csr_to_dense(rp, ci, va, dims[0]), y)
    m = hb.Model(dims, act, loss).configure(hb.HB_F32, 300, sparse_first_layer=True)
    m.set_params(params)
    got = m.worker_eval_loss_csr(rp, ci, va, y, n, 300)
    assert abs(got - ref) <= TOL * abs(ref)
    assert abs(m.worker_eval_loss_csr(rp, ci, va, y, n, 7) - ref) <= TOL * abs(ref)
    after = np.empty_like(params); m.get_params(after)
    np.testing.assert_array_equal(after, params)
    with pytest.raises(hb.HbError):
        m.worker_eval_loss(np.zeros((n, dims[0]), dtype=np.float32), y, n, 300)   # dense rows for a CSR model
    m.destroy()


def test_cpu_and_gpu_workers_share_an_epoch():
    """CPU+GPU Adaptive Hogbatch end to end on synthetic data: one scheduler, one shared host
    model, a CPU worker (Hogwild threads) and the GPU worker running concurrently, the GPU
    replica blended into the host model after every step.  The interleaving is not
    deterministic; what must hold is what the algorithm fixes."""
    import threading
    import paper_2004_08771_amd as hb
    dims, act, loss = (32, 64, 32, 6), hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE
    n = 20000
    rng = np.random.default_rng(12)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    teacher = rng.standard_normal((dims[0], dims[-1]))
    y = np.argmax(X @ teacher, axis=1).astype(np.int32)
    params = hi.xavier_uniform_params(dims, rng)
    before = oracle.batch_loss(dims, act, loss, params, X, y)
    H = params.copy()
    t = 4
    s = hb.Sched(n, [t, 64], [8 * t, 1024], [t, 1024], 2.0)      # CPU starts at its lower, GPU at its upper threshold
    m = hb.Model(dims, act, loss).configure(hb.HB_F32, 1024)
    m.set_params(params)
    out = {}

    def gpu():
        out["gpu"] = m.worker_run_epoch(s, 1, X, y, 0.02 / 64, host_model=H, merge_every=1, merge_weight=0.5)

    def cpu():
        out["cpu"] = hb.cpu_worker_run_epoch(s, 0, dims, act, loss, X, y, H, 0.02 / 64, threads=t, beta=1.0)

    th = [threading.Thread(target=gpu), threading.Thread(target=cpu)]
    for x in th:
        x.start()
    for x in th:
        x.join(timeout=100)
    assert "gpu" in out and "cpu" in out
    ug, steps, _ = out["gpu"]
    uc, batches, _ = out["cpu"]
    m.destroy()
    assert steps >= 1 and batches >= 1 and ug == steps and uc == batches * t
    assert s.remaining() < 64                                    # less than the GPU worker's smallest batch is left
    assert t <= s.batch_size(0) <= 8 * t and 64 <= s.batch_size(1) <= 1024
    assert np.all(np.isfinite(H))
    after = oracle.batch_loss(dims, act, loss, H, X, y)
    assert after < before


def test_two_gpu_workers_on_their_own_streams_share_an_epoch():
    """Two GPU workers (Section 6.2 lets any number of workers share the global model): two
    replicas on the one device, each handle on a stream of its own (default priority), driven by
    two host threads against one scheduler and one host model, each replica blended into the host
    model after every step.  As with the CPU+GPU pair the interleaving is free; what is checked is
    what the algorithm fixes.  Afterwards each handle alone still matches the oracle on its own
    stream: concurrent use has not disturbed it."""
    import threading
    import torch
    import paper_2004_08771_amd as hb
    dims, act, loss = (32, 64, 32, 6), hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE
    n = 60000
    rng = np.random.default_rng(14)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    teacher = rng.standard_normal((dims[0], dims[-1]))
    y = np.argmax(X @ teacher, axis=1).astype(np.int32)
    params = hi.xavier_uniform_params(dims, rng)
    before = oracle.batch_loss(dims, act, loss, params, X, y)
    H = params.copy()
    s = hb.Sched(n, [64, 64], [512, 256], [512, 256], 2.0)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ms = [hb.Model(dims, act, loss).configure(hb.HB_F32, 512, stream=st.cuda_stream) for st in streams]
    for m in ms:
        m.set_params(params)
        # staging buffers and streams are created by a handle's first epoch (milliseconds): do that
        # before the race, with a learning rate of zero, so that both workers get a share of it
        m.worker_run_epoch(hb.Sched(1024, [512], [512], [512]), 0, X, y, 0.0)
    out = {}

    def work(w):
        try:
            out[w] = ms[w].worker_run_epoch(s, w, X, y, 0.02 / 64, host_model=H, merge_every=1, merge_weight=0.5)
        except Exception as e:          # reported by the assertion below
            out[w] = e

    th = [threading.Thread(target=work, args=(w,)) for w in range(2)]
    for x in th:
        x.start()
    for x in th:
        x.join(timeout=100)
    assert all(isinstance(out.get(w), tuple) for w in range(2)), out
    (u0, st0, _), (u1, st1, _) = out[0], out[1]
    assert st0 >= 1 and st1 >= 1 and u0 == st0 and u1 == st1
    # each worker stops at the first request that cannot be served with its batch size
    assert s.remaining() < min(s.batch_size(0), s.batch_size(1))
    assert 64 <= s.batch_size(0) <= 512 and 64 <= s.batch_size(1) <= 256
    assert np.all(np.isfinite(H))
    assert oracle.batch_loss(dims, act, loss, H, X, y) < before
    # one more step on each handle, alone, against the oracle
    for w, m in enumerate(ms):
        p0 = np.empty_like(params)
        m.get_params(p0)
        B = 200 + 56 * w
        l_ref, p_ref = oracle.batch_step(dims, act, loss, p0.astype(np.float64), X[:B], y[:B], 0.05)
        with torch.cuda.stream(streams[w]):
            dX, dy = torch.from_numpy(X[:B]).cuda(), torch.from_numpy(y[:B]).cuda()
        streams[w].synchronize()
        l = m.batch_step(dX, dy, B, 0.05)
        p1 = np.empty_like(params)
        m.get_params(p1)
        assert abs(l - l_ref) <= TOL * abs(l_ref)
        _close(dims, p1, p_ref, TOL)
        m.destroy()


def test_one_call_runs_a_cpu_gpu_epoch():
    """hb_hogbatch_run_epoch: the CPU worker on its own thread, the GPU worker on the caller's,
    one scheduler, one host model, for three epochs with the update counts carried over.  The
    interleaving is free; what the algorithm fixes is checked."""
    import paper_2004_08771_amd as hb
    dims, act, loss = (32, 64, 32, 6), hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE
    n = 20000
    rng = np.random.default_rng(15)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    teacher = rng.standard_normal((dims[0], dims[-1]))
    y = np.argmax(X @ teacher, axis=1).astype(np.int32)
    params = hi.xavier_uniform_params(dims, rng)
    H = params.copy()
    t = 4
    s = hb.Sched(n, [t, 64], [8 * t, 1024], [t, 1024], 2.0)      # worker 0: CPU, worker 1: GPU
    m = hb.Model(dims, act, loss).configure(hb.HB_F32, 1024)
    m.set_params(params)
    losses = [oracle.batch_loss(dims, act, loss, H, X, y)]
    gu = cu = 0.0
    for epoch in range(3):
        gu0, cu0 = gu, cu
        gu, cu, st = hb.hogbatch_run_epoch(s, m, 1, 0, X, y, H, 0.02 / 64, cpu_threads=t, beta=1.0, merge_every=1,
                                           merge_weight=0.5, gpu_updates=gu, cpu_updates=cu)
        assert st["gpu_steps"] >= 1 and st["cpu_batches"] >= 1
        assert gu - gu0 == st["gpu_steps"] and cu - cu0 == st["cpu_batches"] * t
        assert s.remaining() < 64
        assert t <= s.batch_size(0) <= 8 * t and 64 <= s.batch_size(1) <= 1024
        assert np.all(np.isfinite(H))
        losses.append(oracle.batch_loss(dims, act, loss, H, X, y))
        s.new_epoch()
    assert losses[1] < losses[0] and losses[-1] < losses[0]
    # argument errors: same worker twice, no merging, a model that is not fp32 dense
    with pytest.raises(hb.HbError):
        hb.hogbatch_run_epoch(s, m, 1, 1, X, y, H, 0.01)
    with pytest.raises(hb.HbError):
        hb.hogbatch_run_epoch(s, m, 1, 0, X, y, H, 0.01, merge_every=0)
    assert s.remaining() == n                                    # nothing was handed out by the failing calls
    m.destroy()
    mb = hb.Model(dims, act, loss).configure(hb.HB_BF16_F32MASTER, 1024)
    with pytest.raises(hb.HbError):
        hb.hogbatch_run_epoch(s, mb, 1, 0, X, y, H, 0.01)
    mb.destroy()
