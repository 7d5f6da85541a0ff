"""CPU worker of Adaptive Hogbatch (Algorithm 2, CPU worker): host-only code of the library,
checked against the fp64 oracle where the result is deterministic (one thread: sequential
mini-batch SGD) and through what the algorithm fixes where it is not (lock-free threads)."""
import numpy as np
import pytest

import hb_inputs as hi
import oracle
from oracle.sched import AdaptiveSchedule


def _data(n, dims, loss, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    if loss == hi.LOSS_SOFTMAX_CE:
        y = rng.integers(0, dims[-1], size=n).astype(np.int32)
    else:
        y = (2 * rng.integers(0, 2, size=n) - 1).astype(np.int32)
    return X, y, hi.xavier_uniform_params(dims, rng, bias_scale=0.1)


@pytest.mark.parametrize("dims,act,loss", [
    ((12, 9, 5), hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE),
    ((10, 8, 6, 2), hi.ACT_RELU, hi.LOSS_LOGISTIC),
    ((7, 5, 1), hi.ACT_SIGMOID, hi.LOSS_LOGISTIC),
    ((6, 4), hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE),
])
def test_one_thread_is_sequential_minibatch_sgd(dims, act, loss):
    import paper_2004_08771_amd as hb
    n, b, lr_pe = 203, 8, 0.02
    X, y, params = _data(n, dims, loss, 5)
    # oracle: the same batches, one oracle step each
    so = AdaptiveSchedule(n, [b], [b], [b])
    p = params.astype(np.float64)
    u, ref_loss = 0, 0.0
    while True:
        begin, count = so.request(0, u)
        if count == 0:
            break
        l, p = oracle.batch_step(dims, act, loss, p, X[begin:begin + count], y[begin:begin + count],
                                 float(np.float32(lr_pe) * np.float32(count)))
        ref_loss += l
        u += 1
    H = params.copy()
    s = hb.Sched(n, [b], [b], [b])
    uu, batches, loss_sum = hb.cpu_worker_run_epoch(s, 0, dims, act, loss, X, y, H, lr_pe, threads=1, beta=1.0)
    assert batches == u == 25 and uu == 25.0 and s.remaining() == 3
    assert abs(loss_sum - ref_loss) <= 1e-4 * abs(ref_loss)
    assert np.linalg.norm(H - p) <= 1e-4 * np.linalg.norm(p)


@pytest.mark.parametrize("dims,act,loss", [
    ((12, 9, 5), hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE),
    ((10, 8, 6, 2), hi.ACT_RELU, hi.LOSS_LOGISTIC),
    ((7, 5, 1), hi.ACT_SIGMOID, hi.LOSS_LOGISTIC),
])
def test_one_thread_with_batches_of_one_example_is_plain_sgd(dims, act, loss):
    """A sub-batch of one example takes the path that applies the update while the gradient is
    formed (Hogwild's case); with one thread it is plain SGD, one oracle step per example."""
    import paper_2004_08771_amd as hb
    n, lr_pe = 60, 0.05
    X, y, params = _data(n, dims, loss, 6)
    p = params.astype(np.float64)
    ref_loss = 0.0
    for i in range(n):
        l, p = oracle.batch_step(dims, act, loss, p, X[i:i + 1], y[i:i + 1], float(np.float32(lr_pe)))
        ref_loss += l
    H = params.copy()
    s = hb.Sched(n, [1], [1], [1])
    u, batches, loss_sum = hb.cpu_worker_run_epoch(s, 0, dims, act, loss, X, y, H, lr_pe, threads=1, beta=1.0)
    assert batches == n and u == float(n) and s.remaining() == 0
    assert abs(loss_sum - ref_loss) <= 1e-4 * abs(ref_loss)
    assert np.linalg.norm(H - p) <= 1e-4 * np.linalg.norm(p)


def test_hogwild_threads_consume_the_epoch_and_reduce_the_loss():
    import paper_2004_08771_amd as hb
    dims, act, loss = (20, 16, 4), hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE
    n, t = 2000, 4
    rng = np.random.default_rng(8)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    teacher = rng.standard_normal((dims[0], dims[-1]))
    y = np.argmax(X @ teacher, axis=1).astype(np.int32)          # learnable labels
    params = hi.xavier_uniform_params(dims, rng)
    before = oracle.batch_loss(dims, act, loss, params, X, y)
    H = params.copy()
    s = hb.Sched(n, [t], [t], [t])                               # b = t: one example per thread
    u, batches, loss_sum = hb.cpu_worker_run_epoch(s, 0, dims, act, loss, X, y, H, 0.05, threads=t, beta=0.5)
    assert batches == n // t and s.remaining() == 0
    assert u == batches * t * 0.5                                # t * beta updates per batch
    assert np.all(np.isfinite(H)) and not np.array_equal(H, params)
    after = oracle.batch_loss(dims, act, loss, H, X, y)
    assert after < 0.8 * before


def test_update_counts_drive_the_batch_size_of_the_other_worker():
    """The CPU worker reports t updates per small batch; a second worker that asks afterwards
    with fewer updates is sped up (its batch shrinks by alpha), as Algorithm 2 prescribes."""
    import paper_2004_08771_amd as hb
    dims, act, loss = (6, 4), hi.ACT_SIGMOID, hi.LOSS_SOFTMAX_CE
    X, y, params = _data(400, dims, loss, 3)
    s = hb.Sched(400, [2, 16], [2, 256], [2, 256])
    # the other worker takes one batch first, so that 144 rows are left for the CPU worker
    assert s.request(1, 0) == (0, 256)
    H = params.copy()
    u, batches, _ = hb.cpu_worker_run_epoch(s, 0, dims, act, loss, X, y, H, 0.01, threads=2, beta=1.0)
    assert batches == 72 and u == 144.0
    s.new_epoch()
    assert s.request(1, 1) == (0, 128)                           # 1 < 144: halved


def test_cpu_worker_rejects_bad_arguments():
    import paper_2004_08771_amd as hb
    dims = (4, 3)
    X, y, params = _data(16, dims, hi.LOSS_SOFTMAX_CE, 1)
    s = hb.Sched(16, [2], [2], [2])
    H = params.copy()
    for kw in ({"threads": 0}, {"beta": 0.0}, {"beta": 1.5}):
        with pytest.raises(hb.HbError):
            hb.cpu_worker_run_epoch(s, 0, dims, 0, 0, X, y, H, 0.01, **kw)
    with pytest.raises(hb.HbError):
        hb.cpu_worker_run_epoch(s, 0, (4, 3, 5), 0, hi.LOSS_LOGISTIC, X, y, H, 0.01)   # logistic needs d_L <= 2
    with pytest.raises(hb.HbError):
        hb.cpu_worker_run_epoch(s, 0, dims, 0, 0, None, y, H, 0.01)


def test_label_outside_its_domain_is_an_error_not_a_stray_read():
    import paper_2004_08771_amd as hb
    dims = (6, 5, 3)
    rng = np.random.default_rng(3)
    X = rng.standard_normal((32, 6)).astype(np.float32)
    model = hi.xavier_uniform_params(dims, rng, 0.1)
    for loss, bad in ((hb.HB_LOSS_SOFTMAX_CE, 3), (hb.HB_LOSS_SOFTMAX_CE, -1), (hb.HB_LOSS_LOGISTIC, 0)):
        d = dims if loss == hb.HB_LOSS_SOFTMAX_CE else (6, 5, 2)
        y = np.ones(32, np.int32)
        y[20] = bad
        s = hb.Sched(32, [8], [8], [8])
        m = hi.xavier_uniform_params(d, rng, 0.1)
        with pytest.raises(hb.HbError) as e:
            hb.cpu_worker_run_epoch(s, 0, d, hb.HB_ACT_SIGMOID, loss, X, y, m, 0.01)
        assert e.value.code == hb.HB_ERR_INVALID
        assert s.remaining() == 8          # batches 0 and 1 ran, the batch holding row 20 was refused
