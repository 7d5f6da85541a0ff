"""Adaptive Hogbatch batch scheduling (Algorithm 2, coordinator's ScheduleWork handler).
The Python model in oracle/sched.py is pinned by a trace worked by hand from the algorithm and
by the invariants the algorithm implies; the library's hb_sched must then agree with it request
by request.  Host-only: no GPU needed."""
import json
import os

import numpy as np
import pytest

from oracle.sched import AdaptiveSchedule

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    with open(os.path.join(HERE, "golden", "sched_trace.json")) as f:
        return json.load(f)


def _lib_sched(*a, **k):
    import paper_2004_08771_amd as hb
    return hb.Sched(*a, **k)


@pytest.mark.parametrize("make", [AdaptiveSchedule, _lib_sched], ids=["oracle", "library"])
def test_hand_worked_trace(make):
    g = _golden()
    s = make(g["n_examples"], g["min_b"], g["max_b"], g["init_b"], g["alpha"])
    for i, r in enumerate(g["requests"]):
        begin, count = s.request(r["worker"], r["updates"])
        assert (begin, count) == (r["begin"], r["count"]), f"request {i}: {r['why']}"
        b = s.b[r["worker"]] if isinstance(s, AdaptiveSchedule) else s.batch_size(r["worker"])
        assert b == r["b_after"], f"request {i}: {r['why']}"


def _random_run(s, rng, n_workers, n_requests, beta_steps):
    """A seeded sequence of requests; returns what was handed out."""
    u = [0.0] * n_workers
    out = []
    for _ in range(n_requests):
        w = int(rng.integers(0, n_workers))
        begin, count = s.request(w, u[w])
        out.append((w, u[w], begin, count))
        if count > 0:
            u[w] += beta_steps[w]
        elif rng.random() < 0.3:
            s.new_epoch()
    return out


@pytest.mark.parametrize("alpha", [2.0, 1.5, 3.0])
def test_invariants_of_the_oracle(alpha):
    rng = np.random.default_rng(11)
    n, min_b, max_b, init_b = 5000, [1, 16, 7], [12, 1024, 200], [1, 1024, 50]
    s = AdaptiveSchedule(n, min_b, max_b, init_b, alpha)
    prev_b = list(init_b)
    cursor = 0
    u = [0.0, 0.0, 0.0]
    reported = [0.0, 0.0, 0.0]      # what the coordinator has been told so far
    for _ in range(3000):
        w = int(rng.integers(0, 3))
        others = [reported[x] for x in range(3) if x != w]
        begin, count = s.request(w, u[w])
        reported[w] = u[w]
        b = s.b[w]
        assert min_b[w] <= b <= max_b[w]
        # the batch size moves by one factor of alpha (rounded, clipped) and only in the direction
        # the update counts call for
        if u[w] < min(others):
            assert b == max(max(int(np.floor(prev_b[w] / alpha + 0.5)), 1), min_b[w])
        elif u[w] > max(others):
            assert b == min(int(np.floor(prev_b[w] * alpha + 0.5)), max_b[w])
        else:
            assert b == prev_b[w]
        prev_b[w] = b
        # batches are contiguous, in order, disjoint, and never run past the data
        assert begin == cursor
        if count:
            assert count == b and begin + count <= n
            cursor += count
            u[w] += [4.0, 1.0, 0.5][w]      # a CPU worker reports t * beta updates per batch
        else:
            assert b > n - cursor           # nothing is sent only when the batch does not fit
            if rng.random() < 0.5:
                s.new_epoch()
                cursor = 0


def test_single_worker_is_never_rescaled_and_tail_is_dropped():
    s = AdaptiveSchedule(1000, [16], [256], [64], 2.0)
    got = []
    u = 0
    while True:
        begin, count = s.request(0, u)
        if count == 0:
            break
        got.append((begin, count))
        u += 1
    assert got == [(64 * i, 64) for i in range(15)]       # 960 rows; the last 40 do not make a batch
    assert s.remaining() == 40
    s.new_epoch()
    assert s.request(0, u) == (0, 64)


@pytest.mark.parametrize("alpha,seed", [(2.0, 1), (1.5, 2), (2.5, 3), (1.1, 4)])
def test_library_matches_oracle_on_random_request_sequences(alpha, seed):
    n, min_b, max_b, init_b = 20000, [1, 24, 5, 100], [64, 4096, 333, 100], [1, 4096, 5, 100]
    a = AdaptiveSchedule(n, min_b, max_b, init_b, alpha)
    b = _lib_sched(n, min_b, max_b, init_b, alpha)
    ra = _random_run(a, np.random.default_rng(seed), 4, 4000, [8.0, 1.0, 0.75, 1.0])
    rb = _random_run(b, np.random.default_rng(seed), 4, 4000, [8.0, 1.0, 0.75, 1.0])
    assert ra == rb
    assert [b.batch_size(w) for w in range(4)] == a.b
    assert b.remaining() == a.remaining()


def test_library_rejects_bad_arguments():
    import paper_2004_08771_amd as hb
    with pytest.raises(hb.HbError):
        hb.Sched(100, [4], [2], [3], 2.0)          # min_b > max_b
    with pytest.raises(hb.HbError):
        hb.Sched(100, [1], [8], [4], 1.0)          # alpha must exceed 1
    s = hb.Sched(100, [1], [8], [4], 2.0)
    with pytest.raises(hb.HbError):
        s.request(1, 0)                            # no such worker
    with pytest.raises(hb.HbError):
        s.request(0, float("nan"))
    assert s.request(0, 0) == (0, 4)
