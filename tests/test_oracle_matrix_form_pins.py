"""Pins for oracle/matrix_form.py (the mini-batch step with numpy's fp64 matmul as a step, used
where the plain loops of hb_oracle.c are out of reach).  Every check compares it with something
other than itself: the hand-worked values, central finite differences, a scalar reverse-mode
differentiator built from the forward definition, torch's fp64 autograd, closed forms, brute
force over the stored entries of a CSR batch, and the loop oracle.  CPU only."""
import itertools
import json
import math
import os

import numpy as np
import pytest

import hb_inputs as hi
import oracle
from oracle import matrix_form as mf
from test_oracle_pins import (FD_CASES, _min_abs_hidden_preact, _rand_problem, _scalar_net_loss, _torch_loss, _V)

SIG, RELU = mf.ACT_SIGMOID, mf.ACT_RELU
CE, LOGI = mf.LOSS_SOFTMAX_CE, mf.LOSS_LOGISTIC
HERE = os.path.dirname(os.path.abspath(__file__))


def test_hand_worked_golden_cases():
    with open(os.path.join(HERE, "golden", "hand_worked.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        p = np.array(c["params"], dtype=np.float64)
        X = np.array(c["X"], dtype=np.float64)
        y = np.array(c["y"], dtype=np.int32)
        l, g = mf.batch_grad(c["dims"], c["act"], c["loss"], p, X, y)
        assert l == pytest.approx(c["loss_value"], rel=1e-14), c["name"]
        np.testing.assert_allclose(g, c["grad"], rtol=1e-13, atol=1e-15, err_msg=c["name"])
        np.testing.assert_allclose(mf.sgd_update(p, g, c["lr"]), c["params_after"], rtol=1e-13, atol=1e-15)
        assert mf.batch_loss(c["dims"], c["act"], c["loss"], p, X, y) == pytest.approx(l, rel=1e-15)


@pytest.mark.parametrize("dims,act,loss", FD_CASES)
def test_gradient_matches_central_finite_differences(dims, act, loss):
    B, h = 3, 1e-5
    params, X, y = _rand_problem(dims, loss, B, seed=211 + len(dims) + 7 * act + 3 * loss, scale=2.0)
    if act == RELU:
        for attempt in range(50):
            if _min_abs_hidden_preact(dims, params, X) > 100 * h:
                break
            params, X, y = _rand_problem(dims, loss, B, seed=3000 + attempt, scale=2.0)
        assert _min_abs_hidden_preact(dims, params, X) > 100 * h
    _, g = mf.batch_grad(dims, act, loss, params, X, y)
    fd = np.empty_like(g)
    for i in range(params.size):
        pp, pm = params.copy(), params.copy()
        pp[i] += h
        pm[i] -= h
        fd[i] = (mf.batch_loss(dims, act, loss, pp, X, y) - mf.batch_loss(dims, act, loss, pm, X, y)) / (2 * h)
    err = np.abs(fd - g) / np.maximum(np.abs(g), 1e-3)
    assert err.max() < 1e-6, (err.argmax(), err.max())
    assert np.linalg.norm(g) > 1e-3


@pytest.mark.parametrize("dims,act,loss", [((3, 2, 2), SIG, CE), ((3, 4, 3), RELU, CE),
                                           ((4, 3, 2, 1), SIG, LOGI), ((3, 3, 2), RELU, LOGI), ((3, 2), SIG, CE)])
def test_matches_scalar_reverse_mode_on_tiny_nets(dims, act, loss):
    params, X, y = _rand_problem(dims, loss, 4, seed=15 + sum(dims) + act)
    pv = [_V(p) for p in params]
    out = _scalar_net_loss(dims, act, loss, pv, X, y)
    out.backward()
    l, g = mf.batch_grad(dims, act, loss, params, X, y)
    assert l == pytest.approx(out.v, rel=1e-13)
    np.testing.assert_allclose(g, [p.g for p in pv], rtol=1e-11, atol=1e-14)


@pytest.mark.parametrize("dims,act,loss,B", [
    ((54, 48, 48, 7), SIG, CE, 33), ((30, 64, 64, 2), RELU, LOGI, 50), ((30, 64, 1), RELU, LOGI, 50),
    ((20, 40, 40, 40, 100), RELU, CE, 17),
])
def test_matches_torch_fp64_autograd_and_the_loop_oracle(dims, act, loss, B):
    params, X, y = _rand_problem(dims, loss, B, seed=177 + B)
    l, g = mf.batch_grad(dims, act, loss, params, X, y)
    tl, tg = _torch_loss(dims, act, loss, params, X, y)
    assert l == pytest.approx(tl, rel=1e-12)
    np.testing.assert_allclose(g, tg, rtol=1e-9, atol=1e-13)
    lo, go = oracle.batch_grad(dims, act, loss, params, X, y)
    assert l == pytest.approx(lo, rel=1e-12)
    np.testing.assert_allclose(g, go, rtol=1e-9, atol=1e-13)


def test_softmax_and_logistic_regression_closed_forms_and_log_k():
    d, K, B = 7, 5, 12
    params, X, y = _rand_problem((d, K), CE, B, seed=121)
    W, b = params[:K * d].reshape(K, d), params[K * d:]
    Z = X @ W.T + b
    P = np.exp(Z - Z.max(1, keepdims=True))
    P /= P.sum(1, keepdims=True)
    Y = np.eye(K)[y]
    l, g = mf.batch_grad((d, K), SIG, CE, params, X, y)
    assert l == pytest.approx(-np.mean(np.log(P[np.arange(B), y])), rel=1e-13)
    np.testing.assert_allclose(g[:K * d].reshape(K, d), (P - Y).T @ X / B, rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(g[K * d:], (P - Y).sum(0) / B, rtol=1e-11, atol=1e-15)
    d = 6
    params, X, y = _rand_problem((d, 1), LOGI, 15, seed=122)
    z = X @ params[:d] + params[d]
    s = 1.0 / (1.0 + np.exp(y * z))
    l, g = mf.batch_grad((d, 1), RELU, LOGI, params, X, y)
    assert l == pytest.approx(np.mean(np.log1p(np.exp(-y * z))), rel=1e-13)
    np.testing.assert_allclose(g[:d], -(y * s) @ X / 15, rtol=1e-11, atol=1e-15)
    assert g[d] == pytest.approx(-np.mean(y * s), rel=1e-11)
    for dims, loss, expect in [((54, 32, 7), CE, math.log(7)), ((12, 6, 1000), CE, math.log(1000)),
                               ((10, 8, 1), LOGI, math.log(2)), ((10, 8, 2), LOGI, math.log(2))]:
        _, X, y = _rand_problem(dims, loss, 10, seed=1)
        assert mf.batch_loss(dims, RELU, loss, np.zeros(hi.num_params(dims)), X, y) == pytest.approx(expect, rel=1e-14)


def test_csr_batch_with_unsorted_and_duplicate_columns_equals_brute_force_over_the_stored_entries():
    """A row may hold its entries in any order and name a column twice: the layer-1 sums run over
    the stored entries, so duplicates add.  Reference: the batch expanded entry by entry into a
    dense matrix (np.add.at), then the dense path of either oracle."""
    dims = (40, 9, 5, 2)
    rng = np.random.default_rng(5)
    B = 11
    counts = rng.integers(0, 8, size=B)
    counts[3] = 0
    rp = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    ci = rng.integers(0, 12, size=rp[-1]).astype(np.int32)        # 12 columns only: many duplicates
    va = rng.standard_normal(rp[-1])
    assert any(len(set(ci[rp[i]:rp[i + 1]])) < counts[i] for i in range(B))
    y = (2 * rng.integers(0, 2, size=B) - 1).astype(np.int32)
    params = hi.xavier_uniform_params(dims, rng, 0.3).astype(np.float64)
    dense = np.zeros((B, dims[0]))
    for i in range(B):
        np.add.at(dense[i], ci[rp[i]:rp[i + 1]], va[rp[i]:rp[i + 1]])
    for act in (SIG, RELU):
        l_d, g_d = mf.batch_grad(dims, act, LOGI, params, dense, y)
        l_s, g_s = mf.batch_grad(dims, act, LOGI, params, (rp, ci, va), y)
        l_c, g_c = oracle.batch_grad_csr(dims, act, LOGI, params, rp, ci, va, y)
        l_o, g_o = oracle.batch_grad(dims, act, LOGI, params, dense, y)
        for l, g in ((l_s, g_s), (l_c, g_c), (l_o, g_o)):
            assert l == pytest.approx(l_d, rel=1e-13)
            np.testing.assert_allclose(g, g_d, rtol=1e-10, atol=1e-15)


def test_bf16_round_and_storage_variant():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(9)
    v = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, 100000),
                        np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9, 0.0, -0.0, 1e-40], np.float32)])
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(mf.bf16_round(v).view(np.uint32), want.view(np.uint32))
    assert mf.bf16_round(np.float32([1.0 + 2.0 ** -8]))[0] == 1.0                      # tie -> even
    assert mf.bf16_round(np.float32([1.0 + 3 * 2.0 ** -8]))[0] == np.float32(1.0 + 2.0 ** -6)
    # the storage-rounding gradient: against the loop oracle's variant (pinned against torch with the
    # roundings written out in test_oracle_pins.py)
    for dims, act, loss in [((12, 10, 8, 5), SIG, CE), ((12, 10, 8, 5), RELU, CE), ((9, 7, 1), SIG, LOGI)]:
        params, X, y = _rand_problem(dims, loss, 23, seed=177, bias_scale=0.3)
        params, X = params.astype(np.float32), X.astype(np.float32)
        l_o, g_o = oracle.batch_grad_bf16_storage(dims, act, loss, params, X, y)
        l_m, g_m = mf.batch_grad(dims, act, loss, mf.round_weights_bf16(dims, params),
                                 mf.bf16_round(X).astype(np.float64), y, store_bf16=True)
        assert l_m == pytest.approx(l_o, rel=1e-12)
        np.testing.assert_allclose(g_m, g_o, rtol=1e-9, atol=1e-15)


def test_error_scale_is_the_sum_of_absolute_terms_by_brute_force_over_paths():
    """dW_1[j,k] of a 2-hidden-layer net is a sum over (example i, unit path j <- m <- c): the error
    scale must be the same sum with every factor replaced by its absolute value.  For dW_2[m,j] the
    factor A_1[i,j] is replaced by |A_1[i,j]| + |f'| (sum_k |X[i,k]| |W_1[j,k]| + |b_1[j]|)."""
    dims = (3, 2, 3, 2)
    for act in (SIG, RELU):
        params, X, y = _rand_problem(dims, CE, 4, seed=60 + act)
        _, g, s = mf.batch_grad(dims, act, CE, params, X, y, with_error_scale=True)
        assert np.all(s >= np.abs(g) * (1 - 1e-12))
        (W1, b1), (W2, b2), (W3, b3) = mf._views(dims, params)
        acts = mf.forward(dims, act, params, X)
        _, dL = mf.loss_and_delta(CE, acts[-1], y)
        d2 = mf._act_deriv_from_output(act, acts[2])
        d1 = mf._act_deriv_from_output(act, acts[1])
        g1, s1 = np.zeros_like(W1), np.zeros_like(W1)
        for i, j, k, m, c in itertools.product(range(4), range(2), range(3), range(3), range(2)):
            term = dL[i, c] * W3[c, m] * d2[i, m] * W2[m, j] * d1[i, j] * X[i, k]
            g1[j, k] += term
            s1[j, k] += abs(term)
        np.testing.assert_allclose(g[:6].reshape(2, 3), g1, rtol=1e-11, atol=1e-16)
        np.testing.assert_allclose(s[:6].reshape(2, 3), s1, rtol=1e-11, atol=1e-16)
        g2, s2 = np.zeros_like(W2), np.zeros_like(W2)
        for i, m, j, c in itertools.product(range(4), range(3), range(2), range(2)):
            back = dL[i, c] * W3[c, m] * d2[i, m]
            z1_terms = sum(abs(X[i, k]) * abs(W1[j, k]) for k in range(3)) + abs(b1[j])
            g2[m, j] += back * acts[1][i, j]
            s2[m, j] += abs(back) * (abs(acts[1][i, j]) + abs(d1[i, j]) * z1_terms)
        w2 = slice(6 + 2, 6 + 2 + 6)
        np.testing.assert_allclose(g[w2].reshape(3, 2), g2, rtol=1e-11, atol=1e-16)
        np.testing.assert_allclose(s[w2].reshape(3, 2), s2, rtol=1e-11, atol=1e-16)
        # output layer: db_3[c] = sum_i dL[i,c]
        np.testing.assert_allclose(s[-2:], np.abs(dL).sum(0), rtol=1e-12)


def test_relu_decisions_taken_from_elsewhere_against_scalar_reverse_mode():
    """relu_on replaces the derivative decisions of the listed hidden layers: checked against the
    scalar reverse-mode differentiator with the same decisions forced, with a third of the units of
    both hidden layers flipped."""
    dims = (4, 5, 3, 2)
    params, X, y = _rand_problem(dims, CE, 4, seed=91)
    pre = []
    mf.forward(dims, RELU, params, X, pre_activations=pre)
    rng = np.random.default_rng(2)
    relu_on = {l: (pre[l - 1] > 0) ^ (rng.random(pre[l - 1].shape) < 0.33) for l in (1, 2)}
    assert any(((pre[l - 1] > 0) != relu_on[l]).any() for l in (1, 2))
    l0, g0 = mf.batch_grad(dims, RELU, CE, params, X, y)
    l1, g1 = mf.batch_grad(dims, RELU, CE, params, X, y, relu_on=relu_on)
    assert l1 == l0 and not np.allclose(g1, g0)
    pv = [_V(p) for p in params]
    out = _scalar_net_loss(dims, RELU, CE, pv, X, y, relu_on=relu_on)
    out.backward()
    np.testing.assert_allclose(g1, [p.g for p in pv], rtol=1e-11, atol=1e-14)
    # its own decisions given back: the same gradient
    same = {l: pre[l - 1] > 0 for l in (1, 2)}
    np.testing.assert_array_equal(mf.batch_grad(dims, RELU, CE, params, X, y, relu_on=same)[1], g0)
