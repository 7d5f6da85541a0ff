"""Pins for the fp64 CPU oracle: every check here compares it with something other than
itself -- hand-worked values, closed forms, finite differences, a scalar reverse-mode
differentiator built from the forward definition only, torch's fp64 autograd, and
invariants of the mathematics.  CPU only."""
import json
import math
import os

import numpy as np
import pytest

import hb_inputs as hi
import oracle

SIG, RELU = oracle.ACT_SIGMOID, oracle.ACT_RELU
CE, LOGI = oracle.LOSS_SOFTMAX_CE, oracle.LOSS_LOGISTIC
HERE = os.path.dirname(os.path.abspath(__file__))


def _rand_problem(dims, loss, B, seed, bias_scale=0.5, scale=1.0):
    rng = np.random.default_rng(seed)
    params = hi.xavier_uniform_params(dims, rng, bias_scale=bias_scale).astype(np.float64)
    params *= scale
    X = rng.standard_normal((B, dims[0]))
    if loss == CE:
        y = rng.integers(0, dims[-1], size=B).astype(np.int32)
    else:
        y = (2 * rng.integers(0, 2, size=B) - 1).astype(np.int32)
    return params, X, y


# ------------------------------------------------------------------ hand-worked values
def test_hand_worked_golden_cases():
    with open(os.path.join(HERE, "golden", "hand_worked.json")) as f:
        cases = json.load(f)["cases"]
    assert len(cases) >= 4
    for c in cases:
        p = np.array(c["params"], dtype=np.float64)
        X = np.array(c["X"], dtype=np.float64)
        y = np.array(c["y"], dtype=np.int32)
        l, g = oracle.batch_grad(c["dims"], c["act"], c["loss"], p, X, y)
        assert l == pytest.approx(c["loss_value"], rel=1e-14), c["name"]
        np.testing.assert_allclose(g, c["grad"], rtol=1e-13, atol=1e-15, err_msg=c["name"])
        l2, p2 = oracle.batch_step(c["dims"], c["act"], c["loss"], p, X, y, c["lr"])
        assert l2 == l
        np.testing.assert_allclose(p2, c["params_after"], rtol=1e-13, atol=1e-15, err_msg=c["name"])
        assert oracle.batch_loss(c["dims"], c["act"], c["loss"], p, X, y) == pytest.approx(l, rel=1e-15)


# ------------------------------------------------------------------ finite differences
FD_CASES = [
    ((5, 4, 3), SIG, CE), ((5, 4, 3), RELU, CE),
    ((6, 5, 4, 1), SIG, LOGI), ((6, 5, 4, 1), RELU, LOGI),
    ((6, 5, 4, 2), SIG, LOGI), ((6, 5, 4, 2), RELU, LOGI),
    ((4, 3), SIG, CE), ((4, 1), SIG, LOGI),
    ((7, 6, 5, 4, 3), SIG, CE), ((7, 6, 5, 4, 3), RELU, CE),
]


@pytest.mark.parametrize("dims,act,loss", FD_CASES)
def test_gradient_matches_central_finite_differences(dims, act, loss):
    B, h = 3, 1e-5
    params, X, y = _rand_problem(dims, loss, B, seed=11 + len(dims) + 7 * act + 3 * loss, scale=2.0)
    if act == RELU:
        # keep every hidden pre-activation away from the kink: nudge until |Z| > 100 h
        for attempt in range(50):
            if _min_abs_hidden_preact(dims, params, X) > 100 * h:
                break
            params, X, y = _rand_problem(dims, loss, B, seed=1000 + attempt, scale=2.0)
        assert _min_abs_hidden_preact(dims, params, X) > 100 * h
    l0, g = oracle.batch_grad(dims, act, loss, params, X, y)
    fd = np.empty_like(g)
    for i in range(params.size):
        pp, pm = params.copy(), params.copy()
        pp[i] += h
        pm[i] -= h
        fd[i] = (oracle.batch_loss(dims, act, loss, pp, X, y)
                 - oracle.batch_loss(dims, act, loss, pm, X, y)) / (2 * h)
    err = np.abs(fd - g) / np.maximum(np.abs(g), 1e-3)
    assert err.max() < 1e-6, (err.argmax(), err.max())
    assert np.linalg.norm(g) > 1e-3  # the check is not vacuous


def _min_abs_hidden_preact(dims, params, X):
    """numpy forward of the linear parts only, to locate ReLU kinks (test helper)."""
    a, m = X, np.inf
    for l, (wo, bo) in enumerate(hi.param_offsets(dims), start=1):
        W = params[wo:wo + dims[l] * dims[l - 1]].reshape(dims[l], dims[l - 1])
        z = a @ W.T + params[bo:bo + dims[l]]
        if l < len(dims) - 1:
            m = min(m, np.abs(z).min())
            a = np.maximum(z, 0.0)
    return m


# ------------------------------------------------------------------ scalar reverse-mode
class _V:
    """A scalar with a generic chain rule -- knows + * exp log max only.  The network
    below is written from the forward definition; no backprop formula is retyped."""
    __slots__ = ("v", "g", "parents")

    def __init__(self, v, parents=()):
        self.v, self.g, self.parents = float(v), 0.0, parents

    @staticmethod
    def lift(x):
        return x if isinstance(x, _V) else _V(x)

    def __add__(self, o):
        o = _V.lift(o)
        return _V(self.v + o.v, ((self, 1.0), (o, 1.0)))

    __radd__ = __add__

    def __mul__(self, o):
        o = _V.lift(o)
        return _V(self.v * o.v, ((self, o.v), (o, self.v)))

    __rmul__ = __mul__

    def __neg__(self):
        return self * -1.0

    def __sub__(self, o):
        return self + (-_V.lift(o))

    def exp(self):
        e = math.exp(self.v)
        return _V(e, ((self, e),))

    def log(self):
        return _V(math.log(self.v), ((self, 1.0 / self.v),))

    def recip(self):
        return _V(1.0 / self.v, ((self, -1.0 / (self.v * self.v)),))

    def relu(self):
        return _V(max(self.v, 0.0), ((self, 1.0 if self.v > 0 else 0.0),))

    def backward(self):
        order, seen = [], set()

        def visit(n):
            if id(n) in seen:
                return
            seen.add(id(n))
            for p, _ in n.parents:
                visit(p)
            order.append(n)

        visit(self)
        self.g = 1.0
        for n in reversed(order):
            for p, d in n.parents:
                p.g += d * n.g


def _scalar_net_loss(dims, act, loss, pv, X, y, relu_on=None):
    """relu_on: {l: boolean B x d_l} forces the derivative decision of ReLU units (the value
    max(z, 0) is unchanged)."""
    B, L = X.shape[0], len(dims) - 1
    total = _V(0.0)
    offs = hi.param_offsets(dims)
    for i in range(B):
        a = [_V(x) for x in X[i]]
        for l in range(1, L + 1):
            wo, bo = offs[l - 1]
            z = []
            for j in range(dims[l]):
                s = pv[bo + j]
                for k in range(dims[l - 1]):
                    s = s + pv[wo + j * dims[l - 1] + k] * a[k]
                z.append(s)
            if l < L and act == RELU and relu_on is not None and l in relu_on:
                a = [_V(max(t.v, 0.0), ((t, 1.0 if relu_on[l][i, j] else 0.0),)) for j, t in enumerate(z)]
            elif l < L:
                a = [((-t).exp() + 1.0).recip() if act == SIG else t.relu() for t in z]
            else:
                a = z
        if loss == LOGI and dims[-1] == 1:
            total = total + ((a[0] * (-float(y[i]))).exp() + 1.0).log()
        else:
            c = int(y[i]) if loss == CE else (int(y[i]) + 1) // 2
            se = _V(0.0)
            for t in a:
                se = se + t.exp()
            total = total + (se.log() - a[c])
    return total * (1.0 / B)


@pytest.mark.parametrize("dims,act,loss", [((3, 2, 2), SIG, CE), ((3, 4, 3), RELU, CE),
                                           ((4, 3, 2, 1), SIG, LOGI), ((3, 3, 2), RELU, LOGI),
                                           ((3, 2), SIG, CE)])
def test_matches_scalar_reverse_mode_on_tiny_nets(dims, act, loss):
    params, X, y = _rand_problem(dims, loss, 4, seed=5 + sum(dims) + act)
    pv = [_V(p) for p in params]
    out = _scalar_net_loss(dims, act, loss, pv, X, y)
    out.backward()
    l, g = oracle.batch_grad(dims, act, loss, params, X, y)
    assert l == pytest.approx(out.v, rel=1e-13)
    np.testing.assert_allclose(g, [p.g for p in pv], rtol=1e-11, atol=1e-14)


# ------------------------------------------------------------------ library autograd
def _torch_loss(dims, act, loss, params, X, y):
    import torch
    import torch.nn.functional as F
    p = torch.tensor(params, dtype=torch.float64, requires_grad=True)
    a = torch.tensor(X, dtype=torch.float64)
    L = len(dims) - 1
    for l, (wo, bo) in enumerate(hi.param_offsets(dims), start=1):
        W = p[wo:wo + dims[l] * dims[l - 1]].view(dims[l], dims[l - 1])
        a = F.linear(a, W, p[bo:bo + dims[l]])
        if l < L:
            a = torch.sigmoid(a) if act == SIG else torch.relu(a)
    if loss == LOGI and dims[-1] == 1:
        out = F.soft_margin_loss(a[:, 0], torch.tensor(y, dtype=torch.float64))
    else:
        t = torch.tensor(y if loss == CE else (y + 1) // 2, dtype=torch.long)
        out = F.cross_entropy(a, t)
    out.backward()
    return float(out.detach()), p.grad.numpy()


@pytest.mark.parametrize("dims,act,loss,B", [
    ((54, 32, 7), SIG, CE, 64),
    ((54, 48, 48, 7), SIG, CE, 33),
    ((30, 64, 64, 2), RELU, LOGI, 50),
    ((30, 64, 1), RELU, LOGI, 50),
    ((20, 40, 40, 40, 100), RELU, CE, 17),
])
def test_matches_torch_fp64_autograd(dims, act, loss, B):
    params, X, y = _rand_problem(dims, loss, B, seed=77 + B)
    l, g = oracle.batch_grad(dims, act, loss, params, X, y)
    tl, tg = _torch_loss(dims, act, loss, params, X, y)
    assert l == pytest.approx(tl, rel=1e-12)
    np.testing.assert_allclose(g, tg, rtol=1e-9, atol=1e-13)


# ------------------------------------------------------------------ batch reduction
@pytest.mark.parametrize("dims,act,loss", [((6, 5, 4), SIG, CE), ((6, 5, 5, 2), RELU, LOGI)])
def test_batch_gradient_is_mean_of_per_example_gradients(dims, act, loss):
    B = 9
    params, X, y = _rand_problem(dims, loss, B, seed=3)
    l, g = oracle.batch_grad(dims, act, loss, params, X, y)
    ls, gs = zip(*[oracle.batch_grad(dims, act, loss, params, X[i:i + 1], y[i:i + 1]) for i in range(B)])
    assert l == pytest.approx(np.mean(ls), rel=1e-13)
    np.testing.assert_allclose(g, np.mean(gs, axis=0), rtol=1e-11, atol=1e-15)
    perm = np.random.default_rng(0).permutation(B)
    lp, gp = oracle.batch_grad(dims, act, loss, params, X[perm], y[perm])
    assert lp == pytest.approx(l, rel=1e-13)
    np.testing.assert_allclose(gp, g, rtol=1e-11, atol=1e-15)


# ------------------------------------------------------------------ closed forms, no hidden layer
def test_softmax_regression_closed_form():
    d, K, B = 7, 5, 12
    params, X, y = _rand_problem((d, K), CE, B, seed=21)
    W, b = params[:K * d].reshape(K, d), params[K * d:]
    Z = X @ W.T + b
    P = np.exp(Z - Z.max(1, keepdims=True))
    P /= P.sum(1, keepdims=True)
    Y = np.eye(K)[y]
    l, g = oracle.batch_grad((d, K), SIG, CE, params, X, y)
    assert l == pytest.approx(-np.mean(np.log(P[np.arange(B), y])), rel=1e-13)
    np.testing.assert_allclose(g[:K * d].reshape(K, d), (P - Y).T @ X / B, rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(g[K * d:], (P - Y).sum(0) / B, rtol=1e-11, atol=1e-15)


def test_logistic_regression_closed_form():
    d, B = 6, 15
    params, X, y = _rand_problem((d, 1), LOGI, B, seed=22)
    w, b = params[:d], params[d]
    z = X @ w + b
    s = 1.0 / (1.0 + np.exp(y * z))  # sigma(-y z)
    l, g = oracle.batch_grad((d, 1), RELU, LOGI, params, X, y)
    assert l == pytest.approx(np.mean(np.log1p(np.exp(-y * z))), rel=1e-13)
    np.testing.assert_allclose(g[:d], -(y * s) @ X / B, rtol=1e-11, atol=1e-15)
    assert g[d] == pytest.approx(-np.mean(y * s), rel=1e-11)


# ------------------------------------------------------------------ loss values
@pytest.mark.parametrize("dims,loss,expect", [
    ((54, 32, 7), CE, math.log(7)), ((10, 8, 2), CE, math.log(2)),
    ((12, 6, 1000), CE, math.log(1000)), ((10, 8, 1), LOGI, math.log(2)),
    ((10, 8, 2), LOGI, math.log(2)),
])
def test_zero_weights_give_log_k(dims, loss, expect):
    _, X, y = _rand_problem(dims, loss, 10, seed=1)
    z = np.zeros(hi.num_params(dims))
    for act in (SIG, RELU):
        assert oracle.batch_loss(dims, act, loss, z, X, y) == pytest.approx(expect, rel=1e-14)


def test_sigmoid_hidden_units_are_half_at_zero_weights():
    # with W_1 = 0, b_1 = 0 every hidden unit is 1/2, so dW_2[j,:] = 1/2 * db_2[j]
    dims = (4, 3, 5)
    _, X, y = _rand_problem(dims, CE, 8, seed=2)
    p = np.zeros(hi.num_params(dims))
    (w1, b1), (w2, b2) = hi.param_offsets(dims)
    p[w2:w2 + 15] = np.random.default_rng(0).standard_normal(15)
    _, g = oracle.batch_grad(dims, SIG, CE, p, X, y)
    np.testing.assert_allclose(g[w2:w2 + 15].reshape(5, 3), 0.5 * np.repeat(g[b2:b2 + 5, None], 3, 1),
                               rtol=1e-12, atol=1e-16)


# ------------------------------------------------------------------ softmax invariants
def test_softmax_delta_rows_sum_to_zero_and_shift_invariance():
    dims = (6, 5, 4)
    params, X, y = _rand_problem(dims, CE, 7, seed=4)
    l, g = oracle.batch_grad(dims, SIG, CE, params, X, y)
    (_, _), (_, b2) = hi.param_offsets(dims)
    assert abs(g[b2:b2 + 4].sum()) < 1e-15
    shifted = params.copy()
    shifted[b2:b2 + 4] += 3.75
    l2, g2 = oracle.batch_grad(dims, SIG, CE, shifted, X, y)
    assert l2 == pytest.approx(l, rel=1e-13)
    np.testing.assert_allclose(g2, g, rtol=1e-10, atol=1e-15)


def test_two_way_softmax_equals_logistic_on_the_margin():
    dims2, dims1 = (5, 4, 2), (5, 4, 1)
    params2, X, y = _rand_problem(dims2, LOGI, 9, seed=6)
    (w1, b1), (w2, b2) = hi.param_offsets(dims2)
    W2 = params2[w2:w2 + 8].reshape(2, 4)
    bb = params2[b2:b2 + 2]
    params1 = np.concatenate([params2[:w2], W2[1] - W2[0], [bb[1] - bb[0]]])
    for act in (SIG, RELU):
        l2, g2 = oracle.batch_grad(dims2, act, LOGI, params2, X, y)
        l1, g1 = oracle.batch_grad(dims1, act, LOGI, params1, X, y)
        assert l2 == pytest.approx(l1, rel=1e-13)
        np.testing.assert_allclose(g2[:w2], g1[:w2], rtol=1e-11, atol=1e-15)       # hidden layer
        np.testing.assert_allclose(g2[w2 + 4:w2 + 8], g1[w2:w2 + 4], rtol=1e-11, atol=1e-15)
        np.testing.assert_allclose(g2[w2:w2 + 4], -g1[w2:w2 + 4], rtol=1e-11, atol=1e-15)
        # the +-1 labelled two-way loss is the class-indexed softmax cross-entropy
        l3, g3 = oracle.batch_grad(dims2, act, CE, params2, X, (y + 1) // 2)
        assert l3 == l2 and np.array_equal(g3, g2)


# ------------------------------------------------------------------ update
def test_update_is_w_minus_lr_g_and_descends():
    dims = (8, 6, 6, 3)
    params, X, y = _rand_problem(dims, CE, 16, seed=8)
    l, g = oracle.batch_grad(dims, SIG, CE, params, X, y)
    l0, p0 = oracle.batch_step(dims, SIG, CE, params, X, y, 0.0)
    assert l0 == l and np.array_equal(p0, params)
    lr = 0.37
    _, p1 = oracle.batch_step(dims, SIG, CE, params, X, y, lr)
    np.testing.assert_allclose(p1, params - lr * g, rtol=0, atol=1e-16)
    np.testing.assert_array_equal(oracle.sgd_update(params, g, lr), p1)
    # first-order decrease: loss(W - eps g) = loss(W) - eps |g|^2 + O(eps^2)
    eps = 1e-4
    _, p2 = oracle.batch_step(dims, SIG, CE, params, X, y, eps)
    drop = l - oracle.batch_loss(dims, SIG, CE, p2, X, y)
    assert drop == pytest.approx(eps * g @ g, rel=1e-2)


# ------------------------------------------------------------------ CSR path
def test_csr_path_equals_dense_on_densified_batch_and_leaves_untouched_columns():
    dims = (300, 16, 8, 2)
    rng = np.random.default_rng(9)
    row_ptr, col_idx, vals = hi.zipf_csr(40, dims[0], rng, mean_nnz=6, max_nnz=20)
    y = hi.csr_pm1_labels(row_ptr, col_idx, vals, dims[0], rng)
    Xd = hi.csr_to_dense(row_ptr, col_idx, vals, dims[0])
    params = hi.xavier_uniform_params(dims, rng, bias_scale=0.3).astype(np.float64)
    for act in (SIG, RELU):
        ld, gd = oracle.batch_grad(dims, act, LOGI, params, Xd, y)
        ls, gs = oracle.batch_grad_csr(dims, act, LOGI, params, row_ptr, col_idx, vals, y)
        assert ls == pytest.approx(ld, rel=1e-13)
        np.testing.assert_allclose(gs, gd, rtol=1e-11, atol=1e-16)
        _, pd_ = oracle.batch_step(dims, act, LOGI, params, Xd, y, 0.2)
        _, ps = oracle.batch_step_csr(dims, act, LOGI, params, row_ptr, col_idx, vals, y, 0.2)
        np.testing.assert_allclose(ps, pd_, rtol=1e-12, atol=1e-16)
        W1_before = params[:dims[1] * dims[0]].reshape(dims[1], dims[0])
        W1_after = ps[:dims[1] * dims[0]].reshape(dims[1], dims[0])
        untouched = np.setdiff1d(np.arange(dims[0]), col_idx)
        assert untouched.size > 50
        assert np.array_equal(W1_after[:, untouched], W1_before[:, untouched])
        assert not np.array_equal(W1_after[:, np.unique(col_idx)], W1_before[:, np.unique(col_idx)])


def test_csr_with_empty_rows():
    dims = (10, 4, 2)
    row_ptr = np.array([0, 0, 2, 2, 3], dtype=np.int32)
    col_idx = np.array([1, 7, 3], dtype=np.int32)
    vals = np.array([0.5, -1.5, 2.0], dtype=np.float32)
    y = np.array([1, -1, 1, -1], dtype=np.int32)
    params = hi.xavier_uniform_params(dims, np.random.default_rng(1), 0.2).astype(np.float64)
    Xd = hi.csr_to_dense(row_ptr, col_idx, vals, 10)
    ld, gd = oracle.batch_grad(dims, SIG, LOGI, params, Xd, y)
    ls, gs = oracle.batch_grad_csr(dims, SIG, LOGI, params, row_ptr, col_idx, vals, y)
    assert ls == pytest.approx(ld, rel=1e-14)
    np.testing.assert_allclose(gs, gd, rtol=1e-12, atol=1e-16)


# ------------------------------------------------------------------ merge
def test_merge_special_weights():
    rng = np.random.default_rng(3)
    D, H = rng.standard_normal(50), rng.standard_normal(50)
    d0, h0 = oracle.model_merge(D, H, 0.0)
    assert np.array_equal(d0, H) and np.array_equal(h0, H)          # replica <- global
    d1, h1 = oracle.model_merge(D, H, 1.0)
    assert np.array_equal(d1, D) and np.array_equal(h1, D)          # global <- replica
    dm, hm = oracle.model_merge(D, H, 0.5)
    np.testing.assert_allclose(dm, (D + H) / 2, rtol=1e-15)
    assert np.array_equal(dm, hm)
    dq, hq = oracle.model_merge(D, H, 0.25)
    np.testing.assert_allclose(dq, 0.75 * H + 0.25 * D, rtol=1e-15)
    d2, h2 = oracle.model_merge(dq, hq, 0.25)                       # both sides equal already
    np.testing.assert_allclose(d2, dq, rtol=1e-15)
    assert np.array_equal(d2, h2)


# ------------------------------------------------------------------ bf16 rounding
def test_bf16_round_known_values_and_against_torch():
    import torch
    cases = {
        1.0: 1.0,
        1.0 + 2.0 ** -8: 1.0,                 # tie -> even (mantissa ...0)
        1.0 + 2.0 ** -7: 1.0 + 2.0 ** -7,     # representable
        1.0 + 3 * 2.0 ** -8: 1.0 + 2.0 ** -6,  # tie -> even (rounds up)
        1.0 + 2.0 ** -8 + 2.0 ** -20: 1.0 + 2.0 ** -7,  # just above the tie
        -0.3: float(torch.tensor(-0.3).bfloat16().float()),
        0.0: 0.0,
    }
    got = oracle.bf16_round(np.array(list(cases.keys()), dtype=np.float32))
    np.testing.assert_array_equal(got, np.array(list(cases.values()), dtype=np.float32))
    x = (np.random.default_rng(0).standard_normal(100000) *
         np.exp(np.random.default_rng(1).uniform(-20, 20, 100000))).astype(np.float32)
    ref = torch.from_numpy(x).bfloat16().float().numpy()
    np.testing.assert_array_equal(oracle.bf16_round(x), ref)


def test_bf16_rounded_inputs_stay_within_budget():
    dims = (64, 48, 48, 10)
    params, X, y = _rand_problem(dims, CE, 32, seed=12, bias_scale=0.0)
    l, g = oracle.batch_grad(dims, RELU, CE, params, X, y)
    pr = oracle.bf16_round(params.astype(np.float32)).astype(np.float64)
    Xr = oracle.bf16_round(X.astype(np.float32)).astype(np.float64)
    lr_, gr = oracle.batch_grad(dims, RELU, CE, pr, Xr, y)
    assert abs(lr_ - l) / l < 2e-2
    assert np.linalg.norm(gr - g) / np.linalg.norm(g) < 2e-2


# ------------------------------------------------------------------ argument checks
def test_invalid_arguments_return_nan():
    params, X, y = _rand_problem((4, 3), CE, 2, seed=0)
    assert math.isnan(oracle.batch_loss((4, 3), 7, CE, params, X, y))
    assert math.isnan(oracle.batch_loss((4, 3), SIG, 9, params, X, y))
    p3, X3, y3 = _rand_problem((4, 3), LOGI, 2, seed=0)
    assert math.isnan(oracle.batch_loss((4, 3), SIG, LOGI, p3, X3, y3))  # logistic needs d_L <= 2


def test_bf16_storage_gradient_is_the_plain_gradient_up_to_storage_rounding():
    """The mixed-precision variant differs from the plain oracle only by bf16 storage
    rounding of hidden activations and deltas: the two agree to about 2^-8 on a smooth
    (sigmoid) net but are not identical."""
    dims = (32, 24, 24, 6)
    params, X, y = _rand_problem(dims, CE, 40, seed=31, bias_scale=0.2)
    pr = oracle.round_weights_bf16(dims, params.astype(np.float32))
    Xr = oracle.bf16_round(X.astype(np.float32)).astype(np.float64)
    l0, g0 = oracle.batch_grad(dims, SIG, CE, pr, Xr, y)
    l1, g1 = oracle.batch_grad_bf16_storage(dims, SIG, CE, params.astype(np.float32), X, y)
    assert abs(l1 - l0) / l0 < 1e-2
    assert np.linalg.norm(g1 - g0) / np.linalg.norm(g0) < 1e-2
    assert not np.array_equal(g1, g0)
    # no hidden layer: the only stored value is delta_L, so dW = delta_L^T X and
    # db = delta_L^T 1 move by at most the bf16 rounding of delta_L
    dims0 = (16, 4)
    p0, X0, y0 = _rand_problem(dims0, CE, 8, seed=32)
    l_a, ga = oracle.batch_grad_bf16_storage(dims0, SIG, CE, p0.astype(np.float32), X0, y0)
    pr0 = oracle.round_weights_bf16(dims0, p0.astype(np.float32))
    Xr0 = oracle.bf16_round(X0.astype(np.float32)).astype(np.float64)
    l_b, gb = oracle.batch_grad(dims0, SIG, CE, pr0, Xr0, y0)
    assert l_a == l_b                       # the loss sees no stored value
    assert np.linalg.norm(ga - gb) / np.linalg.norm(gb) < 2.0 ** -8


@pytest.mark.parametrize("dims,act,loss", [((12, 10, 8, 5), SIG, CE), ((12, 10, 8, 5), RELU, CE),
                                           ((9, 7, 2), RELU, LOGI), ((9, 7, 1), SIG, LOGI)])
def test_bf16_storage_gradient_against_torch_with_the_roundings_written_out(dims, act, loss):
    """Second route to the mixed-precision gradient: matrix products and the loss derivative
    from torch (fp64, autograd for dl/dz_L), with a bf16 cast wherever a hidden activation or
    a delta is stored.  A missing or misplaced rounding site, a derivative taken from the
    unrounded activation, or a transposed operand in the oracle shows up here."""
    torch = pytest.importorskip("torch")
    B = 23
    params, X, y = _rand_problem(dims, loss, B, seed=77, bias_scale=0.3)
    params = params.astype(np.float32)
    X = X.astype(np.float32)
    l_o, g_o = oracle.batch_grad_bf16_storage(dims, act, loss, params, X, y)

    def st(t):  # what a bf16 store keeps (through fp32, as a kernel would hold it)
        return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)

    Ws, bs = [], []
    for l, (wo, bo) in enumerate(hi.param_offsets(dims), start=1):
        W = torch.from_numpy(params[wo:wo + dims[l] * dims[l - 1]].reshape(dims[l], dims[l - 1]).copy())
        Ws.append(st(W))                                                 # bf16 shadow of the weights
        bs.append(torch.from_numpy(params[bo:bo + dims[l]].copy()).to(torch.float64))  # biases stay fp32
    L = len(Ws)
    acts = [st(torch.from_numpy(X))]
    for l in range(L):
        z = acts[-1] @ Ws[l].T + bs[l]
        if l < L - 1:
            z = st(torch.sigmoid(z) if act == SIG else torch.clamp(z, min=0.0))
        acts.append(z)
    zL = acts[-1].clone().requires_grad_(True)
    yt = torch.from_numpy(y.astype(np.int64))
    if loss == CE:
        lt = torch.nn.functional.cross_entropy(zL, yt, reduction="mean")
    elif dims[-1] == 2:
        lt = torch.nn.functional.cross_entropy(zL, (yt + 1) // 2, reduction="mean")
    else:
        lt = torch.nn.functional.softplus(-yt.to(torch.float64) * zL[:, 0]).mean()
    lt.backward()
    assert l_o == pytest.approx(float(lt.detach()), rel=1e-12)
    D = st(zL.grad)
    grads = [None] * L
    for l in range(L - 1, -1, -1):
        grads[l] = (D.T @ acts[l], D.sum(dim=0))
        if l > 0:
            a = acts[l]
            deriv = a * (1.0 - a) if act == SIG else (a > 0).to(torch.float64)
            D = st((D @ Ws[l]) * deriv)
    flat = np.concatenate([np.concatenate([gw.numpy().ravel(), gb.numpy().ravel()]) for gw, gb in grads])
    np.testing.assert_allclose(g_o, flat, rtol=1e-9, atol=1e-15)
