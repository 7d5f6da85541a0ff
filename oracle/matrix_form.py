"""The mini-batch step in matrix form, numpy fp64.  TEST INFRASTRUCTURE ONLY.

Second statement of what `hb_oracle.c` computes, for the sizes that program's plain loops
cannot reach (a 4096-wide network on thousands of rows): the three products of each layer are
numpy's fp64 `@` (a library matmul as a step), everything else is the definition written out
on whole arrays, in the paper's order.  It imports nothing from the HIP package and shares no
code with it; only the tests, the smoke check and the benchmark's cpu_baseline leg may use it.

What it follows in the paper (Ma & Rusu, "Heterogeneous CPU+GPU Stochastic Gradient Descent
Algorithms", 2020):
  forward pass   Section 3, Eq. (1): A_l = f(A_{l-1} W_l^T + b_l), on a batch a matrix product;
  backward pass  Section 3, Eq. (2): the chain rule from the loss back through the layers
                 (schematic in the paper; the standard recurrences are written out);
  update         Section 3, Eq. (3): W <- W - eta g;
  sigmoid hidden units, softmax output, cross-entropy loss: Section 7.1.
Readings where the paper is silent are those of `hb_oracle.c` (bias vectors, MEAN over the
batch, ReLU with derivative 0 at 0, logistic loss on +-1 labels, 2-way softmax for d_L = 2).

Pinned by tests/test_oracle_pins.py: the hand-worked cases, central finite differences, the
closed forms, and agreement with `hb_oracle.c` (itself pinned the same way) on random nets.

`grad_error_scale` is not part of the method: it gives, for every gradient entry, the sum of the
absolute values of the terms that the chain rule adds up for it (plus the same for the
activation that enters it) -- the scale against which a floating-point evaluation of that entry
can be judged when the terms cancel.
"""
from __future__ import annotations

import numpy as np

ACT_SIGMOID, ACT_RELU = 0, 1
LOSS_SOFTMAX_CE, LOSS_LOGISTIC = 0, 1


def _views(dims, flat):
    """[(W_l, b_l)] views into the flat layout [W_1, b_1, ..., W_L, b_L], W_l is d_l x d_{l-1}."""
    out, off = [], 0
    for l in range(1, len(dims)):
        n = dims[l] * dims[l - 1]
        out.append((flat[off:off + n].reshape(dims[l], dims[l - 1]), flat[off + n:off + n + dims[l]]))
        off += n + dims[l]
    assert off == flat.size, "flat parameter vector has the wrong length"
    return out


def bf16_round(a):
    """Nearest bfloat16 (ties to even) of finite float32 values, returned as float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lower = u & np.uint32(0xffff)
    top = u & np.uint32(0xffff0000)
    up = (lower > 0x8000) | ((lower == 0x8000) & ((top & np.uint32(0x10000)) != 0))
    return (top + np.where(up, np.uint32(0x10000), np.uint32(0))).astype(np.uint32).view(np.float32)


def _stored(v, store_bf16):
    """A value the mixed-precision policy keeps in bf16 between two products: the fp32 result
    rounded to bf16.  Nothing is rounded when store_bf16 is false."""
    return bf16_round(v.astype(np.float32)).astype(np.float64) if store_bf16 else v


def _act(act, z):
    if act == ACT_SIGMOID:
        return 1.0 / (1.0 + np.exp(-z))
    return np.maximum(z, 0.0)


def _act_deriv_from_output(act, a):
    if act == ACT_SIGMOID:
        return a * (1.0 - a)
    return (a > 0.0).astype(np.float64)      # z > 0 <=> a > 0; derivative 0 at 0


def _first_product(X, W1):
    """A_0 W_1^T for dense X, or for a CSR batch (row_ptr, col_idx, vals): sums over the stored
    entries only (scipy's sparse product adds duplicate column indices of a row)."""
    if isinstance(X, tuple):
        import scipy.sparse as sp
        rp, ci, va = X
        # copies: scipy merges duplicate entries in place when it needs a canonical matrix
        S = sp.csr_matrix((np.array(va, np.float64), np.array(ci), np.array(rp)),
                          shape=(len(rp) - 1, W1.shape[1]))
        return np.asarray(S @ W1.T), S
    return X @ W1.T, X


def forward(dims, act, params, X, store_bf16=False, pre_activations=None, pre_activation_scales=None):
    """Eq. (1): list [A_0, A_1, ..., A_{L-1}, Z_L]; A_0 is X (dense array, or scipy CSR).
    pre_activations: an empty list that receives Z_1 .. Z_{L-1}; pre_activation_scales: an empty
    list that receives, for the same entries, |A_{l-1}| |W_l|^T + |b_l| -- the sum of the absolute
    values of the terms of each pre-activation (how close to 0 one has to be for its sign to
    depend on the precision of the sums)."""
    layers = _views(dims, np.asarray(params, dtype=np.float64))
    L = len(layers)
    z, A0 = _first_product(X, layers[0][0])
    acts = [A0]
    for l in range(1, L + 1):
        W, b = layers[l - 1]
        if l > 1:
            z = acts[-1] @ W.T
        z = z + b
        if l < L and pre_activations is not None:
            pre_activations.append(z)
        if l < L and pre_activation_scales is not None:
            pre_activation_scales.append(np.asarray(abs(acts[-1]) @ np.abs(W).T) + np.abs(b))
        acts.append(_stored(_act(act, z), store_bf16) if l < L else z)
    return acts


def loss_and_delta(loss, Z, y, store_bf16=False):
    """Section 7.1: softmax + cross-entropy (or the logistic loss), mean over the batch.
    Returns (mean loss, d(mean loss)/dZ)."""
    B, K = Z.shape
    y = np.asarray(y)
    if loss == LOSS_LOGISTIC and K == 1:
        m = y * Z[:, 0]
        li = np.maximum(-m, 0.0) + np.log1p(np.exp(-np.abs(m)))
        s = np.where(m >= 0.0, np.exp(-np.abs(m)) / (1.0 + np.exp(-np.abs(m))), 1.0 / (1.0 + np.exp(-np.abs(m))))
        delta = (-y * s / B)[:, None]
    else:
        c = (y + 1) // 2 if loss == LOSS_LOGISTIC else y
        mx = Z.max(axis=1, keepdims=True)
        lse = mx + np.log(np.exp(Z - mx).sum(axis=1, keepdims=True))
        li = lse[:, 0] - Z[np.arange(B), c]
        onehot = np.zeros_like(Z)
        onehot[np.arange(B), c] = 1.0
        delta = (np.exp(Z - lse) - onehot) / B
    return float(li.sum() / B), _stored(delta, store_bf16)


def batch_loss(dims, act, loss, params, X, y):
    return loss_and_delta(loss, forward(dims, act, params, X)[-1], y)[0]


def batch_grad(dims, act, loss, params, X, y, store_bf16=False, with_error_scale=False, relu_on=None):
    """(mean loss, flat gradient [dW_1, db_1, ...]) -- Eq. (2) written out:
        dW_l = delta_l^T A_{l-1},  db_l = delta_l^T 1,  delta_{l-1} = (delta_l W_l) * f'(A_{l-1}).
    X: dense B x d_0, or a CSR batch (row_ptr, col_idx, vals).  With store_bf16 the caller passes X
    and the weight matrices already rounded to bf16 and the hidden activations and deltas are
    rounded where the policy stores them.  with_error_scale: also returns grad_error_scale.
    relu_on (ReLU only): {l: boolean B x d_l array} -- the derivative decisions [z > 0] of hidden
    layer l to use in place of this evaluation's own.  A unit whose pre-activation lies within
    rounding of 0 is on or off depending on the precision and order of the sums behind it; both
    are valid evaluations of the same network, and a caller that compares with another evaluation
    passes that one's decisions for exactly those units."""
    params = np.asarray(params, dtype=np.float64)
    layers = _views(dims, params)
    L = len(layers)
    zscale = [] if with_error_scale else None
    acts = forward(dims, act, params, X, store_bf16, pre_activation_scales=zscale)
    mean_loss, delta = loss_and_delta(loss, acts[-1], y, store_bf16)
    grad = np.empty_like(params)
    gl = _views(dims, grad)
    scale = np.empty_like(params) if with_error_scale else None
    sl = _views(dims, scale) if with_error_scale else None
    dabs = np.abs(delta)
    for l in range(L, 0, -1):
        W = layers[l - 1][0]
        Ain = acts[l - 1]
        sparse_in = l == 1 and not isinstance(Ain, np.ndarray)
        gl[l - 1][0][...] = np.asarray((Ain.T @ delta).T) if sparse_in else delta.T @ Ain
        gl[l - 1][1][...] = delta.sum(axis=0)
        fp = None
        if l > 1:
            fp = _act_deriv_from_output(act, Ain)
            if relu_on is not None and (l - 1) in relu_on:
                assert act == ACT_RELU and relu_on[l - 1].shape == fp.shape
                fp = relu_on[l - 1].astype(np.float64)
        if with_error_scale:
            # |delta_l|^T (|A_{l-1}| + f' * (sum of |terms| of Z_{l-1})): the terms of the entry itself,
            # and what the rounding of the sums behind the activation A_{l-1} = f(Z_{l-1}) can move
            Aabs = abs(Ain) if l == 1 else np.abs(Ain) + np.abs(fp) * zscale[l - 2]
            sl[l - 1][0][...] = np.asarray((Aabs.T @ dabs).T) if sparse_in else dabs.T @ Aabs
            sl[l - 1][1][...] = dabs.sum(axis=0)
        if l > 1:
            delta = _stored((delta @ W) * fp, store_bf16)
            if with_error_scale:
                dabs = (dabs @ np.abs(W)) * np.abs(fp)
    if with_error_scale:
        return mean_loss, grad, scale
    return mean_loss, grad


def grad_error_scale(dims, act, loss, params, X, y):
    """For every gradient entry, the magnitude its rounding error is proportional to when the
    entry is evaluated in floating point: the recurrences of batch_grad with every factor replaced
    by its absolute value -- |delta_L|, |W_l|, |f'| going down, and for the entry
    dW_l[j,k] = sum_i delta_l[i,j] A_{l-1}[i,k] the factor |A_{l-1}[i,k]| plus, for l > 1,
    |f'(Z_{l-1}[i,k])| (sum_m |A_{l-2}[i,m]| |W_{l-1}[k,m]| + |b_{l-1}[k]|): an activation is itself
    a rounded sum, and a unit just above the ReLU kink is small next to the terms it was added up
    from.  Without that second part this is the sum of the absolute values of the entry's terms."""
    return batch_grad(dims, act, loss, params, X, y, with_error_scale=True)[2]


def sgd_update(params, grad, lr):
    """Eq. (3)."""
    return np.asarray(params, dtype=np.float64) - lr * np.asarray(grad, dtype=np.float64)


def round_weights_bf16(dims, params):
    """Copy of the flat parameters with every weight matrix rounded to bf16 (biases kept)."""
    out = np.array(params, dtype=np.float64, copy=True)
    for W, _ in _views(dims, out):
        W[...] = bf16_round(W.astype(np.float32))
    return out
