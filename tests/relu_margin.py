"""Input conditioning for ReLU parity cases (test helper, not an oracle).

The ReLU derivative [z > 0] is a discrete decision.  The HIP path takes it on the fp32
pre-activation, the oracle on the fp64 one; the two can only disagree for a unit whose
pre-activation lies within the fp32 accumulation error of zero, and one such unit moves a
whole gradient row by the size of its delta.  Parity inputs are therefore nudged (bias
entries only, by ~1e-3, kept exactly fp32-representable) until no hidden pre-activation lies
within `tau` of the kink, so that the decision is the same in either precision.
"""
import numpy as np

import hb_inputs as hi


def _first_layer(X, W, csr):
    if csr is None:
        return X.astype(np.float64) @ W.T
    import scipy.sparse as sp
    row_ptr, col_idx, vals = csr
    Xs = sp.csr_matrix((vals.astype(np.float64), col_idx.copy(), row_ptr.copy()), shape=(row_ptr.size - 1, W.shape[1]))
    return np.asarray(Xs @ W.T)


def keep_relu_units_off_the_kink(dims, params, X=None, csr=None, tau=2e-6, seed=0, bf16_storage=False):
    """Returns a copy of the flat fp32 `params` whose hidden pre-activations on this batch
    all satisfy |z| >= tau.  X is the dense batch, or csr = (row_ptr, col_idx, vals).
    With bf16_storage the pre-activations are those of the mixed-precision policy (weights,
    X and hidden activations rounded to bf16), the ones the bf16 kernels decide on."""
    import oracle
    rnd = (lambda a: oracle.bf16_round(np.asarray(a, dtype=np.float32)).astype(np.float64)) \
        if bf16_storage else (lambda a: np.asarray(a, dtype=np.float64))
    rng = np.random.default_rng(seed)
    params = np.array(params, dtype=np.float32, copy=True)
    if X is not None:
        X = rnd(X)
    offs = hi.param_offsets(dims)
    L = len(dims) - 1
    a = None
    for l in range(1, L):
        wo, bo = offs[l - 1]
        W = rnd(params[wo:wo + dims[l] * dims[l - 1]].reshape(dims[l], dims[l - 1]))
        lin = _first_layer(X, W, csr) if l == 1 else a @ W.T
        for _ in range(100):
            z = lin + params[bo:bo + dims[l]].astype(np.float64)
            cols = np.unique(np.nonzero(np.abs(z) < tau)[1])
            if cols.size == 0:
                break
            shift = rng.uniform(1e-3, 2e-3, cols.size) * rng.choice([-1.0, 1.0], cols.size)
            params[bo + cols] = (params[bo + cols] + shift).astype(np.float32)
        else:
            raise RuntimeError("could not move every ReLU unit off the kink")
        a = rnd(np.maximum(z, 0.0))
    return params
