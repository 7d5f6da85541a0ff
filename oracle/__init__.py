"""ctypes front end of the fp64 CPU oracle (`hb_oracle.c`).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It imports nothing from the HIP package and shares no code with it.

All arithmetic is in `hb_oracle.c` (fp64, plain loops, following Section 3, Eq. (1)-(3),
Section 6.2 and Section 7.1 of the paper); this file only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hb_oracle.c")
_LIB = os.path.join(_HERE, "libhb_oracle.so")

ACT_SIGMOID = 0
ACT_RELU = 1
LOSS_SOFTMAX_CE = 0
LOSS_LOGISTIC = 1

_lib = None


def build(force: bool = False) -> str:
    """Compile hb_oracle.c with gcc (OpenMP over independent rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    i32p = ctypes.POINTER(ctypes.c_int32)
    f64p = ctypes.POINTER(ctypes.c_double)
    f32p = ctypes.POINTER(ctypes.c_float)
    i64, i32, f64 = ctypes.c_int64, ctypes.c_int32, ctypes.c_double
    lib.hbo_num_params.restype = i64
    lib.hbo_num_params.argtypes = [i32p, i32]
    lib.hbo_max_threads.restype = ctypes.c_int
    lib.hbo_set_threads.argtypes = [ctypes.c_int]
    lib.hbo_batch_loss.restype = f64
    lib.hbo_batch_loss.argtypes = [i32p, i32, ctypes.c_int, ctypes.c_int, f64p, f64p, i32p, i64]
    lib.hbo_batch_grad.restype = f64
    lib.hbo_batch_grad.argtypes = [i32p, i32, ctypes.c_int, ctypes.c_int, f64p, f64p, i32p, i64, f64p]
    lib.hbo_batch_grad_bf16_storage.restype = f64
    lib.hbo_batch_grad_bf16_storage.argtypes = [i32p, i32, ctypes.c_int, ctypes.c_int, f64p, f64p, i32p, i64, f64p]
    lib.hbo_batch_grad_csr.restype = f64
    lib.hbo_batch_grad_csr.argtypes = [i32p, i32, ctypes.c_int, ctypes.c_int, f64p, i32p, i32p,
                                       f64p, i32p, i64, f64p]
    lib.hbo_batch_step.restype = f64
    lib.hbo_batch_step.argtypes = [i32p, i32, ctypes.c_int, ctypes.c_int, f64p, f64p, i32p, i64, f64]
    lib.hbo_batch_step_csr.restype = f64
    lib.hbo_batch_step_csr.argtypes = [i32p, i32, ctypes.c_int, ctypes.c_int, f64p, i32p, i32p,
                                       f64p, i32p, i64, f64]
    lib.hbo_sgd_update.restype = None
    lib.hbo_sgd_update.argtypes = [f64p, f64p, i64, f64]
    lib.hbo_model_merge.restype = None
    lib.hbo_model_merge.argtypes = [f64p, f64p, i64, f64]
    lib.hbo_bf16_round.restype = None
    lib.hbo_bf16_round.argtypes = [f32p, f32p, i64]
    _lib = lib
    return lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _dims(dims):
    d = _i32(list(dims))
    return d, _p(d, ctypes.c_int32), int(d.size)


def max_threads() -> int:
    return int(_load().hbo_max_threads())


def set_threads(n: int) -> None:
    _load().hbo_set_threads(int(n))


def num_params(dims) -> int:
    d, dp, n = _dims(dims)
    return int(_load().hbo_num_params(dp, n))


def batch_loss(dims, act, loss, params, X, y) -> float:
    """Mean batch loss at `params` (forward pass only)."""
    d, dp, n = _dims(dims)
    params, X, y = _f64(params), _f64(X), _i32(y)
    assert params.size == num_params(dims) and X.shape == (y.size, dims[0])
    return float(_load().hbo_batch_loss(dp, n, act, loss, _p(params, ctypes.c_double),
                                        _p(X, ctypes.c_double), _p(y, ctypes.c_int32), y.size))


def batch_grad(dims, act, loss, params, X, y):
    """(mean loss, flat fp64 gradient of the mean loss)."""
    d, dp, n = _dims(dims)
    params, X, y = _f64(params), _f64(X), _i32(y)
    assert params.size == num_params(dims) and X.shape == (y.size, dims[0])
    g = np.empty_like(params)
    l = _load().hbo_batch_grad(dp, n, act, loss, _p(params, ctypes.c_double),
                               _p(X, ctypes.c_double), _p(y, ctypes.c_int32), y.size,
                               _p(g, ctypes.c_double))
    return float(l), g


def round_weights_bf16(dims, params):
    """Copy of the flat parameters with every weight matrix rounded to bf16 (biases kept)."""
    out = np.array(params, dtype=np.float64, copy=True)
    off = 0
    for l in range(1, len(dims)):
        n = dims[l] * dims[l - 1]
        out[off:off + n] = bf16_round(np.asarray(params[off:off + n], dtype=np.float32))
        off += n + dims[l]
    return out


def batch_grad_bf16_storage(dims, act, loss, params, X, y):
    """(mean loss, gradient) under the bf16-storage policy: weights and X are rounded to bf16
    here, hidden activations and deltas inside the oracle; sums stay fp64."""
    d, dp, n = _dims(dims)
    pr = round_weights_bf16(dims, params)
    Xr = _f64(bf16_round(np.asarray(X, dtype=np.float32)))
    y = _i32(y)
    assert pr.size == num_params(dims) and Xr.shape == (y.size, dims[0])
    g = np.empty_like(pr)
    l = _load().hbo_batch_grad_bf16_storage(dp, n, act, loss, _p(pr, ctypes.c_double),
                                            _p(Xr, ctypes.c_double), _p(y, ctypes.c_int32), y.size,
                                            _p(g, ctypes.c_double))
    return float(l), g


def batch_grad_csr(dims, act, loss, params, row_ptr, col_idx, vals, y):
    d, dp, n = _dims(dims)
    params, vals = _f64(params), _f64(vals)
    row_ptr, col_idx, y = _i32(row_ptr), _i32(col_idx), _i32(y)
    assert params.size == num_params(dims) and row_ptr.size == y.size + 1
    assert col_idx.size == vals.size == int(row_ptr[-1]) and row_ptr[0] == 0
    assert col_idx.size == 0 or (col_idx.min() >= 0 and col_idx.max() < dims[0])
    g = np.empty_like(params)
    l = _load().hbo_batch_grad_csr(dp, n, act, loss, _p(params, ctypes.c_double),
                                   _p(row_ptr, ctypes.c_int32), _p(col_idx, ctypes.c_int32),
                                   _p(vals, ctypes.c_double), _p(y, ctypes.c_int32), y.size,
                                   _p(g, ctypes.c_double))
    return float(l), g


def batch_step(dims, act, loss, params, X, y, lr):
    """One SGD step.  Returns (pre-update mean loss, updated flat fp64 parameters)."""
    d, dp, n = _dims(dims)
    new = _f64(params).copy()
    X, y = _f64(X), _i32(y)
    assert new.size == num_params(dims) and X.shape == (y.size, dims[0])
    l = _load().hbo_batch_step(dp, n, act, loss, _p(new, ctypes.c_double),
                               _p(X, ctypes.c_double), _p(y, ctypes.c_int32), y.size, float(lr))
    return float(l), new


def batch_step_csr(dims, act, loss, params, row_ptr, col_idx, vals, y, lr):
    d, dp, n = _dims(dims)
    new = _f64(params).copy()
    vals = _f64(vals)
    row_ptr, col_idx, y = _i32(row_ptr), _i32(col_idx), _i32(y)
    assert new.size == num_params(dims) and row_ptr.size == y.size + 1
    assert col_idx.size == vals.size == int(row_ptr[-1]) and row_ptr[0] == 0
    assert col_idx.size == 0 or (col_idx.min() >= 0 and col_idx.max() < dims[0])
    l = _load().hbo_batch_step_csr(dp, n, act, loss, _p(new, ctypes.c_double),
                                   _p(row_ptr, ctypes.c_int32), _p(col_idx, ctypes.c_int32),
                                   _p(vals, ctypes.c_double), _p(y, ctypes.c_int32), y.size,
                                   float(lr))
    return float(l), new


def sgd_update(params, grad, lr):
    new = _f64(params).copy()
    grad = _f64(grad)
    assert new.size == grad.size
    _load().hbo_sgd_update(_p(new, ctypes.c_double), _p(grad, ctypes.c_double), new.size, float(lr))
    return new


def model_merge(device_replica, host_model, weight):
    """M = (1-w) H + w D.  Returns (new D, new H), both equal to M."""
    D, H = _f64(device_replica).copy(), _f64(host_model).copy()
    assert D.size == H.size
    _load().hbo_model_merge(_p(D, ctypes.c_double), _p(H, ctypes.c_double), D.size, float(weight))
    return D, H


def bf16_round(a):
    """float32 array -> nearest bfloat16 values (ties to even), returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty_like(a)
    _load().hbo_bf16_round(_p(a, ctypes.c_float), _p(out, ctypes.c_float), a.size)
    return out
