"""ctypes binding of libhb.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhb.so")

HB_ACT_SIGMOID, HB_ACT_RELU = 0, 1
HB_LOSS_SOFTMAX_CE, HB_LOSS_LOGISTIC = 0, 1
HB_F32, HB_BF16_F32MASTER = 0, 1
HB_OK, HB_ERR_INVALID, HB_ERR_ALLOC, HB_ERR_DEVICE, HB_ERR_UNSUPPORTED, HB_ERR_STATE = 0, -1, -2, -3, -4, -5

# name -> (restype, argtypes); every symbol include/hb.h declares
_vp, _i32, _i64, _f32, _int = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_int
_i32p = ctypes.POINTER(ctypes.c_int32)
SIGNATURES = {
    "hb_mlp_create": (_vp, [_i32p, _i32, _int, _int]),
    "hb_mlp_configure": (_int, [_vp, _int, _i64, _int, _vp]),
    "hb_model_destroy": (None, [_vp]),
    "hb_model_num_params": (_i64, [_vp]),
    "hb_model_set_params": (_int, [_vp, _vp]),
    "hb_model_get_params": (_int, [_vp, _vp]),
    "hb_model_get_activations": (_int, [_vp, _i32, _i64, _vp]),
    "hb_batch_step": (_f32, [_vp, _vp, _vp, _i64, _f32]),
    "hb_batch_step_async": (_int, [_vp, _vp, _vp, _i64, _f32, _vp]),
    "hb_batch_step_csr": (_f32, [_vp, _vp, _vp, _vp, _i64, _vp, _i64, _f32]),
    "hb_batch_step_csr_async": (_int, [_vp, _vp, _vp, _vp, _i64, _vp, _i64, _f32, _vp]),
    "hb_batch_grad": (_f32, [_vp, _vp, _vp, _i64, _vp]),
    "hb_batch_grad_csr": (_f32, [_vp, _vp, _vp, _vp, _i64, _vp, _i64, _vp]),
    "hb_batch_loss": (_f32, [_vp, _vp, _vp, _i64]),
    "hb_batch_loss_async": (_int, [_vp, _vp, _vp, _i64, _vp]),
    "hb_batch_loss_static": (_int, [_i32p, _i32, _int, _int, _vp, _vp, _vp, _i64, _vp, _vp]),
    "hb_batch_loss_csr": (_f32, [_vp, _vp, _vp, _vp, _i64, _vp, _i64]),
    "hb_batch_loss_csr_async": (_int, [_vp, _vp, _vp, _vp, _i64, _vp, _i64, _vp]),
    "hb_model_merge": (_int, [_vp, _vp, _f32]),
    "hb_last_error": (ctypes.c_char_p, []),
    "hb_version": (ctypes.c_char_p, []),
    "hb_plan_bf16_dw_slices": (_i32, [_i32, _i32, _i64, _i32]),
}

HB_K_NAMES = {0: "fwd_gemm", 1: "da_gemm", 2: "dw_gemm", 3: "loss", 4: "update", 5: "spmm_fwd",
              6: "sparse_dw", 7: "other", 8: "out_layer", 9: "bwd_pair"}


class KernelStat(ctypes.Structure):
    """Mirror of hb_kernel_stat."""
    _fields_ = [("kind", ctypes.c_int32), ("layer", ctypes.c_int32), ("M", ctypes.c_int64),
                ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("launches", ctypes.c_int64),
                ("total_ms", ctypes.c_double), ("flops_per_launch", ctypes.c_double),
                ("bytes_per_launch", ctypes.c_double), ("cache_bytes_per_launch", ctypes.c_double)]


SIGNATURES["hb_last_error_code"] = (_int, [])
SIGNATURES["hb_profile_enable"] = (_int, [_vp, _int])
SIGNATURES["hb_profile_read"] = (_int, [_vp, ctypes.POINTER(KernelStat), _i32, _i32p])

_i64p, _f64, _f64p = ctypes.POINTER(ctypes.c_int64), ctypes.c_double, ctypes.POINTER(ctypes.c_double)
SIGNATURES["hb_sched_create"] = (_vp, [_i64, _i32, _i64p, _i64p, _i64p, _f64])
SIGNATURES["hb_sched_destroy"] = (None, [_vp])
SIGNATURES["hb_sched_request"] = (_int, [_vp, _i32, _f64, _i64p, _i64p])
SIGNATURES["hb_sched_new_epoch"] = (_int, [_vp])
SIGNATURES["hb_sched_batch_size"] = (_i64, [_vp, _i32])
SIGNATURES["hb_sched_remaining"] = (_i64, [_vp])
SIGNATURES["hb_worker_run_epoch"] = (_int, [_vp, _vp, _i32, _vp, _vp, _f32, _vp, _i32, _f32, _f64p, _i64p, _f64p])
SIGNATURES["hb_worker_run_epoch_csr"] = (_int, [_vp, _vp, _i32, _vp, _vp, _vp, _vp, _f32, _vp, _i32, _f32, _f64p, _i64p,
                                                _f64p])
SIGNATURES["hb_worker_eval_loss"] = (_int, [_vp, _vp, _vp, _i64, _i64, _f64p])
SIGNATURES["hb_worker_eval_loss_csr"] = (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _f64p])
SIGNATURES["hb_cpu_worker_run_epoch"] = (_int, [_vp, _i32, _i32p, _i32, _int, _int, _vp, _vp, _vp, _f32, _i32, _f64,
                                                _f64p, _i64p, _f64p])

SIGNATURES["hb_hogbatch_run_epoch"] = (_int, [_vp, _vp, _i32, _i32, _vp, _vp, _vp, _f32, _i32, _f64, _i32, _f32, _f64p,
                                              _f64p, _vp])

_lib = None


class HbError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"hb error {code}: {message}")
        self.code = code


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; "
                              "g.build()'` (or paper_2004_08771_amd/build.py) first")
        l = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def last_error() -> str:
    return lib().hb_last_error().decode()


def _check(rc: int) -> None:
    if rc != HB_OK:
        raise HbError(rc, last_error())


def _check_float(v: float) -> float:
    if v != v:
        raise HbError(int(lib().hb_last_error_code()), last_error())
    return v


def _ptr(t):
    """Device/host address of a torch tensor, numpy array, int or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


class Model:
    """Owner of one hb_model handle.  Methods mirror the C entry points one to one."""

    def __init__(self, layer_dims, activation=HB_ACT_SIGMOID, loss=HB_LOSS_SOFTMAX_CE):
        dims = (ctypes.c_int32 * len(layer_dims))(*[int(d) for d in layer_dims])
        self._h = lib().hb_mlp_create(dims, len(layer_dims), int(activation), int(loss))
        if not self._h:
            raise HbError(HB_ERR_INVALID, last_error())
        self.layer_dims = tuple(int(d) for d in layer_dims)

    def configure(self, dtype=HB_F32, max_B=4096, sparse_first_layer=False, stream=None):
        """stream: a hipStream_t as int (e.g. torch.cuda.current_stream().cuda_stream) or None."""
        _check(lib().hb_mlp_configure(self._h, int(dtype), int(max_B), int(bool(sparse_first_layer)),
                                      stream if stream else None))
        return self

    def destroy(self):
        if getattr(self, "_h", None):
            lib().hb_model_destroy(self._h)
            self._h = None

    __del__ = destroy

    @property
    def num_params(self) -> int:
        return int(lib().hb_model_num_params(self._h))

    def set_params(self, host_flat):
        _check(lib().hb_model_set_params(self._h, _ptr(host_flat)))

    def get_params(self, host_flat):
        _check(lib().hb_model_get_params(self._h, _ptr(host_flat)))

    def get_activations(self, layer, B, host_out):
        _check(lib().hb_model_get_activations(self._h, int(layer), int(B), _ptr(host_out)))

    def batch_step(self, dX, dy, B, lr) -> float:
        v = lib().hb_batch_step(self._h, _ptr(dX), _ptr(dy), int(B), float(lr))
        return _check_float(v)

    def batch_step_async(self, dX, dy, B, lr, d_loss=None):
        _check(lib().hb_batch_step_async(self._h, _ptr(dX), _ptr(dy), int(B), float(lr), _ptr(d_loss)))

    def batch_step_csr(self, d_row_ptr, d_col_idx, d_vals, nnz, dy, B, lr) -> float:
        v = lib().hb_batch_step_csr(self._h, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_vals), int(nnz),
                                    _ptr(dy), int(B), float(lr))
        return _check_float(v)

    def batch_step_csr_async(self, d_row_ptr, d_col_idx, d_vals, nnz, dy, B, lr, d_loss=None):
        _check(lib().hb_batch_step_csr_async(self._h, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_vals),
                                             int(nnz), _ptr(dy), int(B), float(lr), _ptr(d_loss)))

    def batch_grad(self, dX, dy, B, d_grad_flat) -> float:
        v = lib().hb_batch_grad(self._h, _ptr(dX), _ptr(dy), int(B), _ptr(d_grad_flat))
        return _check_float(v)

    def batch_grad_csr(self, d_row_ptr, d_col_idx, d_vals, nnz, dy, B, d_grad_flat) -> float:
        v = lib().hb_batch_grad_csr(self._h, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_vals), int(nnz),
                                    _ptr(dy), int(B), _ptr(d_grad_flat))
        return _check_float(v)

    def batch_loss(self, dX, dy, B) -> float:
        v = lib().hb_batch_loss(self._h, _ptr(dX), _ptr(dy), int(B))
        return _check_float(v)

    def batch_loss_async(self, dX, dy, B, d_loss=None):
        _check(lib().hb_batch_loss_async(self._h, _ptr(dX), _ptr(dy), int(B), _ptr(d_loss)))

    def batch_loss_csr(self, d_row_ptr, d_col_idx, d_vals, nnz, dy, B) -> float:
        v = lib().hb_batch_loss_csr(self._h, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_vals), int(nnz), _ptr(dy),
                                    int(B))
        return _check_float(v)

    def batch_loss_csr_async(self, d_row_ptr, d_col_idx, d_vals, nnz, dy, B, d_loss=None):
        _check(lib().hb_batch_loss_csr_async(self._h, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_vals), int(nnz),
                                             _ptr(dy), int(B), _ptr(d_loss)))

    def model_merge(self, host_model, weight):
        _check(lib().hb_model_merge(self._h, _ptr(host_model), float(weight)))

    def profile_enable(self, on=True):
        _check(lib().hb_profile_enable(self._h, int(bool(on))))

    def profile_read(self, cap=256):
        """List of dicts, one per (kind, layer, shape) launched since the last read."""
        buf = (KernelStat * cap)()
        n = ctypes.c_int32(0)
        _check(lib().hb_profile_read(self._h, buf, cap, ctypes.byref(n)))
        return [{f: getattr(buf[i], f) for f, _ in KernelStat._fields_} for i in range(n.value)]

    def worker_run_epoch(self, sched, worker, host_X, host_y, lr_per_example, host_model=None, merge_every=0,
                         merge_weight=1.0, updates=0.0):
        """hb_worker_run_epoch.  Returns (updates, steps, loss_sum)."""
        u = ctypes.c_double(float(updates))
        steps = ctypes.c_int64(0)
        loss_sum = ctypes.c_double(0.0)
        _check(lib().hb_worker_run_epoch(self._h, sched._h, int(worker), _ptr(host_X), _ptr(host_y),
                                         float(lr_per_example), _ptr(host_model), int(merge_every),
                                         float(merge_weight), ctypes.byref(u), ctypes.byref(steps),
                                         ctypes.byref(loss_sum)))
        return u.value, steps.value, loss_sum.value

    def worker_run_epoch_csr(self, sched, worker, host_row_ptr, host_col_idx, host_vals, host_y, lr_per_example,
                             host_model=None, merge_every=0, merge_weight=1.0, updates=0.0):
        """hb_worker_run_epoch_csr (host_row_ptr: int64).  Returns (updates, steps, loss_sum)."""
        u = ctypes.c_double(float(updates))
        steps = ctypes.c_int64(0)
        loss_sum = ctypes.c_double(0.0)
        _check(lib().hb_worker_run_epoch_csr(self._h, sched._h, int(worker), _ptr(host_row_ptr), _ptr(host_col_idx),
                                             _ptr(host_vals), _ptr(host_y), float(lr_per_example), _ptr(host_model),
                                             int(merge_every), float(merge_weight), ctypes.byref(u),
                                             ctypes.byref(steps), ctypes.byref(loss_sum)))
        return u.value, steps.value, loss_sum.value

    def worker_eval_loss(self, host_X, host_y, n_examples, batch) -> float:
        out = ctypes.c_double(0.0)
        _check(lib().hb_worker_eval_loss(self._h, _ptr(host_X), _ptr(host_y), int(n_examples), int(batch),
                                         ctypes.byref(out)))
        return out.value

    def worker_eval_loss_csr(self, host_row_ptr, host_col_idx, host_vals, host_y, n_examples, batch) -> float:
        out = ctypes.c_double(0.0)
        _check(lib().hb_worker_eval_loss_csr(self._h, _ptr(host_row_ptr), _ptr(host_col_idx), _ptr(host_vals),
                                             _ptr(host_y), int(n_examples), int(batch), ctypes.byref(out)))
        return out.value


def batch_loss_static(layer_dims, activation, loss, d_params, dX, dy, B, d_loss, stream=None):
    """hb_batch_loss_static: forward pass + mean loss without a handle and without any allocation."""
    dims = (ctypes.c_int32 * len(layer_dims))(*[int(d) for d in layer_dims])
    _check(lib().hb_batch_loss_static(dims, len(layer_dims), int(activation), int(loss), _ptr(d_params), _ptr(dX),
                                      _ptr(dy), int(B), _ptr(d_loss), stream if stream else None))


class Sched:
    """Owner of one hb_sched handle (Algorithm 2, ScheduleWork).  Host-only: needs no GPU."""

    def __init__(self, n_examples, min_b, max_b, init_b, alpha=2.0):
        n = len(init_b)
        arr = lambda v: (ctypes.c_int64 * n)(*[int(x) for x in v])
        self._h = lib().hb_sched_create(int(n_examples), n, arr(min_b), arr(max_b), arr(init_b), float(alpha))
        if not self._h:
            raise HbError(int(lib().hb_last_error_code()), last_error())

    def destroy(self):
        if self._h:
            lib().hb_sched_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def request(self, worker, updates):
        """(begin, count); count == 0: nothing sent."""
        b, c = ctypes.c_int64(0), ctypes.c_int64(0)
        _check(lib().hb_sched_request(self._h, int(worker), float(updates), ctypes.byref(b), ctypes.byref(c)))
        return b.value, c.value

    def new_epoch(self):
        _check(lib().hb_sched_new_epoch(self._h))

    def batch_size(self, worker) -> int:
        return int(lib().hb_sched_batch_size(self._h, int(worker)))

    def remaining(self) -> int:
        return int(lib().hb_sched_remaining(self._h))


class EpochStats(ctypes.Structure):
    _fields_ = [("gpu_steps", ctypes.c_int64), ("cpu_batches", ctypes.c_int64),
                ("gpu_loss_sum", ctypes.c_double), ("cpu_loss_sum", ctypes.c_double)]


def hogbatch_run_epoch(sched, gpu_model, gpu_worker, cpu_worker, host_X, host_y, host_model, lr_per_example,
                       cpu_threads=1, beta=1.0, merge_every=1, merge_weight=0.5, gpu_updates=0.0, cpu_updates=0.0):
    """hb_hogbatch_run_epoch.  Returns (gpu_updates, cpu_updates, stats dict)."""
    gu, cu = ctypes.c_double(float(gpu_updates)), ctypes.c_double(float(cpu_updates))
    st = EpochStats()
    _check(lib().hb_hogbatch_run_epoch(sched._h, gpu_model._h, int(gpu_worker), int(cpu_worker), _ptr(host_X),
                                       _ptr(host_y), _ptr(host_model), float(lr_per_example), int(cpu_threads),
                                       float(beta), int(merge_every), float(merge_weight), ctypes.byref(gu),
                                       ctypes.byref(cu), ctypes.byref(st)))
    return gu.value, cu.value, {f: getattr(st, f) for f, _ in EpochStats._fields_}


def cpu_worker_run_epoch(sched, worker, layer_dims, activation, loss, host_X, host_y, host_model, lr_per_example,
                         threads=1, beta=1.0, updates=0.0):
    """hb_cpu_worker_run_epoch.  Returns (updates, batches, loss_sum).  Host-only."""
    dims = (ctypes.c_int32 * len(layer_dims))(*[int(d) for d in layer_dims])
    u = ctypes.c_double(float(updates))
    nb = ctypes.c_int64(0)
    ls = ctypes.c_double(0.0)
    _check(lib().hb_cpu_worker_run_epoch(sched._h, int(worker), dims, len(layer_dims), int(activation), int(loss),
                                         _ptr(host_X), _ptr(host_y), _ptr(host_model), float(lr_per_example),
                                         int(threads), float(beta), ctypes.byref(u), ctypes.byref(nb),
                                         ctypes.byref(ls)))
    return u.value, nb.value, ls.value
