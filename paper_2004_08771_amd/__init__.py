"""MI355X-native GPU-worker mini-batch step of CPU+GPU / Adaptive Hogbatch SGD.

Thin ctypes binding over libhb.so (hand-written HIP for gfx950); see include/hb.h for the
C ABI.  Every step of the path runs in the library's kernels -- this package only
marshals pointers.  There is no CPU fallback: if the library is missing, importing the
binding's entry points raises.
"""
from .binding import (  # noqa: F401
    HB_ACT_RELU, HB_ACT_SIGMOID, HB_BF16_F32MASTER, HB_ERR_ALLOC, HB_ERR_DEVICE,
    HB_ERR_INVALID, HB_ERR_STATE, HB_ERR_UNSUPPORTED, HB_F32, HB_LOSS_LOGISTIC,
    HB_LOSS_SOFTMAX_CE, HB_OK, HbError, Model, Sched, batch_loss_static, cpu_worker_run_epoch, hogbatch_run_epoch, lib, lib_path,
)
