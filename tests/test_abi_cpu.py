"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching a device."""
import os
import re

import numpy as np
import pytest

import paper_2004_08771_amd as hb
from paper_2004_08771_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "hb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hb_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    names = _declared_symbols()
    assert "hb_mlp_create" in names and "hb_batch_step" in names and "hb_model_merge" in names
    assert "hb_batch_grad" in names and len(names) >= 18
    l = hb.lib()
    for n in names:
        assert hasattr(l, n), f"{n} is declared in include/hb.h but not exported"
    # and the binding marshals every one of them
    assert sorted(binding.SIGNATURES) == names


def test_create_validates_on_the_host():
    for dims, act, loss in [((54,), 0, 0), ((), 0, 0), ((54, 0, 7), 0, 0), ((54, -3, 7), 0, 0),
                            ((54, 32, 7), 2, 0), ((54, 32, 7), 0, 5), ((54, 32, 3), 0, 1),
                            (tuple([8] * 40), 0, 0)]:
        with pytest.raises(hb.HbError):
            hb.Model(dims, act, loss)
    m = hb.Model((54, 32, 7))
    assert m.num_params == 54 * 32 + 32 + 32 * 7 + 7
    m.destroy()
    assert hb.lib().hb_model_num_params(None) == -1
    hb.lib().hb_model_destroy(None)  # allowed


def test_calls_before_configure_fail_with_state_error():
    m = hb.Model((8, 4, 2), hb.HB_ACT_RELU, hb.HB_LOSS_LOGISTIC)
    buf = np.zeros(m.num_params, np.float32)
    for call in (lambda: m.set_params(buf), lambda: m.get_params(buf), lambda: m.model_merge(buf, 0.5),
                 lambda: m.batch_step(1, 1, 4, 0.1), lambda: m.batch_grad(1, 1, 4, 1),
                 lambda: m.batch_loss(1, 1, 4), lambda: m.batch_step_async(1, 1, 4, 0.1),
                 lambda: m.batch_step_csr(1, 1, 1, 4, 1, 4, 0.1), lambda: m.profile_enable(True),
                 lambda: m.batch_loss_async(1, 1, 4), lambda: m.batch_loss_csr(1, 1, 1, 4, 1, 4),
                 lambda: m.batch_loss_csr_async(1, 1, 1, 4, 1, 4),
                 lambda: m.worker_eval_loss(buf, buf, 4, 4), lambda: m.worker_eval_loss_csr(buf, buf, buf, buf, 4, 4)):
        with pytest.raises(hb.HbError) as e:
            call()
        assert e.value.code == hb.HB_ERR_STATE
    # the worker loops check the handle before anything else, too
    s = hb.Sched(64, [4], [16], [16])
    for call in (lambda: m.worker_run_epoch(s, 0, buf, buf, 0.01),
                 lambda: m.worker_run_epoch_csr(s, 0, buf, buf, buf, buf, 0.01)):
        with pytest.raises(hb.HbError) as e:
            call()
        assert e.value.code == hb.HB_ERR_STATE
    assert s.remaining() == 64          # nothing was requested from the scheduler
    m.destroy()


def test_configure_validates_before_any_device_call():
    m = hb.Model((8, 4, 2))
    for dtype, max_B, sparse in [(7, 16, 0), (hb.HB_F32, 0, 0), (hb.HB_F32, -5, 0),
                                 (hb.HB_F32, 1 << 40, 0), (hb.HB_BF16_F32MASTER, 16, 1)]:
        with pytest.raises(hb.HbError) as e:
            m.configure(dtype, max_B, sparse)
        assert e.value.code == hb.HB_ERR_INVALID
    m.destroy()
    with pytest.raises(hb.HbError) as e:
        hb.lib().hb_mlp_configure.restype  # keep the symbol referenced
        binding._check(hb.lib().hb_mlp_configure(None, 0, 16, 0, None))
    assert e.value.code == hb.HB_ERR_INVALID


def test_bf16_weight_gradient_slice_buffer_covers_every_batch_size():
    """The slice buffer of the bf16 weight gradient is sized at configure time for max_B; the
    number of slices a smaller batch asks for must never exceed that (it is not monotonic in B:
    an operand beyond 4 GiB is not split at all, so a wide layer can ask for 1 slice at max_B and
    for several at a smaller B)."""
    plan = hb.lib().hb_plan_bf16_dw_slices
    grid_B = [1, 100, 1024, 2047, 2048, 3000, 4096, 8192, 16384, 1 << 16, 1 << 18, 1 << 20, 1 << 21, 1 << 22]
    shapes = [(128, 128), (2048, 2048), (4096, 4096), (4096, 2048), (1000, 4096), (512, 54), (300, 300), (8192, 256)]
    for d_out, d_in in shapes:
        for max_B in grid_B:
            cap = plan(d_out, d_in, max_B, 1)
            assert cap >= 1
            for B in [b for b in grid_B if b <= max_B] + [max_B - 1 if max_B > 1 else 1]:
                got = plan(d_out, d_in, B, 0)
                assert 1 <= got <= cap, (d_out, d_in, max_B, B, got, cap)
    # the case that overflowed a buffer sized from the count at max_B: 2048 x 2048 at max_B = 2^21
    assert plan(2048, 2048, 1 << 21, 0) == 1 and plan(2048, 2048, 8192, 0) == 4 and plan(2048, 2048, 1 << 21, 1) >= 4
    assert plan(0, 5, 5, 0) == 0 and plan(5, 5, 0, 1) == 0


def test_traffic_summaries_have_the_form_the_benchmark_reads():
    """bench.py takes `roofline.traffic` from profiles/hbm_traffic_config<c>_B<B>.json:
    {"bytes_per_launch": {<kernel name as bench.py prints it>: bytes}}.  A summary in another
    form would silently turn the field into null."""
    import glob
    import json
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    files = sorted(glob.glob(os.path.join(root, "profiles", "hbm_traffic_config*_B*.json")))
    assert files, "no traffic summaries under profiles/"
    dominant = {"2": "bwd_pair", "4": "bwd_pair", "5": "fwd_gemm"}
    for f in files:
        with open(f) as fh:
            d = json.load(fh)
        per = d.get("bytes_per_launch")
        assert isinstance(per, dict) and per, f"{f}: no bytes_per_launch table"
        assert all(isinstance(v, (int, float)) and v > 0 for v in per.values()), f
        cfg = os.path.basename(f)[len("hbm_traffic_config")]
        if cfg in dominant:
            assert dominant[cfg] in per, f"{f}: no entry for the dominant kernel {dominant[cfg]}"
        assert os.path.exists(f[:-5] + ".md"), f"{f}: the summary it was taken from is missing"
