#!/usr/bin/env python3
"""Benchmark of the GPU-worker mini-batch step (forward, backward, SGD update) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--batch 4096]

A "step" is one hb_batch_step_async call over one batch of synthetic rows that are already
resident in HBM; successive steps take successive contiguous row ranges of the dataset
(the way the coordinator hands out batches, Algorithm 1 / 2 of the paper).  After W warm-up
steps (and at least half a second of them) five regions of exactly K steps are timed between
synchronisations and the median is reported.  Prints ONE JSON line: throughput in training examples/s, the roofline figures of the dominant kernel
(per-dispatch execution times read from events attached to the kernel launches in a second,
profiled pass over the same steps), and the fp64 CPU oracle timed on a bounded sample of
the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}   # MI355X dense MFMA peaks
PEAK_HBM_GBS = 8000.0
WARM_SECONDS = 0.5     # untimed steps before the timed regions, at least
REPEATS = 5            # timed regions of --steps steps each; the median is reported


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=2, help="workload (hb_inputs.CONFIGS index)")
    ap.add_argument("--batch", type=int, default=4096, help="rows per step (the metric is quoted at 4096)")
    ap.add_argument("--rows", type=int, default=0,
                    help="dataset rows kept on the device (0: the config's size, at most 2 GiB of fp32 rows)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle leg")
    ap.add_argument("--no-from-host", action="store_true",
                    help="skip the worker-loop leg (same steps with the dataset in page-locked host memory)")
    ap.add_argument("--warm-seconds", type=float, default=WARM_SECONDS,
                    help="warm-up lasts at least this long (0 for runs under a counter-collecting profiler)")
    ap.add_argument("--repeats", type=int, default=REPEATS, help="timed regions of --steps steps (the median counts)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device-to-device copy (reference for HBM byte counters)")
    return ap.parse_args()


def make_device_dataset(hi, torch, config, rows):
    """Synthetic dataset of the config's shape on the device: (X, y) or CSR arrays."""
    cfg = hi.CONFIGS[config]
    if cfg.sparse:
        rp, ci, va, y = hi.make_csr_dataset(config, rows)
        return {"row_ptr": rp, "col_idx": ci, "vals": va, "y": y}
    X, y = hi.make_dense_dataset(config, rows)
    return {"X": X, "y": y}


def step_flops(dims, B, first_layer_nnz_per_row=None):
    """Algorithmic flop of one step: forward 2P_w, dW 2P_w, dA 2(P_w - d_1 d_0) per example."""
    pw = sum(dims[l] * dims[l - 1] for l in range(1, len(dims)))
    first = dims[1] * dims[0]
    if first_layer_nnz_per_row is not None:
        pw_eff = pw - first + dims[1] * first_layer_nnz_per_row
        return B * (4.0 * pw_eff + 2.0 * (pw - first))
    return B * (6.0 * pw - 2.0 * first)


def note(msg):
    """Progress on stderr (stdout carries the one JSON line): long silent phases look like hangs."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (each GPU worker owns one device and its own "
              f"replica; there are no inter-GPU collectives on this path); --gpus {args.gpus} is not "
              f"supported.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import hb_inputs as hi
    import paper_2004_08771_amd as hb

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    hb.lib()  # fails loudly if the HIP library was not built
    torch.cuda.set_device(0)

    cfg = hi.CONFIGS[args.config]
    B = args.batch
    rows = args.rows or cfg.n_examples
    if not args.rows and not cfg.sparse:
        # by default no more than 2 GiB of fp32 rows are generated (config 5: 262,144 of its 1,000,000);
        # the step time does not depend on how many batches the steps cycle through
        rows = min(rows, (2 << 30) // (4 * cfg.dims[0]))
    rows = max(rows, B)
    t_gen = time.perf_counter()
    data = make_device_dataset(hi, torch, args.config, rows)
    t_gen = time.perf_counter() - t_gen
    note(f"dataset of {rows} rows generated in {t_gen:.1f} s")
    dtype_name = "bf16" if cfg.dtype == hi.DTYPE_BF16_F32MASTER else "f32"

    model = hb.Model(cfg.dims, cfg.activation, cfg.loss)
    model.configure(hb.HB_BF16_F32MASTER if dtype_name == "bf16" else hb.HB_F32, B, cfg.sparse)
    model.set_params(hi.make_params(args.config))
    lr = 0.1 * B / 256 if args.config in (2, 6, 7) else cfg.lr  # Section 6.2: lr proportional to B

    n_batches = rows // B
    if cfg.sparse:
        rp = data["row_ptr"]
        d_ci = torch.from_numpy(data["col_idx"]).cuda()
        d_va = torch.from_numpy(data["vals"]).cuda()
        d_y = torch.from_numpy(data["y"]).cuda()
        # per-batch row_ptr rebased to 0 (a batch is a contiguous row range)
        batch_rp = [torch.from_numpy((rp[i * B:(i + 1) * B + 1] - rp[i * B]).astype(np.int32)).cuda()
                    for i in range(n_batches)]
        starts = [int(rp[i * B]) for i in range(n_batches)]
        nnzs = [int(rp[(i + 1) * B] - rp[i * B]) for i in range(n_batches)]
        mean_nnz = float(rp[n_batches * B]) / (n_batches * B)

        def one_step(i, d_loss=None):
            j = i % n_batches
            model.batch_step_csr_async(batch_rp[j], d_ci[starts[j]:], d_va[starts[j]:], nnzs[j],
                                       d_y[j * B:], B, lr, d_loss)
    else:
        X = data["X"]
        d_X = torch.from_numpy(X).cuda()
        if dtype_name == "bf16":
            d_X = d_X.to(torch.bfloat16)
        d_y = torch.from_numpy(data["y"]).cuda()
        mean_nnz = None

        row_bytes = d_X.element_size() * cfg.dims[0]
        x_ptr = [d_X.data_ptr() + j * B * row_bytes for j in range(n_batches)]
        y_ptr = [d_y.data_ptr() + j * B * 4 for j in range(n_batches)]

        def one_step(i, d_loss=None):
            j = i % n_batches
            model.batch_step_async(x_ptr[j], y_ptr[j], B, lr, d_loss)

    if args.calibrate_copy:
        # a copy kernel of known size: 256 MiB read + 256 MiB written, for scaling FETCH_SIZE / WRITE_SIZE
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    d_loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    # Warm-up: the W steps asked for, and then more until at least WARM_SECONDS of steps have run --
    # a chip that has been idle takes a few hundred steps to reach its working clocks, and a
    # timed region of a few milliseconds after a handful of steps measures that ramp, not the step.
    it = 0
    t_warm = time.perf_counter()
    while it < args.warmup or time.perf_counter() - t_warm < args.warm_seconds:
        for _ in range(max(1, min(args.warmup, 50))):
            one_step(it, d_loss)
            it += 1
        torch.cuda.synchronize()
    warm_steps = it
    # REPEATS timed regions of exactly K steps each, bracketed by synchronisations; the median counts
    region_ms = []
    for _ in range(max(1, args.repeats)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            one_step(it + i, d_loss)
        torch.cuda.synchronize()
        region_ms.append(1e3 * (time.perf_counter() - t0) / args.steps)
        it += args.steps
    ms_per_step = sorted(region_ms)[len(region_ms) // 2]
    elapsed = 1e-3 * ms_per_step * args.steps
    note(f"{warm_steps} warm-up steps, then {len(region_ms)} x {args.steps} timed steps: "
         + ", ".join(f"{v:.4f}" for v in region_ms) + f" ms per step; median {ms_per_step:.4f}")
    last_loss = float(d_loss.item())
    value = B / (1e-3 * ms_per_step)
    flops = step_flops(cfg.dims, B, mean_nnz)

    # ---- the synchronous entry point (hb_batch_step: the host waits for every step's loss),
    # reported beside the headline figure; dense configs only
    sync_ms_per_step = None
    if not cfg.sparse:
        n_sync = max(1, min(args.steps, 50))
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(n_sync):
            j = (it + i) % n_batches
            model.batch_step(x_ptr[j], y_ptr[j], B, lr)
        sync_ms_per_step = 1e3 * (time.perf_counter() - t1) / n_sync

    # ---- second pass over the same steps with per-dispatch events -> per-kernel times
    roofline, kernels = None, []
    if not args.no_profile:
        n_prof = min(max(args.steps, 100), 1000)   # enough launches for a stable average
        model.profile_enable(True)
        for i in range(n_prof):
            one_step(it + i, d_loss)
        stats = model.profile_read(512)
        model.profile_enable(False)
        for s in stats:
            avg_us = 1e3 * s["total_ms"] / max(s["launches"], 1)
            kernels.append({
                "kernel": hb.binding.HB_K_NAMES.get(s["kind"], "?"), "layer": s["layer"],
                "M": s["M"], "N": s["N"], "K": s["K"], "launches": s["launches"],
                "avg_us": round(avg_us, 3), "share": 0.0,
                "tflops": round(s["flops_per_launch"] / (avg_us * 1e-6) / 1e12, 3) if avg_us > 0 else None,
                "gbs": round(s["bytes_per_launch"] / (avg_us * 1e-6) / 1e9, 1) if avg_us > 0 else None,
                "_total_ms": s["total_ms"], "_flops": s["flops_per_launch"], "_bytes": s["bytes_per_launch"],
            })
            if s["cache_bytes_per_launch"] > 0 and avg_us > 0:     # CSR row gathers: cache-level rate
                kernels[-1]["gathered_gbs"] = round(s["cache_bytes_per_launch"] / (avg_us * 1e-6) / 1e9, 1)
        total = sum(k["_total_ms"] for k in kernels) or 1.0
        for k in kernels:
            k["share"] = round(k["_total_ms"] / total, 4)
        # dominant kernel: merge entries of equal (kernel, shape) -- the hidden layers run the
        # same kernel on the same shape -- and take the group with the largest total time
        groups = {}
        for k in kernels:
            g = groups.setdefault((k["kernel"], k["M"], k["N"], k["K"]),
                                  {"ms": 0.0, "n": 0, "flops": k["_flops"], "bytes": k["_bytes"]})
            g["ms"] += k["_total_ms"]
            g["n"] += k["launches"]
        (name, M, N, K), g = max(groups.items(), key=lambda kv: kv[1]["ms"])
        avg_s = 1e-3 * g["ms"] / g["n"]
        mfma_time = g["flops"] / (PEAK_TFLOPS[dtype_name] * 1e12)
        hbm_time = g["bytes"] / (PEAK_HBM_GBS * 1e9)
        if mfma_time >= hbm_time and g["flops"] > 0:
            ach = g["flops"] / avg_s / 1e12
            roofline = {"bound": "mfma", "achieved": round(ach, 3), "peak": PEAK_TFLOPS[dtype_name],
                        "unit": "TFLOP/s", "frac": round(ach / PEAK_TFLOPS[dtype_name], 4)}
        else:
            ach = g["bytes"] / avg_s / 1e9
            roofline = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": round(ach / PEAK_HBM_GBS, 4)}
        roofline.update({"traffic": None, "kernel": name, "shape": [M, N, K],
                         "avg_kernel_us": round(avg_s * 1e6, 3), "launches": g["n"],
                         "share_of_kernel_time": round(g["ms"] / total, 4),
                         "sum_kernel_us_per_step": round(1e3 * total / n_prof, 2)})
        # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this very
        # command (measured offline, scaled by a plain copy kernel; see profiles/)
        traffic_file = os.path.join(ROOT, "profiles", f"hbm_traffic_config{args.config}_B{B}.json")
        if os.path.exists(traffic_file):
            with open(traffic_file) as f:
                roofline["traffic"] = json.load(f).get("bytes_per_launch", {}).get(name)
                roofline["traffic_source"] = os.path.relpath(traffic_file, ROOT) + \
                    " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command; not measured in this run)"
        for k in kernels:
            for key in ("_total_ms", "_flops", "_bytes"):
                k.pop(key)
    # ---- the GPU worker's loop over the same dataset in page-locked HOST memory (per-batch
    # transfer on a copy stream beside the steps): the PCIe-inclusive rate, reported beside
    # `value`, never as it.  Skipped for datasets above 1 GiB.
    from_host = None
    host_bytes = (data["col_idx"].nbytes + data["vals"].nbytes) if cfg.sparse else \
        rows * cfg.dims[0] * (2 if dtype_name == "bf16" else 4)
    if not args.no_from_host and host_bytes <= (1 << 30) and n_batches >= 2:
        sched = hb.Sched(rows, [B], [B], [B])
        pin = lambda a: torch.from_numpy(np.ascontiguousarray(a)).pin_memory()
        h_y = pin(data["y"])
        if cfg.sparse:
            h_rp = data["row_ptr"].astype(np.int64)
            h_ci, h_va = pin(data["col_idx"]), pin(data["vals"])
            epoch = lambda u: model.worker_run_epoch_csr(sched, 0, h_rp, h_ci, h_va, h_y, lr / B, updates=u)
        else:
            h_X = torch.from_numpy(X)
            h_X = (h_X.to(torch.bfloat16) if dtype_name == "bf16" else h_X).pin_memory()
            epoch = lambda u: model.worker_run_epoch(sched, 0, h_X, h_y, lr / B, updates=u)
        u = 0.0
        n_warm = max(1, min(4, (args.warmup + n_batches - 1) // n_batches + 1))
        for _ in range(n_warm):               # untimed: staging buffers, the runtime's copy paths
            u, _, _ = epoch(u)
            sched.new_epoch()
        n_epochs = max(1, min(8, args.steps // n_batches))
        t2 = time.perf_counter()
        h_steps = 0
        for _ in range(n_epochs):
            u, st_e, _ = epoch(u)
            sched.new_epoch()
            h_steps += st_e
        dt2 = time.perf_counter() - t2
        from_host = {"value": round(h_steps * B / dt2, 1), "unit": "examples/s",
                     "ms_per_step": round(1e3 * dt2 / h_steps, 5), "steps": h_steps,
                     "what": "hb_worker_run_epoch%s: Adaptive Hogbatch scheduler with one worker, dataset in "
                             "page-locked host memory, no merging" % ("_csr" if cfg.sparse else "")}
    model.destroy()
    note("device legs done" + ("" if from_host is None else f"; from host memory {from_host['ms_per_step']:.4f} ms per step"))

    # ---- the oracle as it stands, on the host cores, on a bounded sample of the same workload
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        params64 = hi.make_params(args.config).astype(np.float64)
        cores = oracle.max_threads()

        def oracle_step(nrows):
            t = time.perf_counter()
            if cfg.sparse:
                r, c, v = hi.csr_slice(data["row_ptr"], data["col_idx"], data["vals"], 0, nrows)
                oracle.batch_step_csr(cfg.dims, cfg.activation, cfg.loss, params64, r, c, v,
                                      data["y"][:nrows], lr)
            else:
                Xs = data["X"][:nrows]
                if dtype_name == "bf16":
                    Xs = oracle.bf16_round(Xs)
                oracle.batch_step(cfg.dims, cfg.activation, cfg.loss, params64, Xs, data["y"][:nrows], lr)
            return time.perf_counter() - t

        probe_rows = min(B, 64)
        rate = probe_rows / oracle_step(probe_rows)          # examples/s, B-independent
        # whole batches first (up to 8 oracle steps), a fraction of one batch if even that is too slow
        want = rate * args.cpu_seconds
        if want >= B:
            n_steps, sample = int(min(8, want // B)), B
        else:
            n_steps, sample = 1, int(max(probe_rows, want))
        note(f"oracle on {cores} threads: {rate:.0f} examples/s on a probe of {probe_rows} rows; timing {n_steps} step(s) of {sample} rows")
        dt = 0.0
        for i in range(n_steps):
            dt += oracle_step(sample)
            note(f"oracle step {i + 1} of {n_steps} done")
        # the same oracle on one core, on a small sample (its rate does not depend on B): about 4 s
        oracle.set_threads(1)
        one_rows = int(max(8, min(B, 128, 4.0 * rate / max(cores, 1))))
        one_core = one_rows / oracle_step(one_rows)
        oracle.set_threads(cores)
        note(f"oracle on one thread: {one_core:.1f} examples/s on {one_rows} rows")
        cpu_baseline = {"value": round(n_steps * sample / dt, 2), "unit": "examples/s", "cores": cores,
                        "kind": "oracle", "value_1_core": round(one_core, 2),
                        "sample": f"{n_steps} fp64 oracle step(s) (forward, backward, update) on the first "
                                  f"{sample} rows of the same dataset, {dt:.1f} s"}

    out = {
        "metric": "training examples/sec per SGD batch step at B=4096; % of MFMA peak",
        "value": round(value, 1),
        "unit": "examples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": dtype_name,
        "data": "synthetic",
        "config": {"workload": f"config {args.config}: {cfg.name}", "batch": B, "dataset_rows": rows, "lr": lr,
                   "sparse_first_layer": cfg.sparse},
        "timing": {"warmup_steps_run": warm_steps, "regions_ms_per_step": [round(v, 5) for v in region_ms],
                   "what": f"median of {len(region_ms)} regions of {args.steps} steps after at least {args.warm_seconds} s of warm-up"},
        "step_tflops": round(flops / (elapsed / args.steps) / 1e12, 3),
        "step_frac_of_mfma_peak": round(flops / (elapsed / args.steps) / 1e12 / PEAK_TFLOPS[dtype_name], 4),
        "last_loss": last_loss,
        "sync_ms_per_step": None if sync_ms_per_step is None else round(sync_ms_per_step, 5),
        "from_host": from_host,
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "kernels": kernels,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
