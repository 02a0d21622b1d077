"""Benchmark of the hash-encoding hot path on one MI355X.

A step is one forward plus one backward pass of the encoding over one batch of
synthetic points (inputs resident in HBM): hashgrid_encode_fwd_ws, which also
counts for the backward pass, then hashgrid_encode_bwd_ws (where the
configuration is not served by them: hashgrid_encode_fwd + hashgrid_encode_bwd).
Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published


def algorithmic_bytes(w, s_theta, s_io):
    """Bytes the method itself moves per point: positions, the 2^d * L gathers (or
    fp32 atomic updates, counted once at 4 B) of F scalars, and the output / upstream-gradient row."""
    corners = (1 << w.d) * w.L
    fwd = 4 * w.d + corners * w.F * s_theta + w.L * w.F * s_io
    bwd = 4 * w.d + w.L * w.F * s_io + corners * w.F * 4
    return fwd, bwd


def time_launches(fn, n, torch):
    """Average duration of n back-to-back launches, HIP events on the launch stream."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / n  # ms


def measured_traffic(workload, which):
    """HBM bytes per launch of the dominant pass, from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE scaled by the copy calibration); None when no summary covers it."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.txt")
    try:
        for line in open(path):
            if line.startswith(f"{which}_hbm_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def machine_probes(torch):
    """What this GPU delivers on three elementary access patterns (hashgrid_probe_*): the measured
    denominators next to the published 8 TB/s."""
    from paper_2201_05989_amd import probe_atomic_add, probe_copy, probe_gather

    out = {}
    a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB
    b = torch.empty_like(a)
    probe_copy(a, b)
    out["copy_1GiB_gb_s"] = 2 * a.numel() * 4 / (time_launches(lambda: probe_copy(a, b), 10, torch) * 1e-3) / 1e9
    del b
    sink = torch.empty(1 << 22, dtype=torch.int32, device="cuda")
    n = 1 << 26
    for mib in (2, 64):
        t = a[: mib << 18].view(torch.int32)
        probe_gather(t, n, sink)
        out[f"gather_4B_{mib}MiB_g_per_s"] = n / (time_launches(lambda: probe_gather(t, n, sink), 10, torch) * 1e-3) / 1e9
    n = 1 << 25
    for mib in (4, 128):
        t = a[: mib << 18]
        probe_atomic_add(t, n)
        out[f"atomic_add_f32_{mib}MiB_g_per_s"] = n / (time_launches(lambda: probe_atomic_add(t, n), 5, torch) * 1e-3) / 1e9
    return out


def cpu_baseline(w, x, theta, dy, budget_s=10.0):
    import numpy as np
    from oracle import hashgrid_oracle as orc

    cfg = orc.OracleConfig(w.d, w.L, w.F, w.T, w.N_min, w.N_max)
    nb = min(len(x), 1 << 18)
    xs, dys = x[:nb], dy[:nb].astype(np.float64)
    th = theta.astype(np.float64)
    orc.encode_fwd(cfg, xs[:1024], th)  # load + first touch
    reps, t0 = 0, time.perf_counter()
    while True:
        orc.encode_fwd(cfg, xs, th)
        orc.encode_bwd(cfg, xs, dys)
        reps += 1
        el = time.perf_counter() - t0
        if el >= budget_s or reps >= 1024:
            break
    cores = orc.num_threads()
    # one core, on a smaller sample of the same points (a few seconds)
    n1 = min(nb, 1 << 15)
    orc.set_num_threads(1)
    t1 = time.perf_counter()
    orc.encode_fwd(cfg, xs[:n1], th)
    orc.encode_bwd(cfg, xs[:n1], dys[:n1])
    el1 = time.perf_counter() - t1
    orc.set_num_threads(cores)
    return {"value": nb * reps / el / 1e6, "unit": "Mpoints/s", "cores": cores, "kind": "oracle",
            "sample": f"{reps} fwd+bwd passes over the first {nb} points of the workload, {el:.1f} s",
            "one_core_value": n1 / el1 / 1e6,
            "one_core_sample": f"1 fwd+bwd pass over the first {n1} points, {el1:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="sdf3d")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the machine probes (copy, gather, atomic rates)")
    ap.add_argument("--step-only", action="store_true",
                    help="only the step and its two passes (what the profiles are taken of): no stand-alone "
                         "calls, other entry points, probes or CPU baseline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a 1 GiB device-to-device copy (20 times): the known-size kernel that "
                         "FETCH_SIZE / WRITE_SIZE counter readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2201_05989_amd import HashGrid, synth

    if args.calibrate_copy:
        a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        for _ in range(20):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": a.numel() * 4, "bytes_written": a.numel() * 4, "launches": 20}))
        return

    w = synth.WORKLOADS[args.workload]
    grid = HashGrid(w.d, w.L, w.F, w.T, w.N_min, w.N_max, w.param_dtype, w.io_dtype)
    x, theta, dy = synth.make_inputs(w, grid.n_entries)
    xd, td, gd = (torch.from_numpy(a).cuda() for a in (x, theta, dy))
    y = torch.empty((w.B, w.L * w.F), dtype=grid.io_dtype, device="cuda")
    grad = torch.zeros((grid.n_entries, w.F), dtype=torch.float32, device="cuda")

    def fwd():  # forward alone
        grid.encode_fwd(xd, td, y)

    def bwd():  # backward alone (does its own counting)
        grid.encode_bwd(xd, gd, grad)

    def fwd_counting():
        grid.encode_fwd(xd, td, y, count_for_bwd=True)

    def step():
        fwd_counting()
        bwd()  # skips its counting pass when the forward has done it


    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps

    n = max(args.steps, 20)
    # the two passes as the step runs them, each bracketed by HIP events on the launch stream
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n)]
    for ea, eb, ec in marks:
        ea.record()
        fwd_counting()
        eb.record()
        bwd()
        ec.record()
    torch.cuda.synchronize()
    ms_fwd = sum(ea.elapsed_time(eb) for ea, eb, _ in marks) / n
    ms_bwd = sum(eb.elapsed_time(ec) for _, eb, ec in marks) / n
    extras = {}
    if not args.step_only:
        ms_fwd_alone = time_launches(fwd, n, torch)
        ms_bwd_alone = time_launches(bwd, n, torch)
        ms_zero = time_launches(lambda: grad.zero_(), 20, torch)

        # the same step when the backward pass replaces the gradient instead of adding to it
        # (HG_BWD_OVERWRITE: no clearing pass before it, no reading of the old values in it)
        def step_overwrite():
            fwd_counting()
            grid.encode_bwd(xd, gd, grad, overwrite=True)

        ms_bwd_ow = time_launches(lambda: grid.encode_bwd(xd, gd, grad, overwrite=True), n, torch)
        ms_step_ow = time_launches(step_overwrite, n, torch)
        grad.zero_()

        # next row of the path: the optimiser step on the tables (fp32 master + fp16 working copy,
        # clears the gradient).  Timed as (backward + optimiser) minus backward, because the step
        # skips entries whose gradient is zero and clears the ones it uses.
        from paper_2201_05989_amd import adam_step
        master = td.float()
        m1, m2 = torch.zeros_like(master), torch.zeros_like(master)
        counter = [0]

        def bwd_adam():
            bwd()
            counter[0] += 1
            adam_step(master, grad, m1, m2, counter[0], lr=1e-2, params_half=td if w.param_dtype == "f16" else None)

        grad.zero_()
        ms_bwd_adam = time_launches(bwd_adam, max(args.steps // 2, 10), torch)
        grad.zero_()
        ms_adam = ms_bwd_adam - ms_bwd_alone

        # the whole table-training step when the backward pass replaces the gradient: the optimiser
        # then has nothing to clear
        def train_overwrite():
            fwd_counting()
            grid.encode_bwd(xd, gd, grad, overwrite=True)
            counter[0] += 1
            adam_step(master, grad, m1, m2, counter[0], lr=1e-2, params_half=td if w.param_dtype == "f16" else None,
                      zero_grad=False)

        ms_train_ow = time_launches(train_overwrite, max(args.steps // 2, 10), torch)
        grad.zero_()
        n_scalars = grid.n_entries * w.F
        adam_bytes = n_scalars * (16 + 12 + 4 + (2 if w.param_dtype == "f16" else 0))

        # last row of the path's table: the encoding fused with the paper's 64-64 ReLU network (one output,
        # as for a signed distance function); served for fp16 tables with at most 64 encoded features
        mlp = None
        n_in = w.L * w.F
        if w.param_dtype == "f16" and n_in % 8 == 0 and n_in <= 64 and w.d >= 2:
            import numpy as np
            rng = np.random.default_rng(0)
            W1 = torch.from_numpy((rng.standard_normal((64, n_in)) * np.sqrt(2.0 / n_in)).astype(np.float16)).cuda()
            W2 = torch.from_numpy((rng.standard_normal((64, 64)) * np.sqrt(2.0 / 64)).astype(np.float16)).cuda()
            W3 = torch.from_numpy((rng.standard_normal((1, 64)) / 8.0).astype(np.float16)).cuda()
            o = torch.empty((w.B, 1), dtype=torch.float32, device="cuda")
            grid.encode_mlp_fwd(xd, td, W1, W2, W3, o)
            ms_mlp = time_launches(lambda: grid.encode_mlp_fwd(xd, td, W1, W2, W3, o), max(n // 2, 10), torch)
            flops = 2.0 * (n_in * 64 + 64 * 64 + 64 * 1) * w.B
            mlp = {"ms": ms_mlp, "mpoints_s": w.B / (ms_mlp * 1e-3) / 1e6, "n_out": 1,
                   "network_tflop_s": flops / (ms_mlp * 1e-3) / 1e12, "ms_over_forward_alone": ms_mlp - ms_fwd_alone}
        extras = {
            "ms_grad_zero": ms_zero, "ms_fwd_alone": ms_fwd_alone, "ms_bwd_alone": ms_bwd_alone,
            "overwrite": {"ms_bwd_alone": ms_bwd_ow, "ms_step": ms_step_ow,
                          "mpoints_s": w.B / (ms_step_ow * 1e-3) / 1e6, "train_step_ms": ms_train_ow,
                          "train_step_mpoints_s": w.B / (ms_train_ow * 1e-3) / 1e6},
            "adam": {"ms": ms_adam, "scalars": n_scalars, "algorithmic_bytes": adam_bytes,
                     "achieved_gb_s": adam_bytes / (ms_adam * 1e-3) / 1e9 if ms_adam > 0 else None,
                     "train_step_ms": ms_fwd + ms_bwd + ms_adam,
                     "train_step_mpoints_s": w.B / ((ms_fwd + ms_bwd + ms_adam) * 1e-3) / 1e6},
        }
        if mlp is not None:
            extras["encode_mlp_fwd"] = mlp

    s_theta = 2 if w.param_dtype == "f16" else 4
    s_io = 2 if w.io_dtype == "f16" else 4
    b_fwd, b_bwd = algorithmic_bytes(w, s_theta, s_io)
    dom = ("bwd", ms_bwd, b_bwd) if ms_bwd >= ms_fwd else ("fwd", ms_fwd, b_fwd)
    achieved = dom[2] * w.B / (dom[1] * 1e-3) / 1e9
    kernels = {"fwd": "fwd_point_major (counting)", "bwd": "bin_scan+bin_scatter+bin_accumulate "
                                                            "(one hashgrid_encode_bwd_ws call, counts from the forward)"}
    traffic = measured_traffic(w.name, dom[0])

    out = {
        "metric": "hash-grid encoding fwd+bwd throughput",
        "value": w.B / (ms_step * 1e-3) / 1e6,
        "unit": "Mpoints/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: d={w.d} L={w.L} F={w.F} T=2^{w.T.bit_length() - 1} "
                               f"N_min={w.N_min} N_max={w.N_max} B={w.B} points={w.points}",
                   "param_dtype": w.param_dtype, "io_dtype": w.io_dtype, "grad_dtype": "f32"},
        "fwd_mpoints_s": w.B / (ms_fwd * 1e-3) / 1e6,
        "bwd_mpoints_s": w.B / (ms_bwd * 1e-3) / 1e6,
        "ms_fwd": ms_fwd, "ms_bwd": ms_bwd,
        "roofline": {"bound": "hbm", "kernel": kernels[dom[0]] if grid.bwd_workspace_bytes(w.B) else dom[0],
                     "pass": dom[0], "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes_per_point": {"fwd": b_fwd, "bwd": b_bwd},
                     "fwd_achieved": b_fwd * w.B / (ms_fwd * 1e-3) / 1e9,
                     "bwd_achieved": b_bwd * w.B / (ms_bwd * 1e-3) / 1e9},
    }
    out.update(extras)
    if not args.no_probes and not args.step_only:
        # the pass rates in the elementary operations they stand for, next to what the machine does
        # when it performs those operations one by one at random
        corners = (1 << w.d) * w.L
        probes = machine_probes(torch)
        out["measured_peaks"] = probes
        out["vs_measured"] = {
            "fwd_gathers_g_per_s": corners * w.B / (ms_fwd * 1e-3) / 1e9,
            "fwd_over_gather_2MiB": corners * w.B / (ms_fwd * 1e-3) / 1e9 / probes["gather_4B_2MiB_g_per_s"],
            "bwd_scalar_adds_g_per_s": corners * w.F * w.B / (ms_bwd * 1e-3) / 1e9,
            "bwd_over_atomic_add_4MiB": corners * w.F * w.B / (ms_bwd * 1e-3) / 1e9
            / probes["atomic_add_f32_4MiB_g_per_s"],
            "hbm_frac_of_copy": achieved / probes["copy_1GiB_gb_s"],
        }
    if not args.no_cpu_baseline and not args.step_only:
        out["cpu_baseline"] = cpu_baseline(w, x, theta, dy)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
