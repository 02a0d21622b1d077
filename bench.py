"""Benchmark of the hash-encoding hot path on one MI355X.

A step is one forward plus one backward pass of the encoding over one batch of
synthetic points (inputs resident in HBM): hashgrid_encode_fwd_ws, which also
counts for the backward pass, then hashgrid_encode_bwd_ws (where the
configuration is not served by them: hashgrid_encode_fwd + hashgrid_encode_bwd).
Prints one JSON line: the headline workload first (the configuration the metric is
quoted on), then the same step on the other workloads under "workloads".
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
# What the 256 compute units can take in from their XCDs' L2 caches: 64 bytes per clock each at 2.4 GHz.
# A gather that misses the L1 moves one 128-byte line over this path, however few of its bytes are used.
L2_FILL_PEAK_GBS = 256 * 64 * 2.4
LINE_BYTES = 128
INIT_STEPS = 30  # untimed steps before the warm-up steps: first-call set-up of the library, clocks


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


def time_each(before, fn, n, torch):
    """Average duration of fn over n launches, each bracketed by its own pair of HIP events on the
    launch stream; `before` runs ahead of every launch, outside the bracket."""
    marks = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for e0, e1 in marks:
        before()
        e0.record()
        fn()
        e1.record()
    torch.cuda.synchronize()
    return sum(e0.elapsed_time(e1) for e0, e1 in marks) / n


def profile_figure(name, key):
    """A per-launch figure from a committed rocprofv3 counter summary under profiles/ (`key: value`
    lines); None when no summary holds it."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith(f"{key}:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def machine_probes(torch):
    """What this GPU delivers on elementary access patterns (libhashgrid_probes): the measured
    denominators next to the published 8 TB/s."""
    from paper_2201_05989_amd import probe_atomic_add, probe_copy, probe_gather, probe_gather_lines

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
    # the forward pass's own shape: 2^18 points, 16 levels, 4 lines (2 adjacent words each) per point and
    # level, a barrier per level, a new 2 MiB slice every level
    points, levels, words = 1 << 18, 16, 1 << 19
    t = a[: levels * words].view(torch.int32)
    probe_gather_lines(t, words, levels, points, levels, sink)
    ms = time_launches(lambda: probe_gather_lines(t, words, levels, points, levels, sink), 10, torch)
    out["gather_lines_16x2MiB_g_lines_per_s"] = points * levels * 4 / (ms * 1e-3) / 1e9
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


class Case:
    """One workload resident on the GPU: inputs, outputs and the calls of a step."""

    def __init__(self, w, torch):
        from paper_2201_05989_amd import HashGrid, synth

        self.w, self.torch = w, torch
        self.grid = HashGrid(w.d, w.L, w.F, w.T, w.N_min, w.N_max, w.param_dtype, w.io_dtype)
        self.host = synth.make_inputs(w, self.grid.n_entries)
        self.xd, self.td, self.gd = (torch.from_numpy(a).cuda() for a in self.host)
        self.y = torch.empty((w.B, w.L * w.F), dtype=self.grid.io_dtype, device="cuda")
        self.grad = torch.zeros((self.grid.n_entries, w.F), dtype=torch.float32, device="cuda")
        s_theta = 2 if w.param_dtype == "f16" else 4
        s_io = 2 if w.io_dtype == "f16" else 4
        self.b_fwd, self.b_bwd = algorithmic_bytes(w, s_theta, s_io)
        self.counting = True

    def fwd(self):  # forward alone
        self.grid.encode_fwd(self.xd, self.td, self.y)

    def bwd(self):  # backward; skips its counting pass when the forward has just counted
        self.grid.encode_bwd(self.xd, self.gd, self.grad)

    def fwd_counting(self):
        self.grid.encode_fwd(self.xd, self.td, self.y, count_for_bwd=True)

    def step_fwd(self):  # the forward call of the step: counts for the backward pass where that is the faster pair
        if self.counting:
            self.fwd_counting()
        else:
            self.fwd()

    def step(self):
        self.step_fwd()
        self.bwd()

    def choose_step(self, n=20):
        """The forward can count for the sorted backward pass on the side or leave the counting to it.  Which pair
        of calls is faster depends on the order of the points (samples along rays share voxels between
        neighbouring lanes: there the separate count pass wins), so both are timed once, as a caller would."""
        torch, times = self.torch, {}
        for counting in (True, False):
            self.counting = counting
            for _ in range(3):
                self.step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                self.step()
            torch.cuda.synchronize()
            times[counting] = (time.perf_counter() - t0) / n
        self.counting = times[True] <= 1.01 * times[False]  # (a tie keeps the counting forward)
        return self.counting

    def measure(self, steps, warmup, init=INIT_STEPS, forward_counts="auto"):
        """Wall-clock time of `steps` steps after `init` + `warmup` untimed ones, then the two passes as the
        step runs them, each bracketed by HIP events on the launch stream."""
        torch = self.torch
        for _ in range(init):
            self.step()
        if forward_counts == "auto":
            self.choose_step()
        else:
            self.counting = forward_counts == "yes"
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        ms_step = (time.perf_counter() - t0) * 1e3 / steps
        n = max(steps, 20)
        marks = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n)]
        for ea, eb, ec in marks:
            ea.record()
            self.step_fwd()
            eb.record()
            self.bwd()
            ec.record()
        torch.cuda.synchronize()
        ms_fwd = sum(ea.elapsed_time(eb) for ea, eb, _ in marks) / n
        ms_bwd = sum(eb.elapsed_time(ec) for _, eb, ec in marks) / n
        return ms_step, ms_fwd, ms_bwd

    def fractions(self, ms_step, ms_fwd, ms_bwd):
        """Algorithmic bytes over time, as GB/s and as a fraction of the published HBM rate."""
        B = self.w.B

        def one(nbytes, ms):
            gbs = nbytes * B / (ms * 1e-3) / 1e9
            return {"achieved": gbs, "frac": gbs / HBM_PEAK_GBS}

        return {"fwd": one(self.b_fwd, ms_fwd), "bwd": one(self.b_bwd, ms_bwd),
                "step": one(self.b_fwd + self.b_bwd, ms_step)}

    def describe(self):
        w = self.w
        return (f"{w.name}: d={w.d} L={w.L} F={w.F} T=2^{w.T.bit_length() - 1} "
                f"N_min={w.N_min} N_max={w.N_max} B={w.B} points={w.points}")


def headline_extras(c, ms_fwd, ms_bwd, n, steps, torch):
    """Stand-alone calls, the replacing backward, the optimiser step and the fused network on the headline workload."""
    w, grid, xd, td, gd, grad = c.w, c.grid, c.xd, c.td, c.gd, c.grad
    ms_fwd_alone = time_launches(c.fwd, n, torch)
    ms_bwd_alone = time_launches(c.bwd, n, torch)
    ms_zero = time_launches(lambda: grad.zero_(), 20, torch)

    # the same step when the backward pass replaces the gradient instead of adding to it
    # (HG_BWD_OVERWRITE: no clearing pass before it, no reading of the old values in it)
    def step_overwrite():
        c.step_fwd()
        grid.encode_bwd(xd, gd, grad, overwrite=True)

    ms_bwd_ow = time_launches(lambda: grid.encode_bwd(xd, gd, grad, overwrite=True), n, torch)
    ms_step_ow = time_launches(step_overwrite, n, torch)
    grad.zero_()

    # next row of the path: the optimiser step on the tables (fp32 master + fp16 working copy, clears the
    # gradient).  Every timed launch follows a backward pass, outside its bracket of events, so that it
    # works on a real gradient (the step skips scalars whose gradient is zero and clears the ones it uses).
    from paper_2201_05989_amd import adam_step
    master = td.float()
    m1, m2 = torch.zeros_like(master), torch.zeros_like(master)
    counter = [0]
    half = td if w.param_dtype == "f16" else None

    def adam(zero_grad=True):
        counter[0] += 1
        adam_step(master, grad, m1, m2, counter[0], lr=1e-2, params_half=half, zero_grad=zero_grad)

    grad.zero_()
    ms_adam = time_each(c.bwd, adam, max(steps // 2, 50), torch)

    def train():
        c.step()
        adam()

    ms_train = time_launches(train, max(steps // 2, 10), torch)

    # the whole table-training step when the backward pass replaces the gradient: the optimiser
    # then has nothing to clear
    def train_overwrite():
        step_overwrite()
        adam(zero_grad=False)

    ms_train_ow = time_launches(train_overwrite, max(steps // 2, 10), torch)
    grad.zero_()
    n_scalars = grid.n_entries * w.F
    per_scalar = 16 + 12 + 4 + (2 if w.param_dtype == "f16" else 0)
    adam_bytes = n_scalars * per_scalar
    footprint = n_scalars * (16 + (2 if w.param_dtype == "f16" else 0))

    extras = {
        "ms_grad_zero": ms_zero, "ms_fwd_alone": ms_fwd_alone, "ms_bwd_alone": ms_bwd_alone,
        "overwrite": {"ms_bwd_alone": ms_bwd_ow, "ms_step": ms_step_ow,
                      "mpoints_s": w.B / (ms_step_ow * 1e-3) / 1e6, "train_step_ms": ms_train_ow,
                      "train_step_mpoints_s": w.B / (ms_train_ow * 1e-3) / 1e6},
        "adam": {"ms": ms_adam, "timing": "HIP events around each of the launches, a backward pass before each",
                 "scalars": n_scalars, "algorithmic_bytes": adam_bytes,
                 "achieved_gb_s": adam_bytes / (ms_adam * 1e-3) / 1e9,
                 "footprint_bytes": footprint,
                 "cache_resident": footprint < 256e6,  # then the rate is the memory-side cache's, not HBM's
                 "train_step_ms": ms_train, "train_step_mpoints_s": w.B / (ms_train * 1e-3) / 1e6},
    }
    # half-precision gradients as the paper keeps them: the sorted pass (sums exact, rounded once per call)
    # and the pass of packed two-half atomics
    from paper_2201_05989_amd import HashGrid
    g16 = HashGrid(w.d, w.L, w.F, w.T, w.N_min, w.N_max, w.param_dtype, w.io_dtype, grad_dtype="f16")
    grad16 = torch.zeros((g16.n_entries, w.F), dtype=torch.float16, device="cuda")
    half_grads = {}
    if g16.bwd_workspace_bytes(w.B):
        half_grads["ms_bwd_sorted"] = time_launches(lambda: g16.encode_bwd(xd, gd, grad16, use_workspace=True), n, torch)
        half_grads["ms_bwd_sorted_overwrite"] = time_launches(
            lambda: g16.encode_bwd(xd, gd, grad16, use_workspace=True, overwrite=True), n, torch)
        # the table-training step the way the paper runs it: half-precision gradients (here summed exactly and
        # rounded once), full-precision master copy; the backward pass replaces the gradient
        def train_f16():
            g16.encode_fwd(xd, td, c.y, count_for_bwd=c.counting)
            g16.encode_bwd(xd, gd, grad16, use_workspace=True, overwrite=True)
            counter[0] += 1
            adam_step(master, grad16, m1, m2, counter[0], lr=1e-2, params_half=half, zero_grad=False)

        half_grads["train_step_ms"] = time_launches(train_f16, max(n // 2, 10), torch)
    grad16.zero_()
    half_grads["ms_bwd_atomic"] = time_launches(lambda: g16.encode_bwd(xd, gd, grad16, use_workspace=False), 10, torch)
    extras["grad_f16"] = half_grads
    del g16, grad16

    # last row of the path's table: the encoding fused with the paper's 64-64 ReLU network (one output,
    # as for a signed distance function); served for fp16 tables with at most 64 encoded features
    n_in = w.L * w.F
    if w.param_dtype == "f16" and n_in % 8 == 0 and n_in <= 64 and w.d >= 2:
        import numpy as np
        rng = np.random.default_rng(0)
        # the network's weights in one array (W1 | W2 | W3), so that one optimiser call serves them: fp32
        # master, fp16 working copy, fp32 gradient, the matrices as views
        shapes = [(64, n_in), (64, 64), (1, 64)]
        init = [rng.standard_normal((64, n_in)) * np.sqrt(2.0 / n_in), rng.standard_normal((64, 64)) * np.sqrt(2.0 / 64),
                rng.standard_normal((1, 64)) / 8.0]
        net_master = torch.from_numpy(np.concatenate([a.ravel() for a in init]).astype(np.float32)).cuda()
        net_half, net_grad = net_master.half(), torch.zeros_like(net_master)
        net_m1, net_m2 = torch.zeros_like(net_master), torch.zeros_like(net_master)

        def views(flat):
            out, at = [], 0
            for r, c_ in shapes:
                out.append(flat[at:at + r * c_].view(r, c_))
                at += r * c_
            return out

        W1, W2, W3 = views(net_half)
        o = torch.empty((w.B, 1), dtype=torch.float32, device="cuda")
        grid.encode_mlp_fwd(xd, td, W1, W2, W3, o)
        ms_mlp = time_launches(lambda: grid.encode_mlp_fwd(xd, td, W1, W2, W3, o), max(n // 2, 10), torch)
        flops = 2.0 * (n_in * 64 + 64 * 64 + 64 * 1) * w.B
        extras["encode_mlp_fwd"] = {"ms": ms_mlp, "mpoints_s": w.B / (ms_mlp * 1e-3) / 1e6, "n_out": 1,
                                    "network_tflop_s": flops / (ms_mlp * 1e-3) / 1e12,
                                    "ms_over_forward_alone": ms_mlp - ms_fwd_alone}
        # training the whole model: fused forward that keeps y, the loss's gradient (the workload's loss against a
        # synthetic target), backward of the network, sorted backward of the encoding into the tables, optimiser on
        # the tables and on the network's weights
        from paper_2201_05989_amd import loss_grad, mlp_bwd
        loss_kind = "mape" if w.name.startswith("sdf") else "l2"  # Section 4, "Training"
        target = torch.from_numpy(np.random.default_rng(11).normal(size=(w.B, 1)).astype(np.float32)).cuda()
        dout = torch.empty_like(target)
        loss_sum = torch.zeros(1, dtype=torch.float64, device="cuda")
        yk = torch.empty((w.B, n_in), dtype=torch.float16, device="cuda")
        dyk = torch.empty_like(yk)
        dWs = views(net_grad)
        grid.encode_mlp_fwd(xd, td, W1, W2, W3, o, y=yk)
        ms_net_bwd = time_launches(lambda: mlp_bwd(yk, W1, W2, W3, o, dyk, *dWs), max(n // 2, 10), torch)

        net_counter = [0]

        def model_step():
            grid.encode_mlp_fwd(xd, td, W1, W2, W3, o, y=yk)
            loss_grad(o, target, loss_kind, 1.0, dout, loss_sum)
            mlp_bwd(yk, W1, W2, W3, dout, dyk, *dWs)
            grid.encode_bwd(xd, dyk, grad, overwrite=True)
            adam(zero_grad=False)
            net_counter[0] += 1  # the network's weights: a small learning rate, the gradient cleared for the next step
            adam_step(net_master, net_grad, net_m1, net_m2, net_counter[0], lr=1e-4, params_half=net_half, zero_grad=True,
                      l2_reg=1e-6)

        ms_model = time_launches(model_step, max(n // 2, 10), torch)
        extras["network_training"] = {
            "ms_mlp_bwd": ms_net_bwd, "mlp_bwd_tflop_s": 4.0 * flops / (ms_net_bwd * 1e-3) / 1e12,
            "ms_step": ms_model, "mpoints_s": w.B / (ms_model * 1e-3) / 1e6,
            "loss": loss_kind,
            "step": "encode_mlp_fwd_train + loss_grad + mlp_bwd + encode_bwd_ws (overwrite) + adam_step on the tables + "
                    "adam_step on the network's weights"}
    return extras


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--forward-counts", choices=["auto", "yes", "no"], default="auto",
                    help="whether the step's forward call counts for the sorted backward pass on the side "
                         "(auto: both pairs of calls are timed once and the faster one is kept)")
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="sdf3d")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the machine probes (copy, gather, atomic rates)")
    ap.add_argument("--other-workloads", default="all",
                    help="the workloads whose step is timed after the headline one: all, none, or names separated by commas")
    ap.add_argument("--step-only", action="store_true",
                    help="only the step and its two passes (what the profiles are taken of): no stand-alone "
                         "calls, other entry points, other workloads, probes or CPU baseline")
    ap.add_argument("--probes-only", action="store_true",
                    help="run only the machine probes (for counter runs that check what a probe moves)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a 1 GiB device-to-device copy (20 times): the known-size kernel that "
                         "FETCH_SIZE / WRITE_SIZE counter readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2201_05989_amd import synth

    if args.calibrate_copy:
        a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        for _ in range(20):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": a.numel() * 4, "bytes_written": a.numel() * 4, "launches": 20}))
        return

    if args.probes_only:
        print(json.dumps({"measured_peaks": machine_probes(torch)}))
        return

    w = synth.WORKLOADS[args.workload]
    c = Case(w, torch)
    ms_step, ms_fwd, ms_bwd = c.measure(args.steps, args.warmup, forward_counts=args.forward_counts)
    passes = c.fractions(ms_step, ms_fwd, ms_bwd)
    sorted_path = bool(c.grid.bwd_workspace_bytes(w.B))

    # The dominant kernel: the forward pass is one kernel per call; the backward call is three
    # (bin_scan, bin_scatter, bin_accumulate), none of which takes as long as the forward kernel
    # unless the whole call takes twice as long.
    fwd_dominant = not sorted_path or ms_fwd >= 0.5 * ms_bwd
    dom = "fwd" if fwd_dominant else "bwd"
    kernels = {"fwd": "fwd_point_major (counting variant)" if sorted_path and c.counting else "fwd_point_major",
               "bwd": "bin_scan+bin_scatter+bin_accumulate (one hashgrid_encode_bwd_ws call)" if sorted_path
               else "bwd_general"}
    traffic = {p: profile_figure(f"traffic_{w.name}.txt", f"{p}_hbm_bytes_per_launch") for p in ("fwd", "bwd")}
    roofline = {"bound": "hbm", "kernel": kernels[dom], "pass": dom, "achieved": passes[dom]["achieved"],
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": passes[dom]["frac"], "traffic": traffic[dom],
                "algorithmic_bytes_per_point": {"fwd": c.b_fwd, "bwd": c.b_bwd},
                "duration_ms": ms_fwd if dom == "fwd" else ms_bwd,
                "passes": {p: dict(passes[p], traffic=traffic.get(p)) for p in passes}}
    out = {
        "metric": "hash-grid encoding fwd+bwd throughput",
        "value": w.B / (ms_step * 1e-3) / 1e6,
        "unit": "Mpoints/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": c.describe(), "param_dtype": w.param_dtype, "io_dtype": w.io_dtype, "grad_dtype": "f32",
                   "untimed_steps_before_warmup": INIT_STEPS, "forward_counts_for_backward": bool(c.counting)},
        "fwd_mpoints_s": w.B / (ms_fwd * 1e-3) / 1e6,
        "bwd_mpoints_s": w.B / (ms_bwd * 1e-3) / 1e6,
        "ms_fwd": ms_fwd, "ms_bwd": ms_bwd,
        "roofline": roofline,
    }
    # The forward kernel's gathers are served by the L2, not by HBM: its own roofline is the path from the
    # L2 caches into the compute units.  Lines per launch = TCP_TCC_READ_REQ of the committed counter summary.
    lines = profile_figure(f"ta_tcp_counters_{w.name}.txt", "fwd_l2_read_requests_per_launch")
    if lines is not None:
        gbs = lines * LINE_BYTES / (ms_fwd * 1e-3) / 1e9
        out["roofline_l2"] = {"bound": "l2_fill", "kernel": kernels["fwd"], "lines_per_launch": lines,
                              "line_bytes": LINE_BYTES, "achieved": gbs, "peak": L2_FILL_PEAK_GBS, "unit": "GB/s",
                              "frac": gbs / L2_FILL_PEAK_GBS, "achieved_g_lines_per_s": lines / (ms_fwd * 1e-3) / 1e9}
    if not args.step_only:
        out.update(headline_extras(c, ms_fwd, ms_bwd, max(args.steps, 20), args.steps, torch))
    if not args.no_probes and not args.step_only:
        # the pass rates in the elementary operations they stand for, next to what the machine does
        # when it performs those operations one by one at random
        corners = (1 << w.d) * w.L
        probes = machine_probes(torch)
        out["measured_peaks"] = probes
        out["vs_measured"] = {
            "fwd_gathers_g_per_s": corners * w.B / (ms_fwd * 1e-3) / 1e9,
            "bwd_scalar_adds_g_per_s": corners * w.F * w.B / (ms_bwd * 1e-3) / 1e9,
            "bwd_over_atomic_add_4MiB": corners * w.F * w.B / (ms_bwd * 1e-3) / 1e9
            / probes["atomic_add_f32_4MiB_g_per_s"],
            "step_hbm_frac_of_copy": passes["step"]["achieved"] / probes["copy_1GiB_gb_s"],
        }
        if "roofline_l2" in out:  # the same line fetches, issued in the forward's shape with nothing else to do
            out["roofline_l2"]["probe_g_lines_per_s"] = probes["gather_lines_16x2MiB_g_lines_per_s"]
            out["roofline_l2"]["frac_of_probe"] = (out["roofline_l2"]["achieved_g_lines_per_s"]
                                                   / probes["gather_lines_16x2MiB_g_lines_per_s"])
    host = c.host
    other_names = [n for n in synth.WORKLOADS if n != w.name and args.other_workloads != "none"
                   and (args.other_workloads == "all" or n in args.other_workloads.split(","))]
    if not args.step_only and other_names:
        # the other workloads: the same step, GPU side only, a shorter run each
        del c
        torch.cuda.empty_cache()
        others = []
        for name in other_names:
            o = Case(synth.WORKLOADS[name], torch)
            steps = 100 if o.w.B <= (1 << 18) else 20
            s, f, b = o.measure(steps, 5, init=10, forward_counts=args.forward_counts)
            fr = o.fractions(s, f, b)
            others.append({"name": name, "workload": o.describe(), "B": o.w.B, "steps": steps, "ms_step": s,
                           "mpoints_s": o.w.B / (s * 1e-3) / 1e6, "ms_fwd": f, "ms_bwd": b,
                           "sorted_backward": bool(o.grid.bwd_workspace_bytes(o.w.B)),
                           "forward_counts_for_backward": bool(o.counting),
                           "frac": fr["step"]["frac"], "fwd_frac": fr["fwd"]["frac"], "bwd_frac": fr["bwd"]["frac"],
                           "algorithmic_bytes_per_point": {"fwd": o.b_fwd, "bwd": o.b_bwd}})
            del o
            torch.cuda.empty_cache()
        out["workloads"] = others
    if not args.no_cpu_baseline and not args.step_only:
        out["cpu_baseline"] = cpu_baseline(w, *host)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
