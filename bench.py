#!/usr/bin/env python3
"""Benchmark of the fused FFT-convolution forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2]

A step is one pass of the whole hot path (load u, forward transform, multiply by
k_f, inverse transform, store y) over one batch of seeded synthetic input that
is already resident in HBM.  Prints ONE JSON line: sequences/ms, the roofline of
the dominant kernel (algorithmic bytes / measured duration against the HBM
peak) and the CPU oracle timed on the host cores over a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E peak
MFMA_PEAK_TFLOPS = 2500.0        # MI355X published dense bf16 / fp16 matrix-core peak
COPY_BYTES = 1 << 28             # size of the --copy-calibration kernel's source (and destination)
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.md")


def measured_traffic(workload: str):
    """HBM bytes per launch of the workload's dominant kernel, from the committed rocprofv3 --pmc
    summary (FETCH_SIZE and WRITE_SIZE, each scaled by the copy kernel's reading); None if the table
    has no row for this workload.  Row format: | workload | kernel | fetch bytes | write bytes | total bytes |"""
    try:
        for line in open(TRAFFIC_TABLE):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) >= 5 and cells[0] == workload:
                return float(cells[4])
    except OSError:
        pass
    return None


def algorithmic_bytes(w, gated=False) -> int:
    """Bytes the method must move per launch: u in, y out (I/O dtype) and k_f once
    per channel, counted as 16-bit (re, im) pairs whatever the stored format; the gated
    form reads two more tensors of the shape of u."""
    s = 4 if w.dtype == "f32" else 2
    return (4 if gated else 2) * w.B * w.H * w.N * s + w.H * w.fft_size * 4


def mfma_flops(w, path, factors) -> float:
    """Floating-point operations per launch that the plan's decomposition runs on the matrix cores: complex
    DFT-matrix products at 8 real operations per complex multiply-add, two batch rows per complex transform.
    Single-kernel plans (factors N1, N2, N3): the outermost stage skips its zero half in both directions,
    8 M N1 + 16 M (N2 + N3) per pair (8192-point kernel: N1 = 32 whatever the plan's transform length).
    Multi-pass plans: the inner 8192-point transforms on complex rows, 16 * 8192 * (32 + 16 + 16) per row,
    fft_size / 8192 rows per pair; their outer passes run on the vector ALUs.  Other paths use no matrix cores."""
    pairs = ((w.B + 1) // 2) * w.H
    if path == "fused3":
        if w.fft_size <= 8192:
            groups = 8192 // w.fft_size
            return ((w.B + 2 * groups - 1) // (2 * groups)) * w.H * (8.0 * 8192 * 32 + 16.0 * 8192 * 32)
        n1, n2, n3 = factors
        return pairs * (8.0 * w.fft_size * n1 + 16.0 * w.fft_size * (n2 + n3))
    if path == "multipass":
        return pairs * (w.fft_size // 8192) * 16.0 * 8192 * 64
    return 0.0


def time_oracle(w, u_cpu, k, budget_s=12.0):
    """Oracle throughput on the host cores over a bounded sample of the same workload."""
    import numpy as np
    import oracle

    kext = oracle.extend_filter(k, w.fft_size)
    n_probe = min(w.H, 16)
    t0 = time.perf_counter()
    oracle.fftconv(u_cpu[:1, :n_probe].double().numpy(), kext[:n_probe])
    per_seq = (time.perf_counter() - t0) / n_probe * max(1, oracle.num_threads())   # core-seconds per sequence
    n_seq = int(budget_s * oracle.num_threads() / max(per_seq, 1e-9))
    n_h = min(w.H, max(1, n_seq))
    n_b = min(u_cpu.shape[0], max(1, n_seq // n_h))
    uu = u_cpu[:n_b, :n_h].double().numpy()
    t0 = time.perf_counter()
    oracle.fftconv(uu, kext[:n_h])
    dt = time.perf_counter() - t0
    return {
        "value": n_b * n_h / (dt * 1e3),
        "unit": "sequences/ms",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": "first %d batch rows x first %d channels of the same workload (%d sequences, %.1f s)"
                  % (n_b, n_h, n_b * n_h, dt),
    }


def sustained_power(torch, step, ms_per_step, seconds=2.0):
    """Package power while the step runs back to back for about two seconds (outside the timed region), with the
    board's power cap: the hwmon files of the amdgpu driver, read-only; None where they cannot be read."""
    import glob
    files = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") or \
        glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average")
    if not files:
        return None
    def read(path):
        try:
            with open(path) as f:
                return int(f.read()) / 1e6
        except (OSError, ValueError):
            return None
    cap = read(files[0].rsplit("/", 1)[0] + "/power1_cap")
    n = max(1, int(seconds * 1e3 / ms_per_step / 8))
    samples = []
    for i in range(8):                         # 8 bursts; the sensor is read while the queue is still full
        for _ in range(n):
            step()
        if i >= 3:
            v = read(files[0])
            if v is not None:
                samples.append(v)
        torch.cuda.synchronize()
    if not samples:
        return None
    return {"socket_W": sum(samples) / len(samples), "cap_W": cap, "samples": len(samples)}


def sweep(torch, fftconv, synth, dev, args):
    """Forward pass, bf16, B*H*N = 2^27 elements at every size (B*H >= 1): causal (N = fft/2) or,
    with --circular, the input filling the transform (N = fft)."""
    for lg in range(8, 23):
        M = 1 << lg
        N = M if args.circular else M // 2
        rows = max(1, (1 << 27) // N)
        # at least two batch rows where there are two rows at all: the 16-bit kernels transform rows in pairs,
        # and with B = 1 (config 4's shape, see the default mode) half of every transform is padding
        H = min(768, max(1, rows // 2))
        B = max(1, rows // H)
        plan = fftconv.Plan(N, M, H, "bf16")
        g = torch.Generator(device="cpu").manual_seed(lg)
        k = (torch.randn(H, N, generator=g) * torch.exp(-1e-3 * torch.arange(N))[None]).to(dev)
        kf = plan.filter_fft(k)
        u = torch.randn(B, H, N, generator=g).to(torch.bfloat16).to(dev)
        y = torch.empty_like(u)
        steps = max(3, min(args.steps, 20))
        # settle: the step back to back for about 60 ms (the core clock of an idle chip takes that long to come up)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        spun = 0.0
        while spun < 60.0:
            e0.record()
            for _ in range(8):
                plan.forward(u, kf, out=y)
            e1.record()
            torch.cuda.synchronize()
            spun += e0.elapsed_time(e1)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            plan.forward(u, kf, out=y)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        nbytes = 2 * B * H * N * 2 + H * M * 4
        # Section 3.2, Eq. 2 with this chip's constants: the order it would pick and its cost for this batch
        mach = fftconv.machine_preset(fftconv.MACHINE_MI355X)
        mp, mf, mc = fftconv.plan_order(mach, M)
        print(json.dumps({"fft_size": M, "N": N, "B": B, "H": H, "form": "circular" if args.circular else "causal",
                          "model_order": mp, "model_factors": mf, "model_ms": mc * B * H * 1e3,
                          "path": plan.path, "factors": plan.factors,
                          "ms_per_step": ms, "sequences_per_ms": B * H / ms, "achieved_TBps": nbytes / ms / 1e9}),
              flush=True)
        del plan, kf, u, y, k


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # The paper times each call 30 times (Appendix C).  On this GPU the core clock needs tens of
    # milliseconds of load to settle, so the defaults run longer: ~0.1 s of warm-up, ~0.1 s timed.
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--settle-ms", type=float, default=200.0,
                    help="untimed clock-settle phase before the warm-up: the step runs back to back for at "
                         "least this many milliseconds (0 = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true",
                    help="forward pass over every power-of-two fft size 256 .. 4M at a fixed amount of data "
                         "(one JSON line per size; not the headline metric)")
    ap.add_argument("--circular", action="store_true", help="with --sweep: N = fft_size instead of fft_size / 2")
    ap.add_argument("--backward", action="store_true",
                    help="time the backward pass (du and dk) instead (not the headline metric)")
    ap.add_argument("--gated", action="store_true",
                    help="time the gated form y = v . ((u . w) * k) instead (not the headline metric)")
    ap.add_argument("--digit-keep", default=None,
                    help="comma-separated kept values per digit of the plan's factorisation (Appendix A.4 cut-off "
                         "pattern): time fftconv_forward_freq_sparse_digits against the dense call on the same k_f")
    ap.add_argument("--lean", action="store_true",
                    help="warm-up and timed steps only (no cold figure, settle phase, per-launch events or power "
                         "sampling): the form the counter-collecting rocprofv3 runs use")
    ap.add_argument("--constants", action="store_true",
                    help="measure the machine constants of the cost model (Section 3.2, Appendix C) with the library's "
                         "micro-benchmark kernels and print them beside the built-in preset (not the headline metric)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain elementwise copy of %d MiB (read once, written once) before the "
                         "warm-up, as the known-size reference for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE" % (COPY_BYTES >> 20))
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (sequences are independent: shard channels, then batch "
              "rows, with no collective); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2311_05908_amd import fftconv, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.sweep:
        sweep(torch, fftconv, synth, dev, args)
        return
    if args.constants:
        names = ("sigma_H", "sigma_S", "tau_M", "tau_G")
        runs = [fftconv.measure_machine() for _ in range(3)]
        med = {n: sorted(getattr(r, n) for r in runs)[1] for n in names}
        pre = fftconv.machine_preset(fftconv.MACHINE_MI355X)
        print(json.dumps({"metric": "machine constants of the cost model (Eq. 2), median of 3 measurements",
                          "units": {"sigma_H": "B/s", "sigma_S": "B/s", "tau_M": "FLOP/s", "tau_G": "FLOP/s"},
                          "measured": med, "preset": {n: getattr(pre, n) for n in names},
                          "runs": [{n: getattr(r, n) for n in names} for r in runs], "data": "synthetic", "n_gpus": 1}))
        return
    w = synth.WORKLOADS[args.workload]

    t0 = time.perf_counter()
    u_cpu = synth.gen_u(w)
    k = synth.gen_k(w)
    t_gen = time.perf_counter() - t0
    plan = fftconv.Plan(w.N, w.fft_size, w.H, w.dtype)
    kd = torch.from_numpy(k[:, : w.filter_len].copy()).to(dev)
    bk = synth.block_keep(w) if w.n_blocks else None
    kf = plan.filter_fft(kd, block_keep=bk)
    u = u_cpu.to(dev)
    y = torch.empty_like(u)
    gw = synth.gen_gate(w, "w").to(dev) if args.gated else None
    gv = synth.gen_gate(w, "v").to(dev) if args.gated else None
    torch.cuda.synchronize()

    if args.copy_calibration:
        src = torch.zeros(COPY_BYTES // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)           # one elementwise kernel: COPY_BYTES read, COPY_BYTES written
        torch.cuda.synchronize()
        del src, dst

    if args.digit_keep:
        keep = [int(x) for x in args.digit_keep.split(",")]
        kfd = plan.filter_fft_sparse_digits(kd, keep)
        times = {}
        # two rounds, the second one counts: the core clock is still settling during the first
        for name, fn in 2 * (("dense", lambda: plan.forward(u, kfd, out=y)),
                             ("skipping", lambda: plan.forward_freq_sparse_digits(u, kfd, keep, out=y))):
            for _ in range(min(args.warmup, 20)):
                fn()
            torch.cuda.synchronize()
            b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            n_it = max(3, min(args.steps, 100))
            b0.record()
            for _ in range(n_it):
                fn()
            b1.record()
            torch.cuda.synchronize()
            times[name] = b0.elapsed_time(b1) / n_it
        print(json.dumps({"metric": "digit cut-off FFT-conv ms per call", "unit": "ms", "n_gpus": 1, "data": "synthetic",
                          "dtype": w.dtype, "value": times["skipping"], "higher_is_better": False,
                          "config": {"workload": "%s digit cut-off: B=%d H=%d N=%d fft_size=%d" %
                                     (w.name, w.B, w.H, w.N, w.fft_size),
                                     "factors": plan.factors, "digit_keep": keep, "dense_ms": times["dense"],
                                     "speedup_vs_dense": times["dense"] / times["skipping"], "path": plan.path}}))
        return

    if args.backward:
        dy = synth.gen_gate(w, "dy").to(dev)
        kfa = plan.filter_fft_adjoint(kd)
        dk = torch.empty((w.H, w.filter_len), dtype=torch.float32, device=dev)
        du = torch.empty_like(u)
        times = {}
        # the calls of a training step besides the forward pass: k changes every step, so both filter
        # transforms are part of it
        for name, fn in (("filter_fft", lambda: plan.filter_fft(kd)),
                         ("filter_fft_adjoint", lambda: plan.filter_fft_adjoint(kd)),
                         ("du", lambda: plan.backward_input(dy, kfa, out=du)),
                         ("dk", lambda: plan.backward_filter(u, dy, w.filter_len, out=dk))):
            n_it = max(3, min(args.steps, 30))
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            b0.record()
            for _ in range(n_it):
                fn()
            b1.record()
            torch.cuda.synchronize()
            times[name] = b0.elapsed_time(b1) / n_it
        print(json.dumps({"metric": "backward FFT-conv ms per call", "unit": "ms", "n_gpus": 1, "data": "synthetic",
                          "dtype": w.dtype, "value": times["du"] + times["dk"], "higher_is_better": False,
                          "config": {"workload": "%s backward: B=%d H=%d N=%d fft_size=%d Nk=%d" %
                                     (w.name, w.B, w.H, w.N, w.fft_size, w.filter_len),
                                     "du_ms": times["du"], "dk_ms": times["dk"], "filter_fft_ms": times["filter_fft"],
                                     "filter_fft_adjoint_ms": times["filter_fft_adjoint"], "path": plan.path}}))
        return

    def step():
        if args.gated:
            plan.forward_gated(u, gw, gv, kf, out=y)
        elif bk is not None:
            plan.forward_freq_sparse(u, kf, bk, out=y)
        elif w.Nk:
            plan.forward_partial(u, kf, w.Nk, out=y)
        else:
            plan.forward(u, kf, out=y)

    def timed(n):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(n):
            step()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    # The same protocol on a cold chip first (warm-up, then the timed steps): with a few steps the core
    # clock is still ramping up from idle and the figure is slower; reported as config.ms_per_step_cold.
    for _ in range(0 if args.lean else args.warmup):
        step()
    ms_cold = None if args.lean else timed(args.steps)
    # Clock-settle phase (untimed, disclosed as config.settle_ms): the same step back to back for at least
    # --settle-ms of GPU time, so that the timed region below measures the kernel at the clock the chip
    # sustains under this load, whatever --steps / --warmup are.
    settle_ms = 0.0
    while not args.lean and settle_ms < args.settle_ms:
        n = max(8, int(25.0 / max(ms_cold, 1e-3)))
        settle_ms += timed(n) * n
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # HIP events on the stream the kernels are launched on (torch's current stream).  The timed
    # region is bracketed by two events only: an event per launch would put a marker packet
    # between the kernels and stretch every step.
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t_wall0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    t_wall = time.perf_counter() - t_wall0
    ms_per_step = e0.elapsed_time(e1) / args.steps
    assert torch.isfinite(y.float()).all(), "non-finite output"
    dense_ms = None
    if (bk is not None or w.Nk) and not args.gated and not args.lean:
        # sparse workloads: the dense entry point on the same (masked / truncated) k_f, for the speed-up
        for _ in range(args.warmup):
            plan.forward(u, kf, out=y)
        d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        d0.record()
        for _ in range(args.steps):
            plan.forward(u, kf, out=y)
        d1.record()
        torch.cuda.synchronize()
        dense_ms = d0.elapsed_time(d1) / args.steps

    # distribution over single launches: one event between consecutive launches (the marker packets
    # stretch a step by a few microseconds, which is why the headline figure uses the two-event bracket)
    n_ev = 2 if args.lean else max(2, min(args.steps, 200))
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_ev + 1)]
    torch.cuda.synchronize()
    evs[0].record()
    for i in range(n_ev):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    per = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(n_ev))
    per_launch = {"n": n_ev, "mean": sum(per) / n_ev, "median": per[n_ev // 2], "min": per[0], "max": per[-1]}
    power = None if args.lean else sustained_power(torch, step, ms_per_step)
    nseq = w.B * w.H
    abytes = algorithmic_bytes(w, args.gated)
    avg_kernel_ms = ms_per_step          # one kernel launch per step on the fused paths
    achieved = abytes / (avg_kernel_ms * 1e-3) / 1e9
    flops = mfma_flops(w, plan.path, plan.factors)
    mfma_tflops = flops / (avg_kernel_ms * 1e-3) / 1e12
    hbm_frac, mfma_frac = achieved / HBM_PEAK_GBS, mfma_tflops / MFMA_PEAK_TFLOPS
    out = {
        "metric": ("gated " if args.gated else "") + "FFT-conv sequences/ms + achieved HBM TB/s at B=%d,H=%d,N=%d %s"
                  % (w.B, w.H, w.N, w.dtype),
        "value": nseq / ms_per_step,
        "unit": "sequences/ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: %scausal FFT conv B=%d H=%d N=%d fft_size=%d %s I/O, fp32 accumulate"
                               % (w.name, "gated " if args.gated else "", w.B, w.H, w.N, w.fft_size, w.dtype),
                   "path": plan.path, "factors": plan.factors,
                   "achieved_TBps": achieved / 1e3, "wall_ms_per_step": t_wall / args.steps * 1e3,
                   "input_gen_s": t_gen,
                   "settle_ms": settle_ms, "ms_per_step_cold": ms_cold,
                   "sequences_per_ms_cold": None if ms_cold is None else nseq / ms_cold,
                   "per_launch_ms": per_launch,
                   "power": power,
                   "dense_ms_per_step": dense_ms,
                   "speedup_vs_dense": None if dense_ms is None else dense_ms / ms_per_step},
        # bound: the roof the kernel is nearer to (fraction of the HBM peak on algorithmic bytes against
        # fraction of the matrix-core peak on the decomposition's operations); neither is reached: the
        # profiles show the step paced by vector-instruction issue ("limiter")
        "roofline": {"bound": "hbm" if hbm_frac >= mfma_frac else "mfma", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": hbm_frac, "traffic": None if args.gated else measured_traffic(w.name),
                     "mfma_frac": mfma_frac, "mfma_achieved": mfma_tflops, "mfma_peak": MFMA_PEAK_TFLOPS,
                     "mfma_unit": "TFLOP/s", "mfma_flops": flops,
                     "limiter": ("HBM traffic of the workspace (three passes, measured traffic about 2 x the algorithmic bytes, "
                                 "moved at 3.4-4.7 TB/s; profiles/multipass_cfg4.md)" if plan.path == "multipass" else
                                 "vector-instruction issue (SQ_INSTS_VALU against SQ_BUSY_CYCLES in profiles/)"),
                     "kernel": ("k_fused3_ws" if w.fft_size == 8192 else "k_fused3_big") if plan.path == "fused3" else plan.path,
                     "algorithmic_bytes": abytes},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = time_oracle(w, u_cpu, k)     # the convolution itself; the gates add O(N) per sequence
    print(json.dumps(out))


if __name__ == "__main__":
    main()
