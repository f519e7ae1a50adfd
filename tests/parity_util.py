"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI
and compare it with the CPU oracle on the same seeded inputs."""
import numpy as np
import torch

import oracle
from paper_2311_05908_amd import fftconv, synth

TOL = {"f32": 1e-5, "f16": 1e-2, "bf16": 1e-2}     # max per-sequence relative L2 error


def oracle_filter(w, k):
    """Filter the oracle convolves with, on fft_size taps (fp64)."""
    kext = oracle.extend_filter(k, w.fft_size)
    if w.n_blocks:
        keep = np.repeat(synth.block_keep(w), w.fft_size // w.n_blocks)
        return None, keep, kext
    return kext, None, None


def gpu_forward(w, u_cpu, k, variant="dense"):
    plan = fftconv.Plan(w.N, w.fft_size, w.H, w.dtype)
    kd = torch.from_numpy(k[:, : w.filter_len].copy()).cuda()
    if w.n_blocks:
        bk = synth.block_keep(w)
        kf = plan.filter_fft(kd, block_keep=bk)
        y = plan.forward_freq_sparse(u_cpu.cuda(), kf, bk) if variant == "skip" else plan.forward(u_cpu.cuda(), kf)
    else:
        kf = plan.filter_fft(kd)
        if variant == "skip" and w.Nk:
            y = plan.forward_partial(u_cpu.cuda(), kf, w.Nk)
        else:
            y = plan.forward(u_cpu.cuda(), kf)
    torch.cuda.synchronize()
    return y.cpu(), plan


def check_all_sequences(w, variant="dense"):
    """Every sequence of a (small) workload against the oracle; returns the max error."""
    u = synth.gen_u(w)
    k = synth.gen_k(w)
    y, plan = gpu_forward(w, u, k, variant)
    kext, keep, kfull = oracle_filter(w, k)
    if keep is not None:
        kext = oracle.mask_filter(kfull, keep)
    ref = oracle.fftconv(u.double().numpy(), kext)
    assert torch.isfinite(y.float()).all()
    err = oracle.rel_l2_per_sequence(y.double().numpy(), ref)
    return float(err.max()), plan


def check_sampled_positions(w, n_pos=48, variant="dense", seed=11):
    """Long sequences: every sequence of the workload, but only sampled output positions
    (first and last sample always included), each evaluated by the oracle as its own sum."""
    u = synth.gen_u(w)
    k = synth.gen_k(w)
    y, plan = gpu_forward(w, u, k, variant)
    assert torch.isfinite(y.float()).all()
    kext = oracle.extend_filter(k, w.fft_size)
    g = np.random.Generator(np.random.Philox(key=[seed, w.N]))
    S = w.B * w.H
    idx = g.integers(0, w.N, size=(S, n_pos))
    idx[:, 0] = 0
    idx[:, 1] = w.N - 1
    u_rows = u.double().numpy().reshape(S, w.N)
    k_rows = np.tile(kext, (w.B, 1))
    ref = oracle.fftconv_at(u_rows, k_rows, idx)
    got = np.take_along_axis(y.double().numpy().reshape(S, w.N), idx, axis=1)
    err = oracle.rel_l2_per_sequence(got, ref)          # relative L2 over the sampled positions
    return float(err.max()), plan
