"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI
and compare it with the CPU oracle on the same seeded inputs."""
import numpy as np
import torch

import oracle
from paper_2311_05908_amd import fftconv, synth

TOL = {"f32": 1e-5, "f16": 1e-2, "bf16": 1e-2}     # max per-sequence relative L2 error
ELEM_FACTOR = 8.0                                  # element-wise bound: |y_i - ref_i| <= ELEM_FACTOR * tol * rms(ref)


def parity_error(y, ref, tol, what="", weight=None, floor_rms=None):
    """Compare along the last axis (one sequence per row).  Returns the largest per-sequence relative L2 error
    (the caller asserts it against tol) and itself asserts the element-wise bound

        max_i |y_i - ref_i| <= ELEM_FACTOR * tol * rms(ref)        per sequence.

    The norm alone lets a single wrong element pass once N is large (one element of size rms(ref) moves the
    relative L2 error of a 16384-point row by 1/128); the element-wise bound does not.  With rounding errors
    only, the largest element error of a 16-bit path is about 0.03 rms(ref) (4.5 sigma of an error of relative
    L2 size 5e-3, plus half a unit in the last place of the largest outputs), of an fp32 path about 1e-6.
    weight (same shape as y, optional) multiplies the bound element by element where it exceeds 1: the output
    gate of the gated form scales the convolution's error at position i by |v_i|, and |v_i| reaches 4.
    floor_rms (one value per sequence, optional): rms of the UNTRUNCATED circular result, all fft_size outputs
    of the inverse transform.  Rounding errors are spread evenly over those outputs, so when the N kept ones
    hold almost none of the energy (a late unit tap: y = 0 except for its last sample) the error relative to
    the kept outputs alone says nothing about the arithmetic; both measures then use max(rms(ref), floor_rms)."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert y.shape == ref.shape, (y.shape, ref.shape)
    assert np.isfinite(y).all(), "non-finite output %s" % what
    if y.size == 0:
        return 0.0
    rms = np.sqrt((ref ** 2).mean(axis=-1))
    if floor_rms is not None:
        rms = np.maximum(rms, np.asarray(floor_rms, dtype=np.float64))
    worst = np.abs(y - ref).max(axis=-1)
    bound = ELEM_FACTOR * tol * np.where(rms > 0, rms, 1.0)
    if weight is not None:
        worst = (np.abs(y - ref) / np.maximum(1.0, np.abs(np.asarray(weight, dtype=np.float64)))).max(axis=-1)
    bad = worst > bound
    assert not bad.any(), "element-wise bound exceeded %s: worst |y - ref| / rms(ref) = %.3e (limit %.3e) in sequence %s" % (
        what, float((worst / np.where(rms > 0, rms, 1.0)).max()), ELEM_FACTOR * tol, np.argwhere(bad)[0].tolist())
    if floor_rms is not None:
        return float(np.max(np.sqrt(((y - ref) ** 2).mean(axis=-1)) / np.where(rms > 0, rms, 1.0)))
    return float(np.max(oracle.rel_l2_per_sequence(y, ref)))


def oracle_filter(w, k):
    """Filter the oracle convolves with, on fft_size taps (fp64)."""
    kext = oracle.extend_filter(k, w.fft_size)
    if w.n_blocks:
        keep = np.repeat(synth.block_keep(w), w.fft_size // w.n_blocks)
        return None, keep, kext
    return kext, None, None


def gpu_forward(w, u_cpu, k, variant="dense", path=None):
    plan = fftconv.Plan(w.N, w.fft_size, w.H, w.dtype, path=path)
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


def check_all_sequences(w, variant="dense", path=None):
    """Every sequence of a (small) workload against the oracle; returns the max error.
    path: force a kernel family instead of the cost model's choice."""
    u = synth.gen_u(w)
    k = synth.gen_k(w)
    y, plan = gpu_forward(w, u, k, variant, path)
    kext, keep, kfull = oracle_filter(w, k)
    if keep is not None:
        kext = oracle.mask_filter(kfull, keep)
    ref = oracle.fftconv(u.double().numpy(), kext)
    return parity_error(y.double().numpy(), ref, TOL[w.dtype], "%s %s" % (w.name, variant)), plan


def check_sampled_positions(w, n_pos=48, variant="dense", seed=11, edge=1):
    """Long sequences: every sequence of the workload, but only sampled output positions (the first `edge`
    and the last `edge` positions always included, the rest drawn at random), each evaluated by the oracle
    as its own sum."""
    u = synth.gen_u(w)
    k = synth.gen_k(w)
    y, plan = gpu_forward(w, u, k, variant)
    assert torch.isfinite(y.float()).all()
    kext = oracle.extend_filter(k, w.fft_size)
    g = np.random.Generator(np.random.Philox(key=[seed, w.N]))
    S = w.B * w.H
    idx = g.integers(0, w.N, size=(S, n_pos))
    assert 2 * edge <= n_pos
    idx[:, :edge] = np.arange(edge)[None]
    idx[:, edge:2 * edge] = (w.N - 1 - np.arange(edge))[None]
    u_rows = u.double().numpy().reshape(S, w.N)
    k_rows = np.tile(kext, (w.B, 1))
    ref = oracle.fftconv_at(u_rows, k_rows, idx)
    got = np.take_along_axis(y.double().numpy().reshape(S, w.N), idx, axis=1)
    # relative L2 over the sampled positions, and every sampled element on its own
    return parity_error(got, ref, TOL[w.dtype], "%s sampled positions" % w.name), plan
