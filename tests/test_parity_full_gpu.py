"""Parity at the full benchmark sizes, in the launch configuration bench.py times:
the whole batch runs on the GPU, and a deterministic sample of sequences (all four
corners of the (B, H) grid plus random picks) is compared with the oracle, which
evaluates each sampled sequence on its own."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_05908_amd import fftconv, synth
from parity_util import TOL, parity_error

pytestmark = pytest.mark.gpu
W = synth.WORKLOADS


def run_full(w, n_random, variant="dense"):
    k = synth.gen_k(w)
    plan = fftconv.Plan(w.N, w.fft_size, w.H, w.dtype)
    kd = torch.from_numpy(k[:, : w.filter_len].copy()).cuda()
    bk = synth.block_keep(w) if w.n_blocks else None
    kf = plan.filter_fft(kd, block_keep=bk)
    u_cpu = synth.gen_u(w)
    u = u_cpu.cuda()
    if variant == "skip" and bk is not None:
        y = plan.forward_freq_sparse(u, kf, bk)
    elif variant == "skip" and w.Nk:
        y = plan.forward_partial(u, kf, w.Nk)
    else:
        y = plan.forward(u, kf)
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all()
    pts = synth.sample_sequences(w, n_random)
    kext = oracle.extend_filter(k, w.fft_size)
    if bk is not None:
        hs = sorted({h for _, h in pts})
        keep = np.repeat(bk, w.fft_size // w.n_blocks)
        masked = oracle.mask_filter(kext[hs], keep)
        kext = {h: masked[i] for i, h in enumerate(hs)}
    worst = 0.0
    for b, h in pts:
        ref = oracle.fftconv(u_cpu[b, h].double().numpy()[None, None], np.asarray(kext[h])[None])[0, 0]
        err = parity_error(y[b, h].cpu().double().numpy(), ref, TOL[w.dtype], "%s b=%d h=%d" % (w.name, b, h))
        worst = max(worst, err)
    return worst, plan, y


def test_cfg2_full_size_sampled_sequences():
    w = W["cfg2"]
    worst, plan, y = run_full(w, 44)
    print("cfg2 full: path=%s worst sampled rel L2 = %.3e" % (plan.path, worst), flush=True)
    assert plan.path == "fused3"
    assert worst <= TOL[w.dtype]
    # run-to-run determinism: no atomics on the path, so a second launch is bit-identical
    u = synth.gen_u(w).cuda()
    k = synth.gen_k(w)
    kf = plan.filter_fft(torch.from_numpy(k).cuda())
    y2 = plan.forward(u, kf)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)


def test_cfg3_full_size_sampled_sequences():
    w = W["cfg3"]
    worst, plan, _ = run_full(w, 8)
    print("cfg3 full: path=%s factors=%s worst sampled rel L2 = %.3e" % (plan.path, plan.factors, worst), flush=True)
    assert worst <= TOL[w.dtype]


def test_cfg5a_partial_full_size_both_entry_points():
    w = W["cfg5a"]
    for variant in ("dense", "skip"):
        worst, plan, _ = run_full(w, 12, variant=variant)
        print("cfg5a full %s: path=%s worst sampled rel L2 = %.3e" % (variant, plan.path, worst), flush=True)
        assert worst <= TOL[w.dtype]


def test_cfg5b_frequency_sparse_full_size_both_entry_points():
    w = W["cfg5b"]
    for variant in ("dense", "skip"):
        worst, plan, _ = run_full(w, 4, variant=variant)
        print("cfg5b full %s: path=%s worst sampled rel L2 = %.3e" % (variant, plan.path, worst), flush=True)
        assert worst <= TOL[w.dtype]


def test_cfg4_very_long_full_size_sampled_positions():
    from parity_util import check_sampled_positions
    w = W["cfg4"]
    # 8192 positions per channel: the first 1024, the last 1024 and 6144 drawn at random
    err, plan = check_sampled_positions(w, n_pos=8192, edge=1024)
    print("cfg4 full: path=%s factors=%s worst rel L2 over 8192 sampled positions = %.3e" % (plan.path, plan.factors, err),
          flush=True)
    assert plan.path == "multipass"
    assert err <= TOL[w.dtype]
