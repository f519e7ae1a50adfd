"""Digit cut-off patterns of the frequency-sparse convolution (Appendix A.4) against the oracle: the filter's
spectrum is masked per bin by the pattern, the oracle convolves with Re(IDFT(mask . DFT(k)))."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_05908_amd import fftconv, synth
from parity_util import TOL, parity_error

pytestmark = pytest.mark.gpu
W = synth.WORKLOADS


def run(dtype, B, H, N, M, digit_keep):
    w = synth.scaled(W["cfg2"], B=B, H=H, N=N, fft_size=M, dtype=dtype, alpha=(1e-2, 1e-1))
    u = synth.gen_u(w)
    k = synth.gen_k(w)
    plan = fftconv.Plan(N, M, H, dtype)
    assert len(digit_keep) == len(plan.factors)
    kd = torch.from_numpy(k[:, : w.filter_len].copy()).cuda()
    kf = plan.filter_fft_sparse_digits(kd, digit_keep)
    ud = u.cuda()
    y_dense = plan.forward(ud, kf).cpu()
    y_skip = plan.forward_freq_sparse_digits(ud, kf, digit_keep).cpu()
    torch.cuda.synchronize()
    keep = synth.digit_keep_mask(plan.factors, digit_keep)
    kmasked = oracle.mask_filter(oracle.extend_filter(k, M), keep)
    ref = oracle.fftconv(u.double().numpy(), kmasked)
    e_dense = parity_error(y_dense.double().numpy(), ref, TOL[dtype], "dense")
    e_skip = parity_error(y_skip.double().numpy(), ref, TOL[dtype], "skip")
    print("digits %s B=%d H=%d N=%d M=%d path=%s factors=%s keep=%s kept bins %.1f%% err dense %.3e skip %.3e"
          % (dtype, B, H, N, M, plan.path, plan.factors, list(digit_keep), 100.0 * keep.mean(), e_dense, e_skip), flush=True)
    return plan, e_dense, e_skip


@pytest.mark.parametrize("dtype,B,H,N,M,digit_keep", [
    ("bf16", 4, 3, 4096, 8192, (32, 16, 16)),       # nothing cut: the plain convolution
    ("bf16", 4, 3, 4096, 8192, (32, 16, 8)),        # innermost digit (the paper's first dimension)
    ("f16", 3, 2, 4096, 8192, (8, 16, 16)),         # per-plane loop of the innermost kernel: 8 of 32 planes live
    ("bf16", 2, 2, 4096, 8192, (1, 1, 1)),          # only the bin f = 0
    ("f16", 5, 1, 4096, 8192, (12, 8, 6)),          # every digit cut
    ("bf16", 4, 2, 8192, 16384, (32, 16, 8)),       # the empty tile of the innermost digit is skipped
    ("bf16", 2, 2, 8192, 16384, (10, 16, 16)),
    ("f16", 2, 1, 16384, 32768, (16, 16, 16)),
    ("f16", 2, 1, 16384, 32768, (32, 15, 32)),      # middle digit: its second tile is left out of stages 2 and 3
    ("bf16", 3, 2, 16384, 32768, (8, 15, 15)),      # all three at once: planes, k2 tile, k3 tile
    ("bf16", 2, 2, 16384, 32768, (8, 32, 32)),      # k1 planes only: one live plane per wave
    ("bf16", 4, 2, 8192, 16384, (8, 16, 32)),       # the same at fft 16384
    ("f16", 3, 2, 8192, 16384, (5, 16, 10)),        # planes and the k3 tile
    ("bf16", 2, 1, 8192, 16384, (1, 1, 1)),         # a single live plane in the whole workgroup
    ("bf16", 1, 1, 32768, 65536, (4, 32, 16, 16)),  # outer digit: rows of the inner kernel that are never touched
    ("f16", 2, 1, 32768, 65536, (3, 8, 16, 8)),
    ("bf16", 3, 2, 1 << 17, 1 << 18, (9, 32, 16, 16)),   # odd batch: the last row goes through the real-row passes, sparse
    ("f16", 1, 2, 1 << 16, 1 << 17, (16, 32, 16, 16)),   # a single row, half of the outer digit kept
    ("bf16", 2, 2, 8192, 8192, (1, 32, 16, 4)),     # circular, multi-pass route without an outer transform
    ("f32", 2, 2, 512, 1024, (16, 8)),              # short-transform kernel
    ("f32", 1, 2, 4096, 8192, (16, 16, 4, 2)),      # generic per-stage path
])
def test_digit_patterns(dtype, B, H, N, M, digit_keep):
    plan, e_dense, e_skip = run(dtype, B, H, N, M, digit_keep)
    assert e_dense <= TOL[dtype]
    assert e_skip <= TOL[dtype]


def test_bad_patterns_are_rejected():
    plan = fftconv.Plan(4096, 8192, 2, "bf16")
    k = torch.randn(2, 4096, device="cuda")
    with pytest.raises(fftconv.FFTConvError):
        plan.filter_fft_sparse_digits(k, (32, 16))              # one entry per factor
    with pytest.raises(fftconv.FFTConvError):
        plan.filter_fft_sparse_digits(k, (33, 16, 16))          # more than the digit has
    with pytest.raises(fftconv.FFTConvError):
        plan.filter_fft_sparse_digits(k, (32, 0, 16))
