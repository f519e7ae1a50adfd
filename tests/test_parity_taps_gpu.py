"""Parity on filters with few non-zero taps, every output checked at full length on every path.

Decaying random filters barely weight their late taps, so a wrong mapping of late taps (in the outer
passes of the long plans, in the k_f rows of the multi-pass route) could hide below a 1e-2 norm.  Here
every channel carries a unit tap at 0, 1, L/2 or L-1, or 16 taps of unit magnitude spread over [0, L)
(synth.gen_taps), with L = N for the causal shapes and L = fft_size for the circular ones (where the
wrapped taps are the late ones).  The oracle evaluates the convolution's definition tap by tap
(oracle.fftconv_taps, O(16 N) per sequence), so all N outputs of every sequence are compared, in the
relative L2 norm and element by element."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_05908_amd import fftconv, synth
from parity_util import TOL, parity_error

pytestmark = pytest.mark.gpu
W = synth.WORKLOADS


def run_taps(dtype, B, H, N, M, seed=77):
    w = synth.scaled(W["cfg2"], B=B, H=H, N=N, fft_size=M, dtype=dtype)
    L = M if N == M else N                  # circular shapes: taps anywhere on the circle
    pos, val = synth.gen_taps(H, L, seed)
    k = synth.taps_to_filter(pos, val, L)
    u = synth.gen_u(w)
    plan = fftconv.Plan(N, M, H, dtype)
    kf = plan.filter_fft(torch.from_numpy(k).cuda())
    y = plan.forward(u.cuda(), kf)
    torch.cuda.synchronize()
    ref = oracle.fftconv_taps(u.double().numpy(), pos, val, M)
    # all fft_size outputs of the circular convolution (the input zero-padded to the transform length): a unit
    # tap at N-1 leaves one non-zero sample among the N kept ones, so the error is measured against the rms of
    # the whole result where that is larger (see parity_error)
    upad = np.zeros((B, H, M))
    upad[..., :N] = u.double().numpy()
    full_rms = np.sqrt((oracle.fftconv_taps(upad, pos, val, M) ** 2).mean(axis=-1))
    del upad
    err = parity_error(y.cpu().double().numpy(), ref, TOL[dtype], "taps %s B=%d H=%d N=%d M=%d" % (dtype, B, H, N, M),
                       floor_rms=full_rms)
    print("taps %s B=%d H=%d N=%d M=%d path=%s factors=%s max rel L2 = %.3e" % (dtype, B, H, N, M, plan.path, plan.factors, err),
          flush=True)
    assert err <= TOL[dtype]
    return plan


@pytest.mark.parametrize("dtype,B,H,N,M,path", [
    ("f32", 2, 5, 1024, 2048, "small"),
    ("bf16", 4, 5, 1024, 2048, "fused3"),        # four transforms per work item of the 8192-point kernel
    ("bf16", 2, 5, 4096, 8192, "fused3"),
    ("f16", 3, 5, 4096, 8192, "fused3"),
    ("f16", 3, 5, 8192, 16384, "fused3"),
    ("bf16", 2, 10, 8192, 16384, "fused3"),
    ("bf16", 2, 5, 16384, 32768, "fused3"),
    ("f16", 3, 5, 16384, 32768, "fused3"),
    ("bf16", 2, 5, 1 << 17, 1 << 18, "multipass"),
    ("f16", 1, 5, 1 << 17, 1 << 18, "multipass"),
    ("f32", 2, 5, 4096, 8192, "staged"),
    ("f32", 2, 5, 8192, 16384, "staged"),
    ("f32", 1, 5, 16384, 32768, "staged"),
    ("f32", 1, 5, 1 << 17, 1 << 18, "staged"),
    ("f32", 1, 5, 1 << 20, 1 << 21, "staged"),
])
def test_sparse_tap_filters_causal_all_outputs(dtype, B, H, N, M, path):
    assert run_taps(dtype, B, H, N, M).path == path


@pytest.mark.parametrize("dtype,B,H,M,path", [
    ("f32", 2, 5, 4096, "small"),
    ("bf16", 2, 5, 8192, "multipass"),
    ("f16", 2, 5, 16384, "multipass"),
    ("bf16", 2, 5, 32768, "multipass"),
    ("bf16", 1, 5, 1 << 18, "multipass"),
    ("f16", 2, 5, 1 << 19, "multipass"),
    ("bf16", 2, 5, 1 << 21, "multipass"),
    ("f32", 2, 5, 8192, "staged"),
    ("f32", 1, 5, 32768, "staged"),
    ("f32", 1, 5, 1 << 18, "staged"),
    ("f32", 1, 5, 1 << 21, "staged"),
])
def test_sparse_tap_filters_circular_all_outputs(dtype, B, H, M, path):
    """N = fft_size: the wrapped taps of Eq. 1's circular form are the late ones."""
    assert run_taps(dtype, B, H, M, M).path == path


def test_sparse_tap_filters_very_long_configuration_all_channels():
    """The very long configuration's own shape (B = 1, H = 64, N = 2^20, fft 2^21): every output of all 64 channels."""
    w = W["cfg4"]
    assert run_taps(w.dtype, w.B, w.H, w.N, w.fft_size).path == "multipass"
