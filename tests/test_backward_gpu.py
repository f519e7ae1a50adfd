"""Backward pass through the C ABI against the CPU oracle: du (the forward kernels on the adjoint
spectrum) and dk (batch reduction in frequency space)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_05908_amd import fftconv, synth
from parity_util import TOL, parity_error

pytestmark = pytest.mark.gpu
W = synth.WORKLOADS

SHAPES = [
    ("f32", 2, 3, 256, 512, 256),       # short-transform kernel
    ("f32", 3, 2, 300, 1024, 100),      # ragged N, short filter
    ("f32", 2, 2, 4096, 8192, 4096),    # staged
    ("f32", 2, 2, 256, 256, 256),       # fft_size = N: the wrapped taps take part
    ("bf16", 3, 2, 4096, 8192, 4096),   # fused 8192, odd batch
    ("f16", 2, 3, 4096, 8192, 1000),
    ("bf16", 8, 5, 4096, 8192, 4096),   # several pairs per channel, channels shared out over workgroups
    ("bf16", 1, 2, 1000, 8192, 1000),   # B = 1, ragged N
    ("bf16", 5, 2, 2048, 4096, 2048),   # short transforms grouped on the 8192 kernel: 2 per input, odd batch
    ("f16", 16, 3, 1024, 2048, 300),    # 4 per input
    ("bf16", 37, 2, 512, 1024, 512),    # 8 per input, ragged batch
    ("f16", 9, 1, 256, 512, 256),       # 16 per input
    ("bf16", 70, 2, 128, 256, 128),     # 32 per input: two transforms per row, the odd one in a shifted frame
    ("bf16", 3, 1, 1000, 4096, 1000),   # N < fft/2
    ("bf16", 2, 2, 8192, 16384, 8192),  # fused 16384: its own accumulation kernel
    ("f16", 5, 3, 8192, 16384, 3000),   # odd batch, several channels per workgroup
    ("bf16", 3, 2, 5000, 16384, 5000),  # ragged N
    ("bf16", 1, 1, 8192, 16384, 8192),  # a single row
    ("f16", 2, 1, 16384, 32768, 16384), # fused 32768: four passes over a channel, a quarter of the bins each
    ("bf16", 5, 3, 16384, 32768, 16384), # odd batch, several channels per workgroup
    ("bf16", 3, 2, 9000, 32768, 9000),  # ragged N
    ("bf16", 1, 1, 32768, 65536, 4096), # multi-pass: fp32 transforms of real rows, outer rows ko <= A/2 only (A = 8)
    ("bf16", 3, 2, 40000, 131072, 5000), # A = 16, odd batch (the last row has no partner), ragged N
    ("f32", 3, 2, 8192, 16384, 8192),   # fp32 I/O, A = 2
    ("f16", 2, 1, 16384, 16384, 700),   # circular (N = fft_size) multi-pass plan
    ("bf16", 3, 2, 8192, 8192, 600),    # circular fft 8192: du through the single-kernel route of the multi-pass family
]


@pytest.mark.parametrize("dtype,B,H,N,M,Nk", SHAPES)
def test_backward_input_and_filter(dtype, B, H, N, M, Nk):
    w = synth.scaled(W["cfg1"], B=B, H=H, N=N, fft_size=M, dtype=dtype, alpha=(1e-3, 1e-2))
    u = synth.gen_u(w)
    dy = synth.gen_gate(w, "dy")
    k = synth.gen_k(w)[:, :Nk].copy()
    plan = fftconv.Plan(N, M, H, dtype)
    kd = torch.from_numpy(k).cuda()
    kfa = plan.filter_fft_adjoint(kd)
    du = plan.backward_input(dy.cuda(), kfa)
    dk = plan.backward_filter(u.cuda(), dy.cuda(), Nk)
    torch.cuda.synchronize()
    assert torch.isfinite(du.float()).all() and torch.isfinite(dk).all()
    du_ref = oracle.backward_u(dy.double().numpy(), k, M)
    dk_ref = oracle.backward_k(u.double().numpy(), dy.double().numpy(), M, Nk)
    # single-kernel plans transform u and dy on the matrix cores (16-bit operands); the others in fp32
    tol_k = TOL[dtype] if plan.path == "fused3" else TOL["f32"]
    e_u = parity_error(du.cpu().double().numpy(), du_ref, TOL[dtype], "du")
    e_k = parity_error(dk.cpu().double().numpy(), dk_ref, tol_k, "dk")
    print("backward %s B=%d H=%d N=%d M=%d Nk=%d path=%s du err=%.3e dk err=%.3e" % (dtype, B, H, N, M, Nk, plan.path, e_u, e_k),
          flush=True)
    assert e_u <= TOL[dtype]
    assert e_k <= tol_k
    # the forward pass on the same plan still sees the ordinary spectrum
    y = plan.forward(u.cuda(), plan.filter_fft(kd))
    y_ref = oracle.fftconv(u.double().numpy(), k, M)
    assert parity_error(y.cpu().double().numpy(), y_ref, TOL[dtype], "y") <= TOL[dtype]


@pytest.mark.parametrize("dtype,B,H,N,M,Nk", [
    ("bf16", 2, 1, 1 << 18, 1 << 19, 2000),     # A = 64: both levels of the register outer passes
    ("f16", 1, 2, 1 << 20, 1 << 21, 1000),      # A = 256, config 4's transform, a single row
    ("bf16", 3, 1, 100000, 1 << 18, 300),       # A = 32, ragged N, odd batch
    ("f16", 2, 1, 1 << 17, 1 << 17, 500),       # A = 16, the input fills the transform (circular form)
])
def test_backward_filter_long_rows(dtype, B, H, N, M, Nk):
    """dk of multi-pass plans at lengths where only the filter gradient's oracle (O(N Nk) per row) is affordable."""
    w = synth.scaled(W["cfg1"], B=B, H=H, N=N, fft_size=M, dtype=dtype, alpha=(1e-3, 1e-2))
    u = synth.gen_u(w)
    dy = synth.gen_gate(w, "dy")
    plan = fftconv.Plan(N, M, H, dtype)
    dk = plan.backward_filter(u.cuda(), dy.cuda(), Nk)
    torch.cuda.synchronize()
    dk_ref = oracle.backward_k(u.double().numpy(), dy.double().numpy(), M, Nk)
    e_k = parity_error(dk.cpu().double().numpy(), dk_ref, TOL["f32"], "dk")
    print("backward_filter %s B=%d H=%d N=%d M=%d Nk=%d path=%s dk err=%.3e" % (dtype, B, H, N, M, Nk, plan.path, e_k), flush=True)
    assert plan.path == "multipass"
    assert e_k <= TOL["f32"]


def test_backward_empty_batch_and_errors():
    plan = fftconv.Plan(256, 512, 2, "f32")
    u = torch.zeros((0, 2, 256), device="cuda")
    dk = plan.backward_filter(u, u, 16)
    assert dk.shape == (2, 16) and float(dk.abs().max()) == 0.0
    lib = fftconv.load()
    x = torch.zeros((1, 2, 256), device="cuda")
    out = torch.zeros((2, 16), device="cuda")
    assert lib.fftconv_backward_filter(plan._h, x.data_ptr(), x.data_ptr(), out.data_ptr(), 0, 1, 2, 256, x.data_ptr(), None) == -1
    assert lib.fftconv_backward_filter(plan._h, x.data_ptr(), x.data_ptr(), out.data_ptr(), 16, 1, 2, 256, None, None) == -1
    assert lib.fftconv_backward_filter(plan._h, x.data_ptr(), x.data_ptr(), out.data_ptr(), 16, 1, 3, 256, x.data_ptr(), None) == -1


def test_backward_cfg2_full_size_sampled():
    w = W["cfg2"]
    u = synth.gen_u(w)
    dy = synth.gen_gate(w, "dy")
    k = synth.gen_k(w)
    plan = fftconv.Plan(w.N, w.fft_size, w.H, w.dtype)
    du = plan.backward_input(dy.cuda(), plan.filter_fft_adjoint(torch.from_numpy(k).cuda()))
    dk = plan.backward_filter(u.cuda(), dy.cuda(), w.N)
    torch.cuda.synchronize()
    worst_u = 0.0
    for b, h in synth.sample_sequences(w, 20):
        ref = oracle.backward_u(dy[b, h].double().numpy()[None, None], k[h][None], w.fft_size)[0, 0]
        worst_u = max(worst_u, parity_error(du[b, h].cpu().double().numpy(), ref, TOL[w.dtype], "du b=%d h=%d" % (b, h)))
    worst_k = 0.0
    for h in (0, 401, w.H - 1):
        ref = oracle.backward_k(u[:, h:h + 1].double().numpy(), dy[:, h:h + 1].double().numpy(), w.fft_size, w.N)[0]
        worst_k = max(worst_k, parity_error(dk[h].cpu().double().numpy(), ref, TOL[w.dtype], "dk h=%d" % h))
    print("backward cfg2 full: du worst rel L2 = %.3e, dk worst rel L2 = %.3e" % (worst_u, worst_k), flush=True)
    assert worst_u <= TOL[w.dtype] and worst_k <= TOL[w.dtype]
