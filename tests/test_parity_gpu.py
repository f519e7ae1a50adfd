"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_05908_amd import fftconv, synth
from parity_util import TOL, check_all_sequences, gpu_forward

pytestmark = pytest.mark.gpu
W = synth.WORKLOADS


def test_cfg1_fp32_all_sequences():
    err, plan = check_all_sequences(W["cfg1"])
    print("cfg1 path=%s factors=%s max rel L2 = %.3e" % (plan.path, plan.factors, err), flush=True)
    assert err <= TOL["f32"]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("B,H,N,M", [
    (3, 5, 128, 256),        # smallest transform
    (2, 3, 300, 1024),       # ragged N, N < M/2
    (1, 2, 512, 512),        # circular: fft_size == N
    (2, 2, 700, 1024),       # N > M/2: wrap-around taps matter
    (5, 1, 2048, 4096),
])
def test_small_shapes_all_dtypes(dtype, B, H, N, M):
    w = synth.scaled(W["cfg2"], B=B, H=H, N=N, fft_size=M, dtype=dtype, alpha=(1e-2, 1e-1))
    err, plan = check_all_sequences(w)
    print("%s B=%d H=%d N=%d M=%d path=%s err=%.3e" % (dtype, B, H, N, M, plan.path, err), flush=True)
    # 16-bit causal shapes with N a multiple of 8 share the 8192-point kernel; the rest is the short-transform kernel
    grouped = dtype != "f32" and N <= M // 2 and N % 8 == 0
    assert plan.path == ("fused3" if grouped else "small")
    assert err <= TOL[dtype]


@pytest.mark.parametrize("dtype,B,H,N,M", [
    ("bf16", 37, 3, 100, 256),       # 16 pairs per workgroup pass, a ragged last group, odd batch
    ("f16", 9, 5, 260, 512),         # 8 pairs per pass
    ("f32", 7, 3, 512, 1024),        # 4 pairs per pass
    ("bf16", 4, 3, 1028, 2048),      # three passes, radices 16, 16, 8 (N > fft/2 keeps 16-bit I/O on this kernel)
    ("f32", 3, 2, 4096, 4096),       # one pair per pass, circular
])
def test_small_transform_kernel_group_shapes(dtype, B, H, N, M):
    w = synth.scaled(W["cfg2"], B=B, H=H, N=N, fft_size=M, dtype=dtype, alpha=(1e-2, 1e-1))
    err, plan = check_all_sequences(w)
    print("small %s B=%d H=%d N=%d M=%d path=%s factors=%s err=%.3e" % (dtype, B, H, N, M, plan.path, plan.factors, err),
          flush=True)
    assert plan.path == "small"
    assert err <= TOL[dtype]


@pytest.mark.parametrize("dtype,B,H,N,M", [
    ("bf16", 4, 3, 2048, 4096),      # 2 transforms per pass of the 8192-point kernel, every row present
    ("f16", 5, 2, 2048, 4096),       # odd batch: the last pair and the last group are partly empty
    ("bf16", 16, 2, 1024, 2048),     # 4 per pass
    ("f16", 3, 3, 1000, 2048),       # N < fft/2: the tail of every group's slot is implicit zeros
    ("bf16", 37, 2, 512, 1024),      # 8 per pass, ragged batch
    ("f16", 64, 1, 256, 512),        # 16 per pass
    ("bf16", 7, 2, 200, 512),
    ("bf16", 1, 1, 2048, 4096),      # a single row
    ("bf16", 64, 2, 128, 256),       # 32 per pass: two transforms share an input row, the odd one in a shifted frame
    ("f16", 67, 3, 128, 256),
    ("bf16", 5, 1, 64, 256),         # N < fft/2
])
def test_short_transforms_grouped_on_the_8192_kernel(dtype, B, H, N, M):
    """fft 256 .. 4096, 16-bit I/O: 8192 / fft transforms share one work item of the wave-specialised kernel
    (block-diagonal outermost stage)."""
    w = synth.scaled(W["cfg2"], B=B, H=H, N=N, fft_size=M, dtype=dtype, alpha=(1e-2, 1e-1))
    err, plan = check_all_sequences(w)
    print("grouped %s B=%d H=%d N=%d M=%d path=%s factors=%s err=%.3e" % (dtype, B, H, N, M, plan.path, plan.factors, err),
          flush=True)
    assert plan.path == "fused3"
    assert plan.factors == [M // 256, 16, 16]
    assert err <= TOL[dtype]


@pytest.mark.parametrize("dtype,B,H,N,M", [
    ("f32", 2, 2, 4096, 8192),       # fp32 I/O beyond the short-transform kernel: the whole row in LDS
    ("f32", 1, 2, 5000, 16384),      # ragged N, a single row (no partner in the pair)
    ("f32", 2, 1, 8192, 8192),       # circular
    ("f32", 3, 2, 16384, 32768),     # three kernels: A = 4 outer factor, odd batch
    ("f32", 2, 3, 20000, 65536),     # A = 8, ragged N
])
def test_generic_staged_path(dtype, B, H, N, M):
    w = synth.scaled(W["cfg2"], B=B, H=H, N=N, fft_size=M, dtype=dtype, alpha=(1e-2, 1e-1))
    err, plan = check_all_sequences(w)
    print("staged %s B=%d H=%d N=%d M=%d path=%s factors=%s err=%.3e" % (dtype, B, H, N, M, plan.path, plan.factors, err),
          flush=True)
    assert plan.path == "staged"
    assert err <= TOL[dtype]


@pytest.mark.parametrize("lg,circular", [(16, True), (18, False), (20, False), (22, False)])
def test_fp32_long_rows_sampled_positions(lg, circular):
    """fp32 I/O on the three-kernel route: outer factors 8, 32 = 16 x 2, 128 = 16 x 8, 512 = 16 x 16 x 2."""
    from parity_util import check_sampled_positions
    M = 1 << lg
    w = synth.scaled(W["cfg4"], B=3, H=2, N=M if circular else M // 2, fft_size=M, dtype="f32", alpha=(1e-4, 1e-4))
    err, plan = check_sampled_positions(w, n_pos=16)
    print("fp32 long fft 2^%d path=%s factors=%s err=%.3e" % (lg, plan.path, plan.factors, err), flush=True)
    assert plan.path == "staged"
    assert err <= TOL["f32"]


@pytest.mark.parametrize("dtype,B,H,N,M,paths", [
    ("bf16", 4, 3, 1024, 2048, ("fused3", "small")),          # matrix cores against vector ALUs
    ("f16", 5, 2, 128, 256, ("fused3", "small")),
    ("f16", 3, 2, 4096, 8192, ("fused3", "multipass")),       # one kernel against outer passes through HBM
    ("bf16", 2, 2, 16384, 32768, ("fused3", "multipass")),
])
def test_every_family_that_can_run_a_shape_matches_the_oracle(dtype, B, H, N, M, paths):
    """Where several kernel families can run a shape, plan creation takes the one Eq. 2 prices lowest (the first of
    `paths`); the others can be forced and must return the same convolution."""
    w = synth.scaled(W["cfg2"], B=B, H=H, N=N, fft_size=M, dtype=dtype, alpha=(1e-2, 1e-1))
    _, chosen = check_all_sequences(w)
    assert chosen.path == paths[0]
    for path in paths:
        err, plan = check_all_sequences(w, path=path)
        print("forced %s %s N=%d M=%d factors=%s err=%.3e" % (path, dtype, N, M, plan.factors, err), flush=True)
        assert plan.path == path
        assert err <= TOL[dtype]
    with pytest.raises(fftconv.FFTConvError):
        fftconv.Plan(N, M, H, dtype, path="staged")           # fp32 I/O only


def test_delta_filter_is_identity_and_zero_input_gives_zero():
    N, M, H, B = 1024, 2048, 3, 2
    plan = fftconv.Plan(N, M, H, torch.float32)
    k = torch.zeros(H, N, device="cuda")
    k[:, 0] = 1.0
    kf = plan.filter_fft(k)
    u = torch.randn(B, H, N, device="cuda")
    y = plan.forward(u, kf)
    assert torch.allclose(y, u, atol=2e-5)
    y0 = plan.forward(torch.zeros_like(u), kf)
    assert torch.equal(y0, torch.zeros_like(u))


def test_batch_zero_and_error_paths_on_device():
    plan = fftconv.Plan(256, 512, 2, torch.float32)
    k = torch.randn(2, 256, device="cuda")
    kf = plan.filter_fft(k)
    y = plan.forward(torch.empty(0, 2, 256, device="cuda"), kf)
    assert tuple(y.shape) == (0, 2, 256)
    with pytest.raises(ValueError):
        plan.forward(torch.zeros(1, 3, 256, device="cuda"), kf)      # wrong H
    lib = fftconv.load()
    u = torch.zeros(1, 2, 256, device="cuda")
    rc = lib.fftconv_forward(plan._h, u.data_ptr(), kf.data_ptr(), u.data_ptr(), 1, 2, 256, None, None)
    assert rc == -1                                                   # y aliases u
    rc = lib.fftconv_forward(plan._h, u.data_ptr(), kf.data_ptr(), torch.empty_like(u).data_ptr(), 1, 2, 128, None, None)
    assert rc == -1                                                   # N differs from the plan's


def test_frequency_sparse_filter_matches_masked_oracle_small():
    w = synth.scaled(W["cfg5b"], B=2, H=3, N=256, fft_size=512, dtype="f32", alpha=(1e-2, 1e-1),
                     keep_blocks=(0, 1, 14, 15), n_blocks=16)
    err, _ = check_all_sequences(w)
    assert err <= TOL["f32"]
    err, _ = check_all_sequences(w, variant="skip")
    assert err <= TOL["f32"]


def test_partial_filter_small():
    w = synth.scaled(W["cfg5a"], B=2, H=3, N=512, fft_size=1024, dtype="f32", alpha=(1e-2, 1e-1), Nk=64)
    for variant in ("dense", "skip"):
        err, _ = check_all_sequences(w, variant=variant)
        assert err <= TOL["f32"]


# ---------------------------------------------------------------- fused 3-stage MFMA path

@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("B,H,N", [
    (2, 1, 4096),       # one pair, one channel
    (3, 5, 4096),       # odd batch: the last pair has no partner row
    (8, 3, 4096),
    (1, 2, 4096),       # B = 1
    (4, 2, 2048),       # N < fft_size/2: the tail of the padded half is implicit zeros too
    (2, 2, 1000),       # ragged N (multiple of 8)
])
def test_fused3_fft8192(dtype, B, H, N):
    w = synth.scaled(W["cfg2"], B=B, H=H, N=N, fft_size=8192, dtype=dtype)
    err, plan = check_all_sequences(w)
    print("fused 8192 %s B=%d H=%d N=%d path=%s factors=%s err=%.3e" % (dtype, B, H, N, plan.path, plan.factors, err),
          flush=True)
    assert plan.path == "fused3"
    assert err <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("B,H,N", [
    (2, 2, 8192),
    (5, 3, 8192),       # odd batch
    (2, 1, 4000),       # ragged N
])
def test_fused3_fft16384(dtype, B, H, N):
    w = synth.scaled(W["cfg5a"], B=B, H=H, N=N, fft_size=16384, dtype=dtype, Nk=0)
    err, plan = check_all_sequences(w)
    print("fused 16384 %s B=%d H=%d N=%d path=%s factors=%s err=%.3e" % (dtype, B, H, N, plan.path, plan.factors, err),
          flush=True)
    assert plan.path == "fused3" and plan.factors == [32, 16, 32]
    assert err <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("B,H,N", [
    (2, 1, 16384),      # one pair, one channel
    (3, 2, 16384),      # odd batch: the last pair has no partner row
    (8, 3, 16384),      # several pairs per channel, several channels per workgroup range
    (1, 2, 16384),      # B = 1
    (4, 2, 8192),       # N < fft_size/2
    (2, 2, 10000),      # ragged N (multiple of 8)
])
def test_fused3_fft32768(dtype, B, H, N):
    w = synth.scaled(W["cfg3"], B=B, H=H, N=N, fft_size=32768, dtype=dtype)
    err, plan = check_all_sequences(w)
    print("fused 32768 %s B=%d H=%d N=%d path=%s factors=%s err=%.3e" % (dtype, B, H, N, plan.path, plan.factors, err),
          flush=True)
    assert plan.path == "fused3" and plan.factors == [32, 32, 32]
    assert err <= TOL[dtype]


def test_cfg5_variants_reduced_batch():
    """Partial and frequency-sparse filters on fft 16384 (reduced B, H), dense and skipping entry points."""
    wa = synth.scaled(W["cfg5a"], B=4, H=3)
    wb = synth.scaled(W["cfg5b"], B=4, H=3)
    for w in (wa, wb):
        for variant in ("dense", "skip"):
            err, plan = check_all_sequences(w, variant=variant)
            print("%s %s path=%s err=%.3e" % (w.name, variant, plan.path, err), flush=True)
            assert err <= TOL[w.dtype]


@pytest.mark.parametrize("dtype,B,H,N,M,Nk", [
    ("f16", 3, 2, 16384, 32768, 1024),     # single-kernel 32768 plan: 5 segments per row
    ("bf16", 2, 2, 16384, 32768, 2049),    # the longest filter the segments take (2048 samples of history)
    ("bf16", 2, 1, 12000, 32768, 100),     # ragged N, short filter
    ("bf16", 3, 1, 32768, 65536, 1024),    # multi-pass plan, odd batch
    ("f16", 1, 2, 100000, 262144, 777),    # long row, B = 1
])
def test_partial_convolution_as_segments_on_long_plans(dtype, B, H, N, M, Nk):
    """Partial convolutions (Section 3.3) of plans for fft >= 16384: overlapping 8192-point segments on the
    wave-specialised kernel, against the oracle on the zeroed filter; the dense route on the same k_f as well."""
    w = synth.scaled(W["cfg5a"], B=B, H=H, N=N, fft_size=M, dtype=dtype, Nk=Nk)
    for variant in ("dense", "skip"):
        err, plan = check_all_sequences(w, variant=variant)
        print("partial %s B=%d H=%d N=%d M=%d Nk=%d %s path=%s err=%.3e" % (dtype, B, H, N, M, Nk, variant, plan.path, err),
              flush=True)
        assert err <= TOL[dtype]


# ---------------------------------------------------------------- multi-pass path (Algorithm 4)

@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("B,H,N,M", [
    (3, 2, 32768, 65536),      # outer length 8, odd batch
    (2, 1, 65536, 131072),     # outer length 16
    (1, 1, 20000, 65536),      # ragged N, B = 1
    (3, 1, 20001, 65536),      # odd N: rows start on 2-byte boundaries, element-wise loads and stores; odd batch
])
def test_multipass_all_outputs(dtype, B, H, N, M):
    w = synth.scaled(W["cfg3"], B=B, H=H, N=N, fft_size=M, dtype=dtype)
    err, plan = check_all_sequences(w)
    print("multipass %s B=%d H=%d N=%d M=%d path=%s factors=%s err=%.3e" % (dtype, B, H, N, M, plan.path, plan.factors, err),
          flush=True)
    assert plan.path == "multipass"
    assert err <= TOL[dtype]


@pytest.mark.parametrize("dtype,B,H,N,M", [
    ("bf16", 2, 2, 8192, 8192),      # circular, no outer transform: the inner kernel reads u and writes y itself
    ("f16", 3, 1, 4100, 8192),       # causal, N a multiple of 4 but not of 8: the same single kernel, odd batch
    ("bf16", 5, 3, 6000, 8192),      # N > fft/2 (wrap-around taps), ragged tail inside a lane's range, odd batch
    ("f16", 1, 2, 8192, 8192),       # a lone row: its partner is taken as zero and never stored
    ("bf16", 2, 1, 4, 8192),         # the shortest row the single kernel takes: one 8-byte piece
    ("bf16", 3, 1, 8188, 8192),      # the last piece of a row missing
    ("f16", 2, 2, 4102, 8192),       # N not a multiple of 4: pack, convolve, unpack as three passes
    ("bf16", 3, 2, 16384, 16384),    # circular, outer length 2
    ("f16", 2, 1, 9000, 16384),      # N > fft/2, ragged
    ("bf16", 1, 2, 8190, 16384),     # causal, N not a multiple of 8, outer length 2 with the implicit zero half
    ("bf16", 2, 1, 32768, 32768),    # circular, outer length 4
    ("f16", 1, 1, 65536, 65536),     # circular, outer length 8
    ("bf16", 1, 1, 50000, 65536),    # N > fft/2, wrap-around taps
])
def test_multipass_circular_and_ragged(dtype, B, H, N, M):
    """16-bit shapes with the input filling more than half of the transform (Section 2.1: circular convolution)
    and ragged causal shapes from fft 8192 up: outer passes without the implicit zero half."""
    w = synth.scaled(W["cfg3"], B=B, H=H, N=N, fft_size=M, dtype=dtype)
    err, plan = check_all_sequences(w)
    print("multipass %s B=%d H=%d N=%d M=%d path=%s factors=%s err=%.3e" % (dtype, B, H, N, M, plan.path, plan.factors, err),
          flush=True)
    assert plan.path == "multipass"
    assert err <= TOL[dtype]


@pytest.mark.parametrize("dtype,B,H,N", [
    ("bf16", 6, 300, 8192),        # 900 work items: three or four per workgroup, the software pipeline at full depth
    ("f16", 3, 171, 5004),         # one or two items per workgroup, ragged, every channel's last pair without partner
])
def test_circular_8192_single_kernel_many_items(dtype, B, H, N):
    """fft 8192 with N > fft/2 (Section 2.1: circular convolution): one kernel, several work items per workgroup;
    sampled output positions of every sequence, the first and last ones always."""
    from parity_util import check_sampled_positions
    w = synth.scaled(W["cfg2"], B=B, H=H, N=N, fft_size=8192, dtype=dtype)
    err, plan = check_sampled_positions(w, n_pos=128, edge=2)     # fewer positions: the norm estimate is too noisy
    print("circular 8192 %s B=%d H=%d N=%d path=%s err=%.3e" % (dtype, B, H, N, plan.path, err), flush=True)
    assert plan.path == "multipass"
    assert err <= TOL[dtype]


@pytest.mark.parametrize("B,H,N,M", [
    (2, 1, 1 << 17, 1 << 18),      # outer length 32 = 16 x 2
    (1, 2, 1 << 20, 1 << 21),      # the very long configuration at H = 2: outer length 256 = 16 x 16
])
def test_multipass_long_sampled_positions(B, H, N, M):
    from parity_util import check_sampled_positions
    w = synth.scaled(W["cfg4"], B=B, H=H, N=N, fft_size=M)
    err, plan = check_sampled_positions(w)
    print("multipass long B=%d H=%d N=%d M=%d path=%s factors=%s err=%.3e" % (B, H, N, M, plan.path, plan.factors, err),
          flush=True)
    assert plan.path == "multipass"
    assert err <= TOL[w.dtype]


@pytest.mark.parametrize("B,H,N,Nk", [
    (2, 2, 8192, 1024),     # 3 overlapping 8192-point segments
    (3, 2, 8192, 2049),     # longest filter the segment path takes (2048 samples of history), odd batch
    (2, 1, 8192, 2050),     # one tap more: falls back to the dense 16384-point kernel
    (2, 2, 8192, 1),        # a single tap: no history at all
    (2, 1, 6000, 100),      # ragged length, last segment partly out of range
    (2, 1, 4096, 512),      # sequence fits one segment
])
def test_partial_convolution_segment_path(B, H, N, Nk):
    w = synth.scaled(W["cfg5a"], B=B, H=H, N=N, Nk=Nk)
    err_dense, _ = check_all_sequences(w, variant="dense")
    err_skip, plan = check_all_sequences(w, variant="skip")
    print("partial B=%d H=%d N=%d Nk=%d path=%s dense err=%.3e segments err=%.3e" % (B, H, N, Nk, plan.path, err_dense, err_skip),
          flush=True)
    assert err_dense <= TOL[w.dtype] and err_skip <= TOL[w.dtype]


@pytest.mark.parametrize("dtype,B,H,N,M", [
    ("bf16", 3, 2, 8192, 16384),      # single-kernel plan
    ("f16", 2, 2, 16384, 32768),
    ("bf16", 2, 1, 32768, 65536),     # multi-pass plan: all three of its kernels are gated
])
def test_partial_entry_point_on_a_spectrum_built_for_another_filter_length(dtype, B, H, N, M):
    """fftconv_forward_partial takes the segment route only when k_f carries the short spectrum of exactly that Nk
    (a tag on the device says so); on any other k_f of the plan it must return what fftconv_forward returns."""
    Nk = 1024
    w = synth.scaled(W["cfg5a"], B=B, H=H, N=N, fft_size=M, dtype=dtype, Nk=Nk)
    u = synth.gen_u(w)
    k = synth.gen_k(w)                                    # (H, N), taps >= Nk are zero
    ref = oracle.fftconv(u.double().numpy(), k, M)
    plan = fftconv.Plan(N, M, H, dtype)
    ud = u.cuda()
    kfull = torch.from_numpy(k).cuda()
    kshort = torch.from_numpy(k[:, :Nk].copy()).cuda()
    stale = torch.from_numpy(synth.gen_k(synth.scaled(w, seed_k=999))[:, :Nk].copy()).cuda()
    from parity_util import parity_error
    # 1. the full-length filter with its tail zeroed (no short spectrum is built for Nk = N); the buffer first
    #    holds the short spectrum of ANOTHER filter, which a route that ignored the tag would use
    kf = plan.filter_fft(stale)
    lib = fftconv.load()
    assert lib.fftconv_filter_fft(plan._h, kfull.data_ptr(), N, kf.data_ptr(), None) == 0
    y = plan.forward_partial(ud, kf, Nk)
    assert torch.equal(y, plan.forward(ud, kf))
    assert parity_error(y.cpu().double().numpy(), ref, TOL[dtype], "zeroed tail") <= TOL[dtype]
    # 2. a short spectrum built for a different Nk (more taps, the extra ones zero): still the dense result
    assert lib.fftconv_filter_fft(plan._h, kfull.data_ptr(), Nk + 8, kf.data_ptr(), None) == 0
    y = plan.forward_partial(ud, kf, Nk)
    assert torch.equal(y, plan.forward(ud, kf))
    # 3. the matching one: the segment route runs (a different kernel, so not bit-identical to the dense one)
    kf = plan.filter_fft(kshort)
    y = plan.forward_partial(ud, kf, Nk)
    assert parity_error(y.cpu().double().numpy(), ref, TOL[dtype], "segments") <= TOL[dtype]
    assert not torch.equal(y, plan.forward(ud, kf))
    # 4. a masked and an adjoint spectrum in the same buffer reset the tag
    assert lib.fftconv_filter_fft_adjoint(plan._h, kshort.data_ptr(), Nk, kf.data_ptr(), None) == 0
    assert torch.equal(plan.forward_partial(ud, kf, Nk), plan.forward(ud, kf))
    kf = plan.filter_fft(kshort, block_keep=[1, 1, 0, 0, 0, 0, 1, 1])
    assert torch.equal(plan.forward_partial(ud, kf, Nk), plan.forward(ud, kf))


@pytest.mark.parametrize("keep_blocks", [
    (0, 1, 2, 3, 28, 29, 30, 31),                     # the low-pass of config 5b: one live accumulator slot
    tuple(range(8)) + tuple(range(24, 32)),           # half of the spectrum: two live slots
    (0, 1, 2, 3),                                     # one-sided mask: mirror bins get weight 1/2
    (5, 6, 20, 31),                                   # scattered blocks: nothing can be skipped
    (16,),                                            # only the block at the Nyquist edge
])
def test_frequency_sparse_masks_fft16384(keep_blocks):
    w = synth.scaled(W["cfg5b"], B=3, H=2, keep_blocks=keep_blocks, n_blocks=32)
    for variant in ("dense", "skip"):
        err, plan = check_all_sequences(w, variant=variant)
        print("freq-sparse keep=%s %s path=%s err=%.3e" % (keep_blocks, variant, plan.path, err), flush=True)
        assert err <= TOL[w.dtype]


@pytest.mark.parametrize("dtype,N,M,n_blocks,keep_blocks,path", [
    ("bf16", 4096, 8192, 32, (0, 1, 2, 3, 28, 29, 30, 31), "fused3"),     # the 8192-point kernel's own filter transform
    ("f16", 1024, 2048, 16, (0, 1, 2), "fused3"),                         # a short plan (4 groups), one-sided mask
    ("bf16", 16384, 32768, 64, tuple(range(8)) + tuple(range(56, 64)), "fused3"),   # half-length real transform
    ("bf16", 20000, 65536, 32, (0, 1, 30, 31), "multipass"),              # two-kernel fp32 transform, k_f by the block kernel
    ("f16", 8192, 8192, 8, (0, 7), "multipass"),                          # circular 8192: fp64 rows in LDS
])
def test_block_masks_through_every_filter_transform(dtype, N, M, n_blocks, keep_blocks, path):
    """Frequency-block masks (weights 1 / 1/2 / 0 per bin) are applied inside each plan family's own filter transform."""
    w = synth.scaled(W["cfg5b"], B=2, H=2, N=N, fft_size=M, dtype=dtype, keep_blocks=keep_blocks, n_blocks=n_blocks)
    err, plan = check_all_sequences(w, variant="skip")
    print("block mask %s N=%d M=%d path=%s err=%.3e" % (dtype, N, M, plan.path, err), flush=True)
    assert plan.path == path
    assert err <= TOL[dtype]


# ---------------------------------------------------------------- every transform length the plan accepts

@pytest.mark.parametrize("lg", list(range(8, 23)))
def test_every_power_of_two_fft_size_sampled_positions(lg):
    """fft_size = 256 .. 4M (the paper's range), causal N = fft_size/2, bf16: all paths in turn."""
    from parity_util import check_sampled_positions
    M = 1 << lg
    w = synth.scaled(W["cfg4"], B=2, H=2, N=M // 2, fft_size=M, dtype="bf16", alpha=(1e-4, 1e-4))
    # 128 positions per sequence: the relative L2 error is a ratio of two sums over the sampled positions, and
    # with 16 of them its scatter (about a third of its value) reaches the tolerance from a typical 5.5e-3
    err, plan = check_sampled_positions(w, n_pos=128)
    print("fft 2^%d path=%s factors=%s err=%.3e" % (lg, plan.path, plan.factors, err), flush=True)
    assert err <= TOL["bf16"]
