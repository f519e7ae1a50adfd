"""A check of the hand-rolled synchronisation that is not parity: the library is built a second time with
every LDS-only workgroup barrier of the fused kernels replaced by the full __syncthreads() and with wait
states inserted between the hand-spaced dot products and the conversions that read them
(python -m paper_2311_05908_amd.build --sync-check).  If the release build's lighter barrier or instruction
spacing ever let a wave read a value too early, the two builds would differ; they must agree bit for bit."""
import os

import pytest
import torch

from paper_2311_05908_amd import build as hip_build
from paper_2311_05908_amd import fftconv, synth

pytestmark = pytest.mark.gpu
W = synth.WORKLOADS


def both_builds(w, gated=False, partial=False):
    if not os.path.exists(hip_build.LIB_SYNC_CHECK):
        pytest.fail("libfftconv_synccheck.so is missing: run python -m paper_2311_05908_amd.build --sync-check")
    u = synth.gen_u(w).cuda()
    k = torch.from_numpy(synth.gen_k(w)[:, : w.filter_len].copy()).cuda()
    gw = synth.gen_gate(w, "w").cuda() if gated else None
    gv = synth.gen_gate(w, "v").cuda() if gated else None
    bk = synth.block_keep(w) if w.n_blocks else None
    out = []
    for lib in (fftconv.load(), fftconv.load(hip_build.LIB_SYNC_CHECK)):
        plan = fftconv.Plan(w.N, w.fft_size, w.H, w.dtype, lib=lib)
        kf = plan.filter_fft(k, block_keep=bk)
        if gated:
            y = plan.forward_gated(u, gw, gv, kf)
        elif bk is not None:
            y = plan.forward_freq_sparse(u, kf, bk)
        elif partial:
            y = plan.forward_partial(u, kf, w.Nk)
        else:
            y = plan.forward(u, kf)
        torch.cuda.synchronize()
        out.append((y.clone(), kf.clone(), plan.path))
        plan.close()
    (y0, kf0, path), (y1, kf1, _) = out
    if w.fft_size <= 8192:       # larger plans keep a second spectrum for short filters behind the dense one, unset here
        assert torch.equal(kf0, kf1), "k_f differs between the release and the checking build"
    assert torch.equal(y0.view(torch.int16), y1.view(torch.int16)), "y differs between the release and the checking build"
    return path


@pytest.mark.parametrize("name,kw", [
    ("cfg2", dict(B=16, H=96)),            # wave-specialised 8192-point kernel, several items per workgroup
    ("cfg2", dict(B=5, H=7, N=4000)),      # the guarded instantiation
    ("cfg3", dict(B=4, H=96)),             # 32768-point streamed-table kernel
    ("cfg5b", dict(B=8, H=96)),            # 16384-point kernel with the empty tile skipped, two workgroups per unit
    ("cfg5a", dict(B=4, H=64)),            # dense 16384 kernel
    ("cfg4", dict(H=4, N=1 << 17, fft_size=1 << 18)),     # multi-pass: outer passes and the complex-row inner kernel
])
def test_release_and_checking_builds_agree_bit_for_bit(name, kw):
    w = synth.scaled(W[name], **kw)
    path = both_builds(w)
    print("sync check %s %s path=%s: bit-identical" % (name, kw, path), flush=True)


def test_checking_build_gated_partial_and_fp16():
    both_builds(synth.scaled(W["cfg2"], B=8, H=64), gated=True)
    both_builds(synth.scaled(W["cfg2"], B=8, H=64, dtype="f16"))
    both_builds(synth.scaled(W["cfg5a"], B=4, H=32), partial=True)
