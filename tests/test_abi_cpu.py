"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol,
validates arguments before touching a device, and its host-only helpers are right."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

from paper_2311_05908_amd import fftconv, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fftconv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fftconv_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree_and_library_exports_everything():
    names = declared_functions()
    assert sorted(fftconv.EXPORTS) == names
    lib = fftconv.load()
    for n in names:
        assert getattr(lib, n) is not None


def test_argument_errors_come_before_any_device_use():
    lib = fftconv.load()
    h = ctypes.c_void_p()
    bad = [
        (1024, 1000, 4, 0),        # fft_size not a power of two
        (64, 128, 4, 0),           # fft_size below the paper's range
        (8, 1 << 23, 4, 0),        # above it
        (4096, 2048, 4, 0),        # N > fft_size
        (0, 2048, 4, 0),           # N < 1
        (1024, 2048, 0, 0),        # H < 1
        (1024, 2048, 4, 7),        # unknown dtype
    ]
    for N, M, H, dt in bad:
        rc = lib.fftconv_plan_create(ctypes.byref(h), N, M, H, dt)
        assert rc == -1, (N, M, H, dt)
        assert not h.value
        assert lib.fftconv_last_error().decode() != ""
    assert lib.fftconv_plan_create(None, 1024, 2048, 4, 0) == -1
    assert lib.fftconv_plan_destroy(None) == 0
    assert lib.fftconv_kf_bytes(None) == 0
    assert lib.fftconv_forward(None, None, None, None, 1, 1, 1, None, None) == -1
    assert lib.fftconv_filter_fft(None, None, 1, None, None) == -1
    assert lib.fftconv_strerror(-5).decode() == "no usable GPU"


@pytest.mark.skipif(torch.cuda.is_available(), reason="needs a box without a GPU")
def test_plan_create_without_gpu_fails_cleanly():
    with pytest.raises(fftconv.FFTConvError) as ei:
        fftconv.Plan(1024, 2048, 4, torch.float32)
    assert ei.value.code == -5


def test_sparsity_fraction_reproduces_the_papers_table():
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "sparsity_fraction.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 6
    for a, b, c, d, s in rows:
        frac = fftconv.sparsity_fraction([32, 32, 32, 64], [int(a), int(b), int(c), int(d)])
        assert round(100 * frac) == int(s)
    assert fftconv.sparsity_fraction([32], [8]) == 0.25
    with pytest.raises(ValueError):
        fftconv.sparsity_fraction([32], [33])


def test_synth_is_deterministic_and_subsettable():
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=4, H=3, N=64, fft_size=128)
    u = synth.gen_u(w)
    assert u.dtype == torch.bfloat16 and tuple(u.shape) == (4, 3, 64)
    assert torch.equal(synth.gen_u(w, [2])[0], u[2])
    assert torch.equal(synth.gen_u(w), u)
    k = synth.gen_k(w)
    assert k.dtype == np.float32 and k.shape == (3, 64)
    a = synth.gen_alpha(w)
    assert ((a >= 1e-3) & (a <= 1e-1)).all()
    # the envelope decays: late taps are smaller than early taps on average
    big = synth.gen_k(synth.scaled(w, H=64, N=512))
    assert np.abs(big[:, :32]).mean() > 3 * np.abs(big[:, -32:]).mean()
    wp = synth.scaled(synth.WORKLOADS["cfg5a"], B=1, H=2, N=64, fft_size=128, Nk=16)
    kp = synth.gen_k(wp)
    assert (kp[:, 16:] == 0).all() and (kp[:, :16] != 0).any()
    bk = synth.block_keep(synth.WORKLOADS["cfg5b"])
    assert bk.sum() == 8 and list(np.nonzero(bk)[0]) == [0, 1, 2, 3, 28, 29, 30, 31]
    pts = synth.sample_sequences(synth.WORKLOADS["cfg2"], 16)
    assert len(pts) == 20 and (0, 0) in pts and (63, 767) in pts


def test_workload_table_matches_the_stated_configs():
    W = synth.WORKLOADS
    assert (W["cfg1"].B, W["cfg1"].H, W["cfg1"].N, W["cfg1"].fft_size, W["cfg1"].dtype) == (2, 4, 1024, 2048, "f32")
    assert (W["cfg2"].B, W["cfg2"].H, W["cfg2"].N, W["cfg2"].fft_size, W["cfg2"].dtype) == (64, 768, 4096, 8192, "bf16")
    assert (W["cfg3"].B, W["cfg3"].H, W["cfg3"].N, W["cfg3"].fft_size, W["cfg3"].dtype) == (16, 768, 16384, 32768, "f16")
    assert (W["cfg4"].B, W["cfg4"].H, W["cfg4"].N, W["cfg4"].fft_size, W["cfg4"].dtype) == (1, 64, 1 << 20, 1 << 21, "bf16")
    assert (W["cfg5a"].B, W["cfg5a"].H, W["cfg5a"].N, W["cfg5a"].fft_size, W["cfg5a"].Nk) == (32, 768, 8192, 16384, 1024)
