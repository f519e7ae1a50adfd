"""Pins of the CPU oracle against things it shares no code with.

The paper prints no worked numeric example of a convolution, so the pins are:
Eq. 1 evaluated with dense DFT matrices on tiny inputs, closed forms, exact
integer polynomial products, invariants and library routines (numpy.convolve,
numpy.fft), chosen so that a dropped term, a wrong sign or index, a wrong
stride or a transposed operand fails at least one of them.
"""
import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(12345)


def dft_matrix(M, sign=-1):
    j = np.arange(M)
    return np.exp(sign * 2j * np.pi * np.outer(j, j) / M)


def eq1_dense(u, kext):
    """Eq. 1 literally: F^-1 (F u_pad . F k) with dense M x M DFT matrices."""
    B, H, N = u.shape
    M = kext.shape[1]
    F = dft_matrix(M, -1)
    Fi = dft_matrix(M, +1) / M
    up = np.zeros((B, H, M))
    up[..., :N] = u
    Uf = up @ F.T
    Kf = kext @ F.T
    y = (Uf * Kf[None]) @ Fi.T
    assert np.abs(y.imag).max() < 1e-9
    return y.real[..., :N]


@pytest.mark.parametrize("N,M", [(1, 1), (5, 5), (8, 8), (8, 16), (7, 16), (16, 32), (32, 64), (24, 37), (64, 64)])
def test_matches_eq1_with_dense_dft(N, M):
    B, H = 3, 2
    u = RNG.standard_normal((B, H, N))
    kext = RNG.standard_normal((H, M))          # full-length filter: exercises the wrap-around taps
    y = oracle.fftconv(u, kext)
    assert np.allclose(y, eq1_dense(u, kext), rtol=0, atol=1e-11)


@pytest.mark.parametrize("N", [1, 2, 17, 64, 300])
def test_causal_equals_numpy_convolve(N):
    B, H = 2, 3
    u = RNG.standard_normal((B, H, N))
    k = RNG.standard_normal((H, N))
    y = oracle.fftconv(u, k, M=2 * N)
    for b in range(B):
        for h in range(H):
            assert np.allclose(y[b, h], np.convolve(u[b, h], k[h])[:N], rtol=0, atol=1e-12)


def test_integer_inputs_give_exact_polynomial_product():
    B, H, N = 2, 2, 50
    u = RNG.integers(-9, 10, size=(B, H, N))
    k = RNG.integers(-9, 10, size=(H, N))
    y = oracle.fftconv(u.astype(float), k.astype(float), M=2 * N)
    for b in range(B):
        for h in range(H):
            prod = np.polymul(u[b, h][::-1], k[h][::-1])[::-1]      # exact int64 coefficients
            assert np.array_equal(y[b, h], prod[:N].astype(float))


def test_delta_and_shifted_delta():
    N, M = 40, 80
    u = RNG.standard_normal((2, 1, N))
    k = np.zeros((1, N))
    k[0, 0] = 1.0
    assert np.array_equal(oracle.fftconv(u, k, M=M), u)
    for s in (1, 7, 39):
        k = np.zeros((1, N))
        k[0, s] = 1.0
        y = oracle.fftconv(u, k, M=M)
        assert np.array_equal(y[..., :s], np.zeros_like(y[..., :s]))
        assert np.array_equal(y[..., s:], u[..., : N - s])


def test_circular_wraps_when_fft_size_equals_n():
    N = 16
    u = RNG.standard_normal((1, 1, N))
    for s in (1, 5, 15):
        k = np.zeros((1, N))
        k[0, s] = 1.0
        y = oracle.fftconv(u, k)                      # M = N: circular
        assert np.array_equal(y[0, 0], np.roll(u[0, 0], s))


def test_closed_forms():
    N = 64
    ones = np.ones((1, 1, N))
    y = oracle.fftconv(ones, np.ones((1, N)), M=2 * N)
    assert np.array_equal(y[0, 0], np.arange(1, N + 1, dtype=float))
    r = 0.9
    k = r ** np.arange(N)
    y = oracle.fftconv(ones, k[None], M=2 * N)
    assert np.allclose(y[0, 0], (1 - r ** np.arange(1, N + 1)) / (1 - r), rtol=1e-13)


def test_linearity_and_shift_equivariance():
    B, H, N = 2, 2, 33
    u1, u2 = RNG.standard_normal((2, B, H, N))
    k1, k2 = RNG.standard_normal((2, H, N))
    a, c = 1.7, -0.3
    f = lambda u, k: oracle.fftconv(u, k, M=2 * N)
    assert np.allclose(f(a * u1 + c * u2, k1), a * f(u1, k1) + c * f(u2, k1), atol=1e-12)
    assert np.allclose(f(u1, a * k1 + c * k2), a * f(u1, k1) + c * f(u1, k2), atol=1e-12)
    s = 5
    us = np.zeros_like(u1)
    us[..., s:] = u1[..., : N - s]
    ys = f(us, k1)
    assert np.allclose(ys[..., s:], f(u1, k1)[..., : N - s], atol=1e-12)
    assert np.array_equal(ys[..., :s], np.zeros_like(ys[..., :s]))


def test_filter_row_belongs_to_channel_not_batch():
    # B != H and distinct filters: a swapped (b,h) stride or a filter indexed by b fails here.
    B, H, N = 3, 5, 12
    u = RNG.standard_normal((B, H, N))
    k = RNG.standard_normal((H, N))
    y = oracle.fftconv(u, k, M=32)
    for b in range(B):
        for h in range(H):
            assert np.allclose(y[b, h], np.convolve(u[b, h], k[h])[:N], atol=1e-12)


def test_partial_filter_is_a_sliding_window():
    # Section 3.3: a filter whose later taps are zero only sees the last Nk inputs.
    N, Nk = 96, 8
    u = RNG.standard_normal((1, 1, N))
    k = np.zeros((1, N))
    k[0, :Nk] = RNG.standard_normal(Nk)
    y = oracle.fftconv(u, k, M=2 * N)
    y_short = oracle.fftconv(u, k[:, :Nk], M=2 * N)
    assert np.array_equal(y, y_short)
    u2 = u.copy()
    u2[..., :40] += 100.0
    y2 = oracle.fftconv(u2, k, M=2 * N)
    assert np.array_equal(y2[..., 40 + Nk - 1:], y[..., 40 + Nk - 1:])
    # overlap-add with blocks of length Nk reproduces it
    acc = np.zeros(N + 2 * Nk)
    for c in range(N // Nk):
        blk = u[0, 0, c * Nk:(c + 1) * Nk]
        acc[c * Nk:c * Nk + 2 * Nk - 1] += np.convolve(blk, k[0, :Nk])
    assert np.allclose(acc[:N], y[0, 0], atol=1e-12)


def test_sampled_positions_equal_full_and_direct_dot():
    S, N, M = 3, 200, 512
    u = RNG.standard_normal((S, N))
    kext = np.zeros((S, M))
    kext[:, :N] = RNG.standard_normal((S, N))
    idx = np.stack([RNG.integers(0, N, size=9) for _ in range(S)])
    idx[0, 0], idx[0, 1] = 0, N - 1
    out = oracle.fftconv_at(u, kext, idx)
    for s in range(S):
        full = oracle.fftconv(u[s][None, None], kext[s][None])[0, 0]
        assert np.array_equal(out[s], full[idx[s]])
        for p, i in enumerate(idx[s]):
            assert np.isclose(out[s, p], np.dot(u[s, : i + 1], kext[s, i::-1][: i + 1]), atol=1e-12)
    with pytest.raises(ValueError):
        oracle.fftconv_at(u, kext, np.full((S, 1), N))


def test_mask_filter_identity_and_library_crosscheck():
    H, M = 2, 64
    kext = RNG.standard_normal((H, M))
    assert np.allclose(oracle.mask_filter(kext, np.ones(M)), kext, atol=1e-12)
    assert np.allclose(oracle.mask_filter(kext, np.zeros(M)), 0.0, atol=0)
    keep = (RNG.random(M) < 0.4).astype(np.uint8)             # not Hermitian-symmetric on purpose
    ref = np.fft.ifft(np.fft.fft(kext, axis=1) * keep[None], axis=1).real
    assert np.allclose(oracle.mask_filter(kext, keep), ref, atol=1e-12)


def test_mask_filter_closed_forms_fix_signs_and_scale():
    M, f0 = 32, 3
    t = np.arange(M)
    delta0 = np.zeros((1, M))
    delta0[0, 0] = 1.0
    keep = np.zeros(M)
    keep[[f0, M - f0]] = 1
    assert np.allclose(oracle.mask_filter(delta0, keep)[0], 2.0 / M * np.cos(2 * np.pi * f0 * t / M), atol=1e-14)
    # one non-symmetric bin of a delta at t=1: forward sign -, inverse sign +  =>  cos(2 pi f0 (t-1)/M)/M
    delta1 = np.zeros((1, M))
    delta1[0, 1] = 1.0
    keep = np.zeros(M)
    keep[f0] = 1
    assert np.allclose(oracle.mask_filter(delta1, keep)[0], np.cos(2 * np.pi * f0 * (t - 1) / M) / M, atol=1e-14)


def test_mask_filter_parseval_for_symmetric_mask():
    M = 128
    kext = RNG.standard_normal((1, M))
    keep = np.zeros(M, dtype=np.uint8)
    keep[:20] = 1
    keep[M - 19:] = 1                                           # f and M-f kept together
    kt = oracle.mask_filter(kext, keep)
    K = dft_matrix(M) @ kext[0]
    assert np.isclose((kt ** 2).sum(), (np.abs(K) ** 2 * keep).sum() / M, rtol=1e-12)


def test_bad_sizes_are_rejected():
    with pytest.raises(ValueError):
        oracle.fftconv(np.zeros((1, 1, 8)), np.zeros((1, 4)))        # M < N
    with pytest.raises(ValueError):
        oracle.fftconv(np.zeros((1, 2, 8)), np.zeros((3, 16)))       # filter rows != H


def test_rel_l2_metric():
    y = np.array([[3.0, 4.0], [0.0, 0.0]])
    r = np.array([[3.0, 0.0], [0.0, 0.0]])
    assert np.allclose(oracle.rel_l2_per_sequence(y, r), [4.0 / 3.0, 0.0])


def test_masked_filter_spectrum_is_the_hermitian_part_of_the_masked_spectrum():
    # Re(IDFT(keep . K)) has spectrum K[f] (keep[f] + keep[M-f]) / 2: the form the library stores.
    M = 64
    kext = RNG.standard_normal((1, M))
    keep = np.zeros(M, dtype=np.uint8)
    keep[:8] = 1
    keep[M - 8:] = 1                      # block mask: bin 56 kept, its mirror bin 8 is not
    kt = oracle.mask_filter(kext, keep)[0]
    K = np.fft.fft(kext[0])
    mirror = keep[(-np.arange(M)) % M]
    assert np.allclose(np.fft.fft(kt), K * (keep + mirror) / 2.0, atol=1e-11)
    assert (keep != mirror).sum() == 2    # the asymmetry the weight 1/2 is there for


# ---------------------------------------------------------------- filters given as a list of taps

def test_taps_single_delta_is_a_shift_with_zero_fill_or_wrap():
    # k = delta_s: causal (M >= N + s) gives u shifted right by s with zeros in front (Section 2.1);
    # with M = N the samples pushed out at the end come back in at the front (Eq. 1, circular form)
    B, H, N = 2, 3, 50
    u = RNG.standard_normal((B, H, N))
    for s in (0, 1, 7, 49):
        pos = np.full((H, 1), s)
        val = np.ones((H, 1))
        y = oracle.fftconv_taps(u, pos, val, 2 * N)
        want = np.zeros_like(u)
        want[..., s:] = u[..., : N - s]
        assert np.array_equal(y, want)
        assert np.array_equal(oracle.fftconv_taps(u, pos, val, N), np.roll(u, s, axis=-1))
    # a tap in the padded region (N <= s < M = 2N): output i takes input i - s + M, an input sample only while i < s - N
    s = 70
    y = oracle.fftconv_taps(u, np.full((H, 1), s), np.ones((H, 1)), 2 * N)
    want = np.zeros_like(u)
    want[..., : N - (2 * N - s)] = u[..., 2 * N - s:]
    assert np.array_equal(y, want)


def test_taps_equal_the_dense_definition_and_the_library_convolution():
    B, H, N, M, T = 2, 3, 40, 64, 5
    u = RNG.standard_normal((B, H, N))
    pos = np.stack([RNG.permutation(M)[:T] for _ in range(H)])          # anywhere in [0, M): wrapped taps too
    val = RNG.standard_normal((H, T))
    kext = np.zeros((H, M))
    for h in range(H):
        kext[h, pos[h]] = val[h]
    assert np.allclose(oracle.fftconv_taps(u, pos, val, M), oracle.fftconv(u, kext), rtol=0, atol=1e-13)
    # Eq. 1 written with dense DFT matrices
    n = np.arange(M)
    F = np.exp(-2j * np.pi * np.outer(n, n) / M)
    upad = np.zeros((B, H, M))
    upad[..., :N] = u
    want = np.real(np.einsum("fn,bhf->bhn", np.conj(F) / M, np.einsum("fn,bhn->bhf", F, upad) * (kext @ F.T)[None]))[..., :N]
    assert np.allclose(oracle.fftconv_taps(u, pos, val, M), want, rtol=0, atol=1e-11)
    # causal taps (all below M - N + 1): the library's polynomial product, channel by channel
    posc = np.stack([RNG.permutation(M - N + 1)[:T] for _ in range(H)])
    yc = oracle.fftconv_taps(u, posc, val, M)
    for b in range(B):
        for h in range(H):
            kk = np.zeros(M)
            kk[posc[h]] = val[h]
            assert np.allclose(yc[b, h], np.convolve(u[b, h], kk)[:N], rtol=0, atol=1e-13)


def test_taps_integer_inputs_are_exact_and_bad_arguments_are_rejected():
    u = RNG.integers(-5, 6, (1, 2, 33)).astype(np.float64)
    pos = np.array([[0, 3, 65], [1, 2, 40]])
    val = np.array([[2.0, -1.0, 3.0], [1.0, 1.0, -4.0]])
    y = oracle.fftconv_taps(u, pos, val, 66)
    kext = np.zeros((2, 66))
    for h in range(2):
        kext[h, pos[h]] = val[h]
    assert np.array_equal(y, oracle.fftconv(u, kext))
    with pytest.raises(ValueError):
        oracle.fftconv_taps(u, np.array([[0, 0, 1], [1, 2, 3]]), val, 66)      # a repeated position
    with pytest.raises(ValueError):
        oracle.fftconv_taps(u, np.array([[0, 66, 1], [1, 2, 3]]), val, 66)     # position out of range
    with pytest.raises(ValueError):
        oracle.fftconv_taps(u, pos, val, 32)                                   # M < N


# ---------------------------------------------------------------- gated convolution (Section 3.1 / 4.1)

def test_round_to_matches_library_casts_including_ties():
    import torch
    x = RNG.standard_normal(4096) * np.exp(RNG.uniform(-8, 8, 4096))
    # exact ties of the bf16 grid: 1 + (2j+1) * 2^-8, and of the fp16 grid: 1 + (2j+1) * 2^-11
    ties_b = 1.0 + (2 * np.arange(64) + 1) * 2.0 ** -8
    ties_h = 1.0 + (2 * np.arange(64) + 1) * 2.0 ** -11
    for vals in (x, ties_b, -ties_b, ties_h):
        t = torch.from_numpy(vals.astype(np.float32))
        assert np.array_equal(oracle.round_to(vals.astype(np.float32), "bf16"), t.to(torch.bfloat16).double().numpy())
        assert np.array_equal(oracle.round_to(vals.astype(np.float32), "f16"), t.to(torch.float16).double().numpy())
    assert np.array_equal(oracle.round_to(x, "f32"), x.astype(np.float32).astype(np.float64))


def test_gated_with_unit_gates_is_the_plain_convolution():
    u = RNG.standard_normal((2, 3, 20))
    k = RNG.standard_normal((3, 20))
    ones = np.ones_like(u)
    ref = oracle.fftconv(u.astype(np.float32), k, 40)
    for w, v in ((ones, ones), (None, ones), (ones, None), (None, None)):
        assert np.allclose(oracle.fftconv_gated(u.astype(np.float32), w, v, k, 40), ref, rtol=0, atol=1e-12)


def test_gated_integer_inputs_are_exact():
    B, H, N = 2, 2, 17
    u = RNG.integers(-4, 5, (B, H, N)).astype(np.float64)
    w = RNG.integers(-2, 3, (B, H, N)).astype(np.float64)
    v = RNG.integers(-3, 4, (B, H, N)).astype(np.float64)
    k = RNG.integers(-4, 5, (H, N)).astype(np.float64)
    y = oracle.fftconv_gated(u, w, v, k, 2 * N)
    for b in range(B):
        for h in range(H):
            want = v[b, h] * np.convolve(u[b, h] * w[b, h], k[h])[:N]
            assert np.array_equal(y[b, h], want)


def test_gated_input_gate_as_a_window_and_output_gate_as_a_selector():
    u = RNG.standard_normal((1, 2, 32)).astype(np.float32).astype(np.float64)
    k = RNG.standard_normal((2, 32))
    w = np.zeros_like(u)
    w[..., :10] = 1.0
    ut = u.copy()
    ut[..., 10:] = 0.0
    v = np.zeros_like(u)
    v[..., 5] = 2.0
    y = oracle.fftconv_gated(u, w, v, k, 64)
    ref = oracle.fftconv(ut, k, 64)
    assert np.allclose(y[..., 5], 2.0 * ref[..., 5], rtol=0, atol=1e-12)
    assert np.count_nonzero(np.delete(y, 5, axis=-1)) == 0


def test_gated_product_is_not_rounded_before_the_transform():
    # Section 3.1 defines y = v . ((u . w) * k) in exact arithmetic: (1 + 2^-7)^2 = 1 + 2^-6 + 2^-14 is not a
    # bf16 number, and the oracle must carry it unrounded into the convolution (delta filter: y = u . w);
    # round_to alone shows what one rounding to bf16 would have made of it
    u = np.full((1, 1, 4), 1.0 + 2.0 ** -7)
    w = u.copy()
    k = np.zeros((1, 4))
    k[0, 0] = 1.0
    y = oracle.fftconv_gated(u, w, None, k, 8)
    assert np.array_equal(y, np.full((1, 1, 4), 1.0 + 2.0 ** -6 + 2.0 ** -14))
    assert np.array_equal(oracle.round_to(y, "bf16"), np.full((1, 1, 4), 1.0 + 2.0 ** -6))


def test_gated_is_bilinear_in_u_and_w_and_linear_in_v():
    u, u2, w, v = (RNG.standard_normal((2, 2, 24)) for _ in range(4))
    k = RNG.standard_normal((2, 24))
    f = lambda a, b, c: oracle.fftconv_gated(a, b, c, k, 48)
    assert np.allclose(f(u + 2 * u2, w, v), f(u, w, v) + 2 * f(u2, w, v), rtol=0, atol=1e-11)
    assert np.allclose(f(u, w, v), f(w, u, v), rtol=0, atol=1e-12)          # u . w is symmetric
    assert np.allclose(f(u, w, 3 * v), 3 * f(u, w, v), rtol=0, atol=1e-11)


# ---------------------------------------------------------------- backward pass

def test_backward_is_the_adjoint_of_the_forward_map():
    # y is bilinear in (u, k): <dy, conv(u, k)> = <du, u> = <dk, k> for every u, k, dy
    for (B, H, N, M, Nk) in ((2, 3, 16, 32, 16), (1, 2, 12, 12, 12), (3, 1, 9, 20, 5), (2, 2, 8, 11, 11)):
        u = RNG.standard_normal((B, H, N))
        dy = RNG.standard_normal((B, H, N))
        k = RNG.standard_normal((H, Nk))
        kext = oracle.extend_filter(k, M)
        lhs = float((dy * oracle.fftconv(u, kext)).sum())
        du = oracle.backward_u(dy, kext)
        dk = oracle.backward_k(u, dy, M, Nk)
        assert abs(lhs - float((du * u).sum())) <= 1e-10 * (1 + abs(lhs))
        assert abs(lhs - float((dk * k).sum())) <= 1e-10 * (1 + abs(lhs))


def test_backward_matches_library_correlation_in_the_causal_case():
    B, H, N = 2, 2, 24
    u = RNG.standard_normal((B, H, N))
    dy = RNG.standard_normal((B, H, N))
    k = RNG.standard_normal((H, N))
    du = oracle.backward_u(dy, k, 2 * N)
    dk = oracle.backward_k(u, dy, 2 * N, N)
    for h in range(H):
        want_k = np.zeros(N)
        for b in range(B):
            # du[j] = sum_{i >= j} dy[i] k[i-j]; dk[t] = sum_{i >= t} dy[i] u[i-t]
            assert np.allclose(du[b, h], np.correlate(dy[b, h], k[h], "full")[N - 1:], rtol=0, atol=1e-12)
            want_k += np.correlate(dy[b, h], u[b, h], "full")[N - 1:]
        assert np.allclose(dk[h], want_k, rtol=0, atol=1e-12)


def test_backward_agrees_with_finite_differences_of_the_forward_oracle():
    B, H, N, M, Nk = 1, 2, 6, 8, 8                     # M < 2N: wrapped taps take part
    u = RNG.standard_normal((B, H, N))
    k = RNG.standard_normal((H, Nk))
    dy = RNG.standard_normal((B, H, N))
    kext = oracle.extend_filter(k, M)
    du = oracle.backward_u(dy, kext)
    dk = oracle.backward_k(u, dy, M, Nk)
    loss = lambda uu, kk: float((dy * oracle.fftconv(uu, oracle.extend_filter(kk, M))).sum())
    base = loss(u, k)
    for idx in np.ndindex(u.shape):
        up = u.copy()
        up[idx] += 1.0                                 # the map is linear in u: a unit step is exact
        assert abs((loss(up, k) - base) - du[idx]) <= 1e-10
    for idx in np.ndindex(k.shape):
        kp = k.copy()
        kp[idx] += 1.0
        assert abs((loss(u, kp) - base) - dk[idx]) <= 1e-10


def test_backward_integer_inputs_are_exact_and_channel_reduction_runs_over_the_batch():
    B, H, N = 3, 2, 10
    u = RNG.integers(-3, 4, (B, H, N)).astype(np.float64)
    dy = RNG.integers(-3, 4, (B, H, N)).astype(np.float64)
    dk = oracle.backward_k(u, dy, 2 * N, N)
    per_row = sum(oracle.backward_k(u[b:b + 1], dy[b:b + 1], 2 * N, N) for b in range(B))
    assert np.array_equal(dk, per_row)
    assert np.array_equal(dk, np.round(dk))
