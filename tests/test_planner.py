"""Cost model of Section 3.2 (Eq. 2) and the order it selects: host logic, no GPU."""
import math

import pytest

from paper_2311_05908_amd import fftconv


def a100():
    return fftconv.machine_preset(fftconv.MACHINE_A100_PAPER)


def test_presets_hold_the_papers_table_and_this_chips_constants():
    m = a100()                                    # Appendix C, measured constants for A100-40GB
    assert (m.sigma_H, m.sigma_S, m.tau_M, m.tau_G, m.mu) == (1.35e12, 9.5e12, 234e12, 17.6e12, 16)
    g = fftconv.machine_preset(fftconv.MACHINE_MI355X)
    assert g.mu == 16 and g.sram_seq == 32768
    assert g.sigma_H < 8e12 and g.tau_M < 2.5e15 + 1      # achievable rates stay below the published peaks
    assert g.sigma_S > g.sigma_H and g.tau_M > g.tau_G


def test_equation_2_by_hand():
    m = a100()
    # N = 4096 = 16 * 16 * 16, one sequence: three matrix-unit steps, the first reads HBM, two stay on chip
    want = 3 * 16 * 4096 * 16 / 234e12 + 4 * 4096 * (1 / 1.35e12 + 2 / 9.5e12)
    assert fftconv.cost_model(m, 1, 1, 4096, [16, 16, 16]) == pytest.approx(want, rel=1e-12)
    # scales with B * H
    assert fftconv.cost_model(m, 3, 5, 4096, [16, 16, 16]) == pytest.approx(15 * want, rel=1e-12)
    # a factor below the matrix unit runs at the general arithmetic rate
    want2 = 16 * 256 * (32 / 234e12 + 8 / 17.6e12) + 4 * 256 * (1 / 1.35e12 + 1 / 9.5e12)
    assert fftconv.cost_model(m, 1, 1, 256, [32, 8]) == pytest.approx(want2, rel=1e-12)
    # p = 4: the outer step and the first fused step go through HBM
    want4 = 16 * 65536 * 4 * 16 / 234e12 + 4 * 65536 * (2 / 1.35e12 + 2 / 9.5e12)
    assert fftconv.cost_model(m, 1, 1, 65536, [16, 16, 16, 16]) == pytest.approx(want4, rel=1e-12)
    # p = 3 past the on-chip limit: every intermediate in HBM
    want3 = 16 * 65536 * (64 + 32 + 32) / 234e12 + 4 * 65536 * 3 / 1.35e12
    assert fftconv.cost_model(m, 1, 1, 65536, [64, 32, 32]) == pytest.approx(want3, rel=1e-12)


def test_bad_arguments_are_rejected():
    m = a100()
    with pytest.raises(ValueError):
        fftconv.cost_model(m, 1, 1, 4096, [16, 16, 8])          # product is not N
    with pytest.raises(ValueError):
        fftconv.balanced_factors(3000, 3)
    with pytest.raises(ValueError):
        fftconv.plan_order(m, 2)


def test_balanced_factors():
    assert fftconv.balanced_factors(4096, 3) == [16, 16, 16]
    assert fftconv.balanced_factors(8192, 3) == [32, 16, 16]
    assert fftconv.balanced_factors(1 << 20, 4) == [32, 32, 32, 32]
    assert fftconv.balanced_factors(256, 2) == [16, 16]
    for lg in range(2, 23):
        for p in range(1, 5):
            f = fftconv.balanced_factors(1 << lg, p)
            assert math.prod(f) == 1 << lg and max(f) <= 2 * min(f) and f == sorted(f, reverse=True)


def test_flop_term_grows_as_n_to_the_p_plus_1_over_p():
    """Section 3.2: with equal factors the FLOP cost of order p grows as N^((p+1)/p).  With infinite bandwidths only
    the FLOP term is left; scaling every factor by 2 multiplies N by 2^p and the cost by 2^(p+1)."""
    m = a100()
    m.sigma_H = m.sigma_S = 1e300
    for p, f in ((2, 64), (3, 32), (4, 16)):
        c1 = fftconv.cost_model(m, 1, 1, f ** p, [f] * p)
        c2 = fftconv.cost_model(m, 1, 1, (2 * f) ** p, [2 * f] * p)
        assert c2 / c1 == pytest.approx(2.0 ** (p + 1), rel=1e-12)


def test_the_papers_figure_in_words():
    """Section 3.2 on its cost-model figure (A100): short sequences are cheapest at low order because higher orders
    fall below the matrix unit; order 3 jumps between 32K and 64K when the sequence no longer fits on chip; order 4
    takes over from there."""
    m = a100()
    c = {(p, lg): fftconv.cost_model(m, 1, 1, 1 << lg, fftconv.balanced_factors(1 << lg, p))
         for p in (2, 3, 4) for lg in range(8, 23)}
    for lg in range(8, 11):
        assert c[2, lg] < c[3, lg] and c[2, lg] < c[4, lg]
    # the bump of order 3: doubling N from 32K to 64K costs well over the asymptotic 2^(4/3)
    assert c[3, 16] / c[3, 15] > 3.0
    assert c[3, 15] / c[3, 14] < 2.6 and c[3, 17] / c[3, 16] < 2.6
    for lg in range(12, 16):
        assert fftconv.plan_order(m, 1 << lg)[0] == 3
    for lg in range(16, 23):
        assert c[4, lg] < c[3, lg] < c[2, lg]
        assert fftconv.plan_order(m, 1 << lg)[0] == 4


def test_order_chosen_for_this_chip_matches_the_dispatch_rule():
    """fft 8192 .. 32768 run the order-3 single-kernel path, longer ones the order-4 multi-pass path."""
    g = fftconv.machine_preset(fftconv.MACHINE_MI355X)
    for lg in range(13, 16):
        assert fftconv.plan_order(g, 1 << lg)[0] == 3
    for lg in range(16, 23):
        assert fftconv.plan_order(g, 1 << lg)[0] == 4
    for lg in range(8, 12):
        assert fftconv.plan_order(g, 1 << lg)[0] == 2


def test_a_family_without_a_kernel_for_the_shape_is_refused_before_any_device_is_touched():
    import ctypes
    lib = fftconv.load()
    h = ctypes.c_void_p()
    for N, M, dtype, path in ((4096, 8192, fftconv.FFTCONV_F32, b"fused3"),      # the fused kernels are 16-bit
                              (4096, 8192, fftconv.FFTCONV_BF16, b"small"),       # short transforms only
                              (1024, 2048, fftconv.FFTCONV_BF16, b"multipass"),   # from 8192 up
                              (1000, 8192, fftconv.FFTCONV_BF16, b"staged"),      # fp32 I/O only
                              (4096, 8192, fftconv.FFTCONV_BF16, b"no such family")):
        assert lib.fftconv_plan_create_path(ctypes.byref(h), N, M, 2, dtype, path) == -2
        assert not h.value
        assert b"no kernel of family" in lib.fftconv_last_error()


@pytest.mark.gpu
def test_measured_machine_constants_are_plausible_and_near_the_preset():
    """fftconv_measure_machine runs the micro-benchmarks of Appendix C on the GPU: achievable rates stay below the
    published peaks, are ordered as the model assumes, and the built-in preset (measured the same way) is near a
    fresh measurement: within 40 % for the three rates that are one timing each, within a factor of two for sigma_S,
    which is the DIFFERENCE of two timings (a chain of products with and without the trip through LDS) and moves
    with the clock the board grants each of them (53e12 and 73e12 have both been measured)."""
    m = fftconv.measure_machine()
    g = fftconv.machine_preset(fftconv.MACHINE_MI355X)
    assert 2e12 < m.sigma_H < 8e12 and 0.5e15 < m.tau_M < 2.6e15 and 1e13 < m.tau_G < 157.3e12
    assert m.sigma_S > 2 * m.sigma_H and m.tau_M > 5 * m.tau_G
    assert (m.mu, m.sram_seq) == (g.mu, g.sram_seq)
    for name in ("sigma_H", "tau_M", "tau_G"):
        assert abs(getattr(m, name) / getattr(g, name) - 1.0) < 0.4, (name, getattr(m, name), getattr(g, name))
    assert 0.5 < m.sigma_S / g.sigma_S < 2.0, (m.sigma_S, g.sigma_S)
