"""Seeded synthetic inputs for the FFT-convolution workloads.

This module only draws random numbers and rounds them to the I/O dtype.  It
holds none of the convolution's arithmetic, so that both the HIP path and the
CPU checker used by the tests can be fed identical bytes from it.

The paper benchmarks the convolution on random tensors with batch size 64 and
hidden dimension 768 over power-of-two lengths (Appendix C, "Convolution
Benchmarks"); the decaying random filters stand in for trained long-convolution
filters of Hyena / M2 style models.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    fft_size: int
    dtype: str                      # I/O dtype of u and y: "f32" | "f16" | "bf16"
    alpha: tuple                    # (lo, hi) of the per-channel decay rate; lo == hi -> constant
    seed_u: int
    seed_k: int
    seed_alpha: int
    Nk: int = 0                     # filter support (0 = N); taps t >= Nk are zero ("partial")
    keep_blocks: tuple = field(default=())   # frequency-sparse: kept blocks out of n_blocks
    n_blocks: int = 0

    @property
    def filter_len(self) -> int:
        return self.Nk if self.Nk else self.N


def _lowpass_blocks(n_blocks: int, keep_fraction: float) -> tuple:
    """Blocks of natural-order frequencies nearest DC (both ends of the axis)."""
    n_keep = max(2, int(round(n_blocks * keep_fraction)))
    half = n_keep // 2
    return tuple(list(range(half)) + list(range(n_blocks - (n_keep - half), n_blocks)))


WORKLOADS = {
    # small fp32 case
    "cfg1": Workload("cfg1", 2, 4, 1024, 2048, "f32", (0.01, 0.01), 1001, 1002, 1003),
    # headline: bf16, fft 8192
    "cfg2": Workload("cfg2", 64, 768, 4096, 8192, "bf16", (1e-3, 1e-1), 2001, 2002, 2003),
    # fp16, fft 32768
    "cfg3": Workload("cfg3", 16, 768, 16384, 32768, "f16", (1e-4, 1e-2), 3001, 3002, 3003),
    # very long, fft 2^21
    "cfg4": Workload("cfg4", 1, 64, 1 << 20, 1 << 21, "bf16", (1e-5, 1e-5), 4001, 4002, 4003),
    # sparse variants, fft 16384
    "cfg5a": Workload("cfg5a", 32, 768, 8192, 16384, "bf16", (1e-3, 1e-1), 5001, 5002, 5003, Nk=1024),
    "cfg5b": Workload("cfg5b", 32, 768, 8192, 16384, "bf16", (1e-3, 1e-1), 5001, 5002, 5003,
                      keep_blocks=_lowpass_blocks(32, 0.25), n_blocks=32),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some sizes replaced (reduced test cases)."""
    d = dict(w.__dict__)
    d.update(kw)
    return Workload(**d)


def gen_u(w: Workload, b_indices=None) -> torch.Tensor:
    """u[b] ~ N(0,1) for the listed batch rows, rounded (RNE) to the I/O dtype.

    Every batch row has its own counter-based stream, so any subset of rows can
    be regenerated without drawing the others.  Returns a CPU tensor
    (len(b_indices), H, N).
    """
    if b_indices is None:
        b_indices = range(w.B)
    rows = []
    for b in b_indices:
        g = np.random.Generator(np.random.Philox(key=[w.seed_u, int(b)]))
        x = g.standard_normal((w.H, w.N), dtype=np.float32)
        rows.append(torch.from_numpy(x).to(TORCH_DTYPE[w.dtype]))
    if not rows:
        return torch.empty((0, w.H, w.N), dtype=TORCH_DTYPE[w.dtype])
    return torch.stack(rows, 0)


def gen_gate(w: Workload, which: str, b_indices=None) -> torch.Tensor:
    """Gate tensor of the gated convolution ("w": input gate, "v": output gate) or upstream gradient of
    the backward pass ("dy"): N(0,1) per element,
    rounded to the I/O dtype, one counter-based stream per batch row like gen_u.  Stands in for the
    linear projections of the layer input that Hyena / M2 use as gates."""
    if b_indices is None:
        b_indices = range(w.B)
    seed = w.seed_u + {"w": 100, "v": 200, "dy": 300}[which]
    rows = []
    for b in b_indices:
        g = np.random.Generator(np.random.Philox(key=[seed, int(b)]))
        rows.append(torch.from_numpy(g.standard_normal((w.H, w.N), dtype=np.float32)).to(TORCH_DTYPE[w.dtype]))
    if not rows:
        return torch.empty((0, w.H, w.N), dtype=TORCH_DTYPE[w.dtype])
    return torch.stack(rows, 0)


def gen_alpha(w: Workload) -> np.ndarray:
    lo, hi = w.alpha
    if lo == hi:
        return np.full((w.H,), lo, dtype=np.float64)
    g = np.random.Generator(np.random.Philox(key=[w.seed_alpha, 0]))
    return g.uniform(lo, hi, size=(w.H,))


def gen_k(w: Workload) -> np.ndarray:
    """fp32 filter (H, N): N(0,1) * exp(-alpha_h * t); taps t >= Nk zeroed if Nk is set."""
    g = np.random.Generator(np.random.Philox(key=[w.seed_k, 0]))
    z = g.standard_normal((w.H, w.N))
    t = np.arange(w.N, dtype=np.float64)
    k = (z * np.exp(-gen_alpha(w)[:, None] * t[None, :])).astype(np.float32)
    if w.Nk:
        k[:, w.Nk:] = 0.0
    return k


TAP_KINDS = 5
TAPS = 16


def gen_taps(H: int, L: int, seed: int):
    """Filters with few non-zero taps on [0, L), one kind per channel in turn (h mod 5): a unit tap at position
    0, at 1, at L/2, at L-1, and 16 taps of value +1 or -1, one in each sixteenth of [0, L) at a random offset
    with the last one moved to L-1.  Unlike decaying filters these weight the late taps as much as the early
    ones.  Returns (pos, val), both (H, 16); entries with val 0 are placeholders at distinct unused positions."""
    if L < 4 * TAPS:
        raise ValueError("L too short for 16 separated taps")
    g = np.random.Generator(np.random.Philox(key=[seed, L]))
    pos = np.zeros((H, TAPS), dtype=np.int64)
    val = np.zeros((H, TAPS), dtype=np.float64)
    single = [0, 1, L // 2, L - 1]
    for h in range(H):
        kind = h % TAP_KINDS
        if kind < 4:
            pos[h, 0] = single[kind]
            val[h, 0] = 1.0
            free = [p for p in range(2, 2 + 2 * TAPS) if p not in single][: TAPS - 1]
            pos[h, 1:] = free
        else:
            step = L // TAPS
            pos[h] = np.arange(TAPS) * step + g.integers(0, step, TAPS)
            pos[h, -1] = L - 1
            val[h] = g.choice([-1.0, 1.0], TAPS)
    return pos, val


def taps_to_filter(pos, val, L: int) -> np.ndarray:
    """The taps of gen_taps laid out as a dense fp32 filter (H, L), the form the library takes."""
    H = pos.shape[0]
    k = np.zeros((H, L), dtype=np.float32)
    for h in range(H):
        k[h, pos[h]] = val[h]
    return k


def block_keep(w: Workload) -> np.ndarray:
    """uint8 flag per frequency block (1 = kept); all ones when the workload is dense."""
    if not w.n_blocks:
        return np.ones((1,), dtype=np.uint8)
    m = np.zeros((w.n_blocks,), dtype=np.uint8)
    m[list(w.keep_blocks)] = 1
    return m


def sample_sequences(w: Workload, n_random: int, seed: int = 7) -> list:
    """Deterministic (b, h) sample: every corner of the (B, H) grid plus random picks."""
    pts = {(0, 0), (0, w.H - 1), (w.B - 1, 0), (w.B - 1, w.H - 1)}
    g = np.random.Generator(np.random.Philox(key=[seed, w.seed_u]))
    while len(pts) < min(n_random + 4, w.B * w.H):
        pts.add((int(g.integers(0, w.B)), int(g.integers(0, w.H))))
    return sorted(pts)


def digit_keep_mask(factors, digit_keep) -> np.ndarray:
    """Per-bin 0/1 mask of a digit cut-off pattern: bin f = sum_i d_i w_i (w_0 = 1, w_i = w_{i-1} * factors[i-1])
    is kept when every digit is in its kept set: for digit 0 the digit_keep[0] values nearest zero on the circle
    (ties to the smaller value), for the others the digit_keep[i] values nearest the two ends of the range (the odd
    one at the low end).  Input structure only: no arithmetic of the method."""
    M = int(np.prod(factors))
    f = np.arange(M, dtype=np.int64)
    keep = np.ones(M, dtype=bool)
    for i, (D, kp) in enumerate(zip(factors, digit_keep)):
        d = f % D
        f = f // D
        if i == 0:
            order = sorted(range(D), key=lambda v: (min(v, D - v), v))
        else:
            order = sorted(range(D), key=lambda v: (min(v, D - 1 - v), v))
        kept = np.zeros(D, dtype=bool)
        kept[order[:kp]] = True
        keep &= kept[d]
    return keep.astype(np.uint8)
