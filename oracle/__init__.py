"""fp64 CPU oracle for the FFT-convolution path -- TEST INFRASTRUCTURE ONLY.

Thin numpy front end of ``conv_oracle.c`` (plain C, term-by-term sums in
double precision; see that file's header for the definitions it follows:
paper Section 2.1 for the convolution, Eq. 1 for its circular form, Section
3.3 / Appendix A.4 for partial and frequency-sparse filters, Section 3.1 /
4.1 for the gated form).

Nothing in the product package may import this module; it shares no code with
the HIP library.  Allowed callers: ``tests/``, ``__graft_entry__.smoke()`` and
the ``cpu_baseline`` leg of ``bench.py``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_SO = os.path.join(_HERE, "libconv_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile conv_oracle.c with gcc into libconv_oracle.so next to it."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _SO)
    return _SO


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        p = ctypes.c_void_p
        i64 = ctypes.c_int64
        lib.oracle_fftconv.argtypes = [p, p, p, i64, i64, i64, i64]
        lib.oracle_fftconv.restype = ctypes.c_int
        lib.oracle_fftconv_at.argtypes = [p, p, p, p, i64, i64, i64, i64]
        lib.oracle_fftconv_at.restype = ctypes.c_int
        lib.oracle_fftconv_taps.argtypes = [p, p, p, p, i64, i64, i64, i64, i64]
        lib.oracle_fftconv_taps.restype = ctypes.c_int
        lib.oracle_mask_filter.argtypes = [p, p, p, i64, i64]
        lib.oracle_mask_filter.restype = ctypes.c_int
        lib.oracle_backward_u.argtypes = [p, p, p, i64, i64, i64, i64]
        lib.oracle_backward_u.restype = ctypes.c_int
        lib.oracle_backward_k.argtypes = [p, p, p, i64, i64, i64, i64, i64]
        lib.oracle_backward_k.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def extend_filter(k, M: int) -> np.ndarray:
    """Lay a filter k of shape (H, Nk), Nk <= M, out on M taps (zeros after Nk)."""
    k = _f64(k)
    if k.ndim != 2 or k.shape[1] > M:
        raise ValueError("k must be (H, Nk) with Nk <= M")
    out = np.zeros((k.shape[0], M), dtype=np.float64)
    out[:, : k.shape[1]] = k
    return out


def fftconv(u, kext, M: int | None = None) -> np.ndarray:
    """y[b,h,i] = sum_j u[b,h,j] * kext[h,(i-j) mod M] for 0 <= i < N.

    u: (B,H,N); kext: (H,M) -- or (H,Nk) with M given, zero-extended here.
    """
    u = _f64(u)
    kext = _f64(kext)
    if M is not None and kext.shape[1] != M:
        kext = extend_filter(kext, M)
    B, H, N = u.shape
    if kext.shape[0] != H:
        raise ValueError("filter rows must equal H")
    M = kext.shape[1]
    y = np.empty_like(u)
    rc = _load().oracle_fftconv(u.ctypes.data, kext.ctypes.data, y.ctypes.data, B, H, N, M)
    if rc != 0:
        raise ValueError("oracle_fftconv rejected sizes B=%d H=%d N=%d M=%d" % (B, H, N, M))
    return y


def fftconv_at(u_rows, kext_rows, idx) -> np.ndarray:
    """The same sum at chosen output positions.

    u_rows: (S,N) sequences; kext_rows: (S,M) the filter row of each sequence;
    idx: (S,P) int positions in [0,N).  Returns (S,P).
    """
    u_rows = _f64(u_rows)
    kext_rows = _f64(kext_rows)
    idx = np.ascontiguousarray(np.asarray(idx, dtype=np.int64))
    S, N = u_rows.shape
    if kext_rows.shape[0] != S or idx.shape[0] != S:
        raise ValueError("row counts differ")
    M = kext_rows.shape[1]
    P = idx.shape[1]
    out = np.empty((S, P), dtype=np.float64)
    rc = _load().oracle_fftconv_at(
        u_rows.ctypes.data, kext_rows.ctypes.data, idx.ctypes.data, out.ctypes.data, S, N, M, P
    )
    if rc != 0:
        raise ValueError("oracle_fftconv_at rejected its arguments")
    return out


def fftconv_taps(u, pos, val, M: int) -> np.ndarray:
    """The convolution of fftconv() for a filter with few non-zero taps: channel h has taps val[h,t] at
    positions pos[h,t] in [0,M) (distinct within a channel), zero elsewhere.  O(T N) per sequence.

    u: (B,H,N); pos: (H,T) int; val: (H,T).  Returns (B,H,N).
    """
    u = _f64(u)
    pos = np.ascontiguousarray(np.asarray(pos, dtype=np.int64))
    val = _f64(val)
    B, H, N = u.shape
    if pos.shape != val.shape or pos.ndim != 2 or pos.shape[0] != H:
        raise ValueError("pos and val must both be (H, T)")
    y = np.empty_like(u)
    rc = _load().oracle_fftconv_taps(u.ctypes.data, pos.ctypes.data, val.ctypes.data, y.ctypes.data, B, H, N, int(M),
                                     pos.shape[1])
    if rc != 0:
        raise ValueError("oracle_fftconv_taps rejected its arguments (sizes, or tap positions out of range / repeated)")
    return y


def mask_filter(kext, keep) -> np.ndarray:
    """Time-domain filter of the spectrum DFT_M(kext) with bins keep[f]==0 zeroed.

    kext: (H,M) real; keep: (M,) of 0/1 indexed by natural frequency f.
    Returns Re(IDFT(keep * DFT(kext))), shape (H,M), by naive O(M^2) sums.
    """
    kext = _f64(kext)
    keep = np.ascontiguousarray(np.asarray(keep, dtype=np.uint8))
    H, M = kext.shape
    if keep.shape != (M,):
        raise ValueError("keep must have one entry per frequency bin")
    out = np.empty_like(kext)
    rc = _load().oracle_mask_filter(kext.ctypes.data, keep.ctypes.data, out.ctypes.data, H, M)
    if rc != 0:
        raise RuntimeError("oracle_mask_filter failed (%d)" % rc)
    return out


def round_to(x, dtype: str) -> np.ndarray:
    """Round fp64 values to the I/O dtype ("f32", "f16", "bf16"), nearest even, and return them as fp64.
    A diagnostic helper for tests (how far one rounding moves a value); no oracle result depends on it.

    bf16 is the upper half of fp32: round the fp32 bit pattern to 16 bits (finite inputs only).
    """
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        b = np.ascontiguousarray(x.astype(np.float32)).view(np.uint32).astype(np.uint64)
        b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
        return b.astype(np.uint32).view(np.float32).astype(np.float64)
    raise ValueError("dtype must be f32, f16 or bf16")


def fftconv_gated(u, w, v, kext, M: int | None = None) -> np.ndarray:
    """Gated convolution y = v . ((u . w) * k) (Section 3.1, "Domain-Specific Optimizations"; Section 4.1).

    u, w, v: (B,H,N), w and/or v may be None (no gate on that side).  Exact fp64 throughout: the
    elementwise products and the convolution are evaluated as the definition states them, with no
    intermediate rounding.
    """
    p = _f64(u)
    if w is not None:
        p = p * _f64(w)
    y = fftconv(p, kext, M)
    if v is not None:
        y = y * _f64(v)
    return y


def backward_u(dy, kext, M: int | None = None) -> np.ndarray:
    """du[b,h,j] = sum_i dy[b,h,i] * kext[h,(i-j) mod M]: gradient of fftconv with respect to u."""
    dy = _f64(dy)
    kext = _f64(kext)
    if M is not None and kext.shape[1] != M:
        kext = extend_filter(kext, M)
    B, H, N = dy.shape
    if kext.shape[0] != H:
        raise ValueError("filter rows must equal H")
    du = np.empty_like(dy)
    if _load().oracle_backward_u(dy.ctypes.data, kext.ctypes.data, du.ctypes.data, B, H, N, kext.shape[1]) != 0:
        raise ValueError("oracle_backward_u rejected its sizes")
    return du


def backward_k(u, dy, M: int, Nk: int) -> np.ndarray:
    """dk[h,t] = sum_b sum_i dy[b,h,i] * upad[b,h,(i-t) mod M] for t < Nk: gradient with respect to the filter taps."""
    u = _f64(u)
    dy = _f64(dy)
    if u.shape != dy.shape:
        raise ValueError("u and dy differ in shape")
    B, H, N = u.shape
    dk = np.empty((H, Nk), dtype=np.float64)
    if _load().oracle_backward_k(u.ctypes.data, dy.ctypes.data, dk.ctypes.data, B, H, N, int(M), int(Nk)) != 0:
        raise ValueError("oracle_backward_k rejected its sizes")
    return dk


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def rel_l2_per_sequence(y, y_ref) -> np.ndarray:
    """||y - y_ref||_2 / ||y_ref||_2 over the last axis (the parity metric)."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    num = np.sqrt(((y - y_ref) ** 2).sum(axis=-1))
    den = np.sqrt((y_ref ** 2).sum(axis=-1))
    return num / np.where(den > 0, den, 1.0)
