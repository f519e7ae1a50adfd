"""Python binding of the C-ABI library libfftconv.so (see include/fftconv.h).

Argument marshalling only: every step of the convolution runs in the HIP
kernels of the library.  PyTorch supplies device memory and the stream.  There
is no fallback: if the library cannot be loaded, importing callers fail.
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import build as _build

FFTCONV_F32, FFTCONV_F16, FFTCONV_BF16 = 0, 1, 2
_DTYPE_CODE = {torch.float32: FFTCONV_F32, torch.float16: FFTCONV_F16, torch.bfloat16: FFTCONV_BF16}
_DTYPE_NAME = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}

EXPORTS = [
    "fftconv_plan_create", "fftconv_plan_destroy", "fftconv_kf_bytes", "fftconv_workspace_bytes",
    "fftconv_filter_fft", "fftconv_forward", "fftconv_forward_partial", "fftconv_filter_fft_sparse",
    "fftconv_forward_freq_sparse", "fftconv_sparsity_fraction", "fftconv_plan_path", "fftconv_plan_factors",
    "fftconv_strerror", "fftconv_last_error", "fftconv_workspace_bytes_gated", "fftconv_forward_gated",
    "fftconv_filter_fft_adjoint", "fftconv_backward_input", "fftconv_workspace_bytes_backward_filter",
    "fftconv_backward_filter", "fftconv_machine_preset", "fftconv_cost_model", "fftconv_balanced_factors",
    "fftconv_plan_order", "fftconv_filter_fft_sparse_digits", "fftconv_forward_freq_sparse_digits",
    "fftconv_forward_static", "fftconv_plan_create_path", "fftconv_measure_machine",
]

STATIC_WORKSPACE_BYTES = 64 << 20      # FFTCONV_STATIC_WORKSPACE_BYTES

_libs = {}


class Machine(ctypes.Structure):
    """fftconv_machine: the constants of the cost model (Section 3.2, Eq. 2)."""
    _fields_ = [("sigma_H", ctypes.c_double), ("sigma_S", ctypes.c_double), ("tau_M", ctypes.c_double),
                ("tau_G", ctypes.c_double), ("mu", ctypes.c_int), ("sram_seq", ctypes.c_int64)]


MACHINE_MI355X, MACHINE_A100_PAPER = 0, 1


class FFTConvError(RuntimeError):
    def __init__(self, code: int, detail: str):
        super().__init__("fftconv error %d: %s" % (code, detail))
        self.code = code


def library_path() -> str:
    return _build.LIB


def load(path: str | None = None):
    """Load libfftconv.so (building it first only if no built library exists) and declare its entry points.
    path: another build of the same ABI (the tests load the barrier-checking build this way)."""
    path = os.path.abspath(path) if path else _build.LIB
    if path in _libs:
        return _libs[path]
    if not os.path.exists(path):
        if path != _build.LIB:
            raise FileNotFoundError(path)
        _build.build()
    lib = ctypes.CDLL(path)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    lib.fftconv_plan_create.argtypes = [ctypes.POINTER(vp), i64, i64, i64, ci]
    lib.fftconv_plan_create.restype = ci
    lib.fftconv_plan_create_path.argtypes = [ctypes.POINTER(vp), i64, i64, i64, ci, ctypes.c_char_p]
    lib.fftconv_plan_create_path.restype = ci
    lib.fftconv_plan_destroy.argtypes = [vp]
    lib.fftconv_plan_destroy.restype = ci
    lib.fftconv_kf_bytes.argtypes = [vp]
    lib.fftconv_kf_bytes.restype = ctypes.c_size_t
    lib.fftconv_workspace_bytes.argtypes = [vp, i64]
    lib.fftconv_workspace_bytes.restype = ctypes.c_size_t
    lib.fftconv_filter_fft.argtypes = [vp, vp, i64, vp, vp]
    lib.fftconv_filter_fft.restype = ci
    lib.fftconv_forward.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp]
    lib.fftconv_forward.restype = ci
    lib.fftconv_forward_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp]
    lib.fftconv_forward_static.restype = ci
    lib.fftconv_forward_partial.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp, vp]
    lib.fftconv_forward_partial.restype = ci
    lib.fftconv_filter_fft_sparse.argtypes = [vp, vp, i64, vp, i64, vp, vp]
    lib.fftconv_filter_fft_sparse.restype = ci
    lib.fftconv_forward_freq_sparse.argtypes = [vp, vp, vp, vp, i64, vp, i64, i64, i64, vp, vp]
    lib.fftconv_forward_freq_sparse.restype = ci
    lib.fftconv_workspace_bytes_gated.argtypes = [vp, i64]
    lib.fftconv_workspace_bytes_gated.restype = ctypes.c_size_t
    lib.fftconv_forward_gated.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, vp]
    lib.fftconv_forward_gated.restype = ci
    lib.fftconv_filter_fft_adjoint.argtypes = [vp, vp, i64, vp, vp]
    lib.fftconv_filter_fft_adjoint.restype = ci
    lib.fftconv_backward_input.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp]
    lib.fftconv_backward_input.restype = ci
    lib.fftconv_workspace_bytes_backward_filter.argtypes = [vp, i64]
    lib.fftconv_workspace_bytes_backward_filter.restype = ctypes.c_size_t
    lib.fftconv_backward_filter.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp, vp]
    lib.fftconv_backward_filter.restype = ci
    lib.fftconv_sparsity_fraction.argtypes = [ctypes.POINTER(i64), ctypes.POINTER(i64), ci]
    lib.fftconv_sparsity_fraction.restype = ctypes.c_double
    lib.fftconv_filter_fft_sparse_digits.argtypes = [vp, vp, i64, ctypes.POINTER(i64), ci, vp, vp]
    lib.fftconv_filter_fft_sparse_digits.restype = ci
    lib.fftconv_forward_freq_sparse_digits.argtypes = [vp, vp, vp, ctypes.POINTER(i64), ci, vp, i64, i64, i64, vp, vp]
    lib.fftconv_forward_freq_sparse_digits.restype = ci
    mp = ctypes.POINTER(Machine)
    lib.fftconv_machine_preset.argtypes = [ci, mp]
    lib.fftconv_machine_preset.restype = None
    lib.fftconv_measure_machine.argtypes = [mp]
    lib.fftconv_measure_machine.restype = ci
    lib.fftconv_cost_model.argtypes = [mp, i64, i64, i64, ci, ctypes.POINTER(i64)]
    lib.fftconv_cost_model.restype = ctypes.c_double
    lib.fftconv_balanced_factors.argtypes = [i64, ci, ctypes.POINTER(i64)]
    lib.fftconv_balanced_factors.restype = ci
    lib.fftconv_plan_order.argtypes = [mp, i64, ctypes.POINTER(ci), ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)]
    lib.fftconv_plan_order.restype = ci
    lib.fftconv_plan_path.argtypes = [vp]
    lib.fftconv_plan_path.restype = ctypes.c_char_p
    lib.fftconv_plan_factors.argtypes = [vp, ctypes.POINTER(i64), ci]
    lib.fftconv_plan_factors.restype = ci
    lib.fftconv_strerror.argtypes = [ci]
    lib.fftconv_strerror.restype = ctypes.c_char_p
    lib.fftconv_last_error.argtypes = []
    lib.fftconv_last_error.restype = ctypes.c_char_p
    _libs[path] = lib
    return lib


def _check(rc: int, lib=None):
    if rc != 0:
        lib = lib or load()
        detail = lib.fftconv_last_error().decode() or lib.fftconv_strerror(rc).decode()
        raise FFTConvError(rc, detail)


def _stream_ptr():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def sparsity_fraction(dims, cuts) -> float:
    """fftconv_sparsity_fraction: share of k_f zeroed by per-dimension cut-offs."""
    n = len(dims)
    if len(cuts) != n:
        raise ValueError("dims and cuts differ in length")
    arr = ctypes.c_int64 * max(n, 1)
    v = load().fftconv_sparsity_fraction(arr(*dims), arr(*cuts), n)
    if v < 0:
        raise ValueError("bad sparsity pattern")
    return v


def machine_preset(which: int = MACHINE_MI355X) -> Machine:
    """fftconv_machine_preset."""
    m = Machine()
    load().fftconv_machine_preset(which, ctypes.byref(m))
    return m


def measure_machine() -> Machine:
    """fftconv_measure_machine: the four rates of the cost model measured on the current GPU (about a second)."""
    m = Machine()
    _check(load().fftconv_measure_machine(ctypes.byref(m)))
    return m


def cost_model(machine: Machine, B: int, H: int, N: int, factors) -> float:
    """fftconv_cost_model: Eq. 2 in seconds for the given factors (outermost first)."""
    arr = (ctypes.c_int64 * len(factors))(*factors)
    v = load().fftconv_cost_model(ctypes.byref(machine), B, H, N, len(factors), arr)
    if v < 0:
        raise ValueError("bad decomposition")
    return v


def balanced_factors(N: int, p: int):
    """fftconv_balanced_factors."""
    arr = (ctypes.c_int64 * 8)()
    rc = load().fftconv_balanced_factors(N, p, arr)
    if rc:
        raise ValueError("N must be a power of two and 1 <= p <= 8")
    return [int(arr[i]) for i in range(p)]


def plan_order(machine: Machine, N: int):
    """fftconv_plan_order: (p, factors, cost per sequence in seconds) of the cheapest order in {2, 3, 4}."""
    p = ctypes.c_int()
    arr = (ctypes.c_int64 * 4)()
    c = ctypes.c_double()
    rc = load().fftconv_plan_order(ctypes.byref(machine), N, ctypes.byref(p), arr, ctypes.byref(c))
    if rc:
        raise ValueError("N must be a power of two >= 4")
    return p.value, [int(arr[i]) for i in range(p.value)], c.value


class Plan:
    """fftconv_plan_create / fftconv_plan_destroy and the calls that take a plan."""

    def __init__(self, N: int, fft_size: int, H: int, dtype, lib=None, path: str | None = None):
        if isinstance(dtype, str):
            dtype = _DTYPE_NAME[dtype]
        self.N, self.fft_size, self.H, self.dtype = int(N), int(fft_size), int(H), dtype
        self._lib = lib or load()
        self._h = ctypes.c_void_p()
        # path: force a kernel family (fftconv_plan_create_path); None = the cost model's choice
        self._ok(self._lib.fftconv_plan_create_path(ctypes.byref(self._h), self.N, self.fft_size, self.H, _DTYPE_CODE[dtype],
                                                    path.encode() if path else None))
        self._ws = None

    def _ok(self, rc: int):
        _check(rc, self._lib)

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            self._lib.fftconv_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def path(self) -> str:
        return self._lib.fftconv_plan_path(self._h).decode()

    @property
    def factors(self):
        buf = (ctypes.c_int64 * 8)()
        n = self._lib.fftconv_plan_factors(self._h, buf, 8)
        return [int(buf[i]) for i in range(n)]

    def kf_bytes(self) -> int:
        return int(self._lib.fftconv_kf_bytes(self._h))

    def workspace_bytes(self, B: int) -> int:
        return int(self._lib.fftconv_workspace_bytes(self._h, int(B)))

    def workspace_bytes_gated(self, B: int) -> int:
        return int(self._lib.fftconv_workspace_bytes_gated(self._h, int(B)))

    def _workspace(self, B: int, device, gated: bool = False):
        need = self.workspace_bytes_gated(B) if gated else self.workspace_bytes(B)
        if need == 0:
            return None
        if self._ws is None or self._ws.numel() < need or self._ws.device != device:
            self._ws = torch.empty(need, dtype=torch.uint8, device=device)
        return self._ws

    def _check_k(self, k):
        if k.dtype != torch.float32 or not k.is_cuda or not k.is_contiguous() or k.dim() != 2 or k.shape[0] != self.H:
            raise ValueError("k must be a contiguous CUDA fp32 tensor of shape (H, Nk)")

    def filter_fft(self, k: torch.Tensor, block_keep=None) -> torch.Tensor:
        """fftconv_filter_fft / fftconv_filter_fft_sparse: returns the opaque k_f buffer."""
        self._check_k(k)
        kf = torch.empty(self.kf_bytes(), dtype=torch.uint8, device=k.device)
        if block_keep is None:
            self._ok(self._lib.fftconv_filter_fft(self._h, k.data_ptr(), k.shape[1], kf.data_ptr(), _stream_ptr()))
        else:
            bk = bytes(bytearray(int(x) for x in block_keep))
            self._ok(self._lib.fftconv_filter_fft_sparse(self._h, k.data_ptr(), k.shape[1], bk, len(bk), kf.data_ptr(),
                                                       _stream_ptr()))
        return kf

    def _check_u(self, u):
        if (u.dtype != self.dtype or not u.is_cuda or not u.is_contiguous() or u.dim() != 3
                or u.shape[1] != self.H or u.shape[2] != self.N):
            raise ValueError("u must be a contiguous CUDA tensor (B, H=%d, N=%d) of dtype %s" % (self.H, self.N, self.dtype))

    def forward(self, u: torch.Tensor, kf: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
        """fftconv_forward."""
        self._check_u(u)
        y = torch.empty_like(u) if out is None else out
        ws = self._workspace(u.shape[0], u.device)
        self._ok(self._lib.fftconv_forward(self._h, u.data_ptr(), kf.data_ptr(), y.data_ptr(), u.shape[0], self.H,
                                         self.N, None if ws is None else ws.data_ptr(), _stream_ptr()))
        return y

    def forward_static(self, u: torch.Tensor, kf: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
        """fftconv_forward_static: the caller passes the output; nothing is allocated on the way."""
        self._check_u(u)
        self._ok(self._lib.fftconv_forward_static(self._h, u.data_ptr(), kf.data_ptr(), out.data_ptr(), u.shape[0],
                                                  self.H, self.N, _stream_ptr()))
        return out

    def forward_gated(self, u, w, v, kf, out=None):
        """fftconv_forward_gated: y = v . ((u . w) * k); w and/or v may be None."""
        self._check_u(u)
        for g in (w, v):
            if g is not None:
                self._check_u(g)
                if g.shape != u.shape:
                    raise ValueError("gates must have the shape of u")
        y = torch.empty_like(u) if out is None else out
        ws = self._workspace(u.shape[0], u.device, gated=True)
        self._ok(self._lib.fftconv_forward_gated(self._h, u.data_ptr(), None if w is None else w.data_ptr(),
                                               None if v is None else v.data_ptr(), kf.data_ptr(), y.data_ptr(),
                                               u.shape[0], self.H, self.N, None if ws is None else ws.data_ptr(),
                                               _stream_ptr()))
        return y

    def filter_fft_adjoint(self, k: torch.Tensor) -> torch.Tensor:
        """fftconv_filter_fft_adjoint: the k_f buffer fftconv_backward_input takes."""
        self._check_k(k)
        kf = torch.empty(self.kf_bytes(), dtype=torch.uint8, device=k.device)
        self._ok(self._lib.fftconv_filter_fft_adjoint(self._h, k.data_ptr(), k.shape[1], kf.data_ptr(), _stream_ptr()))
        return kf

    def backward_input(self, dy, kf_adjoint, out=None):
        """fftconv_backward_input: du."""
        self._check_u(dy)
        du = torch.empty_like(dy) if out is None else out
        ws = self._workspace(dy.shape[0], dy.device)
        self._ok(self._lib.fftconv_backward_input(self._h, dy.data_ptr(), kf_adjoint.data_ptr(), du.data_ptr(),
                                                dy.shape[0], self.H, self.N, None if ws is None else ws.data_ptr(),
                                                _stream_ptr()))
        return du

    def backward_filter(self, u, dy, Nk: int, out=None):
        """fftconv_backward_filter: dk, (H, Nk) fp32."""
        self._check_u(u)
        self._check_u(dy)
        if u.shape != dy.shape:
            raise ValueError("u and dy differ in shape")
        dk = torch.empty((self.H, int(Nk)), dtype=torch.float32, device=u.device) if out is None else out
        need = int(self._lib.fftconv_workspace_bytes_backward_filter(self._h, u.shape[0]))
        if getattr(self, "_ws_bk", None) is None or self._ws_bk.numel() < need or self._ws_bk.device != u.device:
            self._ws_bk = torch.empty(max(need, 1), dtype=torch.uint8, device=u.device)
        self._ok(self._lib.fftconv_backward_filter(self._h, u.data_ptr(), dy.data_ptr(), dk.data_ptr(), int(Nk),
                                                 u.shape[0], self.H, self.N, self._ws_bk.data_ptr(), _stream_ptr()))
        return dk

    def forward_partial(self, u, kf, Nk: int, out=None):
        """fftconv_forward_partial."""
        self._check_u(u)
        y = torch.empty_like(u) if out is None else out
        ws = self._workspace(u.shape[0], u.device)
        self._ok(self._lib.fftconv_forward_partial(self._h, u.data_ptr(), kf.data_ptr(), y.data_ptr(), u.shape[0],
                                                 self.H, self.N, int(Nk), None if ws is None else ws.data_ptr(),
                                                 _stream_ptr()))
        return y

    def filter_fft_sparse_digits(self, k, digit_keep):
        """fftconv_filter_fft_sparse_digits: k (H, Nk) fp32 on the device -> opaque k_f."""
        self._check_k(k)
        Nk = k.shape[1]
        kf = torch.empty(self.kf_bytes(), dtype=torch.uint8, device=k.device)
        arr = (ctypes.c_int64 * len(digit_keep))(*[int(x) for x in digit_keep])
        self._ok(self._lib.fftconv_filter_fft_sparse_digits(self._h, k.data_ptr(), Nk, arr, len(digit_keep),
                                                          kf.data_ptr(), _stream_ptr()))
        return kf

    def forward_freq_sparse_digits(self, u, kf, digit_keep, out=None):
        """fftconv_forward_freq_sparse_digits."""
        self._check_u(u)
        y = torch.empty_like(u) if out is None else out
        ws = self._workspace(u.shape[0], u.device)
        arr = (ctypes.c_int64 * len(digit_keep))(*[int(x) for x in digit_keep])
        self._ok(self._lib.fftconv_forward_freq_sparse_digits(self._h, u.data_ptr(), kf.data_ptr(), arr, len(digit_keep),
                                                            y.data_ptr(), u.shape[0], self.H, self.N,
                                                            None if ws is None else ws.data_ptr(), _stream_ptr()))
        return y

    def forward_freq_sparse(self, u, kf, block_keep, out=None):
        """fftconv_forward_freq_sparse."""
        self._check_u(u)
        y = torch.empty_like(u) if out is None else out
        ws = self._workspace(u.shape[0], u.device)
        bk = bytes(bytearray(int(x) for x in block_keep))
        self._ok(self._lib.fftconv_forward_freq_sparse(self._h, u.data_ptr(), kf.data_ptr(), bk, len(bk), y.data_ptr(),
                                                     u.shape[0], self.H, self.N,
                                                     None if ws is None else ws.data_ptr(), _stream_ptr()))
        return y
