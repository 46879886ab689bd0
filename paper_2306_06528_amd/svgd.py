"""Python binding of the C-ABI SVGD library (include/svgd.h): argument marshalling only.

Every step of the method runs in the HIP kernels of libsvgd.so; torch tensors are used here
only as owners of device memory and for the current stream.  Importing this module fails
loudly if the built library is missing - there is no fallback path.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsvgd.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -m paper_2306_06528_amd.build, or "
        "__graft_entry__.build()); there is no fallback implementation")
_lib = ctypes.CDLL(LIB_PATH)

_H = ctypes.c_void_p
_lib.svgd_create.argtypes = [ctypes.POINTER(_H), ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32]
_lib.svgd_set_bandwidth.argtypes = [_H, ctypes.c_double]
_lib.svgd_forget_carry.argtypes = [_H]
_lib.svgd_forget_carry.restype = ctypes.c_int
_lib.svgd_bandwidth.argtypes = [_H, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
                                ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
_lib.svgd_step.argtypes = [_H, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
                           ctypes.c_float, ctypes.c_void_p]
_lib.svgd_phi.argtypes = [_H, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
                          ctypes.c_void_p, ctypes.c_void_p]
_lib.svgd_bandwidth_ld.argtypes = [_H, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                   ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
_lib.svgd_step_ld.argtypes = [_H, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
                              ctypes.c_int64, ctypes.c_float, ctypes.c_void_p]
_lib.svgd_phi_ld.argtypes = [_H, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
                             ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
_lib.svgd_step_rows.argtypes = [_H, ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
                                ctypes.c_int64, ctypes.c_float, ctypes.c_void_p]
_lib.svgd_step_rows.restype = ctypes.c_int
_lib.svgd_get_last.argtypes = [_H, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p, ctypes.c_void_p]
_lib.svgd_destroy.argtypes = [_H]
_lib.svgd_diag_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
_lib.svgd_diag_copy.restype = ctypes.c_int
_lib.svgd_diag_axpy_rows.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                     ctypes.c_float, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
_lib.svgd_diag_axpy_rows.restype = ctypes.c_int
_lib.svgd_diag_read_rows.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                     ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
_lib.svgd_diag_read_rows.restype = ctypes.c_int
_lib.svgd_step_static.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                  ctypes.c_float, ctypes.c_void_p]
_lib.svgd_step_static.restype = ctypes.c_int
_lib.swag_update_moments.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                     ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p]
_lib.swag_update_moments.restype = ctypes.c_int
_lib.svgd_profile_begin.argtypes = [_H]
_lib.svgd_profile_begin_kinds.argtypes = [_H, ctypes.c_uint]
_lib.svgd_profile_begin_kinds.restype = ctypes.c_int
_lib.svgd_profile_end.argtypes = [_H, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)]
_lib.svgd_profile_end_records.argtypes = [_H, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int),
                                          ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float),
                                          ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
_lib.svgd_profile_end_records.restype = ctypes.c_int
_lib.svgd_last_device_error.argtypes = [_H]
_lib.svgd_status_string.argtypes = [ctypes.c_int]
_lib.svgd_status_string.restype = ctypes.c_char_p
for _f in ("svgd_create", "svgd_set_bandwidth", "svgd_bandwidth", "svgd_step", "svgd_phi",
           "svgd_bandwidth_ld", "svgd_step_ld", "svgd_phi_ld",
           "svgd_get_last", "svgd_destroy", "svgd_last_device_error", "svgd_profile_begin",
           "svgd_profile_end"):
    getattr(_lib, _f).restype = ctypes.c_int

SVGD_OK = 0
FLAG_CARRY_GRAM = 1
FLAG_FUSE_MFMA = 2
KERNEL_KINDS = ("gram", "reduce", "bandwidth", "update")
MAX_PARTICLES = 64
STATIC_MAX_D = 1 << 32
MAX_D = 1 << 36


class SvgdError(RuntimeError):
    def __init__(self, status, hip_error=0):
        self.status = status
        self.hip_error = hip_error
        name = _lib.svgd_status_string(status).decode()
        super().__init__(f"{name} ({status})" + (f", hipError {hip_error}" if hip_error else ""))


def status_string(status: int) -> str:
    return _lib.svgd_status_string(status).decode()


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_matrix(t: torch.Tensor, name: str):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.dim() == 2
            and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous 2-D float32 CUDA tensor")
    return t


def padded_rows(n: int, D: int, device="cuda", fill=None):
    """An (n, D) view of a new (n, ld) buffer, ld = D rounded up to 32 floats: every row starts on
    a 128-byte boundary, the layout the update kernels like best.  Returns the view."""
    ld = (D + 31) // 32 * 32
    buf = torch.empty(n, ld, device=device, dtype=torch.float32)
    if fill is not None:
        buf.fill_(fill)
    return buf[:, :D]


def diag_copy(dst: torch.Tensor, src: torch.Tensor, stream=None):
    """Plain copy kernel of known size (calibration of hardware byte counters)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("dst and src must have the same size in bytes")
    rc = _lib.svgd_diag_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr(stream))
    if rc != SVGD_OK:
        raise SvgdError(rc)


def _rows_of(t, name):
    """(n, D, ld) of a 2-D float32 CUDA tensor with contiguous rows."""
    if not isinstance(t, torch.Tensor) or t.dtype is not torch.float32 or not t.is_cuda or t.dim() != 2:
        raise TypeError(f"{name} must be a 2-D float32 CUDA tensor")
    (n, D), st = t.shape, t.stride()
    if (D != 1 and st[1] != 1) or (n != 1 and st[0] < D):
        raise TypeError(f"{name} must have contiguous rows, at least D elements apart")
    return n, D, (st[0] if n != 1 else D)


def diag_axpy_rows(X: torch.Tensor, G: torch.Tensor, s: float, pattern: int, workgroups: int, stream=None):
    """Plain in-place X += s * G over the row streams of X and G (the update's memory traffic and
    nothing else; see svgd_diag_axpy_rows)."""
    shape = _rows_of(X, "X")
    if _rows_of(G, "G") != shape:
        raise ValueError("G must have the shape and row stride of X")
    n, D, ld = shape
    rc = _lib.svgd_diag_axpy_rows(X.data_ptr(), G.data_ptr(), n, D, ld, float(s), int(pattern), int(workgroups),
                                  _stream_ptr(stream))
    if rc != SVGD_OK:
        raise SvgdError(rc)


def diag_read_rows(X: torch.Tensor, sink: torch.Tensor, pattern: int, stream=None):
    """Reads every element of the rows of X once (the pairwise pass's memory traffic and nothing
    else; see svgd_diag_read_rows); sink: float32 CUDA vector, one entry per workgroup, receives the
    workgroups' sums."""
    n, D, ld = _rows_of(X, "X")
    if (not isinstance(sink, torch.Tensor) or sink.dtype is not torch.float32 or not sink.is_cuda
            or sink.dim() != 1 or not sink.is_contiguous() or sink.numel() < 1):
        raise TypeError("sink must be a contiguous 1-D float32 CUDA tensor")
    rc = _lib.svgd_diag_read_rows(X.data_ptr(), n, D, ld, sink.data_ptr(), int(pattern), int(sink.numel()),
                                  _stream_ptr(stream))
    if rc != SVGD_OK:
        raise SvgdError(rc)


def step_static(X: torch.Tensor, G: torch.Tensor, eps: float, stream=None):
    """svgd_step_static: one plain step on the current device with the library's static scratch -
    no handle, nothing allocated.  X and G as in Svgd.step."""
    shape = _rows_of(X, "X")
    if _rows_of(G, "G") != shape:
        raise ValueError("G must have the shape and row stride of X")
    n, D, ld = shape
    with torch.cuda.device(X.device):
        rc = _lib.svgd_step_static(X.data_ptr(), G.data_ptr(), n, D, ld, float(eps), _stream_ptr(stream))
    if rc != SVGD_OK:
        raise SvgdError(rc)


def swag_update_moments(mean: torch.Tensor, sqmean: torch.Tensor, X: torch.Tensor, count: int, stream=None):
    """Multi-SWAG running moments: absorb X into mean / sqmean (in place) after `count` updates."""
    X, mean, sqmean = _dev_matrix(X, "X"), _dev_matrix(mean, "mean"), _dev_matrix(sqmean, "sqmean")
    if mean.shape != X.shape or sqmean.shape != X.shape:
        raise ValueError("mean, sqmean and X must have the same shape")
    n, D = X.shape
    rc = _lib.swag_update_moments(mean.data_ptr(), sqmean.data_ptr(), X.data_ptr(), n, D, int(count),
                                  _stream_ptr(stream))
    if rc != SVGD_OK:
        raise SvgdError(rc)


class Svgd:
    """Handle of the library: svgd_create on construction, svgd_destroy on close()."""

    def __init__(self, max_n: int, max_D: int, device: int = -1, flags: int = 0):
        self._h = _H()
        self._last_n = 0
        rc = _lib.svgd_create(ctypes.byref(self._h), int(max_n), int(max_D), int(device), int(flags))
        if rc != SVGD_OK:
            self._h = _H()
            raise SvgdError(rc)
        self._device = int(device) if device >= 0 else torch.cuda.current_device()

    def _rows(self, t, name):
        """Checks a matrix argument (2-D float32, rows contiguous, on the handle's device - a
        pointer of another GPU would fault) and returns (n, D, ld).  Kept short: at small sizes
        a step costs less than these checks."""
        if not isinstance(t, torch.Tensor) or t.dtype is not torch.float32 or not t.is_cuda or t.dim() != 2:
            raise TypeError(f"{name} must be a 2-D float32 CUDA tensor")
        (n, D), st = t.shape, t.stride()
        if (D != 1 and st[1] != 1) or (n != 1 and st[0] < D):
            raise TypeError(f"{name} must have contiguous rows, at least D elements apart")
        if t.get_device() != self._device:
            raise ValueError(f"{name} is on cuda:{t.get_device()}, the handle on cuda:{self._device}")
        return n, D, (st[0] if n != 1 else D)

    def _same(self, a, b, name):
        if a != b:
            raise ValueError(f"{name} has (n, D, row stride) = {b}, X has {a}")

    def _check(self, rc):
        if rc != SVGD_OK:
            raise SvgdError(rc, _lib.svgd_last_device_error(self._h))

    def set_bandwidth(self, h_fixed: float):
        self._check(_lib.svgd_set_bandwidth(self._h, float(h_fixed)))

    def forget_carry(self):
        self._check(_lib.svgd_forget_carry(self._h))

    def bandwidth(self, X, want_h=True, stream=None):
        n, D, ld = self._rows(X, "X")
        out = ctypes.c_double(0.0)
        self._check(_lib.svgd_bandwidth_ld(self._h, X.data_ptr(), n, D, ld,
                                           ctypes.byref(out) if want_h else None, _stream_ptr(stream)))
        self._last_n = n
        return out.value if want_h else None

    def step(self, X, G, eps: float, stream=None):
        """X <- X + eps * phi(X, G) in place.  X and G: (n, D) with contiguous rows and the same
        row stride (dense, or views like buf[:, :D] of an (n, ld) buffer, see padded_rows)."""
        shape = self._rows(X, "X")
        self._same(shape, self._rows(G, "G"), "G")
        n, D, ld = shape
        self._check(_lib.svgd_step_ld(self._h, X.data_ptr(), G.data_ptr(), n, D, ld, float(eps),
                                      _stream_ptr(stream)))
        self._last_n = n

    def step_rows(self, X_rows, G_rows, eps: float, stream=None):
        """svgd_step_rows: the particles are n separately allocated 1-D float32 CUDA tensors of equal
        length (X_rows[i], updated in place) with their scores (G_rows[i]); nothing is copied."""
        n = len(X_rows)
        if n < 1 or len(G_rows) != n:
            raise ValueError("X_rows and G_rows must be non-empty sequences of the same length")
        D = X_rows[0].numel()
        for name, rows in (("X_rows", X_rows), ("G_rows", G_rows)):
            for t in rows:
                if not (isinstance(t, torch.Tensor) and t.dtype is torch.float32 and t.is_cuda and t.dim() == 1
                        and t.numel() == D and (D == 1 or t.stride(0) == 1)):
                    raise TypeError(f"{name} must hold contiguous 1-D float32 CUDA tensors of one length")
                if t.get_device() != self._device:
                    raise ValueError(f"a row of {name} is on cuda:{t.get_device()}, the handle on cuda:{self._device}")
        xp = (ctypes.c_void_p * n)(*[t.data_ptr() for t in X_rows])
        gp = (ctypes.c_void_p * n)(*[t.data_ptr() for t in G_rows])
        self._check(_lib.svgd_step_rows(self._h, xp, gp, n, D, float(eps), _stream_ptr(stream)))
        self._last_n = n

    def phi(self, X, G, PHI, stream=None):
        shape = self._rows(X, "X")
        self._same(shape, self._rows(G, "G"), "G")
        self._same(shape, self._rows(PHI, "PHI"), "PHI")
        n, D, ld = shape
        self._check(_lib.svgd_phi_ld(self._h, X.data_ptr(), G.data_ptr(), n, D, ld, PHI.data_ptr(),
                                     _stream_ptr(stream)))
        self._last_n = n

    def get_last(self, n: int, stream=None):
        """(h, K) of the most recent call; K is an (n, n) float32 numpy array.  n must be that
        call's particle count: the library copies exactly that many rows and columns."""
        import numpy as np
        if n != self._last_n:
            raise ValueError(f"the last call had n = {self._last_n}, not {n}")
        K = np.empty((n, n), np.float32)
        h = ctypes.c_double(0.0)
        self._check(_lib.svgd_get_last(self._h, ctypes.byref(h), K.ctypes.data_as(ctypes.c_void_p),
                                       _stream_ptr(stream)))
        return h.value, K

    def profile_begin(self, kinds=None):
        """Time every kernel launched from now on, or only the given kinds (names from KERNEL_KINDS)."""
        if kinds is None:
            self._check(_lib.svgd_profile_begin(self._h))
        else:
            mask = 0
            for k in kinds:
                mask |= 1 << KERNEL_KINDS.index(k)
            self._check(_lib.svgd_profile_begin_kinds(self._h, mask))

    def profile_end(self):
        """{kind: (total_ms, launches)} for the kernels launched since profile_begin()."""
        ms = (ctypes.c_double * 4)()
        cnt = (ctypes.c_int * 4)()
        self._check(_lib.svgd_profile_end(self._h, ms, cnt))
        return {k: (ms[i], cnt[i]) for i, k in enumerate(KERNEL_KINDS)}

    def profile_end_records(self, cap: int = 2048):
        """({kind: (total_ms, launches)}, [(kind, ms) per launch, in launch order])."""
        ms = (ctypes.c_double * 4)()
        cnt = (ctypes.c_int * 4)()
        rk = (ctypes.c_int * cap)()
        rm = (ctypes.c_float * cap)()
        nrec = ctypes.c_int(0)
        self._check(_lib.svgd_profile_end_records(self._h, ms, cnt, rk, rm, cap, ctypes.byref(nrec)))
        return ({k: (ms[i], cnt[i]) for i, k in enumerate(KERNEL_KINDS)},
                [(KERNEL_KINDS[rk[r]], rm[r]) for r in range(nrec.value)])

    def close(self):
        if self._h:
            rc = _lib.svgd_destroy(self._h)
            self._h = _H()
            if rc != SVGD_OK:
                raise SvgdError(rc)

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            if self._h:
                _lib.svgd_destroy(self._h)
                self._h = _H()
        except Exception:
            pass
