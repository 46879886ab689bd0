"""ctypes front end of the fp64 CPU oracle in svgd_oracle.c.

TEST INFRASTRUCTURE ONLY.  This module is imported by the tests, by the smoke
check and by the benchmark's CPU-baseline leg; the GPU library and its binding
never import it and it never imports them.

All functions take numpy arrays X, G of shape (n, D), dtype float32 or float64
(both must share one dtype), and compute in fp64, following the paper's App. B.2
SVGD routine in the score/ascent convention:

    d2_ij = |x_i - x_j|^2,  h = median(all n^2 entries of d2)/ln(n+1)  (h<=0 -> 1),
    K_ij = exp(-d2_ij/h),   phi_i = (1/n) sum_j K_ij [ g_j + (2/h)(x_i - x_j) ],
    x_i <- x_i + eps*phi_i  (all phi from the pre-step X).
"""
import ctypes
import numpy as np

from .build_oracle import build as _build

_lib = ctypes.CDLL(_build())
_vp, _dp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_double)
_i, _i64, _d = ctypes.c_int, ctypes.c_int64, ctypes.c_double

_lib.oracle_num_threads.restype = _i
_lib.oracle_pairwise_d2.argtypes = [_vp, _i, _i, _i64, _dp]
_lib.oracle_median_all.argtypes = [_dp, _i]
_lib.oracle_median_all.restype = _d
_lib.oracle_bandwidth.argtypes = [_dp, _i]
_lib.oracle_bandwidth.restype = _d
_lib.oracle_kernel.argtypes = [_dp, _i, _d, _dp, _dp]
_lib.oracle_phi_cols.argtypes = [_vp, _vp, _i, _i, _i64, _dp, _d, _i64, _i64, _dp]
_lib.oracle_step.argtypes = [_vp, _vp, _i, _i, _i64, _d, _d, _dp, _dp, _dp, _dp, _dp, _dp]
_lib.oracle_swag_update.argtypes = [_dp, _dp, _vp, _i, _i64, _i64]


def num_threads() -> int:
    return int(_lib.oracle_num_threads())


def _prep(A):
    A = np.ascontiguousarray(A)
    if A.dtype not in (np.float32, np.float64) or A.ndim != 2:
        raise TypeError("expected a 2-D float32/float64 array")
    return A


def _ptr(A):
    return ctypes.c_void_p(A.ctypes.data)


def _dptr(A):
    return A.ctypes.data_as(_dp)


def pairwise_d2(X):
    X = _prep(X)
    n, D = X.shape
    d2 = np.empty((n, n), np.float64)
    _lib.oracle_pairwise_d2(_ptr(X), int(X.dtype == np.float64), n, D, _dptr(d2))
    return d2


def median_all(d2):
    d2 = np.ascontiguousarray(d2, np.float64)
    return float(_lib.oracle_median_all(_dptr(d2), d2.shape[0]))


def bandwidth(d2):
    d2 = np.ascontiguousarray(d2, np.float64)
    return float(_lib.oracle_bandwidth(_dptr(d2), d2.shape[0]))


def kernel(d2, h):
    d2 = np.ascontiguousarray(d2, np.float64)
    n = d2.shape[0]
    K = np.empty((n, n), np.float64)
    r = np.empty(n, np.float64)
    _lib.oracle_kernel(_dptr(d2), n, float(h), _dptr(K), _dptr(r))
    return K, r


def phi_cols(X, G, K, h, col0, ncols):
    """phi restricted to columns [col0, col0+ncols): (n, ncols) float64."""
    X, G = _prep(X), _prep(G)
    assert X.dtype == G.dtype and X.shape == G.shape
    n, D = X.shape
    assert 0 <= col0 and col0 + ncols <= D
    K = np.ascontiguousarray(K, np.float64)
    out = np.empty((n, ncols), np.float64)
    _lib.oracle_phi_cols(_ptr(X), _ptr(G), int(X.dtype == np.float64), n, D, _dptr(K), float(h),
                         col0, ncols, _dptr(out))
    return out


def step(X, G, eps, h_fixed=0.0, want_phi=True, want_xnew=True):
    """One whole step.  Returns dict(d2, K, r, h, phi, X_new) (fp64)."""
    X, G = _prep(X), _prep(G)
    assert X.dtype == G.dtype and X.shape == G.shape
    n, D = X.shape
    d2 = np.empty((n, n)); K = np.empty((n, n)); r = np.empty(n)
    h = ctypes.c_double(0.0)
    phi = np.empty((n, D)) if want_phi else None
    xn = np.empty((n, D)) if want_xnew else None
    _lib.oracle_step(_ptr(X), _ptr(G), int(X.dtype == np.float64), n, D, float(eps), float(h_fixed),
                     _dptr(d2), _dptr(K), _dptr(r), ctypes.byref(h),
                     _dptr(phi) if want_phi else None, _dptr(xn) if want_xnew else None)
    return dict(d2=d2, K=K, r=r, h=h.value, phi=phi, X_new=xn)


def swag_update(mean, sq, X, count):
    """SWAG running moments, in place: mean, sq are float64 arrays shaped like X (float32/64);
    `count` iterates have been absorbed before this one (paper Sec. 2; Maddox et al.'s recursion)."""
    X = _prep(X)
    assert mean.dtype == np.float64 and sq.dtype == np.float64
    assert mean.shape == X.shape and sq.shape == X.shape
    assert mean.flags.c_contiguous and sq.flags.c_contiguous
    _lib.oracle_swag_update(_dptr(mean), _dptr(sq), _ptr(X), int(X.dtype == np.float64), X.size, int(count))
