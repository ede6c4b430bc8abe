"""TEST INFRASTRUCTURE - not part of the product path.

ctypes binding of the CPU oracle for signature kernels (paper Section 3; see sigkernel_oracle_impl.h
for the arithmetic and the passages it follows).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package.  It shares no code with the HIP path.

All arrays are host numpy arrays, C-contiguous; ``dtype`` is ``np.float64`` (the oracle proper) or
``np.longdouble`` (x87 80-bit, used to arbitrate rounding).
"""
import ctypes as C
import os

import numpy as np

from .build import LIB, build

FLAG_TIME_AUG = 1
FLAG_LEAD_LAG = 8   # same bit as SK_FLAG_LEAD_LAG of the library

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        _lib = C.CDLL(LIB)
        _lib.osk_num_threads.restype = C.c_int
        for suf, creal in (("_f64", C.c_double), ("_f80", C.c_longdouble)):
            f = getattr(_lib, "osk_kernel_from_delta" + suf)
            f.restype = creal
            f.argtypes = [C.c_void_p, C.c_long, C.c_long, C.c_int, C.c_int]
            f = getattr(_lib, "osk_pair_debug" + suf)
            f.restype = creal
            f.argtypes = [C.c_void_p, C.c_void_p, C.c_long, C.c_long, C.c_long, C.c_int, C.c_int, C.c_int,
                          C.c_void_p, C.c_void_p, C.c_void_p]
            f = getattr(_lib, "osk_fwd" + suf)
            f.restype = C.c_int
            f.argtypes = [C.c_void_p] * 3 + [C.c_long] * 4 + [C.c_int] * 3
            f = getattr(_lib, "osk_bwd" + suf)
            f.restype = C.c_int
            f.argtypes = [C.c_void_p] * 6 + [C.c_long] * 4 + [C.c_int] * 3
            f = getattr(_lib, "osk_gram" + suf)
            f.restype = C.c_int
            f.argtypes = [C.c_void_p] * 6 + [C.c_long] * 5 + [C.c_int] * 3
    return _lib


def num_threads() -> int:
    return int(lib().osk_num_threads())


def _suf(dtype):
    dtype = np.dtype(dtype)
    if dtype == np.float64:
        return "_f64"
    if dtype == np.longdouble:
        return "_f80"
    raise TypeError("oracle works in float64 or longdouble, got %s" % dtype)


def _arr(a, dtype):
    return np.ascontiguousarray(np.asarray(a, dtype=dtype))


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def kernel_from_delta(Delta, lam1=0, lam2=0, dtype=np.float64):
    """k computed by Eq. (1) from a given coarse increment Gram matrix Delta[r,q]."""
    D = _arr(Delta, dtype)
    r, q = D.shape
    return getattr(lib(), "osk_kernel_from_delta" + _suf(dtype))(_p(D), r, q, lam1, lam2)


def pair_debug(x, y, lam1=0, lam2=0, flags=0, dtype=np.float64, want_G=True):
    """One pair with intermediates: returns (k, Delta[r,q], grid[m+1,n+1], G=dk/dDelta[r,q])."""
    x = _arr(x, dtype)
    y = _arr(y, dtype)
    L1, d = x.shape
    L2, d2 = y.shape
    assert d == d2
    r, q = max(L1 - 1, 0), max(L2 - 1, 0)
    m, n = r << lam1, q << lam2
    Delta = np.zeros((r, q), dtype=dtype)
    grid = np.ones((m + 1, n + 1), dtype=dtype)
    G = np.zeros((r, q), dtype=dtype) if want_G else None
    k = getattr(lib(), "osk_pair_debug" + _suf(dtype))(_p(x), _p(y), L1, L2, d, lam1, lam2, flags, _p(Delta),
                                                       _p(grid) if r > 0 and q > 0 else None, _p(G))
    return k, Delta, grid, G


def lead_lag(x):
    """The lead-lag transform of Section 4, written out point by point: a path of L points in R^d becomes the path of
    2L - 1 points in R^2d with  lead_i = x[k] for i in {2k - 1, 2k},  lag_i = x[k] for i in {2k, 2k + 1};
    the lead channels come first.  Works on [..., L, d] arrays."""
    x = np.asarray(x)
    L, d = x.shape[-2], x.shape[-1]
    out = np.empty(x.shape[:-2] + (2 * L - 1, 2 * d), dtype=x.dtype)
    for i in range(2 * L - 1):
        k_lead = (i + 1) // 2      # i = 2k or i = 2k - 1
        k_lag = i // 2             # i = 2k or i = 2k + 1
        out[..., i, :d] = x[..., k_lead, :]
        out[..., i, d:] = x[..., k_lag, :]
    return out


def lead_lag_pullback(g):
    """Chain rule through lead_lag: the gradient of a point collects the gradients of every transformed point and
    half that is a copy of it.  g[..., 2L - 1, 2d] -> [..., L, d]."""
    g = np.asarray(g)
    L, d = (g.shape[-2] + 1) // 2, g.shape[-1] // 2
    out = np.zeros(g.shape[:-2] + (L, d), dtype=g.dtype)
    for i in range(2 * L - 1):
        out[..., (i + 1) // 2, :] += g[..., i, :d]
        out[..., i // 2, :] += g[..., i, d:]
    return out


def fwd(x, y, lam1=0, lam2=0, flags=0, dtype=np.float64):
    """x[B,L1,d], y[B,L2,d] -> k[B]."""
    if flags & FLAG_LEAD_LAG:   # transform first, then the (optional) time augmentation of the transformed paths
        return fwd(lead_lag(_arr(x, dtype)), lead_lag(_arr(y, dtype)), lam1, lam2, flags & ~FLAG_LEAD_LAG, dtype)
    x = _arr(x, dtype)
    y = _arr(y, dtype)
    B, L1, d = x.shape
    B2, L2, d2 = y.shape
    assert B == B2 and d == d2
    k = np.empty((B,), dtype=dtype)
    rc = getattr(lib(), "osk_fwd" + _suf(dtype))(_p(x), _p(y), _p(k), B, L1, L2, d, lam1, lam2, flags)
    assert rc == 0
    return k


def bwd(x, y, grad_k, lam1=0, lam2=0, flags=0, dtype=np.float64):
    """Returns (k[B], grad_x[B,L1,d], grad_y[B,L2,d]) for upstream gradients grad_k[B]."""
    if flags & FLAG_LEAD_LAG:
        k, gx, gy = bwd(lead_lag(_arr(x, dtype)), lead_lag(_arr(y, dtype)), grad_k, lam1, lam2,
                        flags & ~FLAG_LEAD_LAG, dtype)
        return k, lead_lag_pullback(gx), lead_lag_pullback(gy)
    x = _arr(x, dtype)
    y = _arr(y, dtype)
    gk = _arr(grad_k, dtype)
    B, L1, d = x.shape
    B2, L2, d2 = y.shape
    assert B == B2 and d == d2 and gk.shape == (B,)
    k = np.empty((B,), dtype=dtype)
    gx = np.empty_like(x)
    gy = np.empty_like(y)
    rc = getattr(lib(), "osk_bwd" + _suf(dtype))(_p(x), _p(y), _p(gk), _p(gx), _p(gy), _p(k), B, L1, L2, d, lam1,
                                                 lam2, flags)
    assert rc == 0
    return k, gx, gy


def gram(X, Y, grad_K=None, lam1=0, lam2=0, flags=0, dtype=np.float64):
    """K[N,M] = k(X[n], Y[m]).  With grad_K[N,M] also returns (grad_X, grad_Y); passing the same array
    object for X and Y selects the symmetric case, where grad_X is the total derivative and grad_Y is None."""
    sym = Y is X
    if flags & FLAG_LEAD_LAG:
        Xl = lead_lag(_arr(X, dtype))
        Yl = Xl if sym else lead_lag(_arr(Y, dtype))
        r = gram(Xl, Yl, grad_K, lam1, lam2, flags & ~FLAG_LEAD_LAG, dtype)
        if grad_K is None:
            return r
        return r[0], lead_lag_pullback(r[1]), (None if sym else lead_lag_pullback(r[2]))
    X = _arr(X, dtype)
    Y = X if sym else _arr(Y, dtype)
    if not sym and Y.ctypes.data == X.ctypes.data:
        Y = Y.copy()   # a slice that starts where X starts: the C entry point takes equal pointers for the symmetric case
    N, L1, d = X.shape
    M, L2, d2 = Y.shape
    assert d == d2
    K = np.empty((N, M), dtype=dtype)
    f = getattr(lib(), "osk_gram" + _suf(dtype))
    if grad_K is None:
        rc = f(_p(X), _p(Y), _p(K), None, None, None, N, M, L1, L2, d, lam1, lam2, flags)
        assert rc == 0
        return K
    W = _arr(grad_K, dtype)
    assert W.shape == (N, M)
    gX = np.empty_like(X)
    gY = None if sym else np.empty_like(Y)
    rc = f(_p(X), _p(Y), _p(K), _p(W), _p(gX), _p(gY), N, M, L1, L2, d, lam1, lam2, flags)
    assert rc == 0
    return K, gX, gY


def mmd2(X, Y, lam1=0, lam2=0, flags=0, dtype=np.float64, want_grads=True):
    """Squared maximum mean discrepancy of two path sets under the signature kernel, written out from its
    definition (biased estimate): mean K(X,X) - 2 mean K(X,Y) + mean K(Y,Y); the gradients by the chain rule
    through gram() with the constant weights 1/N^2, -2/(NM), 1/M^2.  Returns loss or (loss, grad_X, grad_Y)."""
    X = _arr(X, dtype)
    Y = _arr(Y, dtype)
    N, M = X.shape[0], Y.shape[0]
    if not want_grads:
        return (gram(X, X, None, lam1, lam1, flags, dtype).mean() - 2.0 * gram(X, Y, None, lam1, lam2, flags, dtype).mean()
                + gram(Y, Y, None, lam2, lam2, flags, dtype).mean())
    Kxx, gxx, _ = gram(X, X, np.full((N, N), 1.0 / (N * N)), lam1, lam1, flags, dtype)
    Kxy, gxy_x, gxy_y = gram(X, Y, np.full((N, M), -2.0 / (N * M)), lam1, lam2, flags, dtype)
    Kyy, gyy, _ = gram(Y, Y, np.full((M, M), 1.0 / (M * M)), lam2, lam2, flags, dtype)
    return Kxx.mean() - 2.0 * Kxy.mean() + Kyy.mean(), gxx + gxy_x, gyy + gxy_y
