"""ctypes front end of the CPU oracle (oracle/qn_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg; never by the product package.

Array convention: a worker matrix is a numpy array of shape (m, n), C
contiguous, so that worker k's vector is the contiguous row X[k] -- the same
memory layout as the device library's "m contiguous columns of length n".
dtype float32, float64, or uint16 holding bfloat16 bit patterns.
Small matrices (C, V) are returned with shape (m, m) indexed [k, r] =
column k, row r, i.e. V[k] is the eigenvector v_k.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None

F32, BF16, F64, F16 = 0, 1, 2, 3

_i64 = ctypes.c_int64
_int = ctypes.c_int
_dbl = ctypes.c_double
_vp = ctypes.c_void_p


def load_library(path):
    """Opens an oracle shared library and declares its signatures."""
    L = ctypes.CDLL(path)
    L.qno_row_means.argtypes = [_vp, _int, _i64, _int, _i64, _vp]
    L.qno_row_means.restype = None
    L.qno_centre.argtypes = [_vp, _int, _i64, _int, _i64, _vp, _vp]
    L.qno_centre.restype = None
    L.qno_gram.argtypes = [_vp, _i64, _int, _vp]
    L.qno_gram.restype = None
    L.qno_gemv_t.argtypes = [_vp, _i64, _int, _vp, _vp]
    L.qno_gemv_t.restype = None
    L.qno_jacobi_eigh.argtypes = [_vp, _int, _vp, _vp]
    L.qno_jacobi_eigh.restype = _int
    L.qno_sigma_from_mu.argtypes = [_vp, _int, _vp]
    L.qno_sigma_from_mu.restype = None
    L.qno_select_j.argtypes = [_vp, _int, _dbl]
    L.qno_select_j.restype = _int
    L.qno_apply_Hinv_literal.argtypes = [_vp, _vp, _i64, _int, _vp, _vp,
                                         _int, _vp, _vp]
    L.qno_apply_Hinv_literal.restype = None
    L.qno_update_literal.argtypes = [_vp, _vp, _int, _i64, _int, _i64,
                                     _dbl, _dbl, _vp, _vp, _vp, _vp, _vp,
                                     _vp]
    L.qno_update_literal.restype = _int
    L.qno_gram_accumulate.argtypes = [_vp, _int, _i64, _int, _i64, _vp,
                                      _vp]
    L.qno_gram_accumulate.restype = None
    L.qno_coefficients.argtypes = [_vp, _vp, _int, _dbl, _vp, _vp, _vp,
                                   _vp, _vp]
    L.qno_coefficients.restype = _int
    L.qno_apply_closed_form.argtypes = [_vp, _vp, _int, _i64, _int, _i64,
                                        _vp, _dbl, _vp]
    L.qno_apply_closed_form.restype = None
    L.qno_tau_bounded_literal.argtypes = [_dbl, _int, _vp, _vp, _i64, _int, _vp,
                                          _vp, _int, _vp]
    L.qno_tau_bounded_literal.restype = _dbl
    L.qno_tau_bounded_from_gram.argtypes = [_dbl, _int, _vp, _int, _vp, _vp,
                                            _int, _vp]
    L.qno_tau_bounded_from_gram.restype = _dbl
    return L


def lib():
    """The oracle library; QN_ORACLE_LIB names another build of the same source
    (the sanitized one, for the test that runs the pins on it)."""
    global _LIB
    if _LIB is None:
        path = os.environ.get("QN_ORACLE_LIB", "")
        if not path:
            path = _build.LIB
            if not os.path.exists(path):
                _build.build()
        _LIB = load_library(path)
    return _LIB


def _code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float64:
        return F64
    if a.dtype == np.uint16:
        return BF16          # bfloat16 bit patterns (numpy has no such type)
    if a.dtype == np.float16:
        return F16
    raise TypeError(f"unsupported worker-matrix dtype {a.dtype}")


def _worker(a) -> np.ndarray:
    a = np.asarray(a)
    if a.ndim != 2:
        raise ValueError("worker matrix must have shape (m, n)")
    if a.strides[1] != a.itemsize:
        a = np.ascontiguousarray(a)
    return a


def _ld(a: np.ndarray) -> int:
    if a.shape[0] == 1:
        return a.shape[1]
    assert a.strides[0] % a.itemsize == 0
    return a.strides[0] // a.itemsize


def _p(a: np.ndarray):
    return a.ctypes.data_as(_vp)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def row_means(X):
    X = _worker(X)
    m, n = X.shape
    out = np.empty(n, np.float64)
    lib().qno_row_means(_p(X), _code(X), n, m, _ld(X), _p(out))
    return out


def centre(X, mean):
    X = _worker(X)
    m, n = X.shape
    mean = _f64(mean)
    out = np.empty((m, n), np.float64)
    lib().qno_centre(_p(X), _code(X), n, m, _ld(X), _p(mean), _p(out))
    return out


def gram(G):
    G = _f64(G)
    m, n = G.shape
    C = np.empty((m, m), np.float64)
    lib().qno_gram(_p(G), n, m, _p(C))
    return C


def gemv_t(G, z):
    G = _f64(G)
    z = _f64(z)
    m, n = G.shape
    w = np.empty(m, np.float64)
    lib().qno_gemv_t(_p(G), n, m, _p(z), _p(w))
    return w


def jacobi_eigh(C):
    """Returns (mu descending, V with V[k] = v_k, sweeps)."""
    C = _f64(C)
    m = C.shape[0]
    mu = np.empty(m, np.float64)
    V = np.empty((m, m), np.float64)
    sweeps = lib().qno_jacobi_eigh(_p(C), m, _p(mu), _p(V))
    if sweeps < 0:
        raise RuntimeError("oracle Jacobi did not converge")
    return mu, V, sweeps


def sigma_from_mu(mu):
    mu = _f64(mu)
    s = np.empty_like(mu)
    lib().qno_sigma_from_mu(_p(mu), mu.shape[0], _p(s))
    return s


def select_j(sigma, lam: float) -> int:
    sigma = _f64(sigma)
    return int(lib().qno_select_j(_p(sigma), sigma.shape[0], float(lam)))


def apply_Hinv_literal(Theta, G, sigma, V, j: int, z):
    Theta = _f64(Theta)
    G = _f64(G)
    sigma = _f64(sigma)
    V = _f64(V)
    z = _f64(z)
    m, n = G.shape
    out = np.empty(n, np.float64)
    lib().qno_apply_Hinv_literal(_p(Theta), _p(G), n, m, _p(sigma), _p(V),
                                 int(j), _p(z), _p(out))
    return out


def update_literal(thetas, grads, tau: float, lam: float):
    """Eq. (2)-(4) evaluated literally.  Returns a dict with theta_new, j, C,
    w, sigma, V."""
    T = _worker(thetas)
    Gr = _worker(grads)
    assert T.shape == Gr.shape and T.dtype == Gr.dtype
    m, n = T.shape
    if _ld(T) != _ld(Gr):
        T = np.ascontiguousarray(T)
        Gr = np.ascontiguousarray(Gr)
    theta_new = np.empty(n, np.float64)
    j = ctypes.c_int(0)
    C = np.empty((m, m), np.float64)
    w = np.empty(m, np.float64)
    sigma = np.empty(m, np.float64)
    V = np.empty((m, m), np.float64)
    rc = lib().qno_update_literal(_p(T), _p(Gr), _code(T), n, m, _ld(T),
                                  float(tau), float(lam), _p(theta_new),
                                  ctypes.byref(j), _p(C), _p(w), _p(sigma),
                                  _p(V))
    if rc != 0:
        raise RuntimeError("oracle literal update failed")
    return dict(theta_new=theta_new, j=j.value, C=C, w=w, sigma=sigma, V=V)


def gram_accumulate(grads, C_acc=None, w_acc=None):
    """Adds the chunk `grads` (shape (m, rows)) to the running C and w."""
    Gr = _worker(grads)
    m, rows = Gr.shape
    if C_acc is None:
        C_acc = np.zeros((m, m), np.float64)
    if w_acc is None:
        w_acc = np.zeros(m, np.float64)
    lib().qno_gram_accumulate(_p(Gr), _code(Gr), rows, m, _ld(Gr), _p(C_acc),
                              _p(w_acc))
    return C_acc, w_acc


def coefficients(C, w, lam: float):
    """Returns dict(c, j, sigma, V, alpha) from C = G^T G and w = G^T g_bar."""
    C = _f64(C)
    w = _f64(w)
    m = C.shape[0]
    c = np.empty(m, np.float64)
    sigma = np.empty(m, np.float64)
    V = np.empty((m, m), np.float64)
    alpha = np.empty(m, np.float64)
    j = ctypes.c_int(0)
    rc = lib().qno_coefficients(_p(C), _p(w), m, float(lam), _p(c),
                                ctypes.byref(j), _p(sigma), _p(V), _p(alpha))
    if rc != 0:
        raise RuntimeError("oracle coefficients failed")
    return dict(c=c, j=j.value, sigma=sigma, V=V, alpha=alpha)


def apply_closed_form(thetas, grads, c, tau: float):
    T = _worker(thetas)
    Gr = _worker(grads)
    assert T.shape == Gr.shape and T.dtype == Gr.dtype
    if _ld(T) != _ld(Gr):
        T = np.ascontiguousarray(T)
        Gr = np.ascontiguousarray(Gr)
    m, rows = T.shape
    c = _f64(c)
    out = np.empty(rows, np.float64)
    lib().qno_apply_closed_form(_p(T), _p(Gr), _code(T), rows, m, _ld(T),
                                _p(c), float(tau), _p(out))
    return out


def update_streaming(thetas, grads, tau: float, lam: float,
                     chunk_rows: int = 1 << 20):
    """The same step through the chunked closed form (large n)."""
    T = _worker(thetas)
    Gr = _worker(grads)
    m, n = T.shape
    C = np.zeros((m, m), np.float64)
    w = np.zeros(m, np.float64)
    for r0 in range(0, n, chunk_rows):
        gram_accumulate(Gr[:, r0:r0 + chunk_rows], C, w)
    co = coefficients(C, w, lam)
    theta_new = np.empty(n, np.float64)
    for r0 in range(0, n, chunk_rows):
        theta_new[r0:r0 + chunk_rows] = apply_closed_form(
            T[:, r0:r0 + chunk_rows], Gr[:, r0:r0 + chunk_rows], co["c"], tau)
    return dict(theta_new=theta_new, j=co["j"], C=C, w=w, sigma=co["sigma"],
                V=co["V"], c=co["c"], alpha=co["alpha"])


BOUND_SIGMA1, BOUND_SECANT = 1, 2


def tau_bounded_literal(tau: float, mode: int, Theta, G, sigma, V, j: int):
    """(tau_eff, sigma_max) with the norms of G v_k, Theta v_k formed explicitly."""
    Theta = _f64(Theta)
    G = _f64(G)
    m, n = G.shape
    smax = ctypes.c_double(0.0)
    t = lib().qno_tau_bounded_literal(float(tau), int(mode), _p(Theta), _p(G), n, m,
                                      _p(_f64(sigma)), _p(_f64(V)), int(j),
                                      ctypes.byref(smax))
    return t, smax.value


def tau_bounded_from_gram(tau: float, mode: int, Ct, sigma, V, j: int):
    """(tau_eff, sigma_max) from Ct = Theta^T Theta and the eigendecomposition."""
    Ct = _f64(Ct)
    m = Ct.shape[0]
    smax = ctypes.c_double(0.0)
    t = lib().qno_tau_bounded_from_gram(float(tau), int(mode), _p(Ct), m,
                                        _p(_f64(sigma)), _p(_f64(V)), int(j),
                                        ctypes.byref(smax))
    return t, smax.value
