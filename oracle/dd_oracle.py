"""ctypes front end of the CPU oracle (oracle/dd_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The product package never imports it.

Every function takes numpy arrays, widens them exactly to float64 and returns float64
(or int32 for the selection).  See the header of dd_oracle.c for the passages of the
paper each routine follows and for the reading of the rectangular convention.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dd_oracle.c")
_LIB = os.path.join(_HERE, "libdd_oracle.so")

_c_double_p = ctypes.POINTER(ctypes.c_double)
_c_float_p = ctypes.POINTER(ctypes.c_float)
_c_int32_p = ctypes.POINTER(ctypes.c_int32)


def build(force=False):
    """Compile dd_oracle.c with gcc (-O2, OpenMP over token rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.ddo_num_threads.restype = ctypes.c_int
        lib.ddo_materialize.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, _c_int32_p,
                                        _c_double_p, _c_double_p]
        lib.ddo_materialize.restype = None
        lib.ddo_fwd.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, _c_int32_p,
                                _c_double_p, _c_double_p, _c_double_p]
        lib.ddo_fwd.restype = ctypes.c_int
        lib.ddo_bwd_input.argtypes = lib.ddo_fwd.argtypes
        lib.ddo_bwd_input.restype = ctypes.c_int
        lib.ddo_bwd_weight.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       _c_int32_p, _c_double_p, _c_double_p, _c_double_p]
        lib.ddo_bwd_weight.restype = ctypes.c_int
        lib.ddo_bwd_weight_sampled.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, _c_int32_p,
                                               _c_double_p, _c_double_p, ctypes.c_int64,
                                               _c_int32_p, _c_int32_p, _c_double_p]
        lib.ddo_bwd_weight_sampled.restype = None
        lib.ddo_select.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, _c_float_p, _c_int32_p]
        lib.ddo_select.restype = ctypes.c_int
        lib.ddo_soft_topk.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, _c_double_p,
                                      _c_double_p]
        lib.ddo_soft_topk.restype = None
        lib.ddo_soft_topk_bwd.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, _c_double_p,
                                          _c_double_p, _c_double_p]
        lib.ddo_soft_topk_bwd.restype = None
        lib.ddo_scale_values.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, _c_int32_p, _c_double_p,
                                         _c_double_p, _c_double_p]
        lib.ddo_scale_values.restype = None
        lib.ddo_scale_values_bwd.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, _c_int32_p, _c_double_p,
                                             _c_double_p, _c_double_p, _c_double_p, _c_double_p]
        lib.ddo_scale_values_bwd.restype = None
        lib.ddo_diag_magnitude.argtypes = [ctypes.c_int, ctypes.c_int, _c_double_p, _c_double_p]
        lib.ddo_diag_magnitude.restype = None
        lib.ddo_diagheur_update.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, _c_int32_p, _c_float_p,
                                            _c_float_p, _c_int32_p, _c_int32_p]
        lib.ddo_diagheur_update.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _dp(a):
    return a.ctypes.data_as(_c_double_p)


def _ip(a):
    return a.ctypes.data_as(_c_int32_p)


def num_threads():
    return int(_load().ddo_num_threads())


def _check_values(values, K, M, N):
    L = min(M, N)
    if values.shape != (K, L):
        raise ValueError(f"values must be [K={K} x L={L}], got {values.shape}")


def materialize(M, N, offsets, values):
    """Dense W [M x N] holding the K wrapped diagonals (Sec. 3.1 Eq. 1-3, Appendix A)."""
    offsets = _i32(offsets)
    values = _f64(values)
    K = offsets.shape[0]
    _check_values(values, K, M, N)
    W = np.empty((M, N), dtype=np.float64)
    _load().ddo_materialize(M, N, K, _ip(offsets), _dp(values), _dp(W))
    return W


def fwd(X, offsets, values, N):
    """Y = X . W_K."""
    X = _f64(X)
    T, M = X.shape
    offsets = _i32(offsets)
    values = _f64(values)
    _check_values(values, offsets.shape[0], M, N)
    Y = np.empty((T, N), dtype=np.float64)
    if _load().ddo_fwd(T, M, N, offsets.shape[0], _ip(offsets), _dp(values), _dp(X), _dp(Y)):
        raise MemoryError
    return Y


def bwd_input(dY, offsets, values, M):
    """dX = dY . W_K^T."""
    dY = _f64(dY)
    T, N = dY.shape
    offsets = _i32(offsets)
    values = _f64(values)
    _check_values(values, offsets.shape[0], M, N)
    dX = np.empty((T, M), dtype=np.float64)
    if _load().ddo_bwd_input(T, M, N, offsets.shape[0], _ip(offsets), _dp(values), _dp(dY), _dp(dX)):
        raise MemoryError
    return dX


def bwd_weight(X, dY, offsets):
    """dValues [K x L]: the dense gradient X^T dY read back on the K diagonals."""
    X = _f64(X)
    dY = _f64(dY)
    T, M = X.shape
    T2, N = dY.shape
    if T != T2:
        raise ValueError("X and dY disagree on the token count")
    offsets = _i32(offsets)
    K = offsets.shape[0]
    out = np.empty((K, min(M, N)), dtype=np.float64)
    if _load().ddo_bwd_weight(T, M, N, K, _ip(offsets), _dp(X), _dp(dY), _dp(out)):
        raise MemoryError
    return out


def bwd_weight_sampled(X, dY, offsets, sample_k, sample_p):
    """dValues[sample_k[s], sample_p[s]] for each sample, each from the definition."""
    X = _f64(X)
    dY = _f64(dY)
    T, M = X.shape
    N = dY.shape[1]
    offsets = _i32(offsets)
    sample_k = _i32(sample_k)
    sample_p = _i32(sample_p)
    out = np.empty(sample_k.shape[0], dtype=np.float64)
    _load().ddo_bwd_weight_sampled(T, M, N, _ip(offsets), _dp(X), _dp(dY), sample_k.shape[0],
                                   _ip(sample_k), _ip(sample_p), _dp(out))
    return out


def select(scores, K):
    """Indices of the K largest scores per row (ties: lower index; NaN lowest), ascending."""
    scores = np.ascontiguousarray(np.asarray(scores, dtype=np.float32))
    if scores.ndim == 1:
        scores = scores[None, :]
    B, D = scores.shape
    if not 1 <= K <= D:
        raise ValueError("K must be in [1, D]")
    out = np.empty((B, K), dtype=np.int32)
    if _load().ddo_select(B, D, K, scores.ctypes.data_as(_c_float_p), _ip(out)):
        raise MemoryError
    return out


def soft_topk(scores, K, temperature):
    """alpha_tilde = min(K * softmax(scores / temperature), 1), row by row (Sec. 3.2, Eq. 5)."""
    scores = _f64(scores)
    if scores.ndim == 1:
        scores = scores[None, :]
    B, D = scores.shape
    out = np.empty((B, D), dtype=np.float64)
    _load().ddo_soft_topk(B, D, int(K), float(temperature), _dp(scores), _dp(out))
    return out


def soft_topk_bwd(scores, K, temperature, g):
    """Gradient of the loss with respect to the scores, given g = dL/dalpha_tilde."""
    scores = _f64(scores)
    g = _f64(g)
    if scores.ndim == 1:
        scores, g = scores[None, :], g[None, :]
    B, D = scores.shape
    out = np.empty((B, D), dtype=np.float64)
    _load().ddo_soft_topk_bwd(B, D, int(K), float(temperature), _dp(scores), _dp(g), _dp(out))
    return out


def scale_values(offsets, alpha_tilde, V):
    """values_eff[k] = alpha_tilde[offsets[k] mod D] * V[k]  (Eq. 4)."""
    offsets = _i32(offsets)
    alpha_tilde = _f64(alpha_tilde)
    V = _f64(V)
    K, L = V.shape
    out = np.empty((K, L), dtype=np.float64)
    _load().ddo_scale_values(K, L, alpha_tilde.shape[0], _ip(offsets), _dp(alpha_tilde), _dp(V), _dp(out))
    return out


def scale_values_bwd(offsets, alpha_tilde, V, dValues):
    """(dV [K x L], dalpha_tilde [D]) from dValues = dL/dvalues_eff."""
    offsets = _i32(offsets)
    alpha_tilde = _f64(alpha_tilde)
    V = _f64(V)
    dValues = _f64(dValues)
    K, L = V.shape
    D = alpha_tilde.shape[0]
    dV = np.empty((K, L), dtype=np.float64)
    dalpha = np.empty(D, dtype=np.float64)
    _load().ddo_scale_values_bwd(K, L, D, _ip(offsets), _dp(alpha_tilde), _dp(V), _dp(dValues), _dp(dV), _dp(dalpha))
    return dV, dalpha


def diag_magnitude(values):
    """Sum of |v_k[p]| over each diagonal (the appendix on the heuristics-based method)."""
    values = _f64(values)
    K, L = values.shape
    out = np.empty(K, dtype=np.float64)
    _load().ddo_diag_magnitude(K, L, _dp(values), _dp(out))
    return out


def diagheur_update(D, offsets, magnitudes, random, n_drop):
    """(new_offsets [K] ascending, source [K]): drop the n_drop weakest active diagonals, grow the n_drop
    inactive candidates with the largest random score."""
    offsets = _i32(offsets)
    K = offsets.shape[0]
    magnitudes = np.ascontiguousarray(np.asarray(magnitudes, dtype=np.float32))
    random = np.ascontiguousarray(np.asarray(random, dtype=np.float32))
    if magnitudes.shape != (K,) or random.shape != (D,):
        raise ValueError("magnitudes must be [K], random [D]")
    new_offsets = np.empty(K, dtype=np.int32)
    source = np.empty(K, dtype=np.int32)
    rc = _load().ddo_diagheur_update(int(D), K, int(n_drop), _ip(offsets), magnitudes.ctypes.data_as(_c_float_p),
                                     random.ctypes.data_as(_c_float_p), _ip(new_offsets), _ip(source))
    if rc == 1:
        raise ValueError("n_drop must be in [0, min(K, D - K)]")
    if rc:
        raise MemoryError
    return new_offsets, source
