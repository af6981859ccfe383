"""Thin Python binding of libdynadiag.so: argument marshalling only.

Same names as the C ABI (include/dynadiag.h).  Tensors are torch tensors on the GPU; torch is
used for device memory and for the current stream handle, nothing else.  There is no fallback:
if the shared library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch  # imported before the library so that both share one HIP runtime

from .build import LIB_PATH

DD_F32, DD_BF16 = 0, 1
DD_ALGO_AUTO, DD_ALGO_VECTOR, DD_ALGO_MATRIX, DD_ALGO_PREPARED, DD_ALGO_BLOCKS = 0, 1, 2, 3, 4
DD_OP_FWD, DD_OP_BWD_INPUT, DD_OP_BWD_WEIGHT, DD_OP_SELECT, DD_OP_SCALE_VALUES_BWD, DD_OP_PREPARE = 0, 1, 2, 3, 4, 5
DD_OP_DIAGHEUR, DD_OP_BWD_WEIGHT_SCALED, DD_OP_BWD = 6, 7, 8

EXPORTS = ("dd_workspace_bytes", "dd_fwd", "dd_prepare", "dd_prepare_batched", "dd_select_prepare", "dd_prepare_shared", "dd_fwd_shared", "dd_bwd_input_shared",
           "dd_bwd_input", "dd_bwd", "dd_bwd_weight", "dd_bwd_weight_static", "dd_static_scratch_bytes", "dd_select_diagonals",
           "dd_select_soft", "dd_prepare_scaled", "dd_bwd_weight_scaled", "dd_soft_topk", "dd_soft_topk_bwd", "dd_scale_values", "dd_scale_values_bwd", "dd_diag_magnitude",
           "dd_diagheur_update", "dd_status_string")


class DynaDiagError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"dynadiag: {message} (status {status})")
        self.status = status


class dd_layer(ctypes.Structure):
    _fields_ = [("tokens", ctypes.c_int64), ("in_features", ctypes.c_int32), ("out_features", ctypes.c_int32),
                ("K", ctypes.c_int32), ("dtype", ctypes.c_int32), ("algo", ctypes.c_int32)]


_lib = None


def load_library():
    """dlopen libdynadiag.so and declare the prototypes.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise DynaDiagError(-1, f"{LIB_PATH} is not built; run `python -m paper_2506_11449_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
    lp = ctypes.POINTER(dd_layer)
    lib.dd_workspace_bytes.argtypes = [ctypes.c_int, lp, i32]
    lib.dd_workspace_bytes.restype = sz
    lib.dd_fwd.argtypes = [lp, vp, vp, vp, vp, vp, sz, vp]
    lib.dd_prepare.argtypes = [lp, vp, vp, vp, sz, vp]
    lib.dd_select_prepare.argtypes = [lp, vp, vp, vp, vp, sz, vp]
    lib.dd_prepare_batched.argtypes = [lp, i32, vp, vp, vp, sz, vp]
    lib.dd_prepare_batched.restype = ctypes.c_int
    lib.dd_prepare_shared.argtypes = [lp, i32, vp, vp, vp, sz, vp]
    lib.dd_fwd_shared.argtypes = [lp, i32, vp, vp, sz, vp, vp]
    lib.dd_bwd_input_shared.argtypes = [lp, i32, vp, vp, sz, vp, vp]
    lib.dd_bwd_input.argtypes = [lp, vp, vp, vp, vp, vp, sz, vp]
    lib.dd_bwd_weight.argtypes = [lp, vp, vp, vp, vp, vp, sz, vp]
    lib.dd_bwd.argtypes = [lp, vp, vp, vp, vp, vp, sz, vp, vp, vp, sz, vp]
    lib.dd_bwd_weight_static.argtypes = [lp, vp, vp, vp, vp, vp]
    lib.dd_bwd_weight_static.restype = ctypes.c_int
    lib.dd_static_scratch_bytes.argtypes = []
    lib.dd_static_scratch_bytes.restype = sz
    lib.dd_select_diagonals.argtypes = [i32, i32, i32, vp, vp, vp, sz, vp]
    f32 = ctypes.c_float
    lib.dd_select_soft.argtypes = [i32, i32, i32, f32, vp, vp, vp, vp]
    lib.dd_prepare_scaled.argtypes = [lp, vp, vp, vp, vp, sz, vp]
    lib.dd_bwd_weight_scaled.argtypes = [lp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dd_soft_topk.argtypes = [i32, i32, i32, f32, vp, vp, vp]
    lib.dd_soft_topk_bwd.argtypes = [i32, i32, i32, f32, vp, vp, vp, vp]
    lib.dd_scale_values.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.dd_scale_values_bwd.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dd_diag_magnitude.argtypes = [i32, i32, i32, vp, vp, vp]
    lib.dd_diagheur_update.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    for name in ("dd_diag_magnitude", "dd_diagheur_update", "dd_fwd", "dd_prepare", "dd_bwd_input", "dd_bwd_weight", "dd_bwd_weight_static", "dd_static_scratch_bytes", "dd_select_diagonals", "dd_soft_topk",
                 "dd_soft_topk_bwd", "dd_scale_values", "dd_scale_values_bwd"):
        getattr(lib, name).restype = ctypes.c_int
    lib.dd_status_string.argtypes = [ctypes.c_int]
    lib.dd_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(status):
    if status:
        raise DynaDiagError(status, load_library().dd_status_string(status).decode())


_DTYPES = {torch.float32: DD_F32, torch.bfloat16: DD_BF16}


def make_layer(tokens, in_features, out_features, K, dtype, algo=DD_ALGO_AUTO):
    if isinstance(dtype, torch.dtype):
        dtype = _DTYPES[dtype]
    return dd_layer(int(tokens), int(in_features), int(out_features), int(K), int(dtype), int(algo))


_plan_cache = {}


def _plan(op, tokens, in_features, out_features, K, dtype, algo, batch=0):
    """(layer struct, byref(layer), workspace bytes) for one entry point and shape, built once."""
    key = (op, tokens, in_features, out_features, K, dtype, algo, batch)
    hit = _plan_cache.get(key)
    if hit is None:
        layer = make_layer(tokens, in_features, out_features, K, dtype, algo)
        ref = ctypes.byref(layer)
        need = int(load_library().dd_workspace_bytes(int(op), ref, int(batch)))
        hit = _plan_cache[key] = (layer, ref, need)
    return hit


def dd_workspace_bytes(op, layer, batch=0):
    return int(load_library().dd_workspace_bytes(int(op), ctypes.byref(layer), int(batch)))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev(t, dtype, shape, name):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous GPU tensor")
    if t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected {dtype} {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")
    return t


class Workspace:
    """A reusable block of device scratch, grown on demand by the caller's side of the ABI."""

    def __init__(self):
        self.buf = None

    def get(self, nbytes, device):
        if nbytes == 0:
            return None, 0
        if self.buf is None or self.buf.numel() < nbytes or self.buf.device != device:
            self.buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
        return self.buf, self.buf.numel()


_default_ws = Workspace()


def _ws_for(need, device, ws):
    buf, n = (ws or _default_ws).get(need, device)
    return _ptr(buf), n


class Prepared:
    """The block dd_prepare fills for one set of (offsets, values): the dense operands of dd_fwd / dd_bwd_input."""

    def __init__(self, buf, in_features, out_features, K, dtype):
        self.buf, self.in_features, self.out_features, self.K, self.dtype = buf, in_features, out_features, K, dtype


def dd_prepare(offsets, values, in_features, out_features, prepared=None, stream=None):
    """Builds the dense operands of the matrix-core path once; pass the result as `prepared=` to dd_fwd / dd_bwd_input."""
    M, N, K = int(in_features), int(out_features), offsets.shape[0]
    _, ref, need = _plan(DD_OP_PREPARE, 0, M, N, K, values.dtype, DD_ALGO_PREPARED)
    _dev(offsets, torch.int32, (K,), "offsets")
    _dev(values, values.dtype, (K, min(M, N)), "values")
    if prepared is None:
        prepared = Prepared(torch.empty(max(need, 1), dtype=torch.uint8, device=values.device), M, N, K, values.dtype)
    if (prepared.in_features, prepared.out_features, prepared.K, prepared.dtype) != (M, N, K, values.dtype):
        raise ValueError("prepared block belongs to another layer")
    _check(load_library().dd_prepare(ref, _ptr(offsets), _ptr(values), _ptr(prepared.buf), prepared.buf.numel(), _stream(stream)))
    return prepared


def dd_prepare_batched(offsets, values, in_features, out_features, prepared=None, stream=None):
    """dd_prepare for n independent layers of one shape in one launch: offsets int32 [n x K], values [n x K x min(M,N)].

    Returns a list of n Prepared blocks (views into one buffer); pass it back as prepared= to refill it."""
    M, N = int(in_features), int(out_features)
    n, K = offsets.shape
    _, ref, need = _plan(DD_OP_PREPARE, 0, M, N, K, values.dtype, DD_ALGO_PREPARED)
    _dev(offsets, torch.int32, (n, K), "offsets")
    _dev(values, values.dtype, (n, K, min(M, N)), "values")
    if prepared is None:
        buf = torch.empty(max(need * n, 1), dtype=torch.uint8, device=values.device)
        prepared = [Prepared(buf[i * need:(i + 1) * need], M, N, K, values.dtype) for i in range(n)]
        prepared[0].whole = buf
    first = prepared[0]
    if len(prepared) != n or (first.in_features, first.out_features, first.K, first.dtype) != (M, N, K, values.dtype):
        raise ValueError("prepared blocks belong to other layers")
    _check(load_library().dd_prepare_batched(ref, n, _ptr(offsets), _ptr(values), _ptr(first.whole), first.whole.numel(),
                                             _stream(stream)))
    return prepared


def dd_select_prepare(scores, values, in_features, out_features, offsets_out=None, prepared=None, stream=None):
    """dd_select_diagonals on one score vector [D] and dd_prepare on its result, one call: (offsets [K], prepared)."""
    M, N, K = int(in_features), int(out_features), values.shape[0]
    D = max(M, N)
    _, ref, need = _plan(DD_OP_PREPARE, 0, M, N, K, values.dtype, DD_ALGO_PREPARED)
    _dev(scores, torch.float32, (D,), "scores")
    _dev(values, values.dtype, (K, min(M, N)), "values")
    if offsets_out is None:
        offsets_out = torch.empty((K,), dtype=torch.int32, device=values.device)
    _dev(offsets_out, torch.int32, (K,), "offsets_out")
    if prepared is None:
        prepared = Prepared(torch.empty(max(need, 1), dtype=torch.uint8, device=values.device), M, N, K, values.dtype)
    if (prepared.in_features, prepared.out_features, prepared.K, prepared.dtype) != (M, N, K, values.dtype):
        raise ValueError("prepared block belongs to another layer")
    _check(load_library().dd_select_prepare(ref, _ptr(scores), _ptr(values), _ptr(offsets_out), _ptr(prepared.buf),
                                            prepared.buf.numel(), _stream(stream)))
    return offsets_out, prepared


class PreparedShared:
    """The block dd_prepare_shared fills for a group of n_sets layers of one shape that share their input."""

    def __init__(self, buf, n_sets, in_features, out_features, K, dtype):
        self.buf, self.n_sets = buf, n_sets
        self.in_features, self.out_features, self.K, self.dtype = in_features, out_features, K, dtype


def dd_prepare_shared(offsets, values, in_features, out_features, prepared=None, stream=None):
    """offsets int32 [S x K], values [S x K x min(M,N)]: the dense operands of dd_fwd_shared / dd_bwd_input_shared."""
    M, N = int(in_features), int(out_features)
    S, K = offsets.shape
    _, ref, need = _plan(DD_OP_PREPARE, 0, M, N, K, values.dtype, DD_ALGO_PREPARED)
    _dev(offsets, torch.int32, (S, K), "offsets")
    _dev(values, values.dtype, (S, K, min(M, N)), "values")
    if prepared is None:
        prepared = PreparedShared(torch.empty(max(need * S, 1), dtype=torch.uint8, device=values.device), S, M, N, K,
                                  values.dtype)
    if (prepared.n_sets, prepared.in_features, prepared.out_features, prepared.K, prepared.dtype) != \
            (S, M, N, K, values.dtype):
        raise ValueError("prepared block belongs to another group of layers")
    _check(load_library().dd_prepare_shared(ref, S, _ptr(offsets), _ptr(values), _ptr(prepared.buf),
                                            prepared.buf.numel(), _stream(stream)))
    return prepared


def dd_fwd_shared(X, prepared, Y=None, stream=None):
    """Y[s] = X . W_s for every set of the group: X [T x M] -> Y [S x T x N]."""
    T, M, N, S = X.shape[0], prepared.in_features, prepared.out_features, prepared.n_sets
    if prepared.dtype != X.dtype:
        raise ValueError("prepared block belongs to another group of layers")
    ref = make_layer(T, M, N, prepared.K, X.dtype, DD_ALGO_PREPARED)
    _dev(X, X.dtype, (T, M), "X")
    if Y is None:
        Y = torch.empty((S, T, N), dtype=X.dtype, device=X.device)
    _dev(Y, X.dtype, (S, T, N), "Y")
    _check(load_library().dd_fwd_shared(ctypes.byref(ref), S, _ptr(X), _ptr(prepared.buf), prepared.buf.numel(), _ptr(Y),
                                        _stream(stream)))
    return Y


def dd_bwd_input_shared(dY, prepared, dX=None, stream=None):
    """dX = sum over the sets of dY[s] . W_s^T: dY [S x T x N] -> dX [T x M]."""
    M, N, S = prepared.in_features, prepared.out_features, prepared.n_sets
    T = dY.shape[1]
    if prepared.dtype != dY.dtype:
        raise ValueError("prepared block belongs to another group of layers")
    ref = make_layer(T, M, N, prepared.K, dY.dtype, DD_ALGO_PREPARED)
    _dev(dY, dY.dtype, (S, T, N), "dY")
    if dX is None:
        dX = torch.empty((T, M), dtype=dY.dtype, device=dY.device)
    _dev(dX, dY.dtype, (T, M), "dX")
    _check(load_library().dd_bwd_input_shared(ctypes.byref(ref), S, _ptr(dY), _ptr(prepared.buf), prepared.buf.numel(),
                                              _ptr(dX), _stream(stream)))
    return dX


def _product(fn, op, src, offsets, values, n_src, n_dst, M, N, dst, algo, ws, stream, prepared, names):
    T = src.shape[0]
    if prepared is not None:
        if (prepared.in_features, prepared.out_features, prepared.dtype) != (M, N, src.dtype):
            raise ValueError("prepared block belongs to another layer")
        algo, K = (DD_ALGO_BLOCKS if algo == DD_ALGO_BLOCKS else DD_ALGO_PREPARED), prepared.K
        if algo == DD_ALGO_BLOCKS:
            _dev(offsets, torch.int32, (K,), "offsets")
    else:
        K = offsets.shape[0]
        _dev(offsets, torch.int32, (K,), "offsets")
        _dev(values, src.dtype, (K, min(M, N)), "values")
    _, ref, need = _plan(op, T, M, N, K, src.dtype, algo)
    _dev(src, src.dtype, (T, n_src), names[0])
    if dst is None:
        dst = torch.empty((T, n_dst), dtype=src.dtype, device=src.device)
    _dev(dst, src.dtype, (T, n_dst), names[1])
    if prepared is not None:
        wp, wn = _ptr(prepared.buf), prepared.buf.numel()
        _check(fn(ref, _ptr(src), _ptr(offsets) if algo == DD_ALGO_BLOCKS else None, None, _ptr(dst), wp, wn,
                  _stream(stream)))
    else:
        wp, wn = _ws_for(need, src.device, ws)
        _check(fn(ref, _ptr(src), _ptr(offsets), _ptr(values), _ptr(dst), wp, wn, _stream(stream)))
    return dst


def dd_fwd(X, offsets, values, out_features, Y=None, algo=DD_ALGO_AUTO, ws=None, stream=None, prepared=None):
    """Y = X . W_K.  X [T x M], offsets int32 [K], values [K x min(M,N)] -> Y [T x N].

    With prepared= (from dd_prepare) offsets and values are not read and may be None; with algo=DD_ALGO_BLOCKS
    as well, the offsets are read (the product then skips the operand blocks no diagonal crosses)."""
    M, N = X.shape[1], int(out_features)
    return _product(load_library().dd_fwd, DD_OP_FWD, X, offsets, values, M, N, M, N, Y, algo, ws, stream, prepared,
                    ("X", "Y"))


def dd_bwd_input(dY, offsets, values, in_features, dX=None, algo=DD_ALGO_AUTO, ws=None, stream=None, prepared=None):
    """dX = dY . W_K^T.  dY [T x N] -> dX [T x M].  prepared= as for dd_fwd."""
    M, N = int(in_features), dY.shape[1]
    return _product(load_library().dd_bwd_input, DD_OP_BWD_INPUT, dY, offsets, values, N, M, M, N, dX, algo, ws, stream,
                    prepared, ("dY", "dX"))


def dd_bwd_weight(X, dY, offsets, dValues=None, algo=DD_ALGO_AUTO, ws=None, stream=None):
    """dValues [K x min(M,N)] fp32: the gradient of the values on the K diagonals."""
    T, M = X.shape
    N = dY.shape[1]
    K = offsets.shape[0]
    _, ref, need = _plan(DD_OP_BWD_WEIGHT, T, M, N, K, X.dtype, algo)
    _dev(X, X.dtype, (T, M), "X")
    _dev(dY, X.dtype, (T, N), "dY")
    _dev(offsets, torch.int32, (K,), "offsets")
    if dValues is None:
        dValues = torch.empty((K, min(M, N)), dtype=torch.float32, device=X.device)
    _dev(dValues, torch.float32, (K, min(M, N)), "dValues")
    wp, wn = _ws_for(need, X.device, ws)
    _check(_lib.dd_bwd_weight(ref, _ptr(X), _ptr(dY), _ptr(offsets), _ptr(dValues), wp, wn, _stream(stream)))
    return dValues


def dd_bwd(X, dY, offsets, values, dX=None, dValues=None, algo=DD_ALGO_AUTO, ws=None, stream=None, prepared=None):
    """The backward pass as one call: (dX [T x M], dValues [K x min(M,N)] fp32).  prepared= as for dd_fwd."""
    T, M = X.shape
    N = dY.shape[1]
    K = offsets.shape[0]
    if prepared is not None:
        if (prepared.in_features, prepared.out_features, prepared.dtype) != (M, N, X.dtype):
            raise ValueError("prepared block belongs to another layer")
        algo = DD_ALGO_PREPARED
    else:
        _dev(values, X.dtype, (K, min(M, N)), "values")
    _, ref, need = _plan(DD_OP_BWD, T, M, N, K, X.dtype, algo)
    _dev(X, X.dtype, (T, M), "X")
    _dev(dY, X.dtype, (T, N), "dY")
    _dev(offsets, torch.int32, (K,), "offsets")
    if dX is None:
        dX = torch.empty((T, M), dtype=X.dtype, device=X.device)
    if dValues is None:
        dValues = torch.empty((K, min(M, N)), dtype=torch.float32, device=X.device)
    _dev(dX, X.dtype, (T, M), "dX")
    _dev(dValues, torch.float32, (K, min(M, N)), "dValues")
    wp, wn = _ws_for(need, X.device, ws)
    pp, pn = (None, 0) if prepared is None else (_ptr(prepared.buf), prepared.buf.numel())
    _check(load_library().dd_bwd(ref, _ptr(X), _ptr(dY), _ptr(offsets), _ptr(values), pp, pn, _ptr(dX), _ptr(dValues),
                                 wp, wn, _stream(stream)))
    return dX, dValues


def dd_static_scratch_bytes():
    return int(load_library().dd_static_scratch_bytes())


def dd_bwd_weight_static(X, dY, offsets, dValues, algo=DD_ALGO_AUTO, stream=None):
    """dd_bwd_weight without a workspace and without any allocation: dValues [K x min(M,N)] fp32 is the caller's."""
    T, M = X.shape
    N = dY.shape[1]
    K = offsets.shape[0]
    _, ref, _ = _plan(DD_OP_BWD_WEIGHT, T, M, N, K, X.dtype, algo)
    _dev(X, X.dtype, (T, M), "X")
    _dev(dY, X.dtype, (T, N), "dY")
    _dev(offsets, torch.int32, (K,), "offsets")
    _dev(dValues, torch.float32, (K, min(M, N)), "dValues")
    _check(load_library().dd_bwd_weight_static(ref, _ptr(X), _ptr(dY), _ptr(offsets), _ptr(dValues), _stream(stream)))
    return dValues


def dd_select_diagonals(scores, K, offsets_out=None, ws=None, stream=None):
    """Indices of the K largest scores of each row of scores [batch x D], ascending, int32 [batch x K]."""
    if scores.dim() != 2:
        raise ValueError("scores must be [batch x D]")
    B, D = scores.shape
    _dev(scores, torch.float32, (B, D), "scores")
    if offsets_out is None:
        offsets_out = torch.empty((B, K), dtype=torch.int32, device=scores.device)
    _dev(offsets_out, torch.int32, (B, K), "offsets_out")
    _, _, need = _plan(DD_OP_SELECT, 0, D, D, int(K), DD_F32, DD_ALGO_AUTO, batch=B)
    wp, wn = _ws_for(need, scores.device, ws)
    _check(_lib.dd_select_diagonals(B, D, int(K), _ptr(scores), _ptr(offsets_out), wp, wn, _stream(stream)))
    return offsets_out


def dd_select_soft(scores, K, temperature, offsets_out=None, alpha_tilde=None, stream=None):
    """dd_select_diagonals and dd_soft_topk in one launch: (offsets int32 [batch x K], alpha_tilde fp32 [batch x D])."""
    B, D = scores.shape
    _dev(scores, torch.float32, (B, D), "scores")
    if offsets_out is None:
        offsets_out = torch.empty((B, K), dtype=torch.int32, device=scores.device)
    if alpha_tilde is None:
        alpha_tilde = torch.empty_like(scores)
    _dev(offsets_out, torch.int32, (B, K), "offsets_out")
    _dev(alpha_tilde, torch.float32, (B, D), "alpha_tilde")
    _check(load_library().dd_select_soft(B, D, int(K), float(temperature), _ptr(scores), _ptr(offsets_out),
                                         _ptr(alpha_tilde), _stream(stream)))
    return offsets_out, alpha_tilde


def dd_prepare_scaled(offsets, alpha_tilde, V, in_features, out_features, prepared=None, stream=None):
    """dd_prepare on alpha_tilde[o_k] * V[k] without writing the scaled values anywhere."""
    M, N, K = int(in_features), int(out_features), offsets.shape[0]
    _, ref, need = _plan(DD_OP_PREPARE, 0, M, N, K, V.dtype, DD_ALGO_PREPARED)
    _dev(offsets, torch.int32, (K,), "offsets")
    _dev(alpha_tilde, torch.float32, (max(M, N),), "alpha_tilde")
    _dev(V, V.dtype, (K, min(M, N)), "V")
    if prepared is None:
        prepared = Prepared(torch.empty(max(need, 1), dtype=torch.uint8, device=V.device), M, N, K, V.dtype)
    if (prepared.in_features, prepared.out_features, prepared.K, prepared.dtype) != (M, N, K, V.dtype):
        raise ValueError("prepared block belongs to another layer")
    _check(load_library().dd_prepare_scaled(ref, _ptr(offsets), _ptr(alpha_tilde), _ptr(V), _ptr(prepared.buf),
                                            prepared.buf.numel(), _stream(stream)))
    return prepared


def dd_bwd_weight_scaled(X, dY, offsets, alpha_tilde, V, dV=None, d_alpha_tilde=None, algo=DD_ALGO_AUTO, ws=None,
                         stream=None):
    """dd_bwd_weight and dd_scale_values_bwd as one call: (dV [K x L] fp32, d_alpha_tilde [D] fp32)."""
    T, M = X.shape
    N = dY.shape[1]
    K, D, L = offsets.shape[0], max(M, N), min(M, N)
    _, ref, need = _plan(DD_OP_BWD_WEIGHT_SCALED, T, M, N, K, X.dtype, algo)
    _dev(X, X.dtype, (T, M), "X")
    _dev(dY, X.dtype, (T, N), "dY")
    _dev(offsets, torch.int32, (K,), "offsets")
    _dev(alpha_tilde, torch.float32, (D,), "alpha_tilde")
    _dev(V, X.dtype, (K, L), "V")
    if dV is None:
        dV = torch.empty((K, L), dtype=torch.float32, device=X.device)
    if d_alpha_tilde is None:
        d_alpha_tilde = torch.empty((D,), dtype=torch.float32, device=X.device)
    _dev(dV, torch.float32, (K, L), "dV")
    _dev(d_alpha_tilde, torch.float32, (D,), "d_alpha_tilde")
    wp, wn = _ws_for(need, X.device, ws)
    _check(load_library().dd_bwd_weight_scaled(ref, _ptr(X), _ptr(dY), _ptr(offsets), _ptr(alpha_tilde), _ptr(V),
                                               _ptr(dV), _ptr(d_alpha_tilde), wp, wn, _stream(stream)))
    return dV, d_alpha_tilde


def dd_soft_topk(scores, K, temperature, alpha_tilde=None, stream=None):
    """alpha_tilde = min(K * softmax(scores / temperature), 1) for each row of scores [batch x D] (fp32)."""
    B, D = scores.shape
    _dev(scores, torch.float32, (B, D), "scores")
    if alpha_tilde is None:
        alpha_tilde = torch.empty_like(scores)
    _dev(alpha_tilde, torch.float32, (B, D), "alpha_tilde")
    _check(load_library().dd_soft_topk(B, D, int(K), float(temperature), _ptr(scores), _ptr(alpha_tilde),
                                       _stream(stream)))
    return alpha_tilde


def dd_soft_topk_bwd(scores, K, temperature, d_alpha_tilde, d_scores=None, stream=None):
    """Gradient with respect to the scores, from the gradient with respect to alpha_tilde."""
    B, D = scores.shape
    _dev(scores, torch.float32, (B, D), "scores")
    _dev(d_alpha_tilde, torch.float32, (B, D), "d_alpha_tilde")
    if d_scores is None:
        d_scores = torch.empty_like(scores)
    _dev(d_scores, torch.float32, (B, D), "d_scores")
    _check(load_library().dd_soft_topk_bwd(B, D, int(K), float(temperature), _ptr(scores), _ptr(d_alpha_tilde),
                                           _ptr(d_scores), _stream(stream)))
    return d_scores


def dd_scale_values(offsets, alpha_tilde, V, values_eff=None, stream=None):
    """values_eff[k] = alpha_tilde[offsets[k] mod D] * V[k]; alpha_tilde [D] fp32, V [K x L] fp32 or bf16."""
    K, L = V.shape
    D = alpha_tilde.shape[0]
    _dev(offsets, torch.int32, (K,), "offsets")
    _dev(alpha_tilde, torch.float32, (D,), "alpha_tilde")
    _dev(V, V.dtype, (K, L), "V")
    if values_eff is None:
        values_eff = torch.empty_like(V)
    _dev(values_eff, V.dtype, (K, L), "values_eff")
    _check(load_library().dd_scale_values(K, L, D, _DTYPES[V.dtype], _ptr(offsets), _ptr(alpha_tilde), _ptr(V),
                                          _ptr(values_eff), _stream(stream)))
    return values_eff


def dd_scale_values_bwd(offsets, alpha_tilde, V, dValues, ws=None, stream=None):
    """(dV [K x L] fp32, d_alpha_tilde [D] fp32) from dValues = the output of dd_bwd_weight."""
    K, L = V.shape
    D = alpha_tilde.shape[0]
    _dev(offsets, torch.int32, (K,), "offsets")
    _dev(alpha_tilde, torch.float32, (D,), "alpha_tilde")
    _dev(V, V.dtype, (K, L), "V")
    _dev(dValues, torch.float32, (K, L), "dValues")
    dV = torch.empty((K, L), dtype=torch.float32, device=V.device)
    d_alpha = torch.empty((D,), dtype=torch.float32, device=V.device)
    _, _, need = _plan(DD_OP_SCALE_VALUES_BWD, 0, D, D, K, DD_F32, DD_ALGO_AUTO)
    wp, wn = _ws_for(need, V.device, ws)
    _check(load_library().dd_scale_values_bwd(K, L, D, _DTYPES[V.dtype], _ptr(offsets), _ptr(alpha_tilde), _ptr(V),
                                              _ptr(dValues), _ptr(dV), _ptr(d_alpha), wp, wn, _stream(stream)))
    return dV, d_alpha


def dd_diag_magnitude(values, magnitudes=None, stream=None):
    """magnitudes[k] = sum_p |values[k][p]| (fp32) for values [K x L]."""
    K, L = values.shape
    _dev(values, values.dtype, (K, L), "values")
    if magnitudes is None:
        magnitudes = torch.empty(K, dtype=torch.float32, device=values.device)
    _dev(magnitudes, torch.float32, (K,), "magnitudes")
    _check(load_library().dd_diag_magnitude(K, L, _DTYPES[values.dtype], _ptr(values), _ptr(magnitudes),
                                            _stream(stream)))
    return magnitudes


def dd_diagheur_update(D, offsets, magnitudes, random, n_drop, new_offsets=None, source=None, ws=None, stream=None):
    """Drop the n_drop weakest active diagonals, grow the n_drop inactive candidates with the largest random score.

    Returns (new_offsets [K] ascending, source [K]: position in `offsets` or -1 for a grown diagonal)."""
    D, K = int(D), offsets.shape[0]
    _dev(offsets, torch.int32, (K,), "offsets")
    _dev(magnitudes, torch.float32, (K,), "magnitudes")
    _dev(random, torch.float32, (D,), "random")
    if new_offsets is None:
        new_offsets = torch.empty(K, dtype=torch.int32, device=offsets.device)
    if source is None:
        source = torch.empty(K, dtype=torch.int32, device=offsets.device)
    _dev(new_offsets, torch.int32, (K,), "new_offsets")
    _dev(source, torch.int32, (K,), "source")
    _, _, need = _plan(DD_OP_DIAGHEUR, 0, D, D, K, DD_F32, DD_ALGO_AUTO)
    wp, wn = _ws_for(need, offsets.device, ws)
    _check(load_library().dd_diagheur_update(D, K, int(n_drop), _ptr(offsets), _ptr(magnitudes), _ptr(random),
                                             _ptr(new_offsets), _ptr(source), wp, wn, _stream(stream)))
    return new_offsets, source
