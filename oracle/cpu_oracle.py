"""ctypes front-end of the C oracle (test infrastructure, not the product).

Takes numpy arrays (or anything numpy can view), hands raw buffers to
``libmaxsim_oracle.so`` and returns numpy arrays.  16-bit inputs travel as
``uint16`` bit patterns so that no conversion happens on the Python side;
the C code decodes them itself.  Nothing here touches the GPU library.
"""
import ctypes
import os

import numpy as np

from . import build as _build

F32, F16, BF16 = 0, 1, 2
_DTYPE_NAMES = {"f32": F32, "f16": F16, "bf16": BF16}

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        c_i, c_l, c_p = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p
        L.oracle_decode_f16.restype = ctypes.c_double
        L.oracle_decode_f16.argtypes = [ctypes.c_uint16]
        L.oracle_decode_bf16.restype = ctypes.c_double
        L.oracle_decode_bf16.argtypes = [ctypes.c_uint16]
        L.oracle_forward.restype = c_i
        L.oracle_forward.argtypes = [c_p, c_i, c_i, c_p, c_l, c_i, c_p, c_i, c_i, c_p, c_p, c_p, c_i]
        L.oracle_backward.restype = c_i
        L.oracle_backward.argtypes = [c_p, c_i, c_i, c_p, c_l, c_i, c_i, c_i, c_p, c_p, c_p, c_p]
        L.oracle_forward_i8.restype = c_i
        L.oracle_forward_i8.argtypes = [c_p, c_p, c_i, c_i, c_p, c_p, c_l, c_i, c_i, c_p, c_i]
        L.oracle_dot_i8.restype = c_i
        L.oracle_dot_i8.argtypes = [c_p, c_i, c_p, c_i, c_i, c_p]
        L.oracle_quantize_rows_i8.restype = c_i
        L.oracle_quantize_rows_i8.argtypes = [c_p, c_l, c_i, c_i, c_p, c_p]
        L.oracle_ce_grad.restype = c_i
        L.oracle_ce_grad.argtypes = [c_p, c_i, c_i, ctypes.c_double, c_p, c_p]
        _lib = L
    return _lib


def default_threads() -> int:
    return max(1, min(os.cpu_count() or 1, 64))


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else None


def as_raw(x, dtype: str) -> np.ndarray:
    """Contiguous raw buffer for dtype 'f32' (float32) or 'f16'/'bf16' (uint16 bit patterns)."""
    a = np.ascontiguousarray(x)
    if dtype == "f32":
        if a.dtype != np.float32:
            raise TypeError("f32 input must be float32, got %s" % a.dtype)
        return a
    if dtype == "f16" and a.dtype == np.float16:
        return a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("%s input must be uint16 bit patterns (or float16 for f16), got %s" % (dtype, a.dtype))
    return a


def decode_array(raw: np.ndarray, dtype: str) -> np.ndarray:
    """Stored values as float64 (exact): fp32 widened, fp16 / bf16 bit patterns decoded."""
    if dtype == "f32":
        return raw.astype(np.float64)
    if dtype == "f16":
        return raw.view(np.float16).astype(np.float64)
    return (raw.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def forward(Q, D, dtype: str, offsets=None, want_argmax=True, want_margin=True, threads=None):
    """Eq. 1.  Q [n_q,l_q,d]; D [b,l_d,d] (uniform) or [T,d] with int32 offsets [b+1] (ragged).

    Returns (scores float64 [n_q,b], argmax int32 [n_q,b,l_q] or None, margin float64 or None).
    """
    Qr, Dr = as_raw(Q, dtype), as_raw(D, dtype)
    n_q, l_q, d = Qr.shape
    if offsets is None:
        b, l_d, d2 = Dr.shape
        off = None
    else:
        off = np.ascontiguousarray(offsets, dtype=np.int32)
        b, l_d = off.shape[0] - 1, 0
        d2 = Dr.shape[-1]
        if off[0] != 0 or off[-1] != Dr.shape[0] or np.any(np.diff(off) < 0):
            raise ValueError("bad offsets")
    if d2 != d:
        raise ValueError("d mismatch")
    scores = np.empty((n_q, b), np.float64)
    am = np.empty((n_q, b, l_q), np.int32) if want_argmax else None
    mg = np.empty((n_q, b, l_q), np.float64) if want_margin else None
    rc = lib().oracle_forward(_ptr(Qr), n_q, l_q, _ptr(Dr), b, l_d, _ptr(off), d, _DTYPE_NAMES[dtype],
                              _ptr(scores), _ptr(am), _ptr(mg), threads or default_threads())
    if rc != 0:
        raise RuntimeError("oracle_forward failed (%d)" % rc)
    return scores, am, mg


def backward(Q, D, dtype: str, argmax, g):
    """Eqs. 2-3.  Returns (dQ float64 [n_q,l_q,d], dD float64 [b,l_d,d])."""
    Qr, Dr = as_raw(Q, dtype), as_raw(D, dtype)
    n_q, l_q, d = Qr.shape
    b, l_d, _ = Dr.shape
    A = np.ascontiguousarray(argmax, dtype=np.int32)
    G = np.ascontiguousarray(g, dtype=np.float64)
    assert A.shape == (n_q, b, l_q) and G.shape == (n_q, b)
    dQ = np.empty((n_q, l_q, d), np.float64)
    dD = np.empty((b, l_d, d), np.float64)
    rc = lib().oracle_backward(_ptr(Qr), n_q, l_q, _ptr(Dr), b, l_d, d, _DTYPE_NAMES[dtype],
                               _ptr(A), _ptr(G), _ptr(dQ), _ptr(dD))
    if rc != 0:
        raise RuntimeError("oracle_backward failed (%d)" % rc)
    return dQ, dD


def forward_i8(Q_i8, q_scale, D_i8, d_scale, threads=None):
    """Alg. 4 (int8 x int8, deferred dequantisation).  Returns float32 scores [n_q,b]."""
    Qi = np.ascontiguousarray(Q_i8, dtype=np.int8)
    Di = np.ascontiguousarray(D_i8, dtype=np.int8)
    qs = np.ascontiguousarray(q_scale, dtype=np.float32)
    ds = np.ascontiguousarray(d_scale, dtype=np.float32)
    n_q, l_q, d = Qi.shape
    b, l_d, _ = Di.shape
    assert qs.shape == (n_q, l_q) and ds.shape == (b, l_d)
    scores = np.empty((n_q, b), np.float32)
    rc = lib().oracle_forward_i8(_ptr(Qi), _ptr(qs), n_q, l_q, _ptr(Di), _ptr(ds), b, l_d, d,
                                 _ptr(scores), threads or default_threads())
    if rc != 0:
        raise RuntimeError("oracle_forward_i8 failed (%d)" % rc)
    return scores


def _check_offsets(offsets, total):
    off = np.ascontiguousarray(offsets, dtype=np.int64)
    if off[0] != 0 or off[-1] != total or np.any(np.diff(off) < 0):
        raise ValueError("bad offsets")
    return off


def forward_i8_ragged(Q_i8, q_scale, D_i8_packed, d_scale_packed, offsets, threads=None):
    """Alg. 4 over a packed corpus (Sec. "Ragged corpora and kernel family"): document j is rows
    offsets[j]:offsets[j+1] and is scored by the uniform routine on its own; an empty document scores -inf."""
    Dp = np.ascontiguousarray(D_i8_packed, dtype=np.int8)
    sp = np.ascontiguousarray(d_scale_packed, dtype=np.float32)
    off = _check_offsets(offsets, Dp.shape[0])
    n_q, b = np.asarray(Q_i8).shape[0], off.shape[0] - 1
    scores = np.full((n_q, b), -np.inf, np.float32)
    for j in range(b):
        s, e = int(off[j]), int(off[j + 1])
        if e > s:
            scores[:, j] = forward_i8(Q_i8, q_scale, Dp[None, s:e], sp[None, s:e], threads=threads or 1)[:, 0]
    return scores


def backward_ragged(Q, D_packed, dtype: str, offsets, argmax, g):
    """Eqs. 2-3 over a packed corpus: dQ sums the per-document contributions, dD [T,d] is packed like D.
    argmax [n_q,b,l_q] is document-local; negative entries (empty documents) are skipped."""
    Qr, Dr = as_raw(Q, dtype), as_raw(D_packed, dtype)
    n_q, l_q, d = Qr.shape
    off = _check_offsets(offsets, Dr.shape[0])
    b = off.shape[0] - 1
    A = np.ascontiguousarray(argmax, dtype=np.int32)
    G = np.ascontiguousarray(g, dtype=np.float64)
    assert A.shape == (n_q, b, l_q) and G.shape == (n_q, b)
    dQ = np.zeros((n_q, l_q, d), np.float64)
    dD = np.zeros((Dr.shape[0], d), np.float64)
    for j in range(b):
        s, e = int(off[j]), int(off[j + 1])
        if e > s:
            q1, d1 = backward(Qr, Dr[None, s:e], dtype, A[:, j:j + 1], G[:, j:j + 1])
            dQ += q1
            dD[s:e] = d1[0]
    return dQ, dD


def csr_build(argmax, l_d: int):
    """Inverse-grid CSR of the deterministic backward (Sec. "Closed-Form Gradients", Alg. 2): the edge with flat
    index e = (i * b + j) * l_q + s and winning token t = argmax[i, j, s] has destination row dst = j * l_d + t;
    row_ptr = [0, cumsum(bincount(dst))], col_idx = the edges in a STABLE sort by destination (so the edges of a
    row appear in increasing e, i.e. increasing (i, s)).  Entries outside [0, l_d) are not edges.
    Returns (row_ptr int32 [b * l_d + 1], col_idx int32 [number of edges])."""
    A = np.ascontiguousarray(argmax, dtype=np.int64)
    n_q, b, l_q = A.shape
    dst = np.arange(b, dtype=np.int64)[None, :, None] * l_d + A
    valid = (A >= 0) & (A < l_d)
    e = np.flatnonzero(valid.ravel())
    d = dst.ravel()[e]
    order = np.argsort(d, kind="stable")
    col_idx = e[order].astype(np.int32)
    row_ptr = np.concatenate([[0], np.cumsum(np.bincount(d, minlength=b * l_d))]).astype(np.int32)
    return row_ptr, col_idx


def backward_dd_from_csr(Q, dtype: str, b: int, l_d: int, row_ptr, col_idx, g):
    """Eq. 3 evaluated row by row from the CSR (Alg. 2, the row-owned loop): dD[r] = sum over the row's edges, in
    list order, of g[i, j] * Q[i, s].  float64 [b, l_d, d].  (Plain Python loops: small cases only.)"""
    Qr = as_raw(Q, dtype)
    n_q, l_q, d = Qr.shape
    Qd = decode_array(Qr, dtype)
    G = np.asarray(g, dtype=np.float64)
    dD = np.zeros((b * l_d, d), np.float64)
    for r in range(b * l_d):
        acc = np.zeros(d, np.float64)
        for e in col_idx[row_ptr[r]:row_ptr[r + 1]]:
            i, rest = divmod(int(e), b * l_q)
            j, s_ = divmod(rest, l_q)
            acc += G[i, j] * Qd[i, s_]
        dD[r] = acc
    return dD.reshape(b, l_d, d)


def dot_i8(Q_i8, D_i8):
    Qi = np.ascontiguousarray(Q_i8, dtype=np.int8)
    Di = np.ascontiguousarray(D_i8, dtype=np.int8)
    l_q, d = Qi.shape
    l_d, _ = Di.shape
    n = np.empty((l_q, l_d), np.int64)
    rc = lib().oracle_dot_i8(_ptr(Qi), l_q, _ptr(Di), l_d, d, _ptr(n))
    if rc != 0:
        raise RuntimeError("oracle_dot_i8 failed")
    return n


def quantize_rows_i8(X, dtype: str):
    """Per-row symmetric absmax quantiser.  X [..., d] -> (int8 [..., d], float32 scale [...])."""
    Xr = as_raw(X, dtype)
    d = Xr.shape[-1]
    rows = int(np.prod(Xr.shape[:-1]))
    codes = np.empty(Xr.shape, np.int8)
    scale = np.empty(Xr.shape[:-1], np.float32)
    rc = lib().oracle_quantize_rows_i8(_ptr(Xr), rows, d, _DTYPE_NAMES[dtype], _ptr(codes), _ptr(scale))
    if rc != 0:
        raise RuntimeError("oracle_quantize_rows_i8 failed")
    return codes, scale


def ce_grad(scores, tau: float):
    """In-batch-negatives cross-entropy (diagonal labels).  Returns (loss, g float64 [n,b])."""
    S = np.ascontiguousarray(scores, dtype=np.float64)
    n, b = S.shape
    g = np.empty((n, b), np.float64)
    loss = ctypes.c_double(0.0)
    rc = lib().oracle_ce_grad(_ptr(S), n, b, float(tau), ctypes.byref(loss), _ptr(g))
    if rc != 0:
        raise RuntimeError("oracle_ce_grad failed")
    return loss.value, g


def decode_f16(bits: int) -> float:
    return lib().oracle_decode_f16(int(bits))


def decode_bf16(bits: int) -> float:
    return lib().oracle_decode_bf16(int(bits))
