"""Thin ctypes binding of libmaxsim.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/maxsim.h) and takes
torch tensors that live on the GPU; torch is used for device memory and the current
stream, nothing else.  There is no CPU fallback: if the library is missing or a tensor
is not on the device, the call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmaxsim.so")

MAXSIM_F32, MAXSIM_F16, MAXSIM_BF16 = 0, 1, 2
_DTYPE = {torch.float32: MAXSIM_F32, torch.float16: MAXSIM_F16, torch.bfloat16: MAXSIM_BF16}

SYMBOLS = ("maxsim_strerror", "maxsim_init", "maxsim_forward", "maxsim_forward_ragged", "maxsim_forward_streamed", "maxsim_backward", "maxsim_backward_ragged",
           "maxsim_csr_build", "maxsim_backward_csr", "maxsim_backward_csr_static",
           "maxsim_quantize_rows_i8", "maxsim_forward_i8", "maxsim_forward_i8_ragged", "maxsim_forward_i8_streamed", "maxsim_ce_grad")

_lib = None


class MaxSimError(RuntimeError):
    pass


def load():
    """Load libmaxsim.so (once).  torch is imported first so that the HIP runtime the
    library binds to is the one torch already loaded."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MaxSimError("%s is missing: build it with `python -m paper_2605_29517_amd.build` "
                          "(there is no fallback path)" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    i, l, p, f = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p, ctypes.c_float
    L.maxsim_strerror.restype = ctypes.c_char_p
    L.maxsim_strerror.argtypes = [i]
    L.maxsim_forward.restype = i
    L.maxsim_forward.argtypes = [p, i, i, p, l, i, i, i, p, p, p]
    L.maxsim_forward_ragged.restype = i
    L.maxsim_forward_ragged.argtypes = [p, i, i, p, p, l, l, i, i, p, p, p]
    L.maxsim_forward_streamed.restype = i
    L.maxsim_forward_streamed.argtypes = [p, i, i, p, l, i, i, i, l, p, p, p]
    L.maxsim_backward.restype = i
    L.maxsim_backward.argtypes = [p, i, i, p, l, i, i, i, p, p, p, p, p]
    L.maxsim_backward_ragged.restype = i
    L.maxsim_backward_ragged.argtypes = [p, i, i, p, p, l, l, i, i, p, p, p, p, p]
    L.maxsim_csr_build.restype = i
    L.maxsim_csr_build.argtypes = [p, i, l, i, i, p, p, p]
    L.maxsim_backward_csr.restype = i
    L.maxsim_backward_csr.argtypes = [p, i, i, p, l, i, i, i, p, p, p, p, p, p, p]
    L.maxsim_backward_csr_static.restype = i
    L.maxsim_backward_csr_static.argtypes = [p, i, i, p, l, i, i, i, p, p, p, p, p]
    L.maxsim_quantize_rows_i8.restype = i
    L.maxsim_quantize_rows_i8.argtypes = [p, l, i, i, p, p, p]
    L.maxsim_forward_i8.restype = i
    L.maxsim_forward_i8.argtypes = [p, p, i, i, p, p, l, i, i, p, p]
    L.maxsim_forward_i8_ragged.restype = i
    L.maxsim_forward_i8_ragged.argtypes = [p, p, i, i, p, p, p, l, l, i, p, p]
    L.maxsim_forward_i8_streamed.restype = i
    L.maxsim_forward_i8_streamed.argtypes = [p, p, i, i, p, p, l, i, i, l, p, p, p, p]
    L.maxsim_ce_grad.restype = i
    L.maxsim_ce_grad.argtypes = [p, i, i, f, p, p, p]
    L.maxsim_init.restype = i
    L.maxsim_init.argtypes = []
    _lib = L
    return L


def _check(rc: int, what: str):
    if rc != 0:
        raise MaxSimError("%s failed: %s (%d)" % (what, load().maxsim_strerror(rc).decode(), rc))


def _dev(t: torch.Tensor, name: str, dtype=None):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise MaxSimError("%s must be a tensor on the GPU" % name)
    if not t.is_contiguous():
        raise MaxSimError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise MaxSimError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


def _same(t: torch.Tensor, name: str, shape, dtype=None):
    """Shape (and dtype) of a tensor the C side will index with the sizes of the others."""
    if tuple(t.shape) != tuple(shape):
        raise MaxSimError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    if dtype is not None and t.dtype != dtype:
        raise MaxSimError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))


def _same_device(ref: torch.Tensor, **tensors):
    for name, t in tensors.items():
        if t is not None and t.device != ref.device:
            raise MaxSimError("%s must be on %s like the other tensors, got %s" % (name, ref.device, t.device))


def maxsim_init(device=None):
    """Per-device set-up (LDS limits, static scratch): needed before entry points are captured into a HIP graph."""
    L = load()
    with torch.cuda.device(device if device is not None else torch.cuda.current_device()):
        _check(L.maxsim_init(), "maxsim_init")


def _stream(t: torch.Tensor):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


class _on_device:
    """Makes the tensor's GPU current for the call; rejects host tensors before anything else."""

    def __init__(self, t, name):
        _dev(t, name)
        self._ctx = torch.cuda.device(t.device)

    def __enter__(self):
        return self._ctx.__enter__()

    def __exit__(self, *a):
        return self._ctx.__exit__(*a)


def maxsim_forward(Q, D, scores=None, argmax=None, want_argmax=False):
    """Q [n_q,l_q,d], D [b,l_d,d] (same 16/32-bit float dtype) -> scores [n_q,b] fp32 (, argmax int32)."""
    L = load()
    n_q, l_q, d = Q.shape
    b, l_d, d2 = D.shape
    if d2 != d or Q.dtype != D.dtype or Q.dtype not in _DTYPE:
        raise MaxSimError("Q and D must share d and a dtype in {fp32, fp16, bf16}")
    if scores is None:
        scores = torch.empty(n_q, b, dtype=torch.float32, device=Q.device)
    if argmax is None and want_argmax:
        argmax = torch.empty(n_q, b, l_q, dtype=torch.int32, device=Q.device)
    _same(scores, "scores", (n_q, b), torch.float32)
    if argmax is not None:
        _same(argmax, "argmax", (n_q, b, l_q), torch.int32)
    _same_device(Q, D=D, scores=scores, argmax=argmax)
    with _on_device(Q, "Q"):
        rc = L.maxsim_forward(_dev(Q, "Q"), n_q, l_q, _dev(D, "D"), b, l_d, d, _DTYPE[Q.dtype],
                              _dev(scores, "scores", torch.float32),
                              _dev(argmax, "argmax", torch.int32) if argmax is not None else None, _stream(Q))
    _check(rc, "maxsim_forward")
    return (scores, argmax) if argmax is not None else scores


def maxsim_forward_ragged(Q, D_packed, doc_offsets, total_tokens=None, scores=None, argmax=None, want_argmax=False):
    """Q [n_q,l_q,d], D_packed [T,d], doc_offsets int32 [b+1] on the device."""
    L = load()
    n_q, l_q, d = Q.shape
    T, d2 = D_packed.shape
    b = doc_offsets.shape[0] - 1
    if d2 != d or Q.dtype != D_packed.dtype or Q.dtype not in _DTYPE:
        raise MaxSimError("Q and D must share d and a dtype in {fp32, fp16, bf16}")
    if total_tokens is None:
        total_tokens = T
    if scores is None:
        scores = torch.empty(n_q, b, dtype=torch.float32, device=Q.device)
    if argmax is None and want_argmax:
        argmax = torch.empty(n_q, b, l_q, dtype=torch.int32, device=Q.device)
    if b < 1 or int(total_tokens) > T:
        raise MaxSimError("doc_offsets must hold b + 1 >= 2 entries and total_tokens may not exceed the rows of D_packed")
    _same(scores, "scores", (n_q, b), torch.float32)
    if argmax is not None:
        _same(argmax, "argmax", (n_q, b, l_q), torch.int32)
    _same_device(Q, D_packed=D_packed, doc_offsets=doc_offsets, scores=scores, argmax=argmax)
    with _on_device(Q, "Q"):
        rc = L.maxsim_forward_ragged(_dev(Q, "Q"), n_q, l_q, _dev(D_packed, "D_packed"),
                                     _dev(doc_offsets, "doc_offsets", torch.int32), b, int(total_tokens), d,
                                     _DTYPE[Q.dtype], _dev(scores, "scores", torch.float32),
                                     _dev(argmax, "argmax", torch.int32) if argmax is not None else None, _stream(Q))
    _check(rc, "maxsim_forward_ragged")
    return (scores, argmax) if argmax is not None else scores


def maxsim_forward_streamed(Q, D_host, block_docs, staging=None, scores=None):
    """Out-of-core forward: Q on the GPU, D_host [b,l_d,d] a HOST tensor (pinned for asynchronous copies),
    staging a device buffer of 2 * block_docs documents (allocated here if not given)."""
    L = load()
    n_q, l_q, d = Q.shape
    b, l_d, d2 = D_host.shape
    if D_host.is_cuda or not D_host.is_contiguous():
        raise MaxSimError("D_host must be a contiguous host tensor")
    if d2 != d or Q.dtype != D_host.dtype or Q.dtype not in _DTYPE:
        raise MaxSimError("Q and D must share d and a dtype in {fp32, fp16, bf16}")
    block_docs = int(min(block_docs, b))
    if staging is None:
        staging = torch.empty(2 * block_docs, l_d, d, dtype=Q.dtype, device=Q.device)
    if staging.numel() < 2 * block_docs * l_d * d or staging.dtype != Q.dtype:
        raise MaxSimError("staging must hold 2 * block_docs documents of the corpus dtype")
    if scores is None:
        scores = torch.empty(n_q, b, dtype=torch.float32, device=Q.device)
    _same(scores, "scores", (n_q, b), torch.float32)
    _same_device(Q, staging=staging, scores=scores)
    with _on_device(Q, "Q"):
        rc = L.maxsim_forward_streamed(_dev(Q, "Q"), n_q, l_q, ctypes.c_void_p(D_host.data_ptr()), b, l_d, d,
                                       _DTYPE[Q.dtype], block_docs, _dev(staging, "staging"),
                                       _dev(scores, "scores", torch.float32), _stream(Q))
    _check(rc, "maxsim_forward_streamed")
    return scores


def maxsim_backward(Q, D, argmax, dscore, dQ=None, dD=None):
    """Eqs. 2-3: returns (dQ fp32 [n_q,l_q,d], dD fp32 [b,l_d,d])."""
    L = load()
    n_q, l_q, d = Q.shape
    b, l_d, _ = D.shape
    if D.shape[2] != d or D.dtype != Q.dtype or Q.dtype not in _DTYPE:
        raise MaxSimError("Q and D must share d and a dtype in {fp32, fp16, bf16}")
    if tuple(argmax.shape) != (n_q, b, l_q) or tuple(dscore.shape) != (n_q, b):
        raise MaxSimError("argmax must be [n_q,b,l_q] and dscore [n_q,b]")
    if dQ is None:
        dQ = torch.empty(n_q, l_q, d, dtype=torch.float32, device=Q.device)
    if dD is None:
        dD = torch.empty(b, l_d, d, dtype=torch.float32, device=Q.device)
    _same(dQ, "dQ", (n_q, l_q, d), torch.float32)
    _same(dD, "dD", (b, l_d, d), torch.float32)
    _same_device(Q, D=D, argmax=argmax, dscore=dscore, dQ=dQ, dD=dD)
    with _on_device(Q, "Q"):
        rc = L.maxsim_backward(_dev(Q, "Q"), n_q, l_q, _dev(D, "D"), b, l_d, d, _DTYPE[Q.dtype],
                               _dev(argmax, "argmax", torch.int32), _dev(dscore, "dscore", torch.float32),
                               _dev(dQ, "dQ", torch.float32), _dev(dD, "dD", torch.float32), _stream(Q))
    _check(rc, "maxsim_backward")
    return dQ, dD


def maxsim_backward_ragged(Q, D_packed, doc_offsets, argmax, dscore, total_tokens=None, dQ=None, dD=None):
    """Eqs. 2-3 over a packed corpus: returns (dQ fp32 [n_q,l_q,d], dD fp32 [T,d] packed like D_packed)."""
    L = load()
    n_q, l_q, d = Q.shape
    T = D_packed.shape[0]
    b = doc_offsets.shape[0] - 1
    if tuple(argmax.shape) != (n_q, b, l_q) or tuple(dscore.shape) != (n_q, b):
        raise MaxSimError("argmax must be [n_q,b,l_q] and dscore [n_q,b]")
    if total_tokens is None:
        total_tokens = T
    if D_packed.dim() != 2 or D_packed.shape[1] != d or D_packed.dtype != Q.dtype or Q.dtype not in _DTYPE:
        raise MaxSimError("Q and D_packed must share d and a dtype in {fp32, fp16, bf16}")
    if b < 1 or int(total_tokens) > T:
        raise MaxSimError("doc_offsets must hold b + 1 >= 2 entries and total_tokens may not exceed the rows of D_packed")
    if dQ is None:
        dQ = torch.empty(n_q, l_q, d, dtype=torch.float32, device=Q.device)
    if dD is None:
        dD = torch.empty(T, d, dtype=torch.float32, device=Q.device)
    _same(dQ, "dQ", (n_q, l_q, d), torch.float32)
    _same(dD, "dD", (T, d), torch.float32)
    _same_device(Q, D_packed=D_packed, doc_offsets=doc_offsets, argmax=argmax, dscore=dscore, dQ=dQ, dD=dD)
    with _on_device(Q, "Q"):
        rc = L.maxsim_backward_ragged(_dev(Q, "Q"), n_q, l_q, _dev(D_packed, "D_packed"),
                                      _dev(doc_offsets, "doc_offsets", torch.int32), b, int(total_tokens), d,
                                      _DTYPE[Q.dtype], _dev(argmax, "argmax", torch.int32),
                                      _dev(dscore, "dscore", torch.float32), _dev(dQ, "dQ", torch.float32),
                                      _dev(dD, "dD", torch.float32), _stream(Q))
    _check(rc, "maxsim_backward_ragged")
    return dQ, dD


def maxsim_csr_build(argmax, l_d, row_ptr=None, col_idx=None):
    """Alg. 2's inverse-grid CSR of argmax [n_q,b,l_q]: returns (row_ptr int32 [b*l_d+1], col_idx int32 [n_q*b*l_q],
    of which the first row_ptr[-1] entries are the edges)."""
    L = load()
    n_q, b, l_q = argmax.shape
    if row_ptr is None:
        row_ptr = torch.empty(b * l_d + 1, dtype=torch.int32, device=argmax.device)
    if col_idx is None:
        col_idx = torch.empty(n_q * b * l_q, dtype=torch.int32, device=argmax.device)
    if row_ptr.numel() < b * l_d + 1 or col_idx.numel() < n_q * b * l_q:
        raise MaxSimError("row_ptr must hold b*l_d+1 and col_idx n_q*b*l_q entries")
    with _on_device(argmax, "argmax"):
        rc = L.maxsim_csr_build(_dev(argmax, "argmax", torch.int32), n_q, b, l_q, int(l_d),
                                _dev(row_ptr, "row_ptr", torch.int32), _dev(col_idx, "col_idx", torch.int32),
                                _stream(argmax))
    _check(rc, "maxsim_csr_build")
    return row_ptr, col_idx


def maxsim_backward_csr(Q, D, argmax, dscore, row_ptr=None, col_idx=None, dQ=None, dD=None):
    """Eqs. 2-3 with dD through the explicit CSR (Alg. 2): returns (dQ, dD, row_ptr, col_idx)."""
    L = load()
    n_q, l_q, d = Q.shape
    b, l_d, _ = D.shape
    if tuple(argmax.shape) != (n_q, b, l_q) or tuple(dscore.shape) != (n_q, b):
        raise MaxSimError("argmax must be [n_q,b,l_q] and dscore [n_q,b]")
    if row_ptr is None:
        row_ptr = torch.empty(b * l_d + 1, dtype=torch.int32, device=Q.device)
    if col_idx is None:
        col_idx = torch.empty(n_q * b * l_q, dtype=torch.int32, device=Q.device)
    if row_ptr.numel() < b * l_d + 1 or col_idx.numel() < n_q * b * l_q:
        raise MaxSimError("row_ptr must hold b*l_d+1 and col_idx n_q*b*l_q entries")
    if dQ is None:
        dQ = torch.empty(n_q, l_q, d, dtype=torch.float32, device=Q.device)
    if dD is None:
        dD = torch.empty(b, l_d, d, dtype=torch.float32, device=Q.device)
    if D.shape[2] != d or D.dtype != Q.dtype or Q.dtype not in _DTYPE:
        raise MaxSimError("Q and D must share d and a dtype in {fp32, fp16, bf16}")
    _same(dQ, "dQ", (n_q, l_q, d), torch.float32)
    _same(dD, "dD", (b, l_d, d), torch.float32)
    _same_device(Q, D=D, argmax=argmax, dscore=dscore, row_ptr=row_ptr, col_idx=col_idx, dQ=dQ, dD=dD)
    with _on_device(Q, "Q"):
        rc = L.maxsim_backward_csr(_dev(Q, "Q"), n_q, l_q, _dev(D, "D"), b, l_d, d, _DTYPE[Q.dtype],
                                   _dev(argmax, "argmax", torch.int32), _dev(dscore, "dscore", torch.float32),
                                   _dev(row_ptr, "row_ptr", torch.int32), _dev(col_idx, "col_idx", torch.int32),
                                   _dev(dQ, "dQ", torch.float32), _dev(dD, "dD", torch.float32), _stream(Q))
    _check(rc, "maxsim_backward_csr")
    return dQ, dD, row_ptr, col_idx


def maxsim_backward_csr_static(Q, D, argmax, dscore, dQ, dD):
    """maxsim_backward_csr with the CSR in the library's static device array; dQ and dD are the caller's
    (this wrapper allocates nothing either)."""
    L = load()
    n_q, l_q, d = Q.shape
    b, l_d, _ = D.shape
    if tuple(argmax.shape) != (n_q, b, l_q) or tuple(dscore.shape) != (n_q, b):
        raise MaxSimError("argmax must be [n_q,b,l_q] and dscore [n_q,b]")
    if D.shape[2] != d or D.dtype != Q.dtype or Q.dtype not in _DTYPE:
        raise MaxSimError("Q and D must share d and a dtype in {fp32, fp16, bf16}")
    _same(dQ, "dQ", (n_q, l_q, d), torch.float32)
    _same(dD, "dD", (b, l_d, d), torch.float32)
    _same_device(Q, D=D, argmax=argmax, dscore=dscore, dQ=dQ, dD=dD)
    with _on_device(Q, "Q"):
        rc = L.maxsim_backward_csr_static(_dev(Q, "Q"), n_q, l_q, _dev(D, "D"), b, l_d, d, _DTYPE[Q.dtype],
                                          _dev(argmax, "argmax", torch.int32), _dev(dscore, "dscore", torch.float32),
                                          _dev(dQ, "dQ", torch.float32), _dev(dD, "dD", torch.float32), _stream(Q))
    _check(rc, "maxsim_backward_csr_static")
    return dQ, dD


def maxsim_quantize_rows_i8(X, X_i8=None, scale=None):
    """X [..., d] -> (int8 codes [..., d], fp32 scale [...])."""
    L = load()
    d = X.shape[-1]
    rows = X.numel() // d
    if X_i8 is None:
        X_i8 = torch.empty(X.shape, dtype=torch.int8, device=X.device)
    if scale is None:
        scale = torch.empty(X.shape[:-1], dtype=torch.float32, device=X.device)
    if X.dtype not in _DTYPE:
        raise MaxSimError("X must have a dtype in {fp32, fp16, bf16}")
    _same(X_i8, "X_i8", X.shape, torch.int8)
    if scale.numel() != rows:
        raise MaxSimError("scale must hold one entry per row of X")
    _same_device(X, X_i8=X_i8, scale=scale)
    with _on_device(X, "X"):
        rc = L.maxsim_quantize_rows_i8(_dev(X, "X"), rows, d, _DTYPE[X.dtype], _dev(X_i8, "X_i8", torch.int8),
                                       _dev(scale, "scale", torch.float32), _stream(X))
    _check(rc, "maxsim_quantize_rows_i8")
    return X_i8, scale


def maxsim_forward_i8(Q_i8, q_scale, D_i8, d_scale, scores=None):
    """int8 scoring: Q_i8 [n_q,l_q,d] + q_scale [n_q,l_q], D_i8 [b,l_d,d] + d_scale [b,l_d] -> scores [n_q,b]."""
    L = load()
    n_q, l_q, d = Q_i8.shape
    b, l_d, d2 = D_i8.shape
    if scores is None:
        scores = torch.empty(n_q, b, dtype=torch.float32, device=Q_i8.device)
    if d2 != d:
        raise MaxSimError("Q_i8 and D_i8 must share d")
    _same(q_scale, "q_scale", (n_q, l_q), torch.float32)
    _same(d_scale, "d_scale", (b, l_d), torch.float32)
    _same(scores, "scores", (n_q, b), torch.float32)
    _same_device(Q_i8, q_scale=q_scale, D_i8=D_i8, d_scale=d_scale, scores=scores)
    with _on_device(Q_i8, "Q_i8"):
        rc = L.maxsim_forward_i8(_dev(Q_i8, "Q_i8", torch.int8), _dev(q_scale, "q_scale", torch.float32), n_q, l_q,
                                 _dev(D_i8, "D_i8", torch.int8), _dev(d_scale, "d_scale", torch.float32), b, l_d, d,
                                 _dev(scores, "scores", torch.float32), _stream(Q_i8))
    _check(rc, "maxsim_forward_i8")
    return scores


def maxsim_forward_i8_ragged(Q_i8, q_scale, D_i8_packed, d_scale_packed, doc_offsets, total_tokens=None, scores=None):
    """int8 scoring of a packed corpus: D_i8_packed [T,d] + d_scale_packed [T], doc_offsets int32 [b+1] -> scores [n_q,b]."""
    L = load()
    n_q, l_q, d = Q_i8.shape
    T = D_i8_packed.shape[0]
    b = doc_offsets.shape[0] - 1
    if total_tokens is None:
        total_tokens = T
    if scores is None:
        scores = torch.empty(n_q, b, dtype=torch.float32, device=Q_i8.device)
    if D_i8_packed.dim() != 2 or D_i8_packed.shape[1] != d or b < 1 or int(total_tokens) > T:
        raise MaxSimError("D_i8_packed must be [T,d] with Q_i8's d, doc_offsets [b+1], total_tokens <= T")
    _same(q_scale, "q_scale", (n_q, l_q), torch.float32)
    _same(d_scale_packed, "d_scale_packed", (T,), torch.float32)
    _same(scores, "scores", (n_q, b), torch.float32)
    _same_device(Q_i8, q_scale=q_scale, D_i8_packed=D_i8_packed, d_scale_packed=d_scale_packed, doc_offsets=doc_offsets, scores=scores)
    with _on_device(Q_i8, "Q_i8"):
        rc = L.maxsim_forward_i8_ragged(_dev(Q_i8, "Q_i8", torch.int8), _dev(q_scale, "q_scale", torch.float32), n_q, l_q,
                                        _dev(D_i8_packed, "D_i8_packed", torch.int8),
                                        _dev(d_scale_packed, "d_scale_packed", torch.float32),
                                        _dev(doc_offsets, "doc_offsets", torch.int32), b, int(total_tokens), d,
                                        _dev(scores, "scores", torch.float32), _stream(Q_i8))
    _check(rc, "maxsim_forward_i8_ragged")
    return scores


def maxsim_forward_i8_streamed(Q_i8, q_scale, D_i8_host, d_scale_host, block_docs, scores=None):
    """Out-of-core int8 scoring: codes [b,l_d,d] and scales [b,l_d] are HOST tensors (pinned for asynchronous copies)."""
    L = load()
    n_q, l_q, d = Q_i8.shape
    b, l_d, _ = D_i8_host.shape
    if D_i8_host.is_cuda or d_scale_host.is_cuda or not D_i8_host.is_contiguous() or not d_scale_host.is_contiguous():
        raise MaxSimError("D_i8_host and d_scale_host must be contiguous host tensors")
    if D_i8_host.dtype != torch.int8 or d_scale_host.dtype != torch.float32 or tuple(d_scale_host.shape) != (b, l_d):
        raise MaxSimError("D_i8_host must be int8 [b,l_d,d] and d_scale_host float32 [b,l_d]")
    block_docs = int(min(block_docs, b))
    st_c = torch.empty(2 * block_docs, l_d, d, dtype=torch.int8, device=Q_i8.device)
    st_s = torch.empty(2 * block_docs, l_d, dtype=torch.float32, device=Q_i8.device)
    if scores is None:
        scores = torch.empty(n_q, b, dtype=torch.float32, device=Q_i8.device)
    with _on_device(Q_i8, "Q_i8"):
        rc = L.maxsim_forward_i8_streamed(_dev(Q_i8, "Q_i8", torch.int8), _dev(q_scale, "q_scale", torch.float32), n_q, l_q,
                                          ctypes.c_void_p(D_i8_host.data_ptr()), ctypes.c_void_p(d_scale_host.data_ptr()),
                                          b, l_d, d, block_docs, _dev(st_c, "staging_codes"), _dev(st_s, "staging_scales"),
                                          _dev(scores, "scores", torch.float32), _stream(Q_i8))
    _check(rc, "maxsim_forward_i8_streamed")
    # the staging buffers allocated here may be recycled by torch only for later work on this same stream,
    # which runs after the last kernel and hence after the last copy
    return scores


def maxsim_ce_grad(scores, tau, g=None, loss=None):
    """In-batch-negatives cross-entropy gradient of a [n,b] score matrix (labels on the diagonal)."""
    L = load()
    n, b = scores.shape
    if g is None:
        g = torch.empty(n, b, dtype=torch.float32, device=scores.device)
    if loss is None:
        loss = torch.empty(1, dtype=torch.float32, device=scores.device)
    _same(g, "g", (n, b), torch.float32)
    _same_device(scores, g=g, loss=loss)
    with _on_device(scores, "scores"):
        rc = L.maxsim_ce_grad(_dev(scores, "scores", torch.float32), n, b, float(tau), _dev(g, "g", torch.float32),
                              _dev(loss, "loss", torch.float32), _stream(scores))
    _check(rc, "maxsim_ce_grad")
    return g, loss
