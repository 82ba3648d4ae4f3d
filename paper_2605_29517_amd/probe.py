"""ctypes binding of libmaxsim_probe.so (include/maxsim_probe.h): the benchmark's diagnostics, not the operator."""
import ctypes
import os

import torch

from .binding import MaxSimError, _check, _dev, _on_device, _stream

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmaxsim_probe.so")
SYMBOLS = ("maxsim_probe_mfma", "maxsim_probe_read", "maxsim_probe_read_streaming", "maxsim_probe_copy", "maxsim_probe_gather")
PROBE_MFMA_OPS_PER_ITER = {0: 512 * 4 * 4 * 2 * 32 * 32 * 16, 1: 512 * 4 * 4 * 2 * 32 * 32 * 16, 2: 512 * 4 * 4 * 2 * 32 * 32 * 32}

_lib = None


def load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MaxSimError("%s is missing: build it with `python -m paper_2605_29517_amd.build`" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    i, l, p = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p
    L.maxsim_probe_mfma.restype = i
    L.maxsim_probe_mfma.argtypes = [i, p, i, p, p]
    L.maxsim_probe_read.restype = i
    L.maxsim_probe_read.argtypes = [p, l, p, p]
    L.maxsim_probe_read_streaming.restype = i
    L.maxsim_probe_read_streaming.argtypes = [p, l, p, p]
    L.maxsim_probe_copy.restype = i
    L.maxsim_probe_copy.argtypes = [p, p, l, p]
    L.maxsim_probe_gather.restype = l
    L.maxsim_probe_gather.argtypes = [i, p, l, i, p, p]
    _lib = L
    return L


def maxsim_probe_mfma(kind, operands, iters, sink):
    """Register-only MFMA loop.  Returns the number of operations one launch performs."""
    L = load()
    if operands.numel() * operands.element_size() < (1 << 20):
        raise MaxSimError("operands must hold at least 1 MiB")
    with _on_device(operands, "operands"):
        rc = L.maxsim_probe_mfma(int(kind), _dev(operands, "operands"), int(iters), _dev(sink, "sink", torch.float32),
                                 _stream(operands))
    _check(rc, "maxsim_probe_mfma")
    return PROBE_MFMA_OPS_PER_ITER[int(kind)] * int(iters)


def maxsim_probe_read(buf, sink, streaming=False):
    """Streaming read of a whole tensor (streaming=True: with non-temporal loads).  Returns the bytes read."""
    L = load()
    nbytes = buf.numel() * buf.element_size() // 16 * 16
    fn = L.maxsim_probe_read_streaming if streaming else L.maxsim_probe_read
    with _on_device(buf, "buf"):
        rc = fn(_dev(buf, "buf"), nbytes, _dev(sink, "sink", torch.float32), _stream(buf))
    _check(rc, "maxsim_probe_read")
    return nbytes


def maxsim_probe_copy(src, dst):
    """Plain copy of a whole tensor.  Returns the bytes copied."""
    L = load()
    nbytes = min(src.numel() * src.element_size(), dst.numel() * dst.element_size()) // 16 * 16
    with _on_device(src, "src"):
        rc = L.maxsim_probe_copy(_dev(src, "src"), _dev(dst, "dst"), nbytes, _stream(src))
    _check(rc, "maxsim_probe_copy")
    return nbytes


def maxsim_probe_gather(kind, table, iters, sink):
    """Random gathers of 256-byte rows from `table` (the largest power-of-two number of rows it holds is used).
    Returns the bytes gathered by the launch."""
    L = load()
    rows = table.numel() * table.element_size() // 256
    if rows < 1:
        raise MaxSimError("table must hold at least one row of 256 bytes")
    rows = 1 << (rows.bit_length() - 1)
    with _on_device(table, "table"):
        n = L.maxsim_probe_gather(int(kind), _dev(table, "table"), rows, int(iters), _dev(sink, "sink", torch.float32),
                                  _stream(table))
    if n < 0:
        _check(int(n), "maxsim_probe_gather")
    return int(n) * 256
