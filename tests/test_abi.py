"""The C-ABI library loads and exports every entry point the header declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header="maxsim.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(maxsim_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    syms = declared_symbols()
    for name in ("maxsim_forward", "maxsim_forward_ragged", "maxsim_backward", "maxsim_quantize_rows_i8",
                 "maxsim_forward_i8", "maxsim_csr_build", "maxsim_backward_csr", "maxsim_strerror"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    from paper_2605_29517_amd import binding
    assert os.path.exists(binding.LIB_PATH), "build the library first: python -m paper_2605_29517_amd.build"
    import torch  # noqa: F401  (the HIP runtime the library binds to comes with torch)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    assert sorted(binding.SYMBOLS) == declared_symbols()
    assert "maxsim_init" in declared_symbols()


def test_probe_library_exports_its_header():
    """The benchmark's diagnostics live in a library of their own, outside the operator's ABI."""
    from paper_2605_29517_amd import probe
    assert os.path.exists(probe.LIB_PATH), "build the libraries first: python -m paper_2605_29517_amd.build"
    import torch  # noqa: F401
    lib = ctypes.CDLL(probe.LIB_PATH)
    for name in declared_symbols("maxsim_probe.h"):
        assert hasattr(lib, name), name
    assert sorted(probe.SYMBOLS) == declared_symbols("maxsim_probe.h")
    assert not [n for n in declared_symbols() if "probe" in n]
    assert lib.maxsim_probe_mfma(3, None, 1, None, None) == -1      # nothing but argument checks without a GPU


def test_error_codes_without_touching_a_gpu():
    from paper_2605_29517_amd import binding
    L = binding.load()
    assert L.maxsim_strerror(0) == b"ok"
    assert b"invalid" in L.maxsim_strerror(-1)
    assert b"128" not in L.maxsim_strerror(-2) and b"width" in L.maxsim_strerror(-2)
    assert b"scratch" in L.maxsim_strerror(-4)
    # null pointers and bad sizes are rejected before any HIP call
    assert L.maxsim_forward(None, 1, 32, None, 4, 40, 128, 1, None, None, None) == -1
    assert L.maxsim_backward(None, 1, 1, None, 1, 1, 128, 1, None, None, None, None, None) == -1
    assert L.maxsim_forward_i8(None, None, 1, 1, None, None, 1, 1, 128, None, None) == -1
    assert L.maxsim_quantize_rows_i8(None, 1, 128, 0, None, None, None) == -1
    buf = (ctypes.c_char * 4096)()
    addr = (ctypes.addressof(buf) + 255) & ~255
    p = ctypes.c_void_p(addr)
    assert L.maxsim_forward(p, 1, 32, p, 4, 40, 100, 1, p, None, None) == -2      # rows must be a multiple of 64 bytes
    assert L.maxsim_forward(p, 1, 32, p, 4, 40, 16, 1, p, None, None) == -2       # d < 32
    assert L.maxsim_forward(p, 1, 32, p, 4, 40, 16384, 1, p, None, None) == -2    # rows above 16 KB
    assert L.maxsim_backward(p, 1, 1, p, 1, 1, 100, 1, p, p, p, p, None) == -2     # backward: d must be a multiple of 8
    assert L.maxsim_backward(p, 1, 1, p, 1, 1, 16384, 1, p, p, p, p, None) == -2   # ... of at most 8192
    assert L.maxsim_forward_i8(p, p, 1, 2000, p, p, 1, 1, 128, p, None) == -2      # int8 queries above 1024 tokens
    assert L.maxsim_forward_i8(p, p, 1, 20, p, p, 1, 1, 100, p, None) == -2        # int8 rows: a multiple of 32 bytes
    assert L.maxsim_forward_i8(p, p, 1, 20, p, p, 1, 1, 8224, p, None) == -2       # ... of at most 8192
    assert L.maxsim_quantize_rows_i8(p, 4, 24, 1, p, p, None) == -2                # the quantiser likewise
    assert L.maxsim_forward_streamed(p, 1, 32, p, 4, 40, 128, 1, 0, p, p, None) == -1  # block_docs < 1
    assert L.maxsim_forward_i8_ragged(p, p, 1, 32, p, p, None, 4, 100, 128, p, None) == -1  # no offsets
    assert L.maxsim_forward_i8_streamed(p, p, 1, 32, p, p, 4, 10, 128, 2, None, p, p, None) == -1  # no staging buffer
    assert L.maxsim_backward_ragged(p, 1, 1, p, p, 1, 0, 128, 1, p, p, p, p, None) == -1     # total_tokens < 1
    assert L.maxsim_csr_build(None, 1, 1, 1, 1, p, p, None) == -1                  # no argmax
    assert L.maxsim_csr_build(p, 2, 3, 4, 4097, p, p, None) == -2                  # documents above 4096 tokens
    assert L.maxsim_csr_build(p, 70000, 40000, 32, 8, p, p, None) == -2            # more than 2^31 edges
    assert L.maxsim_backward_csr(p, 1, 1, p, 1, 1, 128, 1, p, p, None, p, p, p, None) == -1   # no row_ptr
    assert L.maxsim_backward_csr(p, 1, 1, p, 1, 1, 60, 1, p, p, p, p, p, p, None) == -2      # d must be a multiple of 8
    assert L.maxsim_forward(p, 0, 32, p, 4, 40, 128, 1, p, None, None) == -1      # n_q < 1
    assert L.maxsim_forward(p, 1, 32, p, 4, 40, 128, 7, p, None, None) == -1      # bad dtype
    assert L.maxsim_forward(ctypes.c_void_p(addr + 2), 1, 32, p, 4, 40, 128, 1, p, None, None) == -1  # misaligned


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2605_29517_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libmaxsim.so")
    import pytest
    with pytest.raises(binding.MaxSimError):
        binding.load()


def test_bench_refuses_more_than_one_gpu():
    """This build measures one GPU: `bench.py --gpus N` with N above 1 exits with a message and prints no JSON line."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
