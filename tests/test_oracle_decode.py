"""Pins for the oracle's hand-written fp16 / bf16 decoders: all 65536 bit patterns
against numpy's (fp16) and torch's (bf16) own conversions."""
import numpy as np
import torch

from oracle import cpu_oracle as O


def _same(a, b):
    return (a == b) or (np.isnan(a) and np.isnan(b))


def test_decode_f16_exhaustive():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    for h in range(65536):
        assert _same(O.decode_f16(h), ref[h]), h


def test_decode_bf16_exhaustive():
    bits = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    ref = bits.view(torch.bfloat16).to(torch.float64).numpy()
    for h in range(65536):
        assert _same(O.decode_bf16(h), ref[h]), h
    # bf16 is the upper half of binary32
    with np.errstate(invalid="ignore"):
        as_f32 = (np.arange(65536, dtype=np.uint32) << 16).view(np.float32).astype(np.float64)
    for h in (0x3F80, 0xBF80, 0x0001, 0x7F7F, 0x4049):
        assert O.decode_bf16(h) == as_f32[h]
