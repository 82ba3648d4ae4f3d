"""GPU parity of maxsim_forward_streamed (corpus in host memory, streamed through a two-block device buffer)."""
import numpy as np
import pytest
import torch

from oracle import cpu_oracle as O
from paper_2605_29517_amd import binding as M
from paper_2605_29517_amd import workloads as W
from parity import RTOL_16, check_scores

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("case", [(4, 32, 1000, 50, 128, "f16"), (1, 100, 37, 129, 8, "bf16"), (2, 40, 5, 64, 100, "f32"),
                                  (3, 32, 1, 20, 1, "f16"), (9, 32, 300, 33, 150, "f16")])
def test_streamed_equals_resident_and_oracle(case):
    n_q, l_q, b, l_d, block_docs, dtype = case
    Q = W.unit_rows((n_q, l_q, 128), dtype, 41, DEV)
    D = W.unit_rows((b, l_d, 128), dtype, 42, DEV)
    D_host = torch.empty(D.shape, dtype=D.dtype, pin_memory=True)
    D_host.copy_(D)
    resident = M.maxsim_forward(Q, D)
    staging = torch.empty(2 * min(block_docs, b), l_d, 128, dtype=D.dtype, device=DEV)
    s1 = M.maxsim_forward_streamed(Q, D_host, block_docs, staging=staging)
    s2 = M.maxsim_forward_streamed(Q, D_host, block_docs, staging=staging)  # back to back on the same staging buffer
    torch.cuda.synchronize()
    assert torch.equal(s1, resident) and torch.equal(s2, resident)
    ref, _, _ = O.forward(W.to_raw_numpy(Q), W.to_raw_numpy(D), dtype, want_argmax=False, want_margin=False)
    check_scores(s1, ref, l_q, RTOL_16 if dtype != "f32" else 1e-5)


def test_streamed_from_pageable_memory_and_on_a_side_stream():
    Q = W.unit_rows((2, 32, 128), "f16", 43, DEV)
    D = W.unit_rows((200, 70, 128), "f16", 44, DEV)
    D_host = D.cpu()  # pageable: the copies are staged by the runtime, the result is the same
    resident = M.maxsim_forward(Q, D)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        s = M.maxsim_forward_streamed(Q, D_host, 64)
    side.synchronize()
    assert torch.equal(s, resident)


def test_streamed_rejects_device_corpus():
    Q = W.unit_rows((1, 32, 128), "f16", 45, DEV)
    D = W.unit_rows((4, 10, 128), "f16", 46, DEV)
    with pytest.raises(M.MaxSimError):
        M.maxsim_forward_streamed(Q, D, 2)


@pytest.mark.parametrize("case", [(1, 64, 300, 70, 64), (3, 200, 4500, 20, 4200), (2, 32, 9, 33, 100)])
def test_int8_streamed_equals_resident(case):
    """Blocks of >= 4096 documents take the document-stationary kernel, smaller ones the query-stationary one."""
    n_q, l_q, b, l_d, block_docs = case
    Qf = W.unit_rows((n_q, l_q, 128), "f16", 51, DEV)
    Df = W.unit_rows((b, l_d, 128), "f32", 52, DEV)
    q8, qs = M.maxsim_quantize_rows_i8(Qf)
    d8, ds = M.maxsim_quantize_rows_i8(Df)
    resident = M.maxsim_forward_i8(q8, qs, d8, ds)
    d8h = torch.empty(d8.shape, dtype=torch.int8, pin_memory=True)
    dsh = torch.empty(ds.shape, dtype=torch.float32, pin_memory=True)
    d8h.copy_(d8)
    dsh.copy_(ds)
    s = M.maxsim_forward_i8_streamed(q8, qs, d8h, dsh, block_docs)
    torch.cuda.synchronize()
    assert torch.equal(s, resident)
    oq, oqs = O.quantize_rows_i8(W.to_raw_numpy(Qf), "f16")
    od, ods = O.quantize_rows_i8(W.to_raw_numpy(Df[:50].contiguous()), "f32")
    ref = O.forward_i8(oq, oqs, od, ods)
    assert np.array_equal(s[:, :50].cpu().numpy().view(np.uint32), ref[:, :min(50, b)].view(np.uint32))


def test_int8_streamed_other_width_equals_resident():
    n_q, l_q, b, l_d, d, block_docs = 2, 70, 130, 45, 256, 50
    q8, qs = M.maxsim_quantize_rows_i8(W.unit_rows((n_q, l_q, d), "f16", 61, DEV))
    d8, ds = M.maxsim_quantize_rows_i8(W.unit_rows((b, l_d, d), "f32", 62, DEV))
    resident = M.maxsim_forward_i8(q8, qs, d8, ds)
    d8h = torch.empty(d8.shape, dtype=torch.int8, pin_memory=True)
    dsh = torch.empty(ds.shape, dtype=torch.float32, pin_memory=True)
    d8h.copy_(d8)
    dsh.copy_(ds)
    s = M.maxsim_forward_i8_streamed(q8, qs, d8h, dsh, block_docs)
    torch.cuda.synchronize()
    assert torch.equal(s, resident)
