"""maxsim_backward_csr_static (the CSR backward that allocates nothing: row_ptr / col_idx live in a device array
of the library's image) against maxsim_backward_csr through the C ABI.

Both run the same kernels in the same order, so dQ and dD must be equal bit for bit.  Two calls in a row, the
second with a smaller input: the array keeps the first call's contents and nothing is cleared between calls.
Sizes beyond the array return MAXSIM_ERR_SCRATCH before anything is enqueued.
"""
import ctypes

import numpy as np
import pytest
import torch

from paper_2605_29517_amd import binding as M
from paper_2605_29517_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def one_case(n_q, l_q, b, l_d, dtype, seed):
    Q = W.unit_rows((n_q, l_q, 128), dtype, seed, DEV)
    D = W.unit_rows((b, l_d, 128), dtype, seed + 1, DEV)
    rng = np.random.default_rng(seed)
    A = rng.integers(0, l_d, (n_q, b, l_q)).astype(np.int32)
    A[rng.random(A.shape) < 0.05] = -1
    g = rng.standard_normal((n_q, b)).astype(np.float32)
    At, gt = torch.from_numpy(A).to(DEV), torch.from_numpy(g).to(DEV)
    eQ, eD, _, _ = M.maxsim_backward_csr(Q, D, At, gt)
    dQ = torch.full((n_q, l_q, 128), float("nan"), dtype=torch.float32, device=DEV)
    dD = torch.full((b, l_d, 128), float("nan"), dtype=torch.float32, device=DEV)
    M.maxsim_backward_csr_static(Q, D, At, gt, dQ, dD)
    torch.cuda.synchronize()
    assert torch.equal(dQ.view(torch.int32), eQ.view(torch.int32)), "dQ differs"
    assert torch.equal(dD.view(torch.int32), eD.view(torch.int32)), "dD differs"


def test_static_csr_backward_matches_caller_buffer_variant_twice():
    print("case 1: 24 x 32 queries, 40 x 300 documents, f16", flush=True)
    one_case(24, 32, 40, 300, "f16", 11)
    print("case 2 (smaller, same array): 5 x 33 queries, 7 x 129 documents, bf16", flush=True)
    one_case(5, 33, 7, 129, "bf16", 12)
    print("case 3: 3 x 7 queries, 2 x 31 documents, f32", flush=True)
    one_case(3, 7, 2, 31, "f32", 13)


def test_static_csr_backward_at_its_maximum_size():
    print("case: 256 x 32 queries, 256 x 1024 documents (the array's limits exactly), f16", flush=True)
    one_case(256, 32, 256, 1024, "f16", 14)
    print("then a small one again", flush=True)
    one_case(2, 32, 3, 40, "f16", 15)


def test_sizes_beyond_the_array_are_refused_before_anything_runs():
    L = M.load()
    buf = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    p = ctypes.c_void_p(buf.data_ptr())
    # 257 x 1024 rows > 262144
    assert L.maxsim_backward_csr_static(p, 1, 1, p, 257, 1024, 128, 1, p, p, p, p, None) == -4
    # 2^21 + 32 argmax entries
    assert L.maxsim_backward_csr_static(p, 65537, 32, p, 1, 8, 128, 1, p, p, p, p, None) == -4
    assert b"scratch" in L.maxsim_strerror(-4)
    torch.cuda.synchronize()
