"""GPU parity of the explicit inverse-grid CSR (Alg. 2) through the C ABI.

maxsim_csr_build is integer work: row_ptr and the written part of col_idx must equal the oracle's bit for bit
(the stable order makes the CSR unique).  maxsim_backward_csr is checked against the fp64 oracle to the same
bar as maxsim_backward (max|delta| <= 1e-4 * max|ref|, cosine >= 0.99999) and, because both add a row's
edges in increasing edge id with the same fp32 fused multiply-add, bit for bit against maxsim_backward.
"""
import numpy as np
import pytest
import torch

from oracle import cpu_oracle as O
from paper_2605_29517_amd import binding as M
from paper_2605_29517_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def skewed_argmax(n_q, b, l_q, l_d, seed, holes=0.0):
    """Winning tokens with the skew of real batches: a few hot tokens per document take most of the edges."""
    rng = np.random.default_rng(seed)
    hot = rng.integers(0, l_d, (1, b, 4))
    pick = rng.integers(0, 4, (n_q, b, l_q))
    A = np.where(rng.random((n_q, b, l_q)) < 0.5, np.take_along_axis(np.broadcast_to(hot, (n_q, b, 4)), pick, axis=2),
                 rng.integers(0, l_d, (n_q, b, l_q)))
    A = A.astype(np.int32)
    if holes:
        A[rng.random(A.shape) < holes] = -1
    return A


def check_build(A, l_d):
    rp, ci = O.csr_build(A, l_d)
    n_q, b, l_q = A.shape
    col0 = torch.full((n_q * b * l_q,), -7, dtype=torch.int32, device=DEV)
    grp, gci = M.maxsim_csr_build(torch.from_numpy(A).to(DEV), l_d, col_idx=col0)
    torch.cuda.synchronize()
    assert np.array_equal(grp.cpu().numpy(), rp)
    gci = gci.cpu().numpy()
    assert np.array_equal(gci[:rp[-1]], ci)
    assert np.all(gci[rp[-1]:] == -7)      # nothing is written beyond the edges


@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 3, 4, 5), (3, 2, 70, 3), (5, 7, 33, 129), (16, 18, 32, 257),
                                   (4, 3, 300, 17), (2, 2, 600, 700), (3, 1, 1, 1100), (8, 5, 32, 4096),
                                   (64, 40, 32, 180), (1, 300, 2, 9)])
def test_csr_build_bit_exact(shape):
    n_q, b, l_q, l_d = shape
    check_build(skewed_argmax(n_q, b, l_q, l_d, sum(shape), holes=0.1), l_d)


def test_csr_build_degenerate_inputs():
    check_build(np.full((3, 4, 5), -1, np.int32), 6)                        # no edges at all
    check_build(np.full((70, 2, 40), 3, np.int32), 8)                       # every edge on one token per document
    A = np.arange(2 * 3 * 200, dtype=np.int32).reshape(2, 3, 200) % 250     # entries >= l_d are not edges
    check_build(A, 130)


def test_csr_build_is_reproducible_and_unsupported_sizes_are_refused():
    A = torch.from_numpy(skewed_argmax(12, 9, 48, 300, 3)).to(DEV)
    r1 = M.maxsim_csr_build(A, 300)
    r2 = M.maxsim_csr_build(A, 300)
    torch.cuda.synchronize()
    assert torch.equal(r1[0], r2[0]) and torch.equal(r1[1], r2[1])
    with pytest.raises(M.MaxSimError, match="unsupported"):
        M.maxsim_csr_build(torch.zeros(1, 1, 4, dtype=torch.int32, device=DEV), 4097)


def close(gpu, ref, what):
    g = gpu.detach().cpu().numpy().astype(np.float64)
    scale = np.abs(ref).max()
    err = np.abs(g - ref).max()
    assert err <= 1e-4 * scale + 1e-30, "%s: max|d| %.3e vs scale %.3e" % (what, err, scale)
    if scale > 0:
        cos = (g * ref).sum() / (np.linalg.norm(g) * np.linalg.norm(ref))
        assert cos >= 0.99999, "%s: cosine %.8f" % (what, cos)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 32, 3, 40), (5, 33, 7, 129), (16, 32, 18, 257), (3, 130, 2, 31),
                                   (24, 32, 24, 180)])
def test_backward_csr_parity(shape, dtype):
    n_q, l_q, b, l_d = shape
    Q = W.unit_rows((n_q, l_q, 128), dtype, 5, DEV)
    D = W.unit_rows((b, l_d, 128), dtype, 6, DEV)
    _, A, _ = O.forward(W.to_raw_numpy(Q), W.to_raw_numpy(D), dtype)
    rng = np.random.default_rng(8)
    A = A.copy()
    A[rng.random(A.shape) < 0.1] = -1
    g = rng.standard_normal((n_q, b)).astype(np.float32)
    rQ, rD = O.backward(W.to_raw_numpy(Q), W.to_raw_numpy(D), dtype, A, g.astype(np.float64))
    rp, ci = O.csr_build(A, l_d)
    At, gt = torch.from_numpy(A).to(DEV), torch.from_numpy(g).to(DEV)
    dQ, dD, grp, gci = M.maxsim_backward_csr(Q, D, At, gt)
    eQ, eD = M.maxsim_backward(Q, D, At, gt)
    torch.cuda.synchronize()
    close(dQ, rQ, "dQ")
    close(dD, rD, "dD")
    assert np.array_equal(grp.cpu().numpy(), rp) and np.array_equal(gci.cpu().numpy()[:rp[-1]], ci)
    assert torch.equal(dQ, eQ) and torch.equal(dD, eD)      # same order, same arithmetic: same bits
