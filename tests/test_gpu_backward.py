"""GPU parity of maxsim_backward and maxsim_ce_grad against the CPU oracle (through the C ABI).

The backward is fed the ORACLE's argmax, so dQ / dD are a deterministic function of the
inputs and near-tie argmax choices cannot leak into gradient parity.  Only the fp32
summation order differs from the fp64 oracle: per tensor max|delta| <= 1e-4 * max|ref|
and cosine >= 0.99999.
"""
import numpy as np
import pytest
import torch

from oracle import cpu_oracle as O
from paper_2605_29517_amd import binding as M
from paper_2605_29517_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def close(gpu, ref, what):
    g = gpu.detach().cpu().numpy().astype(np.float64)
    scale = np.abs(ref).max()
    err = np.abs(g - ref).max()
    assert err <= 1e-4 * scale + 1e-30, "%s: max|d| %.3e vs scale %.3e" % (what, err, scale)
    if scale > 0:
        cos = (g * ref).sum() / (np.linalg.norm(g) * np.linalg.norm(ref))
        assert cos >= 0.99999, "%s: cosine %.8f" % (what, cos)
    untouched = ~ref.reshape(-1, ref.shape[-1]).any(axis=1)  # rows no edge points at stay exactly zero
    assert not g.reshape(-1, g.shape[-1])[untouched].any(), what


def run_case(n_q, l_q, b, l_d, dtype, seed, holes=False, d=128):
    Q = W.unit_rows((n_q, l_q, d), dtype, seed, DEV)
    D = W.unit_rows((b, l_d, d), dtype, seed + 1, DEV)
    _, A, _ = O.forward(W.to_raw_numpy(Q), W.to_raw_numpy(D), dtype)
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((n_q, b)).astype(np.float32)
    if holes:
        A = A.copy()
        A[rng.random(A.shape) < 0.2] = -1
    rQ, rD = O.backward(W.to_raw_numpy(Q), W.to_raw_numpy(D), dtype, A, g.astype(np.float64))
    dQ, dD = M.maxsim_backward(Q, D, torch.from_numpy(A).to(DEV), torch.from_numpy(g).to(DEV))
    torch.cuda.synchronize()
    close(dQ, rQ, "dQ")
    close(dD, rD, "dD")
    return dQ, dD


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 32, 3, 40), (5, 33, 7, 129), (3, 7, 6, 300), (16, 32, 18, 257),
                                   (2, 100, 5, 64), (4, 64, 9, 128), (1, 130, 2, 31)])
def test_backward_parity(shape, dtype):
    run_case(*shape, dtype, 7)


# Embedding widths other than 128 (App. "Split-d Speedup": training verified at d = 512 .. 2048): every multiple of 8;
# columns beyond 128 are further slabs of the same kernels.  The explicit CSR must give the same bits.
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("d", [8, 64, 200, 256, 768, 2048])
def test_backward_other_widths(d, dtype):
    dQ, dD = run_case(3, 33, 5, 70, dtype, 31, holes=True, d=d)
    Q = W.unit_rows((3, 33, d), dtype, 31, DEV)
    D = W.unit_rows((5, 70, d), dtype, 32, DEV)
    _, A, _ = O.forward(W.to_raw_numpy(Q), W.to_raw_numpy(D), dtype)
    rng = np.random.default_rng(31)
    g = rng.standard_normal((3, 5)).astype(np.float32)
    A = A.copy()
    A[rng.random(A.shape) < 0.2] = -1
    cQ, cD, _, _ = M.maxsim_backward_csr(Q, D, torch.from_numpy(A).to(DEV), torch.from_numpy(g).to(DEV))
    torch.cuda.synchronize()
    assert torch.equal(cQ, dQ) and torch.equal(cD, dD)


@pytest.mark.parametrize("d", [64, 512, 1024])
def test_backward_other_widths_many_queries(d):
    """Enough query tokens for the document-partitioned dQ (partial sums combined in partition order) and for
    four query tokens per group of sixteen lanes."""
    run_case(72, 32, 40, 80, "f16", 37, d=d)
    run_case(130, 36, 9, 600, "bf16", 38, d=d)


# Twenty or more edges per dD row on average (n_q * l_q >= 20 * l_d): the kernel that sorts the edges inside the
# workgroup.  (n_q, l_q, b, l_d): blocks of 32 rows; 9600 column entries = two rounds; one hot row; blocks of 64 and
# of 128 rows spanning several short documents.
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("shape", [(40, 32, 6, 50), (64, 32, 9, 33), (30, 70, 5, 100), (300, 32, 3, 70), (130, 8, 40, 5),
                                   (33, 32, 1, 1), (70, 32, 4, 100)])
def test_backward_many_edges_per_row(shape, dtype):
    run_case(*shape, dtype, 17, holes=(shape[0] % 2 == 0))


@pytest.mark.parametrize("shape", [(48, 32, 1000, 70), (48, 32, 2000, 70)])
def test_backward_many_edges_per_row_large_blocks(shape):
    run_case(*shape, "f16", 19)


@pytest.mark.parametrize("adjacent", [False, True])
@pytest.mark.parametrize("n_q,l_q,b,l_d", [(96, 32, 7, 90), (300, 32, 3, 50), (64, 32, 40, 33)])
def test_backward_skewed_argmax(n_q, l_q, b, l_d, adjacent):
    """Half of the edges of every document land on four hot tokens (long row lists next to empty rows); the hot
    tokens anywhere in the document, or its first four (several long lists in one wavefront)."""
    rng = np.random.default_rng(23)
    Q = W.unit_rows((n_q, l_q, 128), "f16", 5, DEV)
    D = W.unit_rows((b, l_d, 128), "f16", 6, DEV)
    hot = np.broadcast_to(np.arange(4), (1, b, 4)) if adjacent else rng.integers(0, l_d, (1, b, 4))
    pick = rng.integers(0, 4, (n_q, b, l_q))
    A = np.where(rng.random((n_q, b, l_q)) < 0.5, np.take_along_axis(np.broadcast_to(hot, (n_q, b, 4)), pick, axis=2),
                 rng.integers(0, l_d, (n_q, b, l_q))).astype(np.int32)
    A[rng.random(A.shape) < 0.05] = -1
    g = rng.standard_normal((n_q, b)).astype(np.float32)
    rQ, rD = O.backward(W.to_raw_numpy(Q), W.to_raw_numpy(D), "f16", A, g.astype(np.float64))
    dQ, dD = M.maxsim_backward(Q, D, torch.from_numpy(A).to(DEV), torch.from_numpy(g).to(DEV))
    cQ, cD, _, _ = M.maxsim_backward_csr(Q, D, torch.from_numpy(A).to(DEV), torch.from_numpy(g).to(DEV))
    torch.cuda.synchronize()
    close(dQ, rQ, "dQ")
    close(dD, rD, "dD")
    assert torch.equal(cD, dD)      # long lists are walked by a whole wavefront: same order, same bits


# Rows that are not unit-norm and similarities that are negative throughout: the backward only moves rows and
# multiplies by the upstream gradient, but the forward that feeds it (argmax from the GPU here) has to pick the
# right winners there as well.  Compared with the oracle's backward through the SAME (GPU) argmax, after that
# argmax has itself been checked against the oracle's under the margin rule.
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("scale,q_bias,d_bias", [(1e-3, 0.3, -0.1), (1.0, 1.0, -1.0), (30.0, 0.5, 0.5)])
def test_forward_backward_chain_on_shifted_and_scaled_rows(scale, q_bias, d_bias, dtype):
    n_q, l_q, b, l_d = 40, 32, 7, 150
    Q = W.biased_rows((n_q, l_q, 128), dtype, 81, DEV, bias=q_bias, scale=scale)
    D = W.biased_rows((b, l_d, 128), dtype, 82, DEV, bias=d_bias, scale=scale)
    s, a = M.maxsim_forward(Q, D, want_argmax=True)
    torch.cuda.synchronize()
    _, ra, rm = O.forward(W.to_raw_numpy(Q), W.to_raw_numpy(D), dtype)
    clear = rm > 1e-3
    assert np.array_equal(a.cpu().numpy()[clear], ra[clear])
    rng = np.random.default_rng(83)
    g = rng.standard_normal((n_q, b)).astype(np.float32)
    A = a.cpu().numpy()
    rQ, rD = O.backward(W.to_raw_numpy(Q), W.to_raw_numpy(D), dtype, A, g.astype(np.float64))
    dQ, dD = M.maxsim_backward(Q, D, a, torch.from_numpy(g).to(DEV))
    torch.cuda.synchronize()
    close(dQ, rQ, "dQ")
    close(dD, rD, "dD")


def test_negative_indices_are_skipped():
    run_case(4, 32, 6, 70, "f16", 9, holes=True)


@pytest.mark.parametrize("n,l_d", [(8, 200), (64, 40)])      # few / many edges per dD row: both dD kernels
def test_backward_is_bitwise_reproducible(n, l_d):
    Q = W.unit_rows((n, 32, 128), "f16", 1, DEV)
    D = W.unit_rows((n, l_d, 128), "f16", 2, DEV)
    s, a = M.maxsim_forward(Q, D, want_argmax=True)
    g = torch.randn(n, n, device=DEV, generator=torch.Generator(DEV).manual_seed(3))
    r1 = M.maxsim_backward(Q, D, a, g)
    r2 = M.maxsim_backward(Q, D, a, g)
    r3 = M.maxsim_backward_csr(Q, D, a, g)                   # the explicit CSR adds the same edges in the same order
    torch.cuda.synchronize()
    assert torch.equal(r1[0], r2[0]) and torch.equal(r1[1], r2[1])
    assert torch.equal(r1[0], r3[0]) and torch.equal(r1[1], r3[1])


def test_contrastive_step_small():
    """forward with argmax -> cross-entropy gradient -> backward, all on the GPU, against the oracle chain."""
    n, l_q, l_d, tau = 12, 32, 96, 0.02
    Q, D = W.contrastive_batch(n, l_q, l_d, device=DEV, seed=4)
    s, a = M.maxsim_forward(Q, D, want_argmax=True)
    g, loss = M.maxsim_ce_grad(s, tau)
    dQ, dD = M.maxsim_backward(Q, D, a, g)
    torch.cuda.synchronize()
    # oracle chain on the GPU's fp32 scores (so that the softmax sees identical inputs)
    rs, rA, rm = O.forward(W.to_raw_numpy(Q), W.to_raw_numpy(D), "f16")
    assert np.allclose(s.cpu().numpy(), rs, rtol=2e-3)
    rloss, rg = O.ce_grad(s.cpu().numpy().astype(np.float64), tau)
    assert abs(float(loss) - rloss) <= 1e-5 * max(1.0, abs(rloss))
    assert np.abs(g.cpu().numpy() - rg).max() <= 1e-4 * np.abs(rg).max()
    clear = rm > 1e-3
    assert np.array_equal(a.cpu().numpy()[clear], rA[clear])
    # gradient parity with the oracle's argmax and the GPU's g as inputs
    rQ, rD = O.backward(W.to_raw_numpy(Q), W.to_raw_numpy(D), "f16", rA, g.cpu().numpy().astype(np.float64))
    dQ2, dD2 = M.maxsim_backward(Q, D, torch.from_numpy(rA).to(DEV), g)
    torch.cuda.synchronize()
    close(dQ2, rQ, "dQ")
    close(dD2, rD, "dD")


@pytest.mark.parametrize("n,b", [(1, 1), (4, 6), (37, 50), (256, 256), (40, 700)])
def test_ce_grad(n, b):
    s = (torch.randn(n, b, device=DEV, generator=torch.Generator(DEV).manual_seed(n * 1000 + b)) * 3 + 10).contiguous()
    g, loss = M.maxsim_ce_grad(s, 0.02)
    torch.cuda.synchronize()
    rloss, rg = O.ce_grad(s.cpu().numpy().astype(np.float64), 0.02)
    assert abs(float(loss) - rloss) <= 1e-5 * max(1.0, abs(rloss))
    assert np.abs(g.cpu().numpy() - rg).max() <= 1e-4 * max(np.abs(rg).max(), 1e-30)


def run_ragged_case(n_q, l_q, lens, dtype, seed):
    lens = np.asarray(lens, dtype=np.int64)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(off[-1])
    Q = W.unit_rows((n_q, l_q, 128), dtype, seed, DEV)
    Dp = W.unit_rows((T, 128), dtype, seed + 1, DEV)
    _, A, _ = O.forward(W.to_raw_numpy(Q), W.to_raw_numpy(Dp), dtype, offsets=off)
    g = np.random.default_rng(seed).standard_normal((n_q, len(lens))).astype(np.float32)
    rQ, rD = O.backward_ragged(W.to_raw_numpy(Q), W.to_raw_numpy(Dp), dtype, off, A, g.astype(np.float64))
    dQ, dD = M.maxsim_backward_ragged(Q, Dp, torch.from_numpy(off).to(DEV), torch.from_numpy(A).to(DEV),
                                      torch.from_numpy(g).to(DEV))
    torch.cuda.synchronize()
    close(dQ, rQ, "dQ")
    close(dD, rD, "dD")


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("case", [(1, 1, [1]), (3, 32, [5, 0, 64, 65, 1, 130, 0, 300]), (4, 33, [20] * 30),
                                  (2, 100, [0, 0, 127, 129, 128, 1, 1, 1, 0]), (9, 32, [70, 250, 64, 300, 199])])
def test_backward_ragged_parity(case, dtype):
    run_ragged_case(*case, dtype, 13)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("case", [(40, 32, [5, 0, 64, 65, 1, 130, 0, 30] * 3), (64, 32, [20] * 30), (300, 32, [70, 1, 0, 33]),
                                  (50, 40, [1] * 70 + [0] * 5 + [3] * 20)])
def test_backward_ragged_many_edges_per_row(case, dtype):
    run_ragged_case(*case, dtype, 29)


def test_ragged_forward_argmax_feeds_ragged_backward():
    """End to end on the GPU's own argmax.  The inputs are picked (by the oracle alone) so that every top-2
    margin is clear; the GPU argmax must then equal the oracle's and the gradients follow from it."""
    lens = np.array([40, 70, 0, 33, 5])
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    for seed in range(100, 500):
        Q = W.unit_rows((2, 8, 128), "f16", seed, DEV)
        Dp = W.unit_rows((int(off[-1]), 128), "f16", seed + 1000, DEV)
        _, A, mg = O.forward(W.to_raw_numpy(Q), W.to_raw_numpy(Dp), "f16", offsets=off)
        if mg[A >= 0].min() > 1.1e-3:
            break
    else:
        pytest.fail("no seed with clear margins")
    offd = torch.from_numpy(off).to(DEV)
    s, a = M.maxsim_forward_ragged(Q, Dp, offd, want_argmax=True)
    g = torch.randn(2, len(lens), device=DEV, generator=torch.Generator(DEV).manual_seed(3))
    dQ, dD = M.maxsim_backward_ragged(Q, Dp, offd, a, g)
    torch.cuda.synchronize()
    assert np.array_equal(a.cpu().numpy(), A)
    rQ, rD = O.backward_ragged(W.to_raw_numpy(Q), W.to_raw_numpy(Dp), "f16", off, A, g.cpu().numpy().astype(np.float64))
    close(dQ, rQ, "dQ")
    close(dD, rD, "dD")


def test_autograd_wrapper_matches_the_oracle():
    """loss = sum(w * maxsim(Q, D)) through torch.autograd: gradients equal the oracle's for dscore = w."""
    from paper_2605_29517_amd.autograd import maxsim
    lens = np.array([40, 70, 0, 33, 5])
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    for seed in range(100, 500):  # inputs with clear top-2 margins, chosen by the oracle alone
        Q = W.unit_rows((2, 8, 128), "f16", seed, DEV)
        Dp = W.unit_rows((int(off[-1]), 128), "f16", seed + 1000, DEV)
        _, A, mg = O.forward(W.to_raw_numpy(Q), W.to_raw_numpy(Dp), "f16", offsets=off)
        if mg[A >= 0].min() > 1.1e-3:
            break
    w = torch.randn(2, len(lens), device=DEV, generator=torch.Generator(DEV).manual_seed(5))
    Qg, Dg = Q.clone().requires_grad_(True), Dp.clone().requires_grad_(True)
    s = maxsim(Qg, Dg, torch.from_numpy(off).to(DEV))
    keep = torch.isfinite(s)
    (torch.where(keep, s, torch.zeros_like(s)) * w).sum().backward()
    rQ, rD = O.backward_ragged(W.to_raw_numpy(Q), W.to_raw_numpy(Dp), "f16", off, A, w.cpu().numpy().astype(np.float64))
    # torch wants gradients in the input dtype: the fp32 gradients of the C ABI (bar 1e-4 of the maximum, as in `close`)
    # are rounded to fp16 by the glue, half an ulp = 2^-11 relative per element
    tol = 1e-4 + 2.0 ** -11
    assert np.abs(Qg.grad.float().cpu().numpy() - rQ).max() <= tol * np.abs(rQ).max()
    assert np.abs(Dg.grad.float().cpu().numpy() - rD).max() <= tol * np.abs(rD).max()
    # uniform path, fp32
    Qf = W.unit_rows((3, 16, 128), "f32", 7, DEV).requires_grad_(True)
    Df = W.unit_rows((4, 50, 128), "f32", 8, DEV).requires_grad_(True)
    wf = torch.randn(3, 4, device=DEV, generator=torch.Generator(DEV).manual_seed(6))
    (maxsim(Qf, Df) * wf).sum().backward()
    _, A2, _ = O.forward(W.to_raw_numpy(Qf.detach()), W.to_raw_numpy(Df.detach()), "f32")
    rQ, rD = O.backward(W.to_raw_numpy(Qf.detach()), W.to_raw_numpy(Df.detach()), "f32", A2, wf.cpu().numpy().astype(np.float64))
    close(Qf.grad, rQ, "dQ")
    close(Df.grad, rD, "dD")
