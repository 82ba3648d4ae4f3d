"""Seeded random shapes through every entry point against the oracle: sizes that straddle tile, block, group and
chunk boundaries in combinations the hand-picked cases may miss."""
import numpy as np
import pytest
import torch

from oracle import cpu_oracle as O
from paper_2605_29517_amd import binding as M
from paper_2605_29517_amd import workloads as W

from parity import RTOL_16, RTOL_F32, forward_parity_ragged, forward_parity_uniform

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def pick_shape(rng):
    n_q = int(rng.choice([1, 1, 2, 3, 5, 8, 17, 33, 70]))
    l_q = int(rng.choice([1, 7, 31, 32, 33, 64, 100, 129, 300]))
    if n_q * l_q > 4000:
        l_q = 32
    b = int(rng.integers(1, 80))
    l_d = int(rng.choice([1, 5, 31, 32, 33, 63, 65, 100, 200]))
    return n_q, l_q, b, l_d


@pytest.mark.parametrize("seed", range(48))
def test_forward_random_shape(seed):
    rng = np.random.default_rng(1000 + seed)
    n_q, l_q, b, l_d = pick_shape(rng)
    dtype = ["f16", "bf16", "f32"][seed % 3]
    # register-stationary widths and slab-kernel widths (any multiple of 64 bytes per row)
    d = int(rng.choice([64, 128, 128, 256, 48, 400] if dtype == "f32" else [64, 128, 128, 256, 512, 96, 320, 800]))
    rtol = RTOL_F32 if dtype == "f32" else RTOL_16
    Q = W.unit_rows((n_q, l_q, d), dtype, seed, DEV)
    if seed % 2 == 0:
        D = W.unit_rows((b, l_d, d), dtype, seed + 500, DEV)
        forward_parity_uniform(Q, D, M.maxsim_forward, seed % 4 == 0, rtol)
    else:
        lens = rng.integers(0, 2 * l_d + 1, b)
        lens[rng.integers(0, b)] = max(1, l_d)
        off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(DEV)
        Dp = W.unit_rows((int(lens.sum()), d), dtype, seed + 500, DEV)
        forward_parity_ragged(Q, Dp, off, M.maxsim_forward_ragged, seed % 4 == 1, rtol)


@pytest.mark.parametrize("seed", range(24))
def test_int8_random_shape(seed):
    rng = np.random.default_rng(2000 + seed)
    n_q, l_q, b, l_d = pick_shape(rng)
    if seed % 3 == 0:
        b += 4096  # document-stationary kernel
        l_d = min(l_d, 40)
        n_q, l_q = min(n_q, 3), min(l_q, 100)
    elif seed % 3 == 1 and seed % 2 == 0:
        l_d = int(rng.choice([256, 257, 300, 520]))  # long uniform documents: a workgroup per document
        n_q, l_q, b = min(n_q, 4), min(l_q, 129), min(b, 30)
    lens = rng.integers(0, 2 * l_d + 1, b) if seed % 2 else np.full(b, l_d)
    lens[0] = max(1, l_d)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    Qf = W.unit_rows((n_q, l_q, 128), "f16", seed, DEV)
    Df = W.unit_rows((int(off[-1]), 128), "f32", seed + 700, DEV)
    q8, qs = M.maxsim_quantize_rows_i8(Qf)
    d8, ds = M.maxsim_quantize_rows_i8(Df)
    oq, oqs = O.quantize_rows_i8(W.to_raw_numpy(Qf), "f16")
    od, ods = O.quantize_rows_i8(W.to_raw_numpy(Df), "f32")
    if seed % 2:
        s = M.maxsim_forward_i8_ragged(q8, qs, d8, ds, torch.from_numpy(off).to(DEV))
        ref = O.forward_i8_ragged(oq, oqs, od, ods, off)
    else:
        s = M.maxsim_forward_i8(q8, qs, d8.view(b, l_d, 128), ds.view(b, l_d))
        ref = O.forward_i8(oq, oqs, od.reshape(b, l_d, 128), ods.reshape(b, l_d))
    torch.cuda.synchronize()
    assert np.array_equal(bits(s.cpu().numpy()), bits(ref))


@pytest.mark.parametrize("seed", range(32))
def test_backward_random_shape(seed):
    rng = np.random.default_rng(3000 + seed)
    n_q, l_q, b, l_d = pick_shape(rng)
    dtype = ["f16", "bf16", "f32"][seed % 3]
    lens = rng.integers(0, 2 * l_d + 1, b) if seed % 2 else np.full(b, l_d)
    lens[0] = max(1, l_d)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    Q = W.unit_rows((n_q, l_q, 128), dtype, seed, DEV)
    Dp = W.unit_rows((int(off[-1]), 128), dtype, seed + 900, DEV)
    _, A, _ = O.forward(W.to_raw_numpy(Q), W.to_raw_numpy(Dp), dtype, offsets=off)
    if seed % 4 >= 2:   # a skewed argmax: 40 % of the edges of every document on up to three hot tokens
        A = A.copy()
        for j in range(b):
            if lens[j] > 0:
                hot = rng.integers(0, lens[j], 3)
                take = rng.random((n_q, l_q)) < 0.4
                A[:, j, :] = np.where(take, hot[rng.integers(0, 3, (n_q, l_q))], A[:, j, :])
    g = rng.standard_normal((n_q, b)).astype(np.float32)
    rQ, rD = O.backward_ragged(W.to_raw_numpy(Q), W.to_raw_numpy(Dp), dtype, off, A, g.astype(np.float64))
    At, gt = torch.from_numpy(A).to(DEV), torch.from_numpy(g).to(DEV)
    if seed % 2:
        dQ, dD = M.maxsim_backward_ragged(Q, Dp, torch.from_numpy(off).to(DEV), At, gt)
    else:
        dQ, dD = M.maxsim_backward(Q, Dp.view(b, l_d, 128), At, gt)
        cQ, cD, _, _ = M.maxsim_backward_csr(Q, Dp.view(b, l_d, 128), At, gt)
        assert torch.equal(cQ, dQ) and torch.equal(cD, dD)      # the explicit CSR: same order, same bits
        dD = dD.view(-1, 128)
    torch.cuda.synchronize()
    for got, ref in ((dQ, rQ), (dD, rD)):
        err = np.abs(got.cpu().numpy() - ref).max()
        assert err <= 1e-4 * np.abs(ref).max() + 1e-30
