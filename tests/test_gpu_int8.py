"""GPU parity of maxsim_quantize_rows_i8 and maxsim_forward_i8 against the CPU oracle: bit-exact."""
import numpy as np
import pytest
import torch

from oracle import cpu_oracle as O
from paper_2605_29517_amd import binding as M
from paper_2605_29517_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_quantiser_bit_exact(dtype):
    X = W.unit_rows((777, 128), dtype, 3, DEV)
    X[5] = 0
    X[6] = 0.25
    codes, scale = M.maxsim_quantize_rows_i8(X)
    torch.cuda.synchronize()
    rc, rs = O.quantize_rows_i8(W.to_raw_numpy(X), dtype)
    assert np.array_equal(bits(scale.cpu().numpy()), bits(rs))
    assert np.array_equal(codes.cpu().numpy(), rc)


def test_quantiser_half_to_even():
    X = torch.tensor([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49] + [0.0] * 120], device=DEV)
    codes, scale = M.maxsim_quantize_rows_i8(X)
    torch.cuda.synchronize()
    assert float(scale[0]) == 1.0
    assert codes[0, :8].tolist() == [127, 0, 2, 2, 0, -2, -2, 3]


def test_quantiser_hard_quotients_and_extreme_scales():
    """Rows built to stress the rounding of x / s: elements a few ulps around every half-integer multiple of the
    scale, scales with an all-ones significand, scales from the subnormal range up to 2^100, and a row count that
    leaves the last wavefront partly empty.  Bit-exact against the oracle's IEEE division."""
    rng = np.random.default_rng(12)
    rows = []
    # scales with an all-ones significand: absmax = fl32(127 * s) gives fl32(absmax / 127) = s for most exponents
    cand = (np.arange(60, 200, dtype=np.uint32) << 23 | np.uint32(0x7fffff)).view(np.float32)
    amax = (cand.astype(np.float64) * 127.0).astype(np.float32)
    keep = (amax / np.float32(127.0)).view(np.uint32) & 0x7fffff == 0x7fffff
    assert keep.sum() > 20
    for a in list(amax[keep][:40]) + [np.float32(v) for v in (1e-42, 3e-39, 1e-30, 1e-19, 1e-3, 1.0, 77.7, 1e19, 1e30)]:
        s = np.float32(a) / np.float32(127.0)
        k = rng.integers(-127, 127, 127).astype(np.float32) + np.float32(0.5)
        x = (k * s).astype(np.float32)
        x = (x.view(np.int32) + rng.integers(-3, 4, 127).astype(np.int32)).view(np.float32)   # a few ulps around the tie
        x = np.clip(x, -a, a)
        rows.append(np.concatenate([[a], x]).astype(np.float32))
    for _ in range(150):                                  # random rows of every magnitude
        e = rng.integers(-120, 100)
        rows.append((rng.standard_normal(128) * 2.0 ** e).astype(np.float32))
    Xn = np.stack(rows)
    assert Xn.shape[0] % 16 != 0
    X = torch.from_numpy(Xn).to(DEV)
    codes, scale = M.maxsim_quantize_rows_i8(X)
    torch.cuda.synchronize()
    rc, rs = O.quantize_rows_i8(Xn, "f32")
    assert np.array_equal(bits(scale.cpu().numpy()), bits(rs))
    assert np.array_equal(codes.cpu().numpy(), rc)


def quantised_case(n_q, l_q, b, l_d, seed):
    Qf = W.unit_rows((n_q, l_q, 128), "f16", seed, DEV)
    Df = W.unit_rows((b, l_d, 128), "f32", seed + 1, DEV)
    # oracle quantises its own copies; the GPU quantiser must agree bit for bit
    oq, oqs = O.quantize_rows_i8(W.to_raw_numpy(Qf), "f16")
    od, ods = O.quantize_rows_i8(W.to_raw_numpy(Df), "f32")
    gq, gqs = M.maxsim_quantize_rows_i8(Qf)
    gd, gds = M.maxsim_quantize_rows_i8(Df)
    torch.cuda.synchronize()
    assert np.array_equal(gq.cpu().numpy(), oq) and np.array_equal(bits(gqs.cpu().numpy()), bits(oqs))
    assert np.array_equal(gd.cpu().numpy(), od) and np.array_equal(bits(gds.cpu().numpy()), bits(ods))
    return (gq, gqs, gd, gds), (oq, oqs, od, ods)


@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (1, 32, 9, 64), (2, 33, 5, 65), (1, 100, 7, 31), (3, 32, 11, 200),
                                   (9, 40, 6, 129), (1, 1024, 5, 300), (2, 512, 4, 97), (40, 32, 19, 70)])
def test_forward_i8_bit_exact(shape):
    n_q, l_q, b, l_d = shape
    g, o = quantised_case(n_q, l_q, b, l_d, 17)
    s = M.maxsim_forward_i8(*g)
    torch.cuda.synchronize()
    ref = O.forward_i8(*o)
    assert np.array_equal(bits(s.cpu().numpy()), bits(ref))


def test_forward_i8_extreme_codes_and_negative_maxima():
    Q = torch.full((1, 32, 128), -127, dtype=torch.int8, device=DEV)
    D = torch.full((3, 70, 128), 127, dtype=torch.int8, device=DEV)
    D[1, 5] = -127
    qs = torch.full((1, 32), 0.5, device=DEV)
    ds = torch.rand(3, 70, device=DEV) + 0.01
    s = M.maxsim_forward_i8(Q, qs, D, ds)
    torch.cuda.synchronize()
    ref = O.forward_i8(Q.cpu().numpy(), qs.cpu().numpy(), D.cpu().numpy(), ds.cpu().numpy())
    assert np.array_equal(bits(s.cpu().numpy()), bits(ref))
    assert float(s[0, 0]) < 0 < float(s[0, 1])


def test_forward_i8_rejects_queries_longer_than_one_group():
    Q = torch.zeros((1, 1100, 128), dtype=torch.int8, device=DEV)
    D = torch.zeros((2, 10, 128), dtype=torch.int8, device=DEV)
    with pytest.raises(M.MaxSimError):
        M.maxsim_forward_i8(Q, torch.ones(1, 1100, device=DEV), D, torch.ones(2, 10, device=DEV))


def ragged_case(n_q, l_q, lens, seed):
    """Packed int8 corpus with the given document lengths (GPU quantiser output, checked against the oracle's)."""
    lens = np.asarray(lens, dtype=np.int64)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(off[-1])
    Qf = W.unit_rows((n_q, l_q, 128), "f16", seed, DEV)
    Df = W.unit_rows((T, 128), "f32", seed + 1, DEV)
    oq, oqs = O.quantize_rows_i8(W.to_raw_numpy(Qf), "f16")
    od, ods = O.quantize_rows_i8(W.to_raw_numpy(Df), "f32")
    gq, gqs = M.maxsim_quantize_rows_i8(Qf)
    gd, gds = M.maxsim_quantize_rows_i8(Df)
    torch.cuda.synchronize()
    assert np.array_equal(gd.cpu().numpy(), od) and np.array_equal(bits(gds.cpu().numpy()), bits(ods))
    assert np.array_equal(gq.cpu().numpy(), oq) and np.array_equal(bits(gqs.cpu().numpy()), bits(oqs))
    return (gq, gqs, gd, gds, torch.from_numpy(off).to(DEV)), (oq, oqs, od, ods, off)


@pytest.mark.parametrize("case", [(1, 32, [5, 0, 64, 65, 1, 130, 0]), (3, 40, [33] * 9 + [0, 200]), (2, 512, [31, 97, 300])])
def test_forward_i8_ragged_bit_exact_small(case):
    n_q, l_q, lens = case
    g, o = ragged_case(n_q, l_q, lens, 23)
    s = M.maxsim_forward_i8_ragged(*g)
    torch.cuda.synchronize()
    ref = O.forward_i8_ragged(*o)
    assert np.array_equal(bits(s.cpu().numpy()), bits(ref))


# corpora of >= 4096 documents take the document-stationary kernel (every wavefront on its own run of documents)
@pytest.mark.parametrize("shape", [(1, 32, 4100, 70), (2, 100, 4200, 33), (1, 1024, 4096, 40), (40, 32, 4500, 20), (3, 200, 4100, 65)])
def test_forward_i8_large_corpus_bit_exact(shape):
    n_q, l_q, b, l_d = shape
    g, o = quantised_case(n_q, l_q, b, l_d, 31)
    s = M.maxsim_forward_i8(*g)
    torch.cuda.synchronize()
    ref = O.forward_i8(*o)
    assert np.array_equal(bits(s.cpu().numpy()), bits(ref))


def test_forward_i8_ragged_large_corpus_bit_exact():
    rng = np.random.default_rng(9)
    lens = rng.integers(0, 150, 5000)
    lens[:4] = [0, 1, 32, 33]
    lens[-1] = 0
    for n_q, l_q in ((1, 64), (5, 200)):
        g, o = ragged_case(n_q, l_q, lens, 37)
        s = M.maxsim_forward_i8_ragged(*g)
        torch.cuda.synchronize()
        ref = O.forward_i8_ragged(*o)
        assert np.array_equal(bits(s.cpu().numpy()), bits(ref))


def test_forward_i8_large_corpus_negative_maxima():
    b = 4100
    Q = torch.full((1, 33, 128), -127, dtype=torch.int8, device=DEV)
    D = torch.full((b, 35, 128), 127, dtype=torch.int8, device=DEV)
    D[1::2, 5] = -127
    qs = torch.rand(1, 33, device=DEV) + 0.5
    ds = torch.rand(b, 35, device=DEV) + 0.01
    s = M.maxsim_forward_i8(Q, qs, D, ds)
    torch.cuda.synchronize()
    ref = O.forward_i8(Q.cpu().numpy(), qs.cpu().numpy(), D.cpu().numpy(), ds.cpu().numpy())
    assert np.array_equal(bits(s.cpu().numpy()), bits(ref))
    assert float(s[0, 0]) < 0 < float(s[0, 1])


@pytest.mark.parametrize("b", [7, 4100])
def test_forward_i8_tiny_huge_and_zero_scales(b):
    """Scales far from 1 (but above 2^-100) and all-zero rows: still bit-exact, negative maxima included."""
    rng = np.random.default_rng(77)
    Q = torch.from_numpy(rng.integers(-127, 128, (2, 40, 128), dtype=np.int8)).to(DEV)
    D = torch.from_numpy(rng.integers(-127, 128, (b, 35, 128), dtype=np.int8)).to(DEV)
    D[1] = -Q[0, :35].abs().clamp(min=1)          # mostly negative dot products against query 0 ...
    Q[0] = Q[0].abs().clamp(min=1)                # ... whose rows are made positive
    qs = torch.from_numpy(10.0 ** rng.uniform(-2, 2, (2, 40)).astype(np.float32)).to(DEV)  # row values within 19 binades
    ds = torch.from_numpy(10.0 ** rng.uniform(-25, 10, (b, 35)).astype(np.float32)).to(DEV)
    ds[2] = 0.0
    D[2] = 0
    qs[1, 3] = 0.0
    s = M.maxsim_forward_i8(Q, qs, D, ds)
    torch.cuda.synchronize()
    ref = O.forward_i8(Q.cpu().numpy(), qs.cpu().numpy(), D.cpu().numpy(), ds.cpu().numpy())
    assert np.array_equal(bits(s.cpu().numpy()), bits(ref))
    assert float(s[0, 1]) < 0


# Uniform corpora of long documents (>= 256 tokens), queries of up to 16 column blocks (32 blocks in all) and fewer
# than 4096 documents:
# the wavefronts of a workgroup share each document's tiles and combine their maxima in LDS.
@pytest.mark.parametrize("shape", [(1, 32, 50, 300), (2, 40, 37, 257), (1, 128, 20, 1024), (3, 32, 9, 256),
                                   (8, 32, 5, 270), (1, 97, 1, 999), (2, 100, 600, 260), (1, 512, 12, 300), (2, 300, 9, 257),
                                   (5, 100, 8, 260), (1, 200, 3, 1024)])
def test_forward_i8_shared_documents_bit_exact(shape):
    n_q, l_q, b, l_d = shape
    g, o = quantised_case(n_q, l_q, b, l_d, 23)
    s = M.maxsim_forward_i8(*g)
    torch.cuda.synchronize()
    ref = O.forward_i8(*o)
    assert np.array_equal(bits(s.cpu().numpy()), bits(ref))


def test_forward_i8_shared_documents_negative_maxima():
    Q = torch.full((1, 33, 128), -127, dtype=torch.int8, device=DEV)
    D = torch.full((30, 300, 128), 127, dtype=torch.int8, device=DEV)
    D[1::2, 290] = -127       # one positive cell per odd document, in the last wavefront's share
    qs = torch.rand(1, 33, device=DEV) + 0.5
    ds = torch.rand(30, 300, device=DEV) + 0.01
    s = M.maxsim_forward_i8(Q, qs, D, ds)
    torch.cuda.synchronize()
    ref = O.forward_i8(Q.cpu().numpy(), qs.cpu().numpy(), D.cpu().numpy(), ds.cpu().numpy())
    assert np.array_equal(bits(s.cpu().numpy()), bits(ref))
    assert float(s[0, 0]) < 0 < float(s[0, 1])


# ---- embedding widths other than 128 (every multiple of 32 up to 8192): the slab kernel (multiples of 64) and the
# plain inner loop over d ----

WIDE_D = [32, 64, 96, 256, 320, 768, 1024, 2048]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("d", WIDE_D + [8192])
def test_quantiser_other_widths_bit_exact(d, dtype):
    X = W.unit_rows((53, d), dtype, 300 + d, DEV)
    X[5] = 0
    X[6] = 0.25
    X[7] *= 1e-3 if dtype != "f16" else 1e-2
    codes, scale = M.maxsim_quantize_rows_i8(X)
    torch.cuda.synchronize()
    rc, rs = O.quantize_rows_i8(W.to_raw_numpy(X), dtype)
    assert np.array_equal(bits(scale.cpu().numpy()), bits(rs))
    assert np.array_equal(codes.cpu().numpy(), rc)


def wide_case(n_q, l_q, b, l_d, d, seed):
    Qf = W.unit_rows((n_q, l_q, d), "f16", seed, DEV)
    Df = W.unit_rows((b, l_d, d), "f32", seed + 1, DEV)
    oq, oqs = O.quantize_rows_i8(W.to_raw_numpy(Qf), "f16")
    od, ods = O.quantize_rows_i8(W.to_raw_numpy(Df), "f32")
    gq, gqs = M.maxsim_quantize_rows_i8(Qf)
    gd, gds = M.maxsim_quantize_rows_i8(Df)
    torch.cuda.synchronize()
    assert np.array_equal(gq.cpu().numpy(), oq) and np.array_equal(bits(gqs.cpu().numpy()), bits(oqs))
    assert np.array_equal(gd.cpu().numpy(), od) and np.array_equal(bits(gds.cpu().numpy()), bits(ods))
    return (gq, gqs, gd, gds), (oq, oqs, od, ods)


# (n_q, l_q, b, l_d): one block, ragged tails of blocks and tiles, several queries per workgroup, a query that fills a
# workgroup (32 blocks), more queries than a workgroup holds, more documents than chunks
@pytest.mark.parametrize("d", WIDE_D)
@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (1, 32, 9, 64), (2, 33, 5, 65), (3, 100, 7, 31), (40, 32, 19, 70)])
def test_forward_i8_other_widths_bit_exact(shape, d):
    n_q, l_q, b, l_d = shape
    g, o = wide_case(n_q, l_q, b, l_d, d, 400 + d)
    s = M.maxsim_forward_i8(*g)
    torch.cuda.synchronize()
    ref = O.forward_i8(*o)
    assert np.array_equal(bits(s.cpu().numpy()), bits(ref))


# (the last case: two passes over chunks of more than a thousand documents each, whose first-pass sums wait in LDS)
@pytest.mark.parametrize("case", [(1, 1024, 3, 70, 256), (2, 700, 2100, 40, 64), (5, 300, 6, 130, 768), (1, 600, 1200000, 1, 64)])
def test_forward_i8_other_widths_long_queries_and_many_documents(case):
    n_q, l_q, b, l_d, d = case
    g, o = wide_case(n_q, l_q, b, l_d, d, 77)
    s = M.maxsim_forward_i8(*g)
    torch.cuda.synchronize()
    keep = np.unique(np.concatenate([[0, b - 1], np.random.default_rng(5).integers(0, b, 40)]))
    ref = O.forward_i8(o[0], o[1], np.ascontiguousarray(o[2][keep]), np.ascontiguousarray(o[3][keep]))
    assert np.array_equal(bits(s[:, torch.from_numpy(keep).to(DEV)].cpu().numpy()), bits(ref))


def test_forward_i8_other_widths_extreme_codes():
    """All codes at +-127 and d = 8192: |n| = 127^2 * 8192 is past 2^24, where an fp32 conversion of n would round;
    negative and positive maxima."""
    d = 8192
    Q = torch.full((1, 33, d), -127, dtype=torch.int8, device=DEV)
    D = torch.full((3, 40, d), 127, dtype=torch.int8, device=DEV)
    D[1, 5] = -127
    D[2, :, 1::2] = 126
    qs = torch.full((1, 33), 0.5, device=DEV)
    ds = torch.rand(3, 40, device=DEV, generator=torch.Generator(DEV).manual_seed(3)) + 0.01
    s = M.maxsim_forward_i8(Q, qs, D, ds)
    torch.cuda.synchronize()
    ref = O.forward_i8(Q.cpu().numpy(), qs.cpu().numpy(), D.cpu().numpy(), ds.cpu().numpy())
    assert np.array_equal(bits(s.cpu().numpy()), bits(ref))
    assert float(s[0, 0]) < 0 < float(s[0, 1])


@pytest.mark.parametrize("n_q,l_q", [(3, 40), (2, 700)])
@pytest.mark.parametrize("d", [64, 256, 1024])
def test_forward_i8_ragged_other_widths_bit_exact(d, n_q, l_q):
    lens = np.asarray([5, 0, 64, 65, 1, 130, 0, 33, 0], dtype=np.int64)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    Qf = W.unit_rows((n_q, l_q, d), "f16", 500 + d, DEV)
    Df = W.unit_rows((int(off[-1]), d), "f32", 501 + d, DEV)
    oq, oqs = O.quantize_rows_i8(W.to_raw_numpy(Qf), "f16")
    od, ods = O.quantize_rows_i8(W.to_raw_numpy(Df), "f32")
    gq, gqs = M.maxsim_quantize_rows_i8(Qf)
    gd, gds = M.maxsim_quantize_rows_i8(Df)
    s = M.maxsim_forward_i8_ragged(gq, gqs, gd, gds, torch.from_numpy(off).to(DEV))
    torch.cuda.synchronize()
    ref = O.forward_i8_ragged(oq, oqs, od, ods, off)
    assert np.array_equal(bits(s.cpu().numpy()), bits(ref))
    assert np.isneginf(s.cpu().numpy()[:, lens == 0]).all()


def test_int8_widths_that_are_refused():
    for d in (16, 100, 8224):
        with pytest.raises(M.MaxSimError):
            M.maxsim_quantize_rows_i8(torch.zeros(4, d, device=DEV))
        with pytest.raises(M.MaxSimError):
            M.maxsim_forward_i8(torch.zeros(1, 4, d, dtype=torch.int8, device=DEV), torch.ones(1, 4, device=DEV),
                                torch.zeros(2, 5, d, dtype=torch.int8, device=DEV), torch.ones(2, 5, device=DEV))
