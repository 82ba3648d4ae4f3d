"""Pins of the CSR oracle (inverse map destination row -> source edges of the deterministic backward, Alg. 2):
against a brute-force enumeration, against its structural invariants, and against the edge-order oracle backward
(walking the CSR row by row must reproduce Eq. 3 bit for bit in fp64, because both add a row's edges in increasing
(query, token) order)."""
import numpy as np
import pytest

from oracle import cpu_oracle as O


def brute_csr(A, l_d):
    n_q, b, l_q = A.shape
    rows = [[] for _ in range(b * l_d)]
    for i in range(n_q):              # flat edge order (i, j, s)
        for j in range(b):
            for s in range(l_q):
                t = int(A[i, j, s])
                if 0 <= t < l_d:
                    rows[j * l_d + t].append((i * b + j) * l_q + s)
    row_ptr = [0]
    col = []
    for r in rows:
        col.extend(r)
        row_ptr.append(len(col))
    return np.asarray(row_ptr, np.int32), np.asarray(col, np.int32)


@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 3, 4, 5), (3, 2, 7, 3), (5, 4, 2, 9), (4, 1, 33, 2)])
def test_csr_equals_brute_force(shape):
    n_q, b, l_q, l_d = shape
    rng = np.random.default_rng(sum(shape))
    A = rng.integers(0, l_d, (n_q, b, l_q)).astype(np.int32)
    A[rng.random(A.shape) < 0.1] = -1      # skipped entries (empty documents)
    rp, ci = O.csr_build(A, l_d)
    brp, bci = brute_csr(A, l_d)
    assert np.array_equal(rp, brp) and np.array_equal(ci, bci)


def test_csr_invariants():
    rng = np.random.default_rng(5)
    n_q, b, l_q, l_d = 6, 5, 8, 11
    A = rng.integers(-1, l_d, (n_q, b, l_q)).astype(np.int32)
    rp, ci = O.csr_build(A, l_d)
    n_edges = int((A >= 0).sum())
    assert rp[0] == 0 and rp[-1] == n_edges == ci.size and np.all(np.diff(rp) >= 0)
    assert np.array_equal(np.sort(ci), np.flatnonzero((A >= 0).ravel()))      # a permutation of the valid edges
    for r in range(b * l_d):
        seg = ci[rp[r]:rp[r + 1]]
        assert np.all(np.diff(seg) > 0)                                          # stable: increasing edge index
        i, rest = np.divmod(seg, b * l_q)
        j, s = np.divmod(rest, l_q)
        assert np.all(j == r // l_d) and np.all(A[i, j, s] == r % l_d)           # every edge points at its row
    # all edges on one token: one row holds everything, in order
    A1 = np.full((2, 1, 3), 4, np.int32)
    rp1, ci1 = O.csr_build(A1, 7)
    assert np.array_equal(ci1, np.arange(6)) and rp1[4] == 0 and rp1[5] == 6 and rp1[-1] == 6


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_csr_walk_reproduces_the_edge_order_backward(dtype):
    rng = np.random.default_rng(11)
    n_q, b, l_q, l_d, d = 4, 3, 5, 6, 8
    Qf = rng.standard_normal((n_q, l_q, d)).astype(np.float32)
    Df = rng.standard_normal((b, l_d, d)).astype(np.float32)
    if dtype == "f16":
        Q, D = Qf.astype(np.float16), Df.astype(np.float16)
    elif dtype == "bf16":
        Q, D = (Qf.view(np.uint32) >> 16).astype(np.uint16), (Df.view(np.uint32) >> 16).astype(np.uint16)
    else:
        Q, D = Qf, Df
    A = rng.integers(0, l_d, (n_q, b, l_q)).astype(np.int32)
    g = rng.standard_normal((n_q, b))
    _, dD = O.backward(Q, D, dtype, A, g)
    rp, ci = O.csr_build(A, l_d)
    dD_csr = O.backward_dd_from_csr(Q, dtype, b, l_d, rp, ci, g)
    assert np.array_equal(dD_csr, dD)     # bit for bit in fp64


def test_decode_array_matches_the_scalar_decoders():
    bits = np.asarray([0x0000, 0x8000, 0x3C00, 0xBC00, 0x0001, 0x7BFF, 0x3555, 0x4248], np.uint16)
    assert [O.decode_f16(int(x)) for x in bits] == list(O.decode_array(bits, "f16"))
    assert [O.decode_bf16(int(x)) for x in bits] == list(O.decode_array(bits, "bf16"))
