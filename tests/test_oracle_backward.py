"""Pins for the oracle's backward (Eqs. 2-3) and the cross-entropy helper.  No GPU."""
import numpy as np

from oracle import cpu_oracle as O


def weighted_total(Q, D, w):
    s, _, _ = O.forward(Q.astype(np.float32), D.astype(np.float32), "f32", want_argmax=False, want_margin=False)
    return float((w * s).sum())


def make_case(seed, n_q=2, b=3, l_q=4, l_d=6, d=5):
    """Inputs on a 2^-6 grid (so that +-h perturbations stay exact in fp32) with clear margins."""
    rng = np.random.default_rng(seed)
    while True:
        Q = np.round(rng.standard_normal((n_q, l_q, d)) * 32) / 64
        D = np.round(rng.standard_normal((b, l_d, d)) * 32) / 64
        _, _, m = O.forward(Q.astype(np.float32), D.astype(np.float32), "f32")
        if m.min() > 0.05:
            return Q.astype(np.float32), D.astype(np.float32)


def test_finite_differences():
    Q, D = make_case(0)
    rng = np.random.default_rng(1)
    w = rng.standard_normal((2, 3))
    _, A, m = O.forward(Q, D, "f32")
    dQ, dD = O.backward(Q, D, "f32", A, w)
    # inside an argmax region the total is linear in Q alone and in D alone, so a central
    # difference with an exactly representable step is exact up to fp64 rounding
    h = 2.0 ** -10
    for X, dX, which in ((Q, dQ, 0), (D, dD, 1)):
        for idx in np.ndindex(*X.shape):
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += np.float32(h)
            Xm[idx] -= np.float32(h)
            fp = weighted_total(Xp, D, w) if which == 0 else weighted_total(Q, Xp, w)
            fm = weighted_total(Xm, D, w) if which == 0 else weighted_total(Q, Xm, w)
            assert abs((fp - fm) / (2 * h) - dX[idx]) < 1e-9, (which, idx)


def test_euler_identity_and_row_sums():
    Q, D = make_case(2, n_q=3, b=4, l_q=5, l_d=7, d=6)
    rng = np.random.default_rng(3)
    g = rng.standard_normal((3, 4))
    s, A, _ = O.forward(Q, D, "f32")
    dQ, dD = O.backward(Q, D, "f32", A, g)
    total = (g * s).sum()
    # the score is homogeneous of degree one in Q and in D
    assert abs((dQ * Q).sum() - total) < 1e-12
    assert abs((dD * D).sum() - total) < 1e-12
    # summing dD over a document's tokens collects every query token once
    ref = np.einsum("ij,ik->jk", g, Q.astype(np.float64).sum(1))
    assert np.allclose(dD.sum(1), ref, atol=1e-12)
    # and dQ over documents
    for i in range(3):
        for t in range(5):
            r = sum(g[i, j] * D[j, A[i, j, t]].astype(np.float64) for j in range(4))
            assert np.allclose(dQ[i, t], r, atol=1e-13)


def test_single_edge():
    Q = np.array([[[1.0, -2.0, 0.5]]], np.float32)
    D = np.array([[[0.0, 1.0, 0.0], [2.0, 0.0, 0.0], [1.0, 0.0, 1.0]]], np.float32)
    _, A, _ = O.forward(Q, D, "f32")
    assert A[0, 0, 0] == 1
    dQ, dD = O.backward(Q, D, "f32", A, np.array([[3.0]]))
    assert np.array_equal(dQ[0, 0], 3.0 * D[0, 1])
    assert np.array_equal(dD[0, 1], 3.0 * Q[0, 0])
    assert np.all(dD[0, 0] == 0) and np.all(dD[0, 2] == 0)


def test_negative_indices_are_skipped_and_fp16_inputs_decode():
    rng = np.random.default_rng(5)
    Q = (np.round(rng.standard_normal((2, 3, 4)) * 8) / 8).astype(np.float16)
    D = (np.round(rng.standard_normal((2, 5, 4)) * 8) / 8).astype(np.float16)
    A = np.array([[[0, -1, 4], [2, 2, -1]], [[-1, -1, -1], [1, 0, 3]]], np.int32)
    g = rng.standard_normal((2, 2))
    dQ, dD = O.backward(Q, D, "f16", A, g)
    rQ = np.zeros((2, 3, 4))
    rD = np.zeros((2, 5, 4))
    for q in range(2):
        for b in range(2):
            for i in range(3):
                t = A[q, b, i]
                if t >= 0:
                    rQ[q, i] += g[q, b] * D[b, t].astype(np.float64)
                    rD[b, t] += g[q, b] * Q[q, i].astype(np.float64)
    assert np.allclose(dQ, rQ, atol=1e-14) and np.allclose(dD, rD, atol=1e-14)
    assert np.all(dQ[1, :, :] == g[1, 1] * D[1, [1, 0, 3]].astype(np.float64))


def test_cross_entropy_helper():
    rng = np.random.default_rng(6)
    s = rng.standard_normal((4, 6))
    tau = 0.5
    loss, g = O.ce_grad(s, tau)
    z = s / tau
    ref = np.mean(np.log(np.exp(z).sum(1)) - z[np.arange(4), np.arange(4)])
    assert abs(loss - ref) < 1e-12
    assert np.allclose(g.sum(1), 0, atol=1e-15)
    h = 1e-6
    for idx in np.ndindex(4, 6):
        sp, sm = s.copy(), s.copy()
        sp[idx] += h
        sm[idx] -= h
        fd = (O.ce_grad(sp, tau)[0] - O.ce_grad(sm, tau)[0]) / (2 * h)
        assert abs(fd - g[idx]) < 1e-8
    # one document only: softmax is 1, gradient vanishes, loss is 0
    l1, g1 = O.ce_grad(np.array([[3.7]]), 0.02)
    assert l1 == 0.0 and g1[0, 0] == 0.0
    # large scores at the paper-scale temperature stay finite
    l2, g2 = O.ce_grad(np.array([[30.0, 10.0], [5.0, 31.0]]), 0.02)
    assert np.isfinite(l2) and np.all(np.isfinite(g2))


def test_ragged_backward_against_the_definition_written_out():
    """Packed corpus: dQ[q,i] = sum_j g[q,j] D_j[A[q,j,i]], dD_j[t] = sum over edges landing on t of g[q,j] Q[q,i]."""
    rng = np.random.default_rng(5)
    n_q, l_q, d = 3, 4, 6
    lens = np.array([5, 0, 1, 7])
    off = np.concatenate([[0], np.cumsum(lens)])
    Q = rng.standard_normal((n_q, l_q, d)).astype(np.float32)
    Dp = rng.standard_normal((int(off[-1]), d)).astype(np.float32)
    g = rng.standard_normal((n_q, len(lens)))
    _, A, _ = O.forward(Q, Dp, "f32", offsets=off)
    assert np.all(A[:, 1] == -1)
    dQ, dD = O.backward_ragged(Q, Dp, "f32", off, A, g)
    rQ = np.zeros((n_q, l_q, d))
    rD = np.zeros((int(off[-1]), d))
    for q in range(n_q):
        for j in range(len(lens)):
            for i in range(l_q):
                t = A[q, j, i]
                if t < 0:
                    continue
                rQ[q, i] += g[q, j] * Dp[off[j] + t].astype(np.float64)
                rD[off[j] + t] += g[q, j] * Q[q, i].astype(np.float64)
    assert np.allclose(dQ, rQ, rtol=1e-12, atol=1e-12) and np.allclose(dD, rD, rtol=1e-12, atol=1e-12)
    # Euler identity (the score is homogeneous of degree one in Q and in D)
    s, _, _ = O.forward(Q, Dp, "f32", offsets=off)
    fin = np.isfinite(s)
    total = float((g[fin] * s[fin]).sum())
    assert abs((dQ * Q).sum() - total) < 1e-9 and abs((dD * Dp).sum() - total) < 1e-9
    # equal lengths: identical to the uniform routine
    D = rng.standard_normal((3, 5, d)).astype(np.float32)
    _, A2, _ = O.forward(Q, D, "f32")
    g2 = rng.standard_normal((n_q, 3))
    uQ, uD = O.backward(Q, D, "f32", A2, g2)
    pQ, pD = O.backward_ragged(Q, D.reshape(15, d), "f32", np.arange(4) * 5, A2, g2)
    assert np.allclose(pQ, uQ, rtol=0, atol=1e-12) and np.array_equal(pD.reshape(3, 5, d), uD)
