"""Pins for the oracle's int8 scoring (Alg. 4) and the per-token absmax quantiser.  No GPU."""
import numpy as np

from oracle import cpu_oracle as O


def test_integer_dot_against_numpy_int64():
    rng = np.random.default_rng(0)
    Q = rng.integers(-127, 128, (7, 128), dtype=np.int8)
    D = rng.integers(-127, 128, (9, 128), dtype=np.int8)
    n = O.dot_i8(Q, D)
    assert np.array_equal(n, Q.astype(np.int64) @ D.astype(np.int64).T)
    # extreme magnitude stays exact
    Qx = np.full((1, 128), -127, np.int8)
    Dx = np.full((1, 128), 127, np.int8)
    assert O.dot_i8(Qx, Dx)[0, 0] == -127 * 127 * 128


def test_unit_scales_give_exact_integer_scores():
    rng = np.random.default_rng(1)
    Q = rng.integers(-20, 21, (2, 5, 16), dtype=np.int8)
    D = rng.integers(-20, 21, (3, 7, 16), dtype=np.int8)
    s = O.forward_i8(Q, np.ones((2, 5), np.float32), D, np.ones((3, 7), np.float32), threads=2)
    n = np.einsum("qik,bjk->qbij", Q.astype(np.int64), D.astype(np.int64))
    assert np.array_equal(s.astype(np.int64), n.max(3).sum(2))
    assert s.dtype == np.float32


def test_matches_float_oracle_on_dequantised_values():
    """<Q_deq, D_deq> = q_s d_s <Q_i8, D_i8> (App. "INT8 Kernel")."""
    rng = np.random.default_rng(2)
    Qf = rng.standard_normal((2, 6, 32)).astype(np.float32)
    Df = rng.standard_normal((4, 9, 32)).astype(np.float32)
    Qi, qs = O.quantize_rows_i8(Qf, "f32")
    Di, ds = O.quantize_rows_i8(Df, "f32")
    s8 = O.forward_i8(Qi, qs, Di, ds)
    Qd = (Qi.astype(np.float64) * qs[..., None].astype(np.float64))
    Dd = (Di.astype(np.float64) * ds[..., None].astype(np.float64))
    S = np.einsum("qik,bjk->qbij", Qd, Dd)
    ref = S.max(3).sum(2)
    assert np.allclose(s8, ref, rtol=1e-6, atol=0)
    # and the order of operations the oracle fixes: per-cell d_s, max, then q_s, all in fp32
    n = np.einsum("qik,bjk->qbij", Qi.astype(np.int64), Di.astype(np.int64))
    v = (n.astype(np.float64) * ds[None, :, None, :].astype(np.float64)).astype(np.float32)
    m = v.max(3)
    r = (m.astype(np.float64) * qs[:, None, :].astype(np.float64)).astype(np.float32)
    assert np.array_equal(s8, r.astype(np.float64).sum(2).astype(np.float32))


def test_negative_maxima_and_scale_order():
    """The max is taken after the per-token document scale: a small-scale token can win."""
    Q = np.array([[[-1, 0]]], np.int8)
    D = np.array([[[10, 0], [1, 0]]], np.int8)  # dots: -10, -1
    s = O.forward_i8(Q, np.array([[2.0]], np.float32), D, np.array([[0.01, 1.0]], np.float32))
    assert s[0, 0] == np.float32(2.0) * np.float32(-10 * np.float32(0.01))


def test_quantiser_properties():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((50, 128)).astype(np.float32)
    X[7] = 0.0
    X[8, :] = 0.25  # every element is the absmax
    codes, s = O.quantize_rows_i8(X, "f32")
    a = np.abs(X).max(1)
    assert np.array_equal(s, (a.astype(np.float64) / 127.0).astype(np.float32))
    assert np.all(codes[7] == 0) and s[7] == 0.0
    assert np.all(codes[8] == 127)
    for r in range(50):
        if r == 7:
            continue
        assert np.abs(codes[r]).max() == 127
        assert np.abs(codes[r][np.abs(X[r]).argmax()]) == 127
        err = np.abs(codes[r].astype(np.float64) * float(s[r]) - X[r].astype(np.float64))
        assert err.max() <= 0.5 * float(s[r]) * (1 + 1e-6)
        assert np.array_equal(np.sign(codes[r]) * (codes[r] != 0), np.sign(X[r]) * (codes[r] != 0))


def test_quantiser_rounds_half_to_even_and_accepts_16bit():
    # absmax 127 -> scale exactly 1, so x/scale = x and halves are visible
    X = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49]], np.float32)
    codes, s = O.quantize_rows_i8(X, "f32")
    assert s[0] == 1.0
    assert codes[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 3]
    Xh = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5]], np.float16)
    ch, sh = O.quantize_rows_i8(Xh, "f16")
    assert sh[0] == 1.0 and ch[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 4]


def test_ragged_equals_uniform_when_lengths_are_equal_and_brute_force_otherwise():
    rng = np.random.default_rng(11)
    Q = rng.integers(-127, 128, (2, 5, 16), dtype=np.int8)
    qs = rng.random((2, 5)).astype(np.float32) + 0.1
    D = rng.integers(-127, 128, (4, 6, 16), dtype=np.int8)
    ds = rng.random((4, 6)).astype(np.float32) + 0.1
    off = np.arange(5) * 6
    s_r = O.forward_i8_ragged(Q, qs, D.reshape(24, 16), ds.reshape(24), off)
    assert np.array_equal(s_r.view(np.uint32), O.forward_i8(Q, qs, D, ds).view(np.uint32))
    # unequal lengths incl. an empty document: the definition written out with numpy (float32 per-cell scaling)
    off = np.array([0, 1, 1, 9, 24])
    s_r = O.forward_i8_ragged(Q, qs, D.reshape(24, 16), ds.reshape(24), off)
    assert np.all(np.isneginf(s_r[:, 1]))
    n = np.einsum("qik,tk->qit", Q.astype(np.int64), D.reshape(24, 16).astype(np.int64))
    for j in (0, 2, 3):
        v = (n[:, :, off[j]:off[j + 1]].astype(np.float64) * ds.reshape(24)[off[j]:off[j + 1]].astype(np.float64)).astype(np.float32)
        r = (qs.astype(np.float64) * v.max(2).astype(np.float64)).astype(np.float32)
        assert np.array_equal(s_r[:, j], r.astype(np.float64).sum(1).astype(np.float32))
