"""Pins for the oracle's forward (Eq. 1, tie rule, ragged layout).  No GPU.

Each pin is something other than the oracle's own formula: a materialise-then-reduce
brute force written independently (Listing 1's order), a hand-computed integer case,
closed forms and invariants of the operator.
"""
import os

import numpy as np
import pytest

from oracle import cpu_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_force(Q, D):
    """Listing 1 in slow motion: build S[q,b,i,j] with python floats (k ascending), then
    max over j (first occurrence), then sum over i."""
    n_q, l_q, d = Q.shape
    b, l_d, _ = D.shape
    S = np.zeros((n_q, b, l_q, l_d))
    for q in range(n_q):
        for x in range(b):
            for i in range(l_q):
                for j in range(l_d):
                    s = 0.0
                    for k in range(d):
                        s += float(Q[q, i, k]) * float(D[x, j, k])
                    S[q, x, i, j] = s
    mx = S.max(axis=3)
    am = S.argmax(axis=3)  # numpy: first occurrence
    scores = np.zeros((n_q, b))
    for q in range(n_q):
        for x in range(b):
            t = 0.0
            for i in range(l_q):
                t += mx[q, x, i]
            scores[q, x] = t
    srt = np.sort(S, axis=3)
    margin = srt[..., -1] - srt[..., -2] if l_d > 1 else np.full(mx.shape, np.inf)
    return scores, am.astype(np.int32), margin


def unit(rng, *shape):
    x = rng.standard_normal(shape).astype(np.float32)
    return x / np.linalg.norm(x, axis=-1, keepdims=True).astype(np.float32)


def test_hand_example_from_fixture():
    lines = [l for l in open(os.path.join(GOLDEN, "hand_example.txt")) if not l.startswith("#")]
    it = iter(lines)
    mats = {}
    out = {}
    for line in it:
        tok = line.split()
        if tok[0] in ("Q", "D"):
            r, c = int(tok[1]), int(tok[2])
            mats[tok[0]] = np.array([[float(v) for v in next(it).split()] for _ in range(r)], np.float32)
            assert mats[tok[0]].shape == (r, c)
        else:
            out[tok[0]] = [float(v) for v in tok[1:]]
    s, a, m = O.forward(mats["Q"][None], mats["D"][None], "f32")
    assert s[0, 0] == out["score"][0]
    assert a[0, 0].tolist() == [int(v) for v in out["argmax"]]
    assert m[0, 0].tolist() == out["margin"]
    # the same data in fp16 and bf16 storage (small integers are exact in both)
    s16, a16, _ = O.forward(mats["Q"][None].astype(np.float16), mats["D"][None].astype(np.float16), "f16")
    assert s16[0, 0] == out["score"][0] and a16[0, 0].tolist() == a[0, 0].tolist()
    import torch
    qb = torch.from_numpy(mats["Q"][None]).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    db = torch.from_numpy(mats["D"][None]).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    sb, ab, _ = O.forward(qb, db, "bf16")
    assert sb[0, 0] == out["score"][0] and ab[0, 0].tolist() == a[0, 0].tolist()


@pytest.mark.parametrize("shape", [(1, 1, 1, 1, 1), (2, 3, 5, 7, 4), (3, 4, 2, 6, 3), (1, 2, 4, 1, 5)])
def test_brute_force_bit_for_bit(shape):
    n_q, b, l_q, l_d, d = shape
    rng = np.random.default_rng(100 + sum(shape))
    Q = rng.standard_normal((n_q, l_q, d)).astype(np.float32)
    D = rng.standard_normal((b, l_d, d)).astype(np.float32)
    s, a, m = O.forward(Q, D, "f32", threads=3)
    bs, ba, bm = brute_force(Q, D)
    assert np.array_equal(s, bs)  # bit for bit in fp64
    assert np.array_equal(a, ba)
    assert np.array_equal(m, bm)


def test_brute_force_fp16_inputs():
    rng = np.random.default_rng(7)
    Q = rng.standard_normal((2, 3, 4)).astype(np.float16)
    D = rng.standard_normal((3, 5, 4)).astype(np.float16)
    s, a, _ = O.forward(Q, D, "f16")
    bs, ba, _ = brute_force(Q.astype(np.float64), D.astype(np.float64))
    assert np.array_equal(s, bs) and np.array_equal(a, ba)


def test_single_token_document_closed_form():
    rng = np.random.default_rng(1)
    Q = unit(rng, 2, 9, 16)
    D = unit(rng, 5, 1, 16)
    s, a, m = O.forward(Q, D, "f32")
    ref = np.einsum("qk,bk->qb", Q.astype(np.float64).sum(1), D[:, 0].astype(np.float64))
    assert np.allclose(s, ref, rtol=0, atol=1e-13)
    assert np.all(a == 0) and np.all(np.isinf(m))


def test_single_query_token_is_plain_max():
    rng = np.random.default_rng(2)
    Q = unit(rng, 1, 1, 8)
    D = unit(rng, 4, 11, 8)
    s, a, _ = O.forward(Q, D, "f32")
    S = D.astype(np.float64) @ Q[0, 0].astype(np.float64)
    assert np.allclose(s[0], S.max(1), atol=1e-14)
    assert np.array_equal(a[0, :, 0], S.argmax(1))


def test_permuting_document_tokens():
    rng = np.random.default_rng(3)
    Q = unit(rng, 2, 6, 16)
    D = unit(rng, 3, 13, 16)
    s, a, _ = O.forward(Q, D, "f32")
    perm = rng.permutation(13)
    Dp = D[:, perm]
    sp, ap, _ = O.forward(Q, Dp, "f32")
    # each max is over the same set of fp64 values, so the score is bit-identical
    assert np.array_equal(s, sp)
    assert np.array_equal(perm[ap], a)


def test_document_contains_query_unit_rows():
    rng = np.random.default_rng(4)
    Q = unit(rng, 1, 5, 32)
    D = unit(rng, 2, 20, 32)
    pos = np.array([3, 17, 0, 9, 12])
    D[1, pos] = Q[0]
    s, a, _ = O.forward(Q, D, "f32")
    norms = (Q[0].astype(np.float64) ** 2).sum()
    assert abs(s[0, 1] - norms) < 1e-13  # Cauchy-Schwarz: nothing beats the copy
    assert abs(s[0, 1] - 5.0) < 1e-5
    assert np.array_equal(a[0, 1], pos)
    assert s[0, 0] < s[0, 1]


def test_chunk_additivity_over_query_tokens():
    rng = np.random.default_rng(5)
    Q = unit(rng, 1, 10, 16)
    D = unit(rng, 4, 9, 16)
    s, a, _ = O.forward(Q, D, "f32")
    s1, a1, _ = O.forward(Q[:, :4], D, "f32")
    s2, a2, _ = O.forward(Q[:, 4:], D, "f32")
    assert np.allclose(s, s1 + s2, atol=1e-14)
    assert np.array_equal(a, np.concatenate([a1, a2], axis=2))


def test_homogeneity_monotonicity_duplicates():
    rng = np.random.default_rng(6)
    Q = unit(rng, 2, 4, 8)
    D = unit(rng, 3, 6, 8)
    s, a, _ = O.forward(Q, D, "f32")
    s2, a2, _ = O.forward((Q * np.float32(2.0)), D, "f32")  # exact scaling by a power of two
    assert np.array_equal(s2, 2.0 * s) and np.array_equal(a, a2)
    # adding tokens can only raise each max
    Dm = np.concatenate([D, unit(rng, 3, 3, 8)], axis=1)
    sm, _, _ = O.forward(Q, Dm, "f32")
    assert np.all(sm >= s)
    # appending copies of existing tokens changes nothing; the first copy keeps the argmax
    Dd = np.concatenate([D, D[:, ::-1]], axis=1)
    sd, ad, md = O.forward(Q, Dd, "f32")
    assert np.array_equal(sd, s) and np.array_equal(ad, a)
    assert np.all(md == 0.0)


def test_sign_and_transpose_sensitivity():
    """A flipped sign or swapped operand roles must change the answer on this input."""
    Q = np.array([[[1.0, 2.0]]], np.float32)
    D = np.array([[[1.0, 0.0], [-3.0, 0.0], [0.0, 1.0]]], np.float32)
    s, a, m = O.forward(Q, D, "f32")
    assert s[0, 0] == 2.0 and a[0, 0, 0] == 2 and m[0, 0, 0] == 1.0
    # roles swapped (3 "query" tokens against 1 "document" token): sum of all three products
    s2, _, _ = O.forward(D, Q, "f32")
    assert s2[0, 0] == 1.0 - 3.0 + 2.0


def test_ragged_equals_uniform_and_per_doc_calls():
    rng = np.random.default_rng(8)
    Q = unit(rng, 2, 5, 16)
    D = unit(rng, 4, 7, 16)
    s, a, m = O.forward(Q, D, "f32")
    off = np.arange(5, dtype=np.int32) * 7
    sr, ar, mr = O.forward(Q, D.reshape(-1, 16), "f32", offsets=off)
    assert np.array_equal(s, sr) and np.array_equal(a, ar) and np.array_equal(m, mr)
    lens = [1, 31, 32, 33, 2]
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    Dp = unit(rng, int(off[-1]), 16)
    sr, ar, _ = O.forward(Q, Dp, "f32", offsets=off, threads=2)
    for x, n in enumerate(lens):
        su, au, _ = O.forward(Q, Dp[off[x]:off[x + 1]][None], "f32")
        assert np.array_equal(sr[:, x], su[:, 0])
        assert np.array_equal(ar[:, x], au[:, 0])
        assert ar[:, x].max() < n


def test_empty_document_in_ragged_corpus():
    rng = np.random.default_rng(9)
    Q = unit(rng, 1, 3, 8)
    Dp = unit(rng, 5, 8)
    off = np.array([0, 2, 2, 5], np.int32)
    s, a, _ = O.forward(Q, Dp, "f32", offsets=off)
    assert s[0, 1] == -np.inf and np.all(a[0, 1] == -1)
    assert np.isfinite(s[0, 0]) and np.isfinite(s[0, 2])


def test_thread_count_does_not_matter():
    rng = np.random.default_rng(10)
    Q = unit(rng, 2, 4, 8)
    D = unit(rng, 9, 5, 8)
    r1 = O.forward(Q, D, "f32", threads=1)
    r5 = O.forward(Q, D, "f32", threads=5)
    for x, y in zip(r1, r5):
        assert np.array_equal(x, y)


def test_paper_size_figures():
    """The byte model used for the roofline numbers reproduces the sizes the paper prints."""
    vals = {}
    for line in open(os.path.join(GOLDEN, "paper_sizes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, v, unit_ = line.split("|")[0].split()
        vals[key] = (float(v), unit_)
    d = 128
    assert round(1000 * 1024 * d * 2 / 1e9, 2) == vals["fused_traffic_colpali_b1000"][0]
    assert round(10000 * 1024 * 1024 * 2 / 1e9) == vals["unfused_S_colpali_b10000_fp16"][0]
    assert round(10000 * 1024 * 1024 * 4 / 1e9) == vals["unfused_S_colpali_b10000_fp32"][0]
    assert round(64 * 64 * 1024 * 4 / 2 ** 20) == vals["argmax_colpali_b64"][0]
    assert round(128 * 128 * 1024 * 4 / 2 ** 20) == vals["argmax_colpali_b128"][0]
