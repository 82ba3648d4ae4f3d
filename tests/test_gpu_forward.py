"""GPU parity of maxsim_forward / maxsim_forward_ragged against the CPU oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

from paper_2605_29517_amd import binding as M
from paper_2605_29517_amd import workloads as W

from parity import RTOL_16, RTOL_F32, forward_parity_ragged, forward_parity_uniform

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_config1_tiny_fp32_with_argmax():
    Q, D = W.tiny_forward()
    worst = forward_parity_uniform(Q.to(DEV), D.to(DEV), M.maxsim_forward, True, RTOL_F32)
    print("config 1 max rel err %.2e" % worst)


# (n_q, l_q, b, l_d): streaming kernel (<= 4 column blocks), every tile-kernel width, ragged tails,
# single-token documents, one document, a query longer than one workgroup's 1024 tokens
SHAPES = [
    (1, 32, 37, 128), (1, 1, 5, 1), (1, 31, 9, 33), (2, 33, 11, 31), (4, 32, 50, 100), (1, 100, 20, 65),
    (3, 17, 1, 300), (8, 32, 40, 64), (5, 40, 13, 97), (16, 32, 70, 200), (2, 256, 9, 130),
    (64, 32, 33, 150), (1, 1024, 6, 260), (3, 700, 5, 95), (1, 1100, 4, 70), (2, 2100, 3, 40),
    # several wavefronts of the streaming kernel sharing a run of documents (2, 3 and 4 groups)
    (12, 32, 45, 130), (3, 64, 21, 77), (4, 96, 17, 140), (7, 50, 30, 33), (6, 1, 9, 5),
    # one long query of 5-16 blocks: tile kernel with one or two blocks per wavefront and a ring of tiles in flight
    (1, 200, 7, 90), (1, 256, 5, 64), (1, 300, 4, 100), (1, 512, 3, 70), (2, 160, 9, 45),
]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("want_argmax", [False, True])
@pytest.mark.parametrize("shape", SHAPES)
def test_uniform_16bit(shape, want_argmax, dtype):
    n_q, l_q, b, l_d = shape
    Q = W.unit_rows((n_q, l_q, 128), dtype, 11 + l_q, DEV)
    D = W.unit_rows((b, l_d, 128), dtype, 12 + l_d, DEV)
    forward_parity_uniform(Q, D, M.maxsim_forward, want_argmax, RTOL_16)


@pytest.mark.parametrize("want_argmax", [False, True])
@pytest.mark.parametrize("shape", [(1, 32, 9, 40), (2, 32, 7, 33), (3, 32, 21, 100), (9, 20, 30, 70), (40, 32, 5, 64)])
def test_uniform_fp32(shape, want_argmax):
    n_q, l_q, b, l_d = shape
    Q = W.unit_rows((n_q, l_q, 128), "f32", 21, DEV)
    D = W.unit_rows((b, l_d, 128), "f32", 22, DEV)
    forward_parity_uniform(Q, D, M.maxsim_forward, want_argmax, RTOL_F32)


def _ragged_case(n_q, l_q, lens, dtype, seed):
    lens = np.asarray(lens)
    off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(DEV)
    Dp = W.unit_rows((int(lens.sum()), 128), dtype, seed, DEV)
    Q = W.unit_rows((n_q, l_q, 128), dtype, seed + 1, DEV)
    return Q, Dp, off


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("want_argmax", [False, True])
@pytest.mark.parametrize("n_q,l_q", [(1, 32), (3, 32), (5, 32), (8, 30), (3, 40), (7, 33), (64, 32), (2, 300)])
def test_ragged_edge_lengths(n_q, l_q, want_argmax, dtype):
    lens = [1, 31, 32, 33, 0, 64, 300, 0, 0, 2, 65, 128, 1, 97]
    Q, Dp, off = _ragged_case(n_q, l_q, lens, dtype, 31)
    forward_parity_ragged(Q, Dp, off, M.maxsim_forward_ragged, want_argmax, RTOL_F32 if dtype == "f32" else RTOL_16)


@pytest.mark.parametrize("n_q", [1, 4, 6, 64])
def test_ragged_colbert_like(n_q):
    Q, Dp, off, _ = W.colbert_rerank(n_q=n_q, n_docs=700, device=DEV)
    forward_parity_ragged(Q, Dp, off, M.maxsim_forward_ragged, n_q == 4, RTOL_16)


def test_leading_and_trailing_empty_documents():
    Q, Dp, off = _ragged_case(2, 32, [0, 0, 5, 0, 40, 0, 0], "f16", 41)
    forward_parity_ragged(Q, Dp, off, M.maxsim_forward_ragged, True, RTOL_16)


def test_duplicate_tokens_keep_first_index():
    """Exact ties: the lowest index wins ("Tied maxima"), also across tiles and lane halves."""
    Q = W.unit_rows((1, 32, 128), "f16", 51, DEV)
    base = W.unit_rows((1, 5, 128), "f16", 52, DEV)
    D = base.repeat(1, 20, 1).contiguous()  # 100 tokens, every token repeated 20 times, period 5
    s, a = M.maxsim_forward(Q, D, want_argmax=True)
    torch.cuda.synchronize()
    assert int(a.max()) < 5
    s1, a1 = M.maxsim_forward(Q, base.contiguous(), want_argmax=True)
    torch.cuda.synchronize()
    assert torch.equal(a, a1) and torch.equal(s, s1)


# Similarities that are negative throughout, partly, or shifted per document (token rows of real encoders share a
# mean direction): the argmax fold of the tile kernel orders cells through their bit patterns, which is only right
# among non-negative values, and falls back to compare-and-select while a running maximum is negative.
# (n_q, l_q, b, l_d): tile kernel with 4, 2 and 1 blocks per wavefront; streaming kernel; ragged
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("shape", [(40, 32, 6, 200), (2, 256, 5, 130), (1, 1024, 3, 100), (1, 200, 4, 90), (2, 32, 9, 70)])
@pytest.mark.parametrize("q_bias,d_bias", [(1.0, -1.0), (0.6, 0.6), (0.4, -0.2)])
def test_argmax_with_negative_and_shifted_similarities(shape, q_bias, d_bias, dtype):
    n_q, l_q, b, l_d = shape
    Q = W.biased_rows((n_q, l_q, 128), dtype, 61, DEV, bias=q_bias)
    D = W.biased_rows((b, l_d, 128), dtype, 62, DEV, bias=d_bias)
    D[b // 2:] = W.biased_rows((b - b // 2, l_d, 128), dtype, 63, DEV, bias=-d_bias)   # half of the documents the other way
    rtol = RTOL_F32 if dtype == "f32" else RTOL_16
    forward_parity_uniform(Q, D.contiguous(), M.maxsim_forward, True, rtol)
    lens = np.array([l_d, 1, 33, 0, l_d // 2, 70])
    off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(DEV)
    Dp = W.biased_rows((int(lens.sum()), 128), dtype, 64, DEV, bias=d_bias)
    forward_parity_ragged(Q, Dp, off, M.maxsim_forward_ragged, True, rtol)


# Rows that are not unit-norm (the ABI does not ask for it): similarities of 1e-6 and of 1e+6
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("want_argmax", [False, True])
@pytest.mark.parametrize("scale", [1e-3, 30.0, 1e3])
@pytest.mark.parametrize("shape", [(40, 32, 6, 200), (1, 32, 20, 100), (3, 300, 4, 70)])
def test_rows_that_are_not_unit_norm(shape, scale, want_argmax, dtype):
    if dtype == "f16" and scale > 100:
        pytest.skip("fp16 cannot hold rows of that magnitude times each other")
    n_q, l_q, b, l_d = shape
    Q = W.biased_rows((n_q, l_q, 128), dtype, 71, DEV, bias=0.3, scale=scale)
    D = W.biased_rows((b, l_d, 128), dtype, 72, DEV, bias=-0.1, scale=scale)
    # the absolute slack for scores that sit at zero scales with the similarities (scale^2)
    forward_parity_uniform(Q, D, M.maxsim_forward, want_argmax, RTOL_F32 if dtype == "f32" else RTOL_16,
                           atol_per_token=1e-6 * scale * scale)


def test_argument_errors():
    Q = W.unit_rows((1, 32, 128), "f16", 1, DEV)
    D = W.unit_rows((4, 40, 128), "f16", 2, DEV)
    with pytest.raises(M.MaxSimError):
        M.maxsim_forward(Q.cpu(), D)
    with pytest.raises(M.MaxSimError):
        M.maxsim_forward(Q[..., :100].contiguous(), D[..., :100].contiguous())  # rows of 200 bytes: not a multiple of 64
    L = M.load()
    assert L.maxsim_forward(None, 1, 32, None, 4, 40, 128, 1, None, None, None) == -1


# Other embedding widths (rows of 128, 512 and 1024 bytes): stream and tile kernels, several passes, ragged, argmax
WIDTH_SHAPES = [(1, 32, 9, 40), (3, 17, 5, 100), (8, 32, 12, 65), (2, 200, 6, 130), (1, 1030, 3, 70), (40, 32, 7, 33)]


@pytest.mark.parametrize("dtype,d", [("f16", 64), ("f16", 256), ("f16", 512), ("bf16", 64), ("bf16", 256), ("bf16", 512),
                                     ("f32", 64), ("f32", 256)])
@pytest.mark.parametrize("want_argmax", [False, True])
@pytest.mark.parametrize("shape", WIDTH_SHAPES)
def test_uniform_other_widths(shape, want_argmax, dtype, d):
    n_q, l_q, b, l_d = shape
    Q = W.unit_rows((n_q, l_q, d), dtype, 61 + l_q, DEV)
    D = W.unit_rows((b, l_d, d), dtype, 62 + l_d, DEV)
    forward_parity_uniform(Q, D, M.maxsim_forward, want_argmax, RTOL_F32 if dtype == "f32" else RTOL_16)


@pytest.mark.parametrize("dtype,d", [("f16", 64), ("bf16", 256), ("f16", 512), ("f32", 256)])
@pytest.mark.parametrize("n_q,l_q", [(1, 32), (5, 40), (2, 300)])
def test_ragged_other_widths(n_q, l_q, dtype, d):
    lens = np.asarray([1, 31, 32, 33, 0, 64, 150, 0, 2, 65, 97])
    off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(DEV)
    Dp = W.unit_rows((int(lens.sum()), d), dtype, 71, DEV)
    Q = W.unit_rows((n_q, l_q, d), dtype, 72, DEV)
    forward_parity_ragged(Q, Dp, off, M.maxsim_forward_ragged, True, RTOL_F32 if dtype == "f32" else RTOL_16)


# Widths without a register-stationary kernel go through the slab-streaming ("split-d") kernel: rows that are any
# multiple of 64 bytes.  Shapes: one block, ragged column tail, more than one group of 16 blocks (several queries),
# a query of more than 16 blocks (two passes), documents shorter and longer than a macro tile of 128 tokens.
SPLITD_SHAPES = [(1, 32, 9, 40), (3, 17, 5, 300), (8, 32, 12, 65), (2, 200, 6, 130), (1, 1030, 3, 70), (40, 32, 7, 33),
                 (3, 600, 4, 257)]
SPLITD_WIDTHS = [("f16", 32), ("f16", 96), ("bf16", 160), ("f16", 384), ("bf16", 768), ("f16", 1024), ("bf16", 2048),
                 ("f32", 48), ("f32", 80), ("f32", 512)]


@pytest.mark.parametrize("dtype,d", SPLITD_WIDTHS)
@pytest.mark.parametrize("want_argmax", [False, True])
@pytest.mark.parametrize("shape", SPLITD_SHAPES)
def test_uniform_split_d(shape, want_argmax, dtype, d):
    n_q, l_q, b, l_d = shape
    Q = W.unit_rows((n_q, l_q, d), dtype, 81 + l_q, DEV)
    D = W.unit_rows((b, l_d, d), dtype, 82 + l_d, DEV)
    forward_parity_uniform(Q, D, M.maxsim_forward, want_argmax, RTOL_F32 if dtype == "f32" else RTOL_16)


@pytest.mark.parametrize("dtype,d", [("f16", 96), ("bf16", 768), ("f16", 1024), ("f32", 48)])
@pytest.mark.parametrize("n_q,l_q", [(1, 32), (5, 40), (2, 300), (1, 700)])
def test_ragged_split_d(n_q, l_q, dtype, d):
    lens = np.asarray([1, 31, 32, 33, 0, 64, 150, 0, 2, 65, 97, 128, 129, 300])
    off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(DEV)
    Dp = W.unit_rows((int(lens.sum()), d), dtype, 91, DEV)
    Q = W.unit_rows((n_q, l_q, d), dtype, 92, DEV)
    forward_parity_ragged(Q, Dp, off, M.maxsim_forward_ragged, True, RTOL_F32 if dtype == "f32" else RTOL_16)


# Ragged corpora scored by more than 16 queries of one column block take 32-row windows over the packed rows (a window
# may hold the end of one document and the start of the next).  Length mixes: runs of tiny documents (several
# boundaries close together, a document that lies inside one window whole), empty documents at the start, in a row
# and at the end, lengths around the window size, and long documents.
PACK_LENGTHS = {
    "tiny": [1, 1, 1, 2, 1, 3, 1, 1, 5, 1, 1, 1, 40, 1, 1],
    "empties": [0, 0, 7, 0, 33, 0, 0, 0, 31, 1, 0, 64, 0],
    "window": [32, 32, 31, 33, 1, 63, 64, 65, 32, 16, 16, 16, 16],
    "long": [300, 64, 129, 5, 700, 31, 257],
}


@pytest.mark.parametrize("dtype,d", [("f16", 128), ("bf16", 128), ("f16", 64), ("f32", 64)])
@pytest.mark.parametrize("n_q,l_q", [(5, 32), (6, 9), (7, 32), (8, 31), (9, 32), (10, 32), (12, 7), (13, 32), (16, 32), (17, 32), (40, 20), (64, 32), (33, 1)])
@pytest.mark.parametrize("mix", sorted(PACK_LENGTHS))
def test_ragged_packed_windows(mix, n_q, l_q, dtype, d):
    lens = np.asarray(PACK_LENGTHS[mix] * 3)
    off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(DEV)
    Dp = W.unit_rows((int(lens.sum()), d), dtype, 101, DEV)
    Q = W.unit_rows((n_q, l_q, d), dtype, 102, DEV)
    forward_parity_ragged(Q, Dp, off, M.maxsim_forward_ragged, False, RTOL_F32 if dtype == "f32" else RTOL_16)


@pytest.mark.parametrize("n_q", [6, 8, 11, 48])
def test_ragged_packed_windows_many_chunks(n_q):
    # enough documents that every workgroup gets its own chunk, with chunk borders inside runs of short documents
    # (workgroups of two, four and eight wavefronts)
    rng = np.random.default_rng(7)
    lens = rng.integers(0, 90, size=6000)
    off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(DEV)
    Dp = W.unit_rows((int(lens.sum()), 128), "f16", 103, DEV)
    Q = W.unit_rows((n_q, 32, 128), "f16", 104, DEV)
    forward_parity_ragged(Q, Dp, off, M.maxsim_forward_ragged, False, RTOL_16)


@pytest.mark.parametrize("dtype,d", [("f16", 128), ("bf16", 64)])
@pytest.mark.parametrize("n_q,l_q", [(5, 32), (8, 32), (11, 32), (14, 3), (17, 32), (64, 20)])
@pytest.mark.parametrize("b,l_d", [(50, 1), (33, 7), (21, 33), (40, 100), (9, 300), (700, 45), (30, 64), (12, 256), (3000, 32)])
def test_uniform_packed_windows(b, l_d, n_q, l_q, dtype, d):
    """Uniform corpora whose documents are not a whole number of 32-row tiles take the packed windows as well, and so
    do corpora of whole tiles at 5-16 queries."""
    Q = W.unit_rows((n_q, l_q, d), dtype, 111, DEV)
    D = W.unit_rows((b, l_d, d), dtype, 112, DEV)
    forward_parity_uniform(Q, D, M.maxsim_forward, False, RTOL_16)


# Five to sixteen column blocks on a corpus of thousands of documents: the workgroups of two and four wavefronts with
# four blocks each (tile kernel: argmax or queries of several blocks; packed windows otherwise), uniform and ragged.
@pytest.mark.parametrize("dtype,d", [("f16", 128), ("bf16", 128), ("f32", 64)])
@pytest.mark.parametrize("n_q,l_q,want_argmax", [(1, 200, False), (1, 256, True), (3, 130, True), (2, 250, False), (7, 32, True),
                                                 (12, 32, True), (6, 32, False), (14, 20, False)])
@pytest.mark.parametrize("ragged", [False, True])
def test_mid_block_counts_on_many_documents(ragged, n_q, l_q, want_argmax, dtype, d):
    b = 4500
    rtol = RTOL_F32 if dtype == "f32" else RTOL_16
    Q = W.unit_rows((n_q, l_q, d), dtype, 131, DEV)
    if ragged:
        lens = np.random.default_rng(n_q * 1000 + l_q).integers(0, 50, size=b)
        lens[:3] = [0, 33, 1]
        off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(DEV)
        Dp = W.unit_rows((int(lens.sum()), d), dtype, 132, DEV)
        forward_parity_ragged(Q, Dp, off, M.maxsim_forward_ragged, want_argmax, rtol)
    else:
        D = W.unit_rows((b, 32 if l_q > 100 else 40, d), dtype, 132, DEV)
        forward_parity_uniform(Q, D, M.maxsim_forward, want_argmax, rtol)
