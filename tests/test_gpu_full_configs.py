"""Parity at the full sizes of the benchmark's configs, in the launch configuration bench.py times.

The oracle cannot run these sizes whole, so the GPU result is checked on sampled outputs the
oracle computes one by one (first, last, shortest, longest and random documents), plus
properties that hold at any size.
"""
import numpy as np
import pytest
import torch

from oracle import cpu_oracle as O
from paper_2605_29517_amd import binding as M
from paper_2605_29517_amd import workloads as W

from parity import ARGMAX_MARGIN, RTOL_16, check_argmax, check_scores, decode

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def sample_docs(n_docs, lengths=None, k=24, seed=0):
    rng = np.random.default_rng(seed)
    pick = {0, n_docs - 1}
    if lengths is not None:
        pick |= {int(np.argmin(lengths)), int(np.argmax(lengths))}
    pick |= set(int(x) for x in rng.integers(0, n_docs, k))
    return np.array(sorted(pick))


@pytest.fixture(scope="module")
def config2():
    Q, Dp, off, lens = W.colbert_rerank(device=DEV)
    return Q, Dp, off, lens.cpu().numpy()


@pytest.mark.parametrize("n_q", [1, 64])
def test_config2_ragged_rerank_full_size(config2, n_q):
    Q, Dp, off, lens = config2
    Qn = Q[:n_q].contiguous()
    n_docs = lens.shape[0]
    s = M.maxsim_forward_ragged(Qn, Dp, off)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(s).all())
    pick = sample_docs(n_docs, lens, k=40, seed=n_q)
    off_c = off.cpu().numpy().astype(np.int64)
    rows = np.concatenate([np.arange(off_c[d], off_c[d + 1]) for d in pick])
    sub_off = np.concatenate([[0], np.cumsum(lens[pick])]).astype(np.int32)
    Dsub = Dp[torch.from_numpy(rows).to(DEV)]
    ref, _, _ = O.forward(W.to_raw_numpy(Qn), W.to_raw_numpy(Dsub), "f16", offsets=sub_off, want_argmax=False,
                          want_margin=False)
    check_scores(s[:, torch.from_numpy(pick).to(DEV)], ref, 32, RTOL_16)
    # a score is a sum of 32 cosines of unit-norm rows
    assert float(s.abs().max()) <= 32.0 * 1.001


def test_config2_full_size_with_argmax_four_queries(config2):
    """Config 2 with four queries and the argmax output (the tile kernel's ragged argmax path at full size)."""
    Q, Dp, off, lens = config2
    Qn = Q[:4].contiguous()
    n_docs = lens.shape[0]
    s, a = M.maxsim_forward_ragged(Qn, Dp, off, want_argmax=True)
    s_plain = M.maxsim_forward_ragged(Qn, Dp, off)
    torch.cuda.synchronize()
    a_np = a.cpu().numpy()
    assert a_np.min() >= 0 and bool((a_np < lens[None, :, None]).all())
    assert float((s - s_plain).abs().max()) <= 2e-3 * 32      # with and without argmax: the same scores within the bar
    pick = sample_docs(n_docs, lens, k=60, seed=44)
    off_c = off.cpu().numpy().astype(np.int64)
    rows = np.concatenate([np.arange(off_c[d], off_c[d + 1]) for d in pick])
    sub_off = np.concatenate([[0], np.cumsum(lens[pick])]).astype(np.int32)
    Dsub = Dp[torch.from_numpy(rows).to(DEV)]
    ref, ra, rm = O.forward(W.to_raw_numpy(Qn), W.to_raw_numpy(Dsub), "f16", offsets=sub_off)
    pick_t = torch.from_numpy(pick).to(DEV)
    check_scores(s[:, pick_t], ref, 32, RTOL_16)
    Dd = decode(Dsub)
    check_argmax(a[:, pick_t], ra, rm, Qn, lambda b: Dd[sub_off[b]:sub_off[b + 1]])


def test_config3_colpali_page_as_query_full_size():
    Q, D = W.colpali_page_as_query(device=DEV)
    n_docs = D.shape[0]
    s = M.maxsim_forward(Q, D)
    s_a, a = M.maxsim_forward(Q, D, want_argmax=True)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(s).all())
    # 64 documents: first, last, drawn ones, and both sides of the borders between the runs of documents that
    # workgroups take (a run is ceil(10000 / n) documents for n a small multiple of the CU count)
    pick = set(int(x) for x in sample_docs(n_docs, k=24, seed=3))
    for per_run in (10, 20, 40, 79, 157):
        for k in (1, 3, n_docs // per_run):
            pick |= {min(n_docs - 1, k * per_run - 1), min(n_docs - 1, k * per_run)}
    pick = np.array(sorted(pick))[:64]
    pick_t = torch.from_numpy(pick).to(DEV)
    Dsub = D[pick_t]
    ref, ra, rm = O.forward(W.to_raw_numpy(Q), W.to_raw_numpy(Dsub), "bf16")
    check_scores(s[:, pick_t], ref, 1024, RTOL_16)
    check_scores(s_a[:, pick_t], ref, 1024, RTOL_16)
    Dd = decode(Dsub)
    check_argmax(a[:, pick_t], ra, rm, Q, lambda b: Dd[b])
    a_min, a_max = int(a.min()), int(a.max())
    assert a_min >= 0 and a_max < 1024
    # a score is a sum of 1024 cosines of unit-norm rows
    assert float(s.abs().max()) <= 1024.0 * 1.01


def test_config4_contrastive_step_full_size():
    n, l_q, l_d, tau = 256, 32, 1024, 0.02
    Q, D = W.contrastive_batch(n, l_q, l_d, device=DEV)
    s, a = M.maxsim_forward(Q, D, want_argmax=True)
    g, loss = M.maxsim_ce_grad(s, tau)
    torch.cuda.synchronize()
    a_np = a.cpu().numpy()
    assert a_np.min() >= 0 and a_np.max() < l_d
    Qr, Dr = W.to_raw_numpy(Q), W.to_raw_numpy(D)

    # forward on sampled documents (all queries) and sampled queries (all documents)
    docs = sample_docs(n, k=4, seed=4)
    qs = sample_docs(n, k=4, seed=5)
    ref_d, arg_d, mar_d = O.forward(Qr, Dr[docs], "f16")
    check_scores(s[:, torch.from_numpy(docs).to(DEV)], ref_d, l_q, RTOL_16)
    clear = mar_d > ARGMAX_MARGIN
    assert np.array_equal(a_np[:, docs][clear], arg_d[clear])
    ref_q, arg_q, mar_q = O.forward(Qr[qs], Dr, "f16")
    check_scores(s[torch.from_numpy(qs).to(DEV)], ref_q, l_q, RTOL_16)
    clear = mar_q > ARGMAX_MARGIN
    assert np.array_equal(a_np[qs][clear], arg_q[clear])

    # cross-entropy gradient on the GPU's own fp32 scores
    rloss, rg = O.ce_grad(s.cpu().numpy().astype(np.float64), tau)
    assert abs(float(loss) - rloss) <= 1e-5 * max(1.0, abs(rloss))
    assert np.abs(g.cpu().numpy() - rg).max() <= 1e-4 * np.abs(rg).max()

    # backward at full size.  The argmax handed to the GPU is its own, overwritten with the
    # oracle's on the sampled slices, so that the sampled gradient rows are a function of
    # oracle-side indices only.
    a_in = a_np.copy()
    a_in[:, docs] = arg_d
    a_in[qs] = arg_q
    g_np = g.cpu().numpy()
    dQ, dD = M.maxsim_backward(Q, D, torch.from_numpy(a_in).to(DEV), g)
    torch.cuda.synchronize()
    # dD of a document depends on that document's argmax column only
    _, rD = O.backward(Qr, Dr[docs], "f16", np.ascontiguousarray(a_in[:, docs]), g_np[:, docs].astype(np.float64))
    got = dD[torch.from_numpy(docs).to(DEV)].cpu().numpy()
    assert np.abs(got - rD).max() <= 1e-4 * np.abs(rD).max()
    # dQ of a query depends on that query's argmax rows only
    rQ, _ = O.backward(Qr[qs], Dr, "f16", np.ascontiguousarray(a_in[qs]), g_np[qs].astype(np.float64))
    got = dQ[torch.from_numpy(qs).to(DEV)].cpu().numpy()
    assert np.abs(got - rQ).max() <= 1e-4 * np.abs(rQ).max()
    # properties over the whole tensors: Euler identity (degree-one homogeneity) and column sums
    total = float((g.double() * s.double()).sum())
    eq = float((dQ.double() * Q.double()).sum())
    ed = float((dD.double() * D.double()).sum())
    scale = float((g.double().abs() * s.double().abs()).sum())
    assert abs(eq - total) <= 1e-4 * scale and abs(ed - total) <= 1e-4 * scale
    col = torch.einsum("ij,ik->jk", g.double(), Q.double().sum(1))
    assert float((dD.double().sum(1) - col).abs().max()) <= 1e-4 * float(col.abs().max())

    # the explicit CSR at full size: the whole structure against the oracle's (integer work, bit-exact), and the
    # gradients through it against the default backward (same summation order and arithmetic: same bits)
    a_dev = torch.from_numpy(a_in).to(DEV)
    cQ, cD, row_ptr, col_idx = M.maxsim_backward_csr(Q, D, a_dev, g)
    torch.cuda.synchronize()
    rp, ci = O.csr_build(a_in, l_d)
    assert np.array_equal(row_ptr.cpu().numpy(), rp)
    assert np.array_equal(col_idx.cpu().numpy()[:rp[-1]], ci)
    assert torch.equal(cQ, dQ) and torch.equal(cD, dD)


def test_config5_int8_corpus_full_size():
    n_docs, l, chunk = 400_000, 1024, 10_000
    Qh = W.int8_query(l, device=DEV)
    D8 = torch.empty(n_docs, l, 128, dtype=torch.int8, device=DEV)
    ds = torch.empty(n_docs, l, dtype=torch.float32, device=DEV)
    for ci in range(n_docs // chunk):
        X = W.int8_corpus_chunk(ci, chunk, l, device=DEV)
        M.maxsim_quantize_rows_i8(X, X_i8=D8[ci * chunk:(ci + 1) * chunk], scale=ds[ci * chunk:(ci + 1) * chunk])
        del X
    Q8, qs = M.maxsim_quantize_rows_i8(Qh)
    s = M.maxsim_forward_i8(Q8, qs, D8, ds)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(s).all())
    # the oracle quantises its own copies of the float rows of the sampled documents
    oq, oqs = O.quantize_rows_i8(W.to_raw_numpy(Qh), "f16")
    assert np.array_equal(Q8.cpu().numpy(), oq)
    assert np.array_equal(qs.cpu().numpy().view(np.uint32), oqs.view(np.uint32))
    pick = sample_docs(n_docs, k=10, seed=5)
    for d in pick:
        ci, within = divmod(int(d), chunk)
        X = W.int8_corpus_chunk(ci, chunk, l, device=DEV)[within].cpu()
        od, ods = O.quantize_rows_i8(W.to_raw_numpy(X), "f32")
        assert np.array_equal(D8[d].cpu().numpy(), od)
        assert np.array_equal(ds[d].cpu().numpy().view(np.uint32), ods.view(np.uint32))
        ref = O.forward_i8(oq, oqs, od[None], ods[None])
        assert ref.view(np.uint32)[0, 0] == s[0, d].cpu().numpy().view(np.uint32), int(d)
