"""The library only enqueues kernels on the caller's stream (no allocation, no memset, no synchronisation), so a
training step can be captured into a HIP graph.  Replays are interleaved with eager work and synchronisations and
every replay must reproduce the eager result bit for bit (the kernels are deterministic)."""
import numpy as np
import pytest
import torch

from paper_2605_29517_amd import binding as M
from paper_2605_29517_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_training_step_replays_from_a_graph():
    n, l_q, l_d = 24, 32, 200
    Q, D = W.contrastive_batch(n, l_q, l_d, device=DEV)
    s = torch.empty(n, n, device=DEV)
    a = torch.empty(n, n, l_q, dtype=torch.int32, device=DEV)
    g = torch.empty(n, n, device=DEV)
    loss = torch.empty(1, device=DEV)
    dQ = torch.empty(n, l_q, 128, device=DEV)
    dD = torch.empty(n, l_d, 128, device=DEV)
    q8 = torch.empty(n, l_q, 128, dtype=torch.int8, device=DEV)
    qs = torch.empty(n, l_q, device=DEV)
    d8, ds = M.maxsim_quantize_rows_i8(D)
    s8 = torch.empty(n, n, device=DEV)
    # a corpus large enough for the document-stationary int8 kernel (dynamic LDS above 64 KB)
    big8, bigs = M.maxsim_quantize_rows_i8(W.unit_rows((4200, 40, 128), "f32", 8, DEV))
    s8b = torch.empty(n, 4200, device=DEV)
    cQ = torch.empty(n, l_q, 128, device=DEV)
    cD = torch.empty(n, l_d, 128, device=DEV)
    row_ptr = torch.empty(n * l_d + 1, dtype=torch.int32, device=DEV)
    col_idx = torch.empty(n * n * l_q, dtype=torch.int32, device=DEV)
    outs = (s, a, g, loss, dQ, dD, s8, s8b, cQ, cD, row_ptr, col_idx)

    def step():
        M.maxsim_forward(Q, D, scores=s, argmax=a)
        M.maxsim_ce_grad(s, 0.02, g=g, loss=loss)
        M.maxsim_backward(Q, D, a, g, dQ=dQ, dD=dD)
        M.maxsim_quantize_rows_i8(Q, X_i8=q8, scale=qs)
        M.maxsim_forward_i8(q8, qs, d8, ds, scores=s8)
        M.maxsim_forward_i8(q8, qs, big8, bigs, scores=s8b)
        M.maxsim_backward_csr(Q, D, a, g, row_ptr=row_ptr, col_idx=col_idx, dQ=cQ, dD=cD)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in outs]
    assert torch.equal(cQ, dQ) and torch.equal(cD, dD)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()  # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(4):
        for t in outs:
            t.fill_(0) if t.dtype != torch.int32 else t.fill_(-7)   # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outs, want):
            assert torch.equal(got, ref), "replay %d differs from the eager result" % rep


def test_forward_variants_replay_from_a_graph():
    """The packed-window kernel (ragged corpus, many short queries) and the slab kernel (wide rows, more than
    64 KB of dynamic LDS) under capture, after one eager call each."""
    lens = np.asarray([5, 0, 64, 33, 1, 1, 200, 31, 90] * 4)
    off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(DEV)
    Dp = W.unit_rows((int(lens.sum()), 128), "f16", 21, DEV)
    Qs = W.unit_rows((40, 32, 128), "f16", 22, DEV)
    Qw = W.unit_rows((2, 70, 768), "bf16", 23, DEV)
    Dw = W.unit_rows((9, 150, 768), "bf16", 24, DEV)
    s1 = torch.empty(40, len(lens), device=DEV)
    s2 = torch.empty(2, 9, device=DEV)
    a2 = torch.empty(2, 9, 70, dtype=torch.int32, device=DEV)

    def step():
        M.maxsim_forward_ragged(Qs, Dp, off, scores=s1)
        M.maxsim_forward(Qw, Dw, scores=s2, argmax=a2)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (s1, s2, a2)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        s1.fill_(0), s2.fill_(0), a2.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((s1, s2, a2), want):
            assert torch.equal(got, ref), "replay %d differs from the eager result" % rep


def test_capture_without_a_warm_up_of_the_captured_shapes():
    """maxsim_init does the per-device set-up (LDS limits of every instantiation), so a shape class may meet its
    first launch under capture: the int8 document-stationary kernel with 24 column blocks, the fp32 slab kernel
    with argmax and the int8 slab kernel (two passes, 157 KB of LDS) are captured here without an eager call of
    theirs before, and checked against eager calls after."""
    M.maxsim_init()
    big8, bigs = M.maxsim_quantize_rows_i8(W.unit_rows((4100, 36, 128), "f32", 31, DEV))
    q8, qs = M.maxsim_quantize_rows_i8(W.unit_rows((1, 700, 128), "f16", 32, DEV))
    s8 = torch.empty(1, 4100, device=DEV)
    Qw = W.unit_rows((1, 40, 320), "f32", 33, DEV)
    Dw = W.unit_rows((7, 90, 320), "f32", 34, DEV)
    sw = torch.empty(1, 7, device=DEV)
    aw = torch.empty(1, 7, 40, dtype=torch.int32, device=DEV)
    q8w, qsw = M.maxsim_quantize_rows_i8(W.unit_rows((1, 600, 256), "f16", 35, DEV))
    d8w, dsw = M.maxsim_quantize_rows_i8(W.unit_rows((6, 50, 256), "f32", 36, DEV))
    s8w = torch.empty(1, 6, device=DEV)

    def step():
        M.maxsim_forward_i8(q8, qs, big8, bigs, scores=s8)
        M.maxsim_forward(Qw, Dw, scores=sw, argmax=aw)
        M.maxsim_forward_i8(q8w, qsw, d8w, dsw, scores=s8w)

    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    got = []
    for rep in range(2):
        s8.fill_(0), sw.fill_(0), aw.fill_(-7), s8w.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got.append([t.clone() for t in (s8, sw, aw, s8w)])
    s8.fill_(0), sw.fill_(0), aw.fill_(-7), s8w.fill_(0)
    step()
    torch.cuda.synchronize()
    for rep in range(2):
        for g_, ref in zip(got[rep], (s8, sw, aw, s8w)):
            assert torch.equal(g_, ref), "replay %d differs from the eager result" % rep
