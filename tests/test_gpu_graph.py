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

    def step():
        M.maxsim_forward(Q, D, scores=s, argmax=a)
        M.maxsim_ce_grad(s, 0.02, g=g, loss=loss)
        M.maxsim_backward(Q, D, a, g, dQ=dQ, dD=dD)
        M.maxsim_quantize_rows_i8(Q, X_i8=q8, scale=qs)
        M.maxsim_forward_i8(q8, qs, d8, ds, scores=s8)
        M.maxsim_forward_i8(q8, qs, big8, bigs, scores=s8b)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (s, a, g, loss, dQ, dD, s8, s8b)]

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
        for t in (s, a, g, loss, dQ, dD, s8, s8b):
            t.fill_(0) if t.dtype != torch.int32 else t.fill_(-7)   # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((s, a, g, loss, dQ, dD, s8, s8b), want):
            assert torch.equal(got, ref), "replay %d differs from the eager result" % rep
