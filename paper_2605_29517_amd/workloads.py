"""Seeded synthetic inputs shaped like the paper's workloads (Tab. "shapes", Tab. "varlen").

This module only draws random tensors, normalises token rows and rounds them to the
storage dtype.  It contains none of the scoring, gradient or quantisation arithmetic and
is the one piece shared by the CPU oracle's tests and the GPU path's tests/benchmark.
The paper times its kernels on synthetic tensors of ColBERT / ColPali shapes; these
generators stand in for the BEIR / REAL-MM-RAG corpora its quality tables use.
"""
import math

import numpy as np
import torch

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def unit_rows(shape, dtype: str, seed: int, device="cpu", generator=None) -> torch.Tensor:
    """i.i.d. N(0,1) entries, each last-axis row divided by its l2 norm in fp32, then rounded to dtype."""
    g = generator if generator is not None else _gen(seed, device)
    x = torch.randn(*shape, generator=g, device=device, dtype=torch.float32)
    x = x / x.norm(dim=-1, keepdim=True).clamp_min(1e-30)
    return x.to(TORCH_DTYPE[dtype]).contiguous()


def biased_rows(shape, dtype: str, seed: int, device="cpu", bias: float = 0.0, scale: float = 1.0,
                direction_seed: int = 7) -> torch.Tensor:
    """Rows (noise + bias * v) / norm * scale: noise i.i.d. N(0, 1/d) (norm about 1), v one fixed unit direction
    shared by every call with the same direction_seed.  bias > 0 pulls all rows towards v, bias < 0 away from it
    (two tensors with opposite biases have negative inner products throughout); scale gives rows that are not
    unit-norm.  Normalised in fp32, then scaled and rounded to dtype."""
    d = shape[-1]
    v = torch.randn(d, generator=_gen(direction_seed, device), device=device, dtype=torch.float32)
    v = v / v.norm()
    x = torch.randn(*shape, generator=_gen(seed, device), device=device, dtype=torch.float32) / math.sqrt(d)
    x = x + bias * v
    x = x / x.norm(dim=-1, keepdim=True).clamp_min(1e-30) * scale
    return x.to(TORCH_DTYPE[dtype]).contiguous()


def tiny_forward(seed: int = 0, n_docs: int = 1000, l_q: int = 32, l_d: int = 128, d: int = 128):
    """Config 1: one query, fp32, numpy default_rng(seed); Q drawn first, then D; rows l2-normalised."""
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((1, l_q, d)).astype(np.float32)
    D = rng.standard_normal((n_docs, l_d, d)).astype(np.float32)
    Q /= np.linalg.norm(Q, axis=-1, keepdims=True).astype(np.float32)
    D /= np.linalg.norm(D, axis=-1, keepdims=True).astype(np.float32)
    return torch.from_numpy(Q), torch.from_numpy(D)


def ragged_lengths(n_docs: int, lo: int, hi: int, seed: int, device="cpu"):
    """Document lengths uniform on [lo, hi] and their exclusive-cumsum int32 offsets [n_docs+1]."""
    g = _gen(seed, device)
    lengths = torch.randint(lo, hi + 1, (n_docs,), generator=g, device=device, dtype=torch.int64)
    offsets = torch.zeros(n_docs + 1, dtype=torch.int64, device=device)
    offsets[1:] = torch.cumsum(lengths, 0)
    if int(offsets[-1]) >= 2 ** 31:
        raise ValueError("packed corpus too long for int32 offsets")
    return lengths.to(torch.int32), offsets.to(torch.int32)


def colbert_rerank(n_q: int = 64, l_q: int = 32, n_docs: int = 100_000, lo: int = 64, hi: int = 300,
                   d: int = 128, dtype: str = "f16", seed: int = 2, device="cpu"):
    """Config 2: ragged ColBERT-style corpus, packed [T,d] + offsets, unit-norm rows."""
    lengths, offsets = ragged_lengths(n_docs, lo, hi, seed, device)
    total = int(offsets[-1])
    g = _gen(seed + 1000, device)
    D = unit_rows((total, d), dtype, 0, device, generator=g)
    Q = unit_rows((n_q, l_q, d), dtype, 0, device, generator=g)
    return Q, D, offsets, lengths


def colpali_pages(n_pages: int, l: int = 1024, d: int = 128, dtype: str = "bf16", seed: int = 3,
                  device="cpu", cosine: float = 0.3, chunk: int = 512) -> torch.Tensor:
    """Config 3 pages: rows = N(0,1) + alpha * (per-page mean vector), normalised.

    alpha = sqrt(c/(1-c)) makes the expected cosine between two rows of a page about c,
    so that many document tokens compete for each query token's maximum.
    """
    alpha = math.sqrt(cosine / (1.0 - cosine))
    g = _gen(seed, device)
    out = torch.empty(n_pages, l, d, dtype=TORCH_DTYPE[dtype], device=device)
    for p0 in range(0, n_pages, chunk):
        p1 = min(n_pages, p0 + chunk)
        mu = torch.randn(p1 - p0, 1, d, generator=g, device=device, dtype=torch.float32)
        x = torch.randn(p1 - p0, l, d, generator=g, device=device, dtype=torch.float32) + alpha * mu
        x = x / x.norm(dim=-1, keepdim=True)
        out[p0:p1] = x.to(TORCH_DTYPE[dtype])
    return out


def colpali_page_as_query(n_q: int = 4, n_docs: int = 10_000, l: int = 1024, d: int = 128,
                          dtype: str = "bf16", seed: int = 3, device="cpu"):
    """Config 3: query pages and document pages from the same page model."""
    Q = colpali_pages(n_q, l, d, dtype, seed, device)
    D = colpali_pages(n_docs, l, d, dtype, seed + 1000, device)
    return Q, D


def contrastive_batch(n: int = 256, l_q: int = 32, l_d: int = 1024, d: int = 128, dtype: str = "f16",
                      seed: int = 4, device="cpu"):
    """Config 4: in-batch negatives, n queries and n documents, unit-norm rows."""
    g = _gen(seed, device)
    Q = unit_rows((n, l_q, d), dtype, 0, device, generator=g)
    D = unit_rows((n, l_d, d), dtype, 0, device, generator=g)
    return Q, D


def int8_corpus_chunk(chunk_index: int, docs: int, l_d: int = 1024, d: int = 128, seed: int = 5,
                      device="cpu") -> torch.Tensor:
    """Config 5: fp32 unit-norm rows of one corpus chunk (quantised by the caller).

    Each chunk has its own seed so that any chunk can be regenerated alone when
    sampled documents are checked against the oracle.
    """
    return unit_rows((docs, l_d, d), "f32", seed * 1_000_003 + 17 * chunk_index + 1, device)


def int8_query(l_q: int = 1024, d: int = 128, seed: int = 5, device="cpu") -> torch.Tensor:
    """Config 5 query: fp16 unit-norm rows [1, l_q, d]."""
    return unit_rows((1, l_q, d), "f16", seed, device)


def to_raw_numpy(t: torch.Tensor) -> np.ndarray:
    """Host copy as the oracle wants it: float32 as is, 16-bit types as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.float16, torch.bfloat16):
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def dtype_name(t: torch.Tensor) -> str:
    return {torch.float32: "f32", torch.float16: "f16", torch.bfloat16: "bf16"}[t.dtype]
