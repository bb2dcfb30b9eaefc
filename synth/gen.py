"""Seeded synthetic workloads shaped like the paper's retrieval experiments.

This module only draws inputs: document vector sets, query vector sets,
candidate lists and projection matrices.  It holds none of the method's
arithmetic (no hashing, no collision counting, no ranking) and is the one
module the CPU oracle's tests and the HIP library's tests both import; every
array it returns is handed to both sides as plain bytes, so differences in
random-number streams between devices can never look like a kernel error.

The five presets follow the benchmark configurations of this build (token
embedding sets of dimension 128, about 32 query vectors and about 70 document
vectors, the hyper-parameters C=7, L=32 of the paper's App. B first setting);
they stand in for the MS MARCO / LoTTE ColBERT embeddings and the GloVe sets
of the paper's Sec. 6, which are not available here.

All draws go through ``torch`` generators so that the same code fills host
memory (small presets, CPU tests) or device memory (large presets that do not
fit the host).  A given (preset, seed, device type) is reproducible; CPU and
GPU streams differ, which is harmless because the data, not the seed, is what
both implementations consume.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import torch

SEED_CENTRES, SEED_DOCS, SEED_LENGTHS, SEED_QUERIES, SEED_CANDS, SEED_PROJ = range(6)


@dataclasses.dataclass
class Preset:
    """Shape of one synthetic workload (no data)."""
    name: str
    cfg: int
    n_docs: int
    length_law: str          # "const", "uniform", "truncnorm"
    length_args: tuple
    d: int
    dtype: str               # "i8" or "f16"
    n_centres: int
    sigma: float             # total noise norm relative to a unit centre
    L: int
    C: int
    proj_kind: str           # "rademacher" or "gaussian"
    n_queries: int
    q_len: int
    sigma_q: float
    planted_per_query: int
    n_cand: int              # 0 = score every document
    k: int


PRESETS = {
    1: Preset("cfg1_tiny_exhaustive", 1, 1_000, "const", (32,), 128, "i8", 64, 0.3,
              16, 6, "rademacher", 10, 8, 0.2, 1, 0, 10),
    2: Preset("cfg2_exhaustive_mid", 2, 100_000, "uniform", (16, 128), 128, "i8", 1024, 0.3,
              32, 7, "rademacher", 64, 32, 0.2, 1, 0, 100),
    3: Preset("cfg3_candidate_rerank", 3, 1_000_000, "truncnorm", (70.0, 25.0, 8, 180), 128, "i8", 1024, 0.3,
              32, 7, "rademacher", 256, 32, 0.2, 8, 4096, 10),
    4: Preset("cfg4_large_exhaustive", 4, 8_000_000, "truncnorm", (70.0, 25.0, 8, 180), 128, "i8", 1024, 0.3,
              32, 7, "rademacher", 32, 32, 0.2, 1, 0, 100),
    5: Preset("cfg5_fp16_stress", 5, 500_000, "uniform", (32, 256), 256, "f16", 4096, 0.3,
              64, 8, "gaussian", 64, 128, 0.2, 1, 0, 10),
}


def sweep_preset(m: int, n_queries: int = 16) -> Preset:
    """The paper's synthetic experiment (Sec. 6.1): 1000 documents of exactly m vectors, queries are whole
    documents with added noise, L = 8 tables of C = log2(m) + 1 one-bit hashes (m a power of two, 2..1024).
    Stand-in for the GloVe vectors used there: the same clustered int8 vectors as the other presets."""
    if m < 2 or m > 1024 or m & (m - 1):
        raise ValueError("m must be a power of two in 2..1024")
    return Preset(f"sweep_m{m}", 6, 1_000, "const", (m,), 128, "i8", 1024, 0.3,
                  8, int(math.log2(m)) + 1, "rademacher", n_queries, m, 0.2, 1, 0, 10)


@dataclasses.dataclass
class Workload:
    preset: Preset
    docs: torch.Tensor                 # [V, d] int8 or float16
    lengths: torch.Tensor              # [N] int64, CPU
    offsets: torch.Tensor              # [N+1] int64, CPU (exclusive scan of lengths)
    queries: torch.Tensor              # [B*q_len, d] same dtype as docs
    q_lengths: torch.Tensor            # [B] int64, CPU
    planted: torch.Tensor              # [B, planted_per_query] int64, CPU
    cand_ids: Optional[torch.Tensor]   # [B, n_cand] int64 on the docs' device, or None
    proj: torch.Tensor                 # [L*C, d] int8 (+-1) or float32

    @property
    def n_docs(self) -> int:
        return int(self.lengths.numel())

    @property
    def n_vectors(self) -> int:
        return int(self.offsets[-1])


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _seed(p: Preset, which: int, seed_base: Optional[int]) -> int:
    base = 1000 * p.cfg if seed_base is None else seed_base
    return base + which


def draw_lengths(p: Preset, n_docs: int, seed: int) -> torch.Tensor:
    """Document lengths m_i on the CPU (int64)."""
    g = _gen(seed, "cpu")
    if p.length_law == "const":
        return torch.full((n_docs,), int(p.length_args[0]), dtype=torch.int64)
    if p.length_law == "uniform":
        lo, hi = p.length_args
        return torch.randint(int(lo), int(hi) + 1, (n_docs,), generator=g, dtype=torch.int64)
    if p.length_law == "truncnorm":
        mean, sd, lo, hi = p.length_args
        out = torch.empty(n_docs, dtype=torch.int64)
        todo = torch.arange(n_docs)
        while todo.numel():
            z = torch.randn(todo.numel(), generator=g, dtype=torch.float64) * sd + mean
            r = torch.round(z).to(torch.int64)
            ok = (r >= lo) & (r <= hi)
            out[todo[ok]] = r[ok]
            todo = todo[~ok]
        return out
    raise ValueError(p.length_law)


def quantize(v: torch.Tensor, dtype: str) -> torch.Tensor:
    """Unit-norm float rows -> storage dtype (int8: round-half-even of 127*v)."""
    if dtype == "i8":
        return torch.clamp(torch.round(v * 127.0), -127, 127).to(torch.int8)
    if dtype == "f16":
        return v.to(torch.float16)
    raise ValueError(dtype)


def _normalize(v: torch.Tensor) -> torch.Tensor:
    return v / v.norm(dim=1, keepdim=True).clamp_min(1e-12)


def draw_centres(p: Preset, seed: int, device) -> torch.Tensor:
    g = _gen(seed, device)
    return torch.randn(p.n_centres, p.d, generator=g, device=device, dtype=torch.float32) / math.sqrt(p.d)


def draw_docs(p: Preset, n_vectors: int, centres: torch.Tensor, seed: int, device,
              chunk: int = 1 << 21) -> torch.Tensor:
    """All document vectors, concatenated in document order: [V, d]."""
    g = _gen(seed, device)
    tdtype = torch.int8 if p.dtype == "i8" else torch.float16
    out = torch.empty(n_vectors, p.d, dtype=tdtype, device=device)
    scale = p.sigma / math.sqrt(p.d)
    for s in range(0, n_vectors, chunk):
        n = min(chunk, n_vectors - s)
        c = torch.randint(0, p.n_centres, (n,), generator=g, device=device)
        v = centres[c] + scale * torch.randn(n, p.d, generator=g, device=device, dtype=torch.float32)
        out[s:s + n] = quantize(_normalize(v), p.dtype)
    return out


def draw_projection(p: Preset, seed: int, device) -> torch.Tensor:
    """[L*C, d] projection rows; row t*C+c is sign bit c of table t."""
    g = _gen(seed, "cpu")
    P = p.L * p.C
    if p.proj_kind == "rademacher":
        bits = torch.randint(0, 2, (P, p.d), generator=g, dtype=torch.int8)
        return (bits * 2 - 1).to(torch.int8).to(device)
    return torch.randn(P, p.d, generator=g, dtype=torch.float32).to(device)


def make(cfg, device="cpu", n_docs: Optional[int] = None, n_queries: Optional[int] = None,
         n_cand: Optional[int] = None, seed_base: Optional[int] = None) -> Workload:
    """Build preset ``cfg`` (a number, or a Preset such as sweep_preset(m)); ``n_docs`` / ``n_queries`` /
    ``n_cand`` shrink it for tests."""
    p = dataclasses.replace(cfg if isinstance(cfg, Preset) else PRESETS[cfg])
    if n_docs is not None:
        p.n_docs = int(n_docs)
    if n_queries is not None:
        p.n_queries = int(n_queries)
    if n_cand is not None:
        p.n_cand = int(n_cand)
    if p.n_cand:
        p.n_cand = min(p.n_cand, p.n_docs)
    device = torch.device(device)

    lengths = draw_lengths(p, p.n_docs, _seed(p, SEED_LENGTHS, seed_base))
    offsets = torch.zeros(p.n_docs + 1, dtype=torch.int64)
    torch.cumsum(lengths, 0, out=offsets[1:])
    V = int(offsets[-1])
    centres = draw_centres(p, _seed(p, SEED_CENTRES, seed_base), device)
    docs = draw_docs(p, V, centres, _seed(p, SEED_DOCS, seed_base), device)

    # Queries: noisy copies of vectors taken from planted documents.
    gq = _gen(_seed(p, SEED_QUERIES, seed_base), "cpu")
    B, mq, pp = p.n_queries, p.q_len, p.planted_per_query
    planted = torch.stack([torch.randperm(p.n_docs, generator=gq)[:pp] if p.n_docs >= pp
                           else torch.randint(0, p.n_docs, (pp,), generator=gq) for _ in range(B)]) \
        if B else torch.zeros(0, pp, dtype=torch.int64)
    rows = torch.empty(B, mq, dtype=torch.int64)
    per = mq // pp
    for b in range(B):
        pos = 0
        for j in range(pp):
            doc = int(planted[b, j])
            take = per if j < pp - 1 else mq - pos
            m = int(lengths[doc])
            if m >= take:
                pick = torch.randperm(m, generator=gq)[:take]
            else:
                pick = torch.randint(0, m, (take,), generator=gq)
            rows[b, pos:pos + take] = offsets[doc] + pick
            pos += take
    src = docs[rows.reshape(-1).to(device)].to(torch.float32)
    if p.dtype == "i8":
        src = src / 127.0
    gqd = _gen(_seed(p, SEED_QUERIES, seed_base) + 7919, device)
    noise = torch.randn(src.shape, generator=gqd, device=device, dtype=torch.float32)
    queries = quantize(_normalize(_normalize(src) + (p.sigma_q / math.sqrt(p.d)) * noise), p.dtype)
    q_lengths = torch.full((B,), mq, dtype=torch.int64)

    cand_ids = None
    if p.n_cand:
        gc = _gen(_seed(p, SEED_CANDS, seed_base), "cpu")
        cand = torch.empty(B, p.n_cand, dtype=torch.int64)
        for b in range(B):
            # distinct ids: the planted documents plus uniform random others, shuffled
            need = p.n_cand
            chosen = planted[b][:min(pp, need)].clone()
            while chosen.numel() < need:
                extra = torch.randint(0, p.n_docs, (2 * (need - chosen.numel()) + 16,), generator=gc)
                chosen = torch.cat([chosen, extra])
                # keep first occurrences, order preserved
                uniq, inv = torch.unique(chosen, return_inverse=True)
                first = torch.full((uniq.numel(),), chosen.numel(), dtype=torch.int64)
                first.scatter_reduce_(0, inv, torch.arange(chosen.numel()), reduce="amin")
                chosen = chosen[torch.sort(first).values][:need]
            cand[b] = chosen[torch.randperm(need, generator=gc)]
        cand_ids = cand.to(device)

    proj = draw_projection(p, _seed(p, SEED_PROJ, seed_base), device)
    return Workload(p, docs, lengths, offsets, queries, q_lengths, planted, cand_ids, proj)


def filter_centroids(w: Workload, n_centroids: Optional[int] = None, seed_base: Optional[int] = None) -> torch.Tensor:
    """Centroids for the candidate filter (int8 [K, d], on the documents' device).

    Stand-in for k-means on a sample of the vectors: with K equal to the number of mixture
    centres the quantised centres themselves (what k-means would converge to on this data),
    otherwise K document vectors drawn without replacement."""
    p = w.preset
    if p.dtype != "i8":
        raise ValueError("filter centroids are generated for int8 presets only")
    K = p.n_centres if n_centroids is None else int(n_centroids)
    device = w.docs.device
    if K == p.n_centres:
        centres = draw_centres(p, _seed(p, SEED_CENTRES, seed_base), device)
        return quantize(_normalize(centres), "i8")
    g = _gen(_seed(p, SEED_CENTRES, seed_base) + 104729, "cpu")
    pick = torch.randperm(w.n_vectors, generator=g)[:K]
    return w.docs[pick.to(device)].clone()
