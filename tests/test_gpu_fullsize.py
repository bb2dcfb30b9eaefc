"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot score every pair of the large presets in reasonable time, so these tests check
  - hash codes of sampled documents (every vector of each sampled document) bit for bit,
  - raw scores of sampled (query set, document) pairs and of every document the GPU ranks, bit for bit,
  - the top-k of every query set re-derived by the oracle's selection from the GPU's full score dump
    (exact, including the tie rule), and
  - properties that hold at any size (score range, planted documents rank first / in the top-k).
Inputs are generated on the device from fixed seeds and handed to the oracle as bytes.
"""
import dataclasses
import sys

import numpy as np
import pytest
import torch

import paper_2210_15748_amd as dz
from oracle import oracle as orc
from synth import gen

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print("[case]", msg, flush=True)
    sys.stdout.flush()


def oracle_codes_of_docs(w, doc_ids):
    """Oracle hash of every vector of the given documents -> (codes, offsets over the subset)."""
    off = w.offsets.numpy()
    rows = np.concatenate([np.arange(off[i], off[i + 1]) for i in doc_ids]) if len(doc_ids) else np.zeros(0, np.int64)
    sub = w.docs[torch.from_numpy(rows).to(w.docs.device)].cpu().numpy()
    codes = orc.hash_i8(sub, w.proj.cpu().numpy(), w.preset.L, w.preset.C)
    sub_off = np.concatenate([[0], np.cumsum(off[np.asarray(doc_ids) + 1] - off[np.asarray(doc_ids)])])
    return rows, codes, sub_off


def check_candidate_rerank(w, min_planted_hits):
    p = w.preset
    ix = dz.create(p.d, p.L, p.C, proj=w.proj)
    codes, offsets = dz.build_index(ix, w.docs, w.lengths)
    assert torch.equal(offsets.cpu(), w.offsets)
    cand = w.cand_ids.to(torch.int32).contiguous()
    ids, sc = dz.search(ix, w.queries, w.q_lengths, p.k, cand_ids=cand)
    raw = dz.scores(ix, w.queries, w.q_lengths, cand_ids=cand).cpu().numpy().reshape(p.n_queries, p.n_cand)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    cand_np = w.cand_ids.cpu().numpy()
    qc = orc.hash_i8(w.queries.cpu().numpy(), w.proj.cpu().numpy(), p.L, p.C)

    # (1) top-k of every query set from the dumped scores, by the oracle's selection
    for b in range(p.n_queries):
        want_ids, want_sc = orc.topk(raw[b], p.k, cand_np[b])
        assert np.array_equal(ids[b], want_ids) and np.array_equal(sc[b], want_sc), b
    assert raw.min() >= 0 and raw.max() <= p.q_len * p.L

    # (2) sampled pairs: 3 whole query sets + 3000 random pairs + every ranked document
    rng = np.random.default_rng(3)
    pairs = [(b, c) for b in (0, 101, 255) for c in range(p.n_cand)]
    pairs += list(zip(rng.integers(0, p.n_queries, 3000).tolist(), rng.integers(0, p.n_cand, 3000).tolist()))
    pos_of = {}
    for b in range(p.n_queries):
        order = np.argsort(cand_np[b], kind="stable")
        where = np.searchsorted(cand_np[b][order], ids[b].astype(np.int64))
        pairs += [(b, int(order[x])) for x in where]
    pb = np.array([x[0] for x in pairs]); pc = np.array([x[1] for x in pairs])
    docs_needed = np.unique(cand_np[pb, pc])
    rows, dcodes, sub_off = oracle_codes_of_docs(w, docs_needed)
    # (3) hash parity on every vector of the sampled documents
    assert np.array_equal(codes[torch.from_numpy(rows).to(DEV)].cpu().numpy(), dcodes)
    local = np.searchsorted(docs_needed, cand_np[pb, pc])
    for b in np.unique(pb):
        sel = pb == b
        want = orc.scores(dcodes, sub_off, qc[b * p.q_len:(b + 1) * p.q_len], local[sel])
        assert np.array_equal(raw[b, pc[sel]], want), b
    # (4) most planted documents reach the top-10 (each supplied only 4 of the 32 query vectors)
    hits = [len(set(w.planted[b].tolist()) & set(ids[b].tolist())) for b in range(p.n_queries)]
    assert np.mean(hits) >= min_planted_hits, np.mean(hits)


def test_cfg3_full_candidate_rerank():
    say("cfg3 full: 1M docs, 256 query sets x 4096 candidates, k=10")
    check_candidate_rerank(gen.make(3, device=DEV), 5.0)


@pytest.mark.parametrize("L,Cb,n_cand", [(32, 6, 8192), (32, 7, 16384), (64, 7, 4096), (128, 8, 4096), (16, 4, 4096)])
def test_cfg3_full_with_the_papers_hyperparameter_settings(L, Cb, n_cand):
    """The candidate-rerank preset at full size with the settings the paper selects (App. B: (L, C, filter_k) =
    (32, 6, 8192), (32, 7, 16384), (64, 7, 4096)) and the two corners of its grid (L = 128, C = 8: hashed in two
    table groups; L = 16, C = 4)."""
    say(f"cfg3 full with L={L} C={Cb}, {n_cand} candidates per query set")
    preset = dataclasses.replace(gen.PRESETS[3], L=L, C=Cb, n_cand=n_cand)
    check_candidate_rerank(gen.make(preset, device=DEV), 0.1)


def test_cfg2_full_exhaustive():
    say("cfg2 full: 100k docs x 64 query sets exhaustive, k=100")
    w = gen.make(2, device=DEV)
    p = w.preset
    ix = dz.create(p.d, p.L, p.C, proj=w.proj)
    codes, offsets = dz.build_index(ix, w.docs, w.lengths)
    ids, sc = dz.search(ix, w.queries, w.q_lengths, p.k)
    raw = dz.scores(ix, w.queries, w.q_lengths).cpu().numpy()
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    R = w.proj.cpu().numpy()
    dcodes = orc.hash_i8(w.docs.cpu().numpy(), R, p.L, p.C)          # all 7.2M vectors
    assert np.array_equal(codes.cpu().numpy(), dcodes)
    qc = orc.hash_i8(w.queries.cpu().numpy(), R, p.L, p.C)
    off = w.offsets.numpy()
    for b in range(p.n_queries):
        want_ids, want_sc = orc.topk(raw[b], p.k)
        assert np.array_equal(ids[b], want_ids) and np.array_equal(sc[b], want_sc), b
        assert ids[b, 0] == int(w.planted[b, 0])
    rng = np.random.default_rng(2)
    for b in (0, 17, 63):                                           # three query sets against every document
        assert np.array_equal(raw[b], orc.scores(dcodes, off, qc[b * p.q_len:(b + 1) * p.q_len])), b
    for b in range(p.n_queries):                                    # everywhere: ranked docs + a random sample
        sel = np.unique(np.concatenate([ids[b].astype(np.int64), rng.integers(0, w.n_docs, 500)]))
        assert np.array_equal(raw[b, sel], orc.scores(dcodes, off, qc[b * p.q_len:(b + 1) * p.q_len], sel)), b


def test_cfg5_fp16_gaussian_tolerance_path():
    """fp16 vectors x fp32 Gaussian projections, L=64, C=8, |Q|=128 (four mask-table chunks per query set).

    Tolerances of this configuration: code-bit mismatch rate <= 1e-4, every mismatch at a projection with
    |p| < 1e-3*||x||, top-10 overlap with the oracle >= 0.99.  The scoring of GPU codes is itself exact, which
    is checked by scoring the GPU's own codes with the oracle."""
    say("cfg5 reduced to 8k docs: fp16 / Gaussian, L=64 C=8, 16 query sets x 128 vectors, exhaustive, k=10")
    w = gen.make(5, device=DEV, n_docs=8000, n_queries=16)
    p = w.preset
    ix = dz.create(p.d, p.L, p.C, dtype=dz.F16, proj_kind=dz.PROJ_GAUSSIAN_F32, proj=w.proj)
    codes, _ = dz.build_index(ix, w.docs, w.lengths)
    ids, sc = dz.search(ix, w.queries, w.q_lengths, p.k)
    raw = dz.scores(ix, w.queries, w.q_lengths).cpu().numpy()
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    R = w.proj.cpu().numpy()
    off = w.offsets.numpy()

    # hashing: sampled documents, all their vectors
    rng = np.random.default_rng(5)
    sample = np.unique(np.concatenate([rng.integers(0, w.n_docs, 800), w.planted[:, 0].numpy()]))
    rows = np.concatenate([np.arange(off[i], off[i + 1]) for i in sample])
    X = w.docs[torch.from_numpy(rows).to(DEV)].cpu().numpy()
    want, proj = orc.hash_fp(X, R, p.L, p.C, want_proj=True)
    got = codes[torch.from_numpy(rows).to(DEV)].cpu().numpy()
    diff = np.unpackbits(got[..., None], axis=2, bitorder="little") != np.unpackbits(want[..., None], axis=2, bitorder="little")
    assert diff.mean() <= 1e-4, diff.mean()
    norms = np.linalg.norm(X.astype(np.float64), axis=1)
    margins = np.abs(proj.reshape(X.shape[0], p.L, p.C))
    assert np.all(margins[diff] < 1e-3 * np.broadcast_to(norms[:, None, None], margins.shape)[diff])

    # scoring and top-k are exact given the GPU's own codes
    gcodes = codes.cpu().numpy()
    qcodes_gpu = dz.hash(ix, w.queries).cpu().numpy()
    for b in (0, 7, 15):
        q = qcodes_gpu[b * p.q_len:(b + 1) * p.q_len]
        assert np.array_equal(raw[b], orc.scores(gcodes, off, q)), b
    for b in range(p.n_queries):
        want_ids, want_sc = orc.topk(raw[b], p.k)
        assert np.array_equal(ids[b], want_ids) and np.array_equal(sc[b], want_sc), b

    # end to end against the oracle's own codes: top-10 overlap
    ocodes = orc.hash_fp(w.docs.cpu().numpy(), R, p.L, p.C)
    oq = orc.hash_fp(w.queries.cpu().numpy(), R, p.L, p.C)
    overlap = []
    for b in range(p.n_queries):
        s = orc.scores(ocodes, off, oq[b * p.q_len:(b + 1) * p.q_len])
        o_ids, _ = orc.topk(s, p.k)
        overlap.append(len(set(o_ids.tolist()) & set(ids[b].tolist())) / p.k)
        assert ids[b, 0] == int(w.planted[b, 0])
    assert np.mean(overlap) >= 0.99, overlap


def test_cfg3_full_candidate_filter_sampled():
    """Candidate filter at the benchmark's size (1M documents, 65536 centroids, probe 1, filter_k 4096).

    The oracle's brute-force assignment costs 8.4M multiply-adds per vector here, so it runs on samples:
      - closest centroid of sampled document vectors, bit for bit;
      - for sampled documents, the set of buckets that hold the document = the set of centroids the oracle
        assigns its vectors to;
      - for two query sets, the count of every sampled document (oracle: number of query vectors whose closest
        centroid is among the document's) against the filter's output, including the cut at filter_k;
      - properties at any size: bucket offsets, no document twice in a bucket, output order and padding."""
    say("cfg3 full: candidate filter, 65536 centroids, probe 1, filter_k 4096")
    w = gen.make(3, device=DEV)
    p = w.preset
    K, probe, filter_k = 65536, 1, 4096
    Cn = gen.filter_centroids(w, K)
    ix = dz.create(p.d, p.L, p.C, proj=w.proj)
    dz.build_index(ix, w.docs, w.lengths)
    assign, b_off, b_docs = dz.filter_build(ix, Cn, w.docs)
    ids, cnt = dz.filter_query(ix, w.queries, w.q_lengths, probe, filter_k)
    ids_np, cnt_np = ids.cpu().numpy(), cnt.cpu().numpy()
    Cn_np = Cn.cpu().numpy()
    off = w.offsets.numpy()
    rng = np.random.default_rng(33)

    # bucket structure
    bo = b_off.cpu().numpy().astype(np.int64)
    assert bo[0] == 0 and np.all(np.diff(bo) >= 0) and bo[-1] <= w.n_vectors
    entries = b_docs[: int(bo[-1])].to(torch.int64)
    bucket_of_entry = torch.searchsorted(b_off.to(torch.int64), torch.arange(int(bo[-1]), device=DEV), right=True) - 1
    pair = bucket_of_entry * w.n_docs + entries
    assert torch.unique(pair).numel() == pair.numel()          # a document appears once per bucket
    del pair

    # sampled vectors: closest centroid
    rows = rng.integers(0, w.n_vectors, 1500)
    want = orc.assign_centroids(w.docs[torch.from_numpy(rows).to(DEV)].cpu().numpy(), Cn_np)
    assert np.array_equal(assign[torch.from_numpy(rows).to(DEV)].cpu().numpy().astype(np.int64), want.astype(np.int64))

    # sampled documents: buckets that hold them, and their counts for two query sets
    qsets = (5, 200)
    sample = set(rng.integers(0, w.n_docs, 30).tolist())
    for b in qsets:
        sample |= set(w.planted[b].tolist()) | set(int(x) for x in ids_np[b][:12]) | set(int(x) for x in ids_np[b][-6:])
    sample.discard(0xFFFFFFFF)
    sample = sorted(sample)
    cent_of_doc = {}
    for dcm in sample:
        X = w.docs[off[dcm]:off[dcm + 1]].cpu().numpy()
        cs = set(orc.assign_centroids(X, Cn_np).tolist())
        cent_of_doc[dcm] = cs
        pos = torch.nonzero(entries == dcm).reshape(-1)
        got = set(bucket_of_entry[pos].cpu().tolist())
        assert got == cs, dcm
    for b in qsets:
        qv = w.queries[b * p.q_len:(b + 1) * p.q_len].cpu().numpy()
        qc = orc.assign_centroids(qv, Cn_np).tolist()                  # probe = 1: the closest centroid
        real = ids_np[b] != 0xFFFFFFFF
        assert np.all(cnt_np[b][real] >= 1) and np.all(cnt_np[b][~real] == -1) and np.all(cnt_np[b] <= p.q_len * probe)
        key = cnt_np[b][real].astype(np.int64) * (1 << 32) - ids_np[b][real].astype(np.int64)
        assert np.all(np.diff(key) < 0)                                  # count descending, then id ascending, no repeats
        assert not np.any(real[1:] & ~real[:-1])                         # padding only at the end
        where = {int(i): int(c) for i, c in zip(ids_np[b][real], cnt_np[b][real])}
        last = (int(cnt_np[b][real][-1]), -int(ids_np[b][real][-1])) if real.all() else (0, 0)
        for dcm in sample:
            c = sum(1 for x in qc if x in cent_of_doc[dcm])
            if dcm in where:
                assert where[dcm] == c, (b, dcm)
            else:
                assert c == 0 or (c, -dcm) < last, (b, dcm, c, last)


def test_cfg4_full_large_exhaustive_sampled():
    """The large exhaustive preset at full size (8M documents, 560M vectors = 72 GB of int8 in HBM, 32 query sets,
    k = 100).  The oracle cannot score 2.6e8 pairs, so: hash codes and raw scores of sampled documents (4000 random
    ones, every document the GPU ranks, every planted one) for all 32 query sets, bit for bit; the top-100 of every
    query set re-derived by the oracle's selection from the GPU's score dump restricted to scores >= the 100th."""
    say("cfg4 full: generating 8M documents on the device")
    w = gen.make(4, device=DEV)
    p = w.preset
    say(f"cfg4 full: {w.n_vectors} vectors generated; build + search")
    ix = dz.create(p.d, p.L, p.C, proj=w.proj)
    codes, offsets = dz.build_index(ix, w.docs, w.lengths)
    ids, sc = dz.search(ix, w.queries, w.q_lengths, p.k)
    raw_dev = dz.scores(ix, w.queries, w.q_lengths)
    torch.cuda.synchronize()
    say("cfg4 full: scores computed; checking the top-k against the dump")
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    raw = raw_dev.cpu().numpy().reshape(p.n_queries, w.n_docs)
    del raw_dev
    assert raw.min() >= 0 and raw.max() <= p.q_len * p.L
    for b in range(p.n_queries):
        kth = sc[b, -1]
        assert int((raw[b] > kth).sum()) < p.k                      # the cut is in the right place
        cand = np.nonzero(raw[b] >= kth)[0]
        want_ids, want_sc = orc.topk(raw[b][cand], p.k, cand)
        assert np.array_equal(ids[b], want_ids) and np.array_equal(sc[b], want_sc), b
        assert ids[b, 0] == int(w.planted[b, 0])
    say("cfg4 full: oracle on sampled documents")
    rng = np.random.default_rng(4)
    sample = np.unique(np.concatenate([rng.integers(0, w.n_docs, 4000), ids.reshape(-1).astype(np.int64),
                                       w.planted.numpy().reshape(-1)]))
    rows, dcodes, sub_off = oracle_codes_of_docs(w, sample)
    assert np.array_equal(codes[torch.from_numpy(rows).to(DEV)].cpu().numpy(), dcodes)
    qc = orc.hash_i8(w.queries.cpu().numpy(), w.proj.cpu().numpy(), p.L, p.C)
    for b in range(p.n_queries):
        want = orc.scores(dcodes, sub_off, qc[b * p.q_len:(b + 1) * p.q_len])
        assert np.array_equal(raw[b, sample], want), b
    off_last = offsets[-1].item()
    assert off_last == w.n_vectors


def test_cfg5_full_fp16_sampled():
    """The fp16 / Gaussian preset at full size (500k documents, 72M vectors of d = 256 = 37 GB, L = 64, C = 8, 64 query
    sets of 128 vectors, k = 10): hashing tolerance on sampled documents, the top-10 of every query set re-derived from
    the GPU's score dump, planted documents first, and raw scores of sampled documents within the bound that the
    tolerated bit flips allow (a flipped code bit changes at most one table of one vector pair)."""
    say("cfg5 full: generating 500k fp16 documents on the device")
    w = gen.make(5, device=DEV)
    p = w.preset
    say(f"cfg5 full: {w.n_vectors} vectors generated; build + search")
    ix = dz.create(p.d, p.L, p.C, dtype=dz.F16, proj_kind=dz.PROJ_GAUSSIAN_F32, proj=w.proj)
    codes, _ = dz.build_index(ix, w.docs, w.lengths)
    ids, sc = dz.search(ix, w.queries, w.q_lengths, p.k)
    raw = dz.scores(ix, w.queries, w.q_lengths).cpu().numpy()
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    say("cfg5 full: checking the top-k against the dump")
    for b in range(p.n_queries):
        kth = sc[b, -1]
        assert int((raw[b] > kth).sum()) < p.k
        cand = np.nonzero(raw[b] >= kth)[0]
        want_ids, want_sc = orc.topk(raw[b][cand], p.k, cand)
        assert np.array_equal(ids[b], want_ids) and np.array_equal(sc[b], want_sc), b
        assert ids[b, 0] == int(w.planted[b, 0])
    say("cfg5 full: oracle hashing of sampled documents")
    rng = np.random.default_rng(55)
    off = w.offsets.numpy()
    sample = np.unique(np.concatenate([rng.integers(0, w.n_docs, 300), w.planted[:, 0].numpy()]))
    rows = np.concatenate([np.arange(off[i], off[i + 1]) for i in sample])
    X = w.docs[torch.from_numpy(rows).to(DEV)].cpu().numpy()
    R = w.proj.cpu().numpy()
    want, proj = orc.hash_fp(X, R, p.L, p.C, want_proj=True)
    got = codes[torch.from_numpy(rows).to(DEV)].cpu().numpy()
    diff = np.unpackbits(got[..., None], axis=2, bitorder="little") != np.unpackbits(want[..., None], axis=2, bitorder="little")
    assert diff.mean() <= 1e-4, diff.mean()
    norms = np.linalg.norm(X.astype(np.float64), axis=1)
    margins = np.abs(proj.reshape(X.shape[0], p.L, p.C))
    assert np.all(margins[diff] < 1e-3 * np.broadcast_to(norms[:, None, None], margins.shape)[diff])
    # scores of the sampled documents from the oracle's own codes: equal up to the flipped bits
    sub_off = np.concatenate([[0], np.cumsum(off[sample + 1] - off[sample])])
    oq = orc.hash_fp(w.queries.cpu().numpy(), R, p.L, p.C)
    flips = int(diff.sum())
    for b in (0, 31, 63):
        s = orc.scores(want, sub_off, oq[b * p.q_len:(b + 1) * p.q_len])
        d = np.abs(raw[b, sample].astype(np.int64) - s)
        assert d.sum() <= 2 * (flips + 64) and (d == 0).mean() >= 0.95, (d.sum(), flips)
