"""GPU parity of the mask-table scoring kernel over every instantiation its dispatcher can reach, element by
element against the oracle: the paper's hyper-parameter grid (App. B: C in 4..8, L in 16..128; Alg. 2 inner
loops) plus L = 8 and the 16-bit code shapes, each as
  cand    candidate lists, one query set per workgroup;
  pair    every document for a batch of three query sets (two sets per workgroup where the paired table fits);
  split   query sets longer than 32 vectors on a small grid (their 32-vector chunks dealt to several workgroups);
  chunks  query sets longer than 32 vectors on a grid large enough that one workgroup takes all chunks;
with raw counts, the Eq. 1 remap, a weighted sum of a tabulated phi, and the mean of count / L plain and weighted.  Every test also asserts which
instantiation the launch picked."""
import re
import sys

import numpy as np
import pytest
import torch

import paper_2210_15748_amd as dz
from oracle import oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
EMPTY = 0xFFFFFFFF

NARROW = [(L, Cb) for L in (8, 16, 32, 64, 128) for Cb in (4, 5, 6, 7, 8)]
WIDE = [(8, 9), (8, 10), (8, 11), (16, 9), (16, 10), (32, 9)]
EDGE_LENGTHS = [0, 1, 7, 8, 9, 15, 16, 17, 31, 33, 64, 65, 2, 180, 0, 3]


def say(msg):
    print("[case]", msg, flush=True)
    sys.stdout.flush()


def clustered(rng, n, d, pool, spread):
    return np.clip(pool[rng.integers(0, len(pool), n)] + rng.integers(-spread, spread + 1, (n, d)), -127, 127).astype(np.int8)


def pair_ok(L, Cb):
    size = L * (1 << max(Cb, 6)) * 8
    return size <= 32 * 1024 or (L <= 32 and size <= 64 * 1024)


def make_reference(form, dc, off, Cb):
    """form -> (score transform, weights flag, oracle function of (query codes, weights, doc ids))."""
    if form == "raw":
        return dz.SCORE_RAW_COUNTS, False, lambda q, w, sel: orc.scores(dc, off, q, sel)
    if form == "eq1":
        return dz.SCORE_EQ1_Q16, False, lambda q, w, sel: orc.scores_eq1(dc, off, q, Cb, sel)
    if form == "weighted":
        return dz.SCORE_MAX_SIGMOID_Q16, True, lambda q, w, sel: orc.scores_general(dc, off, q, orc.PHI_SIGMOID, orc.SIGMA_MAX,
                                                                                      weights=w, doc_ids=sel)
    # sigma = mean of count / L (Sec. 4.1), plain and weighted
    return dz.SCORE_MEAN_IDENTITY_Q16, form == "mean_weighted", lambda q, w, sel: orc.scores_general(
        dc, off, q, orc.PHI_IDENTITY, orc.SIGMA_MEAN, weights=w, doc_ids=sel)


def launched(ix):
    m = re.fullmatch(r"score_masklut_kernel<(\d+), (\d+), (\d+), (\d+), (\d+), (true|false)>", dz.last_score_kernel(ix))
    assert m, dz.last_score_kernel(ix)
    return tuple(int(x) for x in m.groups()[:5]) + (m.group(6) == "true",)


@pytest.mark.parametrize("form", ["raw", "eq1", "weighted", "mean", "mean_weighted"])
@pytest.mark.parametrize("mode", ["cand", "pair", "split"])
@pytest.mark.parametrize("L,Cb", NARROW + WIDE)
def test_masklut_instantiation_matches_oracle(L, Cb, mode, form):
    say(f"mask-table grid L={L} C={Cb} mode={mode} form={form}")
    rng = np.random.default_rng(L * 1000 + Cb * 10 + len(mode) + len(form))
    d = 64
    lens = np.concatenate([np.array(EDGE_LENGTHS), rng.integers(0, 40, 150)]).astype(np.int64)
    rng.shuffle(lens)
    N, V = len(lens), int(lens.sum())
    pool = rng.integers(-100, 101, (15, d))
    X = clustered(rng, V, d, pool, 12)
    q_lens = np.array({"cand": [32, 5, 17, 1], "pair": [32, 9, 20], "split": [70, 33, 5]}[mode], dtype=np.int64)
    nq = int(q_lens.sum())
    Q = clustered(rng, nq, d, pool, 8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, dz.HASH_AUTO, dz.SCORE_MASKLUT)
    codes, _ = dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    assert np.array_equal(codes.cpu().numpy(), dc)
    off = np.concatenate([[0], np.cumsum(lens)])
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    transform, weighted, ref = make_reference(form, dc, off, Cb)
    dz.set_score_transform(ix, transform)
    w = None
    if weighted:
        w = rng.integers(0, 65537, nq).astype(np.uint32)
        w[:3] = [65536, 0, 1]
        dz.set_query_weights(ix, torch.from_numpy(w.view(np.int32)).to(DEV))
    wq = lambda b: None if w is None else w[qo[b]:qo[b + 1]]
    Qd = torch.from_numpy(Q).to(DEV)
    want_remap = {"raw": 0, "eq1": 1, "weighted": 2, "mean": 3, "mean_weighted": 4}[form]
    cb = max(Cb, 6)
    some = False
    if mode in ("pair", "split"):                    # every document for every query set
        got = dz.scores(ix, Qd, q_lens).cpu().numpy()
        kl = launched(ix)
        assert kl[:4] == (L, cb, 2 if Cb > 8 else 1, want_remap), kl
        if mode == "pair":
            assert kl[4:] == (2 if pair_ok(L, Cb) and want_remap < 3 else 1, False), kl
        else:
            assert kl[4:] == (1, True), kl
        for b in range(len(q_lens)):
            want = ref(qc[qo[b]:qo[b + 1]], wq(b), None)
            some = some or want.max() > 0
            assert np.array_equal(got[b], want), b
    if mode in ("cand", "split"):                    # candidate lists: ragged, repeated ids, empty slots, an empty list
        cands = [rng.integers(0, N, 300), np.array([], dtype=np.int64), np.arange(N), np.array([5, 5, 0, N - 1, 3])][:len(q_lens)]
        co = np.concatenate([[0], np.cumsum([len(c) for c in cands])])
        flat = np.concatenate(cands).astype(np.int64)
        empty = rng.random(flat.shape[0]) < 0.05
        flat_dev = torch.from_numpy(np.where(empty, EMPTY, flat).astype(np.uint32).view(np.int32)).to(DEV)
        got = dz.scores(ix, Qd, q_lens, cand_ids=flat_dev, cand_offsets=co).cpu().numpy()
        kl = launched(ix)
        assert kl == (L, cb, 2 if Cb > 8 else 1, want_remap, 1, mode == "split"), kl
        for b, c in enumerate(cands):
            want = ref(qc[qo[b]:qo[b + 1]], wq(b), c) if len(c) else np.zeros(0, np.int32)
            some = some or (len(want) and want.max() > 0)
            want = np.where(empty[co[b]:co[b + 1]], -1, want)
            assert np.array_equal(got[co[b]:co[b + 1]], want), b
    assert some


@pytest.mark.parametrize("L,Cb", [(L, Cb) for L in (8, 16, 32, 64, 128) for Cb in (6, 7, 8)] + WIDE)
def test_masklut_long_query_sets_on_a_large_grid(L, Cb):
    """Query sets of 40 and 70 vectors with enough (query set, document block) pairs that the chunks of a set stay in
    one workgroup: the second chunk's table is rebuilt in place and its partial scores are added by plain stores."""
    say(f"mask-table grid L={L} C={Cb} mode=chunks")
    rng = np.random.default_rng(L * 77 + Cb)
    d, N, B, n_cand = 64, 3000, 34, 4096
    lens = rng.integers(0, 6, N).astype(np.int64)
    V = int(lens.sum())
    pool = rng.integers(-100, 101, (15, d))
    X = clustered(rng, V, d, pool, 12)
    q_lens = np.array([40, 70] * (B // 2), dtype=np.int64)
    Q = clustered(rng, int(q_lens.sum()), d, pool, 8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, dz.HASH_AUTO, dz.SCORE_MASKLUT)
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    off = np.concatenate([[0], np.cumsum(lens)])
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    cand = rng.integers(0, N, (B, n_cand)).astype(np.int64)
    got = dz.scores(ix, torch.from_numpy(Q).to(DEV), q_lens,
                    cand_ids=torch.from_numpy(cand.astype(np.int32)).to(DEV)).cpu().numpy().reshape(B, n_cand)
    kl = launched(ix)
    assert kl == (L, max(Cb, 6), 2 if Cb > 8 else 1, 0, 1, False), kl
    for b in range(B):
        assert np.array_equal(got[b], orc.scores(dc, off, qc[qo[b]:qo[b + 1]], cand[b])), b
