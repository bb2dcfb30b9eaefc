"""GPU parity for the other inner aggregations (sigma = max / mean of phi(count / L), Sec. 4.1) and the weighted
outer sum (Sec. 4.2), against oracle_scores_general, bit for bit."""
import sys

import numpy as np
import pytest
import torch

import paper_2210_15748_amd as dz
from oracle import oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# transform -> (phi, sigma) of the oracle
KINDS = {dz.SCORE_EQ1_Q16: (orc.PHI_EQ1, orc.SIGMA_MAX),
         dz.SCORE_MAX_IDENTITY_Q16: (orc.PHI_IDENTITY, orc.SIGMA_MAX),
         dz.SCORE_MAX_EXPM1_Q16: (orc.PHI_EXPM1, orc.SIGMA_MAX),
         dz.SCORE_MAX_SIGMOID_Q16: (orc.PHI_SIGMOID, orc.SIGMA_MAX),
         dz.SCORE_MEAN_IDENTITY_Q16: (orc.PHI_IDENTITY, orc.SIGMA_MEAN),
         dz.SCORE_MEAN_EXPM1_Q16: (orc.PHI_EXPM1, orc.SIGMA_MEAN),
         dz.SCORE_MEAN_SIGMOID_Q16: (orc.PHI_SIGMOID, orc.SIGMA_MEAN)}


def say(msg):
    print("[case]", msg, flush=True)
    sys.stdout.flush()


def build_case(seed, d, L, Cb):
    rng = np.random.default_rng(seed)
    lens = np.concatenate([np.array([0, 1, 7, 8, 9, 70, 0, 31, 33, 64, 65, 2, 300]), rng.integers(0, 40, 200)])
    V = int(lens.sum())
    pool = rng.integers(-100, 101, (15, d))
    X = np.clip(pool[rng.integers(0, 15, V)] + rng.integers(-12, 13, (V, d)), -127, 127).astype(np.int8)
    q_lens = np.array([1, 32, 33, 70, 7], dtype=np.int64)
    nq = int(q_lens.sum())
    Q = np.clip(pool[rng.integers(0, 15, nq)] + rng.integers(-8, 9, (nq, d)), -127, 127).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    return rng, lens, X, q_lens, Q, R


@pytest.mark.parametrize("transform", sorted(KINDS))
@pytest.mark.parametrize("weighted", [False, True])
@pytest.mark.parametrize("L,Cb,algo", [(32, 7, dz.SCORE_AUTO), (32, 7, dz.SCORE_BYTECMP), (8, 11, dz.SCORE_AUTO),
                                       (12, 5, dz.SCORE_AUTO), (64, 8, dz.SCORE_AUTO), (16, 3, dz.SCORE_MASKLUT)])
def test_aggregations_match_oracle(transform, weighted, L, Cb, algo):
    phi, sigma = KINDS[transform]
    if algo == dz.SCORE_MASKLUT and sigma == orc.SIGMA_MEAN and phi != orc.PHI_IDENTITY:
        pytest.skip("of the means only phi = identity has a mask-table form (the others are checked as an error below)")
    say(f"aggregation transform={transform} weighted={weighted} L={L} C={Cb} algo={algo}")
    rng, lens, X, q_lens, Q, R = build_case(L * 100 + Cb + transform, 64, L, Cb)
    ix = dz.create(64, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, dz.HASH_AUTO, algo)
    dz.set_score_transform(ix, transform)
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    off = np.concatenate([[0], np.cumsum(lens)])
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    w = None
    if weighted:
        w = rng.integers(0, 65537, Q.shape[0]).astype(np.uint32)
        w[:3] = [65536, 0, 1]
        dz.set_query_weights(ix, torch.from_numpy(w.view(np.int32)).to(DEV))
    want_masklut = algo != dz.SCORE_BYTECMP and (L, Cb) != (12, 5) and (sigma == orc.SIGMA_MAX or phi == orc.PHI_IDENTITY)
    ref = lambda b, sel=None: orc.scores_general(dc, off, qc[qo[b]:qo[b + 1]], phi, sigma, weights=None if w is None else w[qo[b]:qo[b + 1]],
                                                 doc_ids=sel, eq1_C=Cb)
    Qd = torch.from_numpy(Q).to(DEV)
    got = dz.scores(ix, Qd, q_lens).cpu().numpy()
    assert dz.last_score_kernel(ix).startswith("score_masklut_kernel" if want_masklut else "score_bytecmp_kernel"), dz.last_score_kernel(ix)
    for b in range(len(q_lens)):
        assert np.array_equal(got[b], ref(b)), b
    # candidate lists with an empty slot, then top-k
    n_docs = len(lens)
    cands = [rng.integers(0, n_docs, 50) for _ in q_lens]
    co = np.concatenate([[0], np.cumsum([len(c) for c in cands])])
    flat = np.concatenate(cands).astype(np.int64)
    flat_dev = flat.copy(); flat_dev[7] = 0xFFFFFFFF
    got = dz.scores(ix, Qd, q_lens, cand_ids=torch.from_numpy(flat_dev.astype(np.uint32).view(np.int32)).to(DEV), cand_offsets=co).cpu().numpy()
    for b, c in enumerate(cands):
        want = ref(b, c)
        if b == 0:
            want = want.copy(); want[7] = -1
        assert np.array_equal(got[co[b]:co[b + 1]], want), b
    ids, sc = dz.search(ix, Qd, q_lens, 10)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    for b in range(len(q_lens)):
        want_ids, want_sc = orc.topk(ref(b), 10)
        assert np.array_equal(ids[b], want_ids) and np.array_equal(sc[b], want_sc), b
    # removing the weights restores the unweighted scores
    if weighted:
        dz.set_query_weights(ix, None)
        got = dz.scores(ix, Qd, q_lens).cpu().numpy()
        assert np.array_equal(got[1], orc.scores_general(dc, off, qc[qo[1]:qo[2]], phi, sigma, eq1_C=Cb))


def test_aggregation_argument_errors():
    rng, lens, X, q_lens, Q, R = build_case(1, 64, 32, 7)
    ix = dz.create(64, 32, 7, proj=torch.from_numpy(R).to(DEV))
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    Qd = torch.from_numpy(Q).to(DEV)
    with pytest.raises(dz.DessertError):
        dz.set_score_transform(ix, 8)
    w = torch.full((Q.shape[0],), 65536, dtype=torch.int32, device=DEV)
    dz.set_query_weights(ix, w)
    with pytest.raises(dz.DessertError, match="fixed-point"):
        dz.scores(ix, Qd, q_lens)                      # raw counts take no weights
    dz.set_score_transform(ix, dz.SCORE_MAX_IDENTITY_Q16)
    dz.set_query_weights(ix, w[:-1])
    with pytest.raises(dz.DessertError, match="query weights"):
        dz.scores(ix, Qd, q_lens)                      # wrong number of weights
    dz.set_query_weights(ix, None)
    dz.set_score_transform(ix, dz.SCORE_MEAN_EXPM1_Q16)
    dz.set_algo(ix, dz.HASH_AUTO, dz.SCORE_MASKLUT)
    with pytest.raises(dz.DessertError, match="code-compare"):
        dz.scores(ix, Qd, q_lens)
    # switching transforms back and forth gives the same results as a fresh index
    dz.set_algo(ix, dz.HASH_AUTO, dz.SCORE_AUTO)
    a = dz.scores(ix, Qd, q_lens).cpu().numpy()
    dz.set_score_transform(ix, dz.SCORE_RAW_COUNTS)
    raw = dz.scores(ix, Qd, q_lens).cpu().numpy()
    dz.set_score_transform(ix, dz.SCORE_MEAN_EXPM1_Q16)
    assert np.array_equal(a, dz.scores(ix, Qd, q_lens).cpu().numpy())
    dc, qc = orc.hash_i8(X, R, 32, 7), orc.hash_i8(Q, R, 32, 7)
    off = np.concatenate([[0], np.cumsum(lens)])
    assert np.array_equal(raw[0], orc.scores(dc, off, qc[:1]))
