"""GPU parity for wide codes (9..16 one-bit hashes per table, 16-bit codes) and for L = 8 tables: the shapes of the
paper's synthetic experiment (Sec. 6.1: 1000 documents of m vectors, L = 8, C = log2(m) + 1, queries = documents
with noise).  Everything is compared with the oracle bit for bit."""
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


def clustered(rng, n, d, pool, spread):
    return np.clip(pool[rng.integers(0, len(pool), n)] + rng.integers(-spread, spread + 1, (n, d)), -127, 127).astype(np.int8)


@pytest.mark.parametrize("d,L,Cb,n", [(128, 8, 11, 1000), (128, 8, 9, 33), (64, 4, 16, 257), (100, 12, 10, 64),
                                      (128, 32, 9, 129), (128, 8, 2, 500), (128, 8, 8, 65)])
def test_hash_wide_and_l8_bit_exact(d, L, Cb, n):
    say(f"hash d={d} L={L} C={Cb} n={n}")
    rng = np.random.default_rng(d + L + Cb)
    X = rng.integers(-127, 128, (n, d)).astype(np.int8)
    X[0] = 0
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    got = dz.hash(ix, torch.from_numpy(X).to(DEV))
    want = orc.hash_i8(X, R, L, Cb)
    assert got.cpu().numpy().dtype == want.dtype
    assert np.array_equal(got.cpu().numpy(), want)
    # the seed-derived matrix: same rule on both sides
    ix2 = dz.create(d, L, Cb, seed=99)
    assert np.array_equal(dz.hash(ix2, torch.from_numpy(X).to(DEV)).cpu().numpy(),
                          orc.hash_i8(X, orc.rademacher(99, L * Cb, d), L, Cb))


@pytest.mark.parametrize("algo", [dz.HASH_SCALAR, dz.HASH_MFMA])
@pytest.mark.parametrize("d,L,Cb", [(128, 8, 11), (128, 8, 9), (64, 8, 16), (256, 8, 10), (128, 16, 12), (64, 32, 9),
                                    (128, 32, 16), (256, 16, 13), (128, 8, 1), (64, 8, 8), (256, 8, 5), (128, 8, 7),
                                    # 128 bytes of code row: two launches of 32 tables each
                                    (128, 64, 9), (64, 64, 16), (256, 32, 12), (256, 64, 9), (128, 128, 9)])
@pytest.mark.parametrize("n", [1, 63, 64, 65, 1000, 4099])
def test_hash_mfma_wide_and_l8_shapes(algo, d, L, Cb, n):
    say(f"hash algo={algo} d={d} L={L} C={Cb} n={n}")
    rng = np.random.default_rng(d + L + Cb + n)
    X = rng.integers(-127, 128, (n, d)).astype(np.int8)
    X[0] = 0
    if n > 2:
        X[2] = -X[1]
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, algo, dz.SCORE_AUTO)
    got = dz.hash(ix, torch.from_numpy(X).to(DEV)).cpu().numpy()
    assert np.array_equal(got, orc.hash_i8(X, R, L, Cb))


def test_hash_wide_fp16_gaussian_within_tolerance():
    say("hash fp16/gaussian L=8 C=11")
    rng = np.random.default_rng(3)
    d, L, Cb, n = 128, 8, 11, 3000
    X = rng.standard_normal((n, d)).astype(np.float32)
    X = (X / np.linalg.norm(X, axis=1, keepdims=True)).astype(np.float16)
    R = rng.standard_normal((L * Cb, d)).astype(np.float32)
    ix = dz.create(d, L, Cb, dtype=dz.F16, proj_kind=dz.PROJ_GAUSSIAN_F32, proj=torch.from_numpy(R).to(DEV))
    got = dz.hash(ix, torch.from_numpy(X).to(DEV)).cpu().numpy()
    want, proj = orc.hash_fp(X, R, L, Cb, want_proj=True)
    gb = (got[..., None].astype(np.int64) >> np.arange(Cb)) & 1
    wb = (want[..., None].astype(np.int64) >> np.arange(Cb)) & 1
    diff = gb != wb
    assert diff.mean() <= 1e-4
    norms = np.linalg.norm(X.astype(np.float64), axis=1)
    margins = np.abs(proj.reshape(n, L, Cb))
    assert np.all(margins[diff] < 1e-3 * np.broadcast_to(norms[:, None, None], margins.shape)[diff])
    assert got.max() < 2 ** Cb


def scoring_case(rng, d, L, Cb, algo, eq1=False):
    lens = np.array([0, 1, 7, 8, 9, 70, 0, 31, 33, 64, 65, 2, 200, 0, 16, 1030], dtype=np.int64)
    lens = np.concatenate([lens, rng.integers(0, 40, 300)])
    V = int(lens.sum())
    pool = rng.integers(-100, 101, (15, d))
    X = clustered(rng, V, d, pool, 12)
    q_lens = np.array([1, 32, 33, 70, 7, 64], dtype=np.int64)
    Q = clustered(rng, int(q_lens.sum()), d, pool, 8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, dz.HASH_AUTO, algo)
    if eq1:
        dz.set_score_transform(ix, dz.SCORE_EQ1_Q16)
    codes, _ = dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    assert np.array_equal(codes.cpu().numpy(), dc)
    off = np.concatenate([[0], np.cumsum(lens)])
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    ref = (lambda q, sel=None: orc.scores_eq1(dc, off, q, Cb, sel)) if eq1 else (lambda q, sel=None: orc.scores(dc, off, q, sel))
    got = dz.scores(ix, torch.from_numpy(Q).to(DEV), q_lens).cpu().numpy()
    some = False
    for b in range(len(q_lens)):
        want = ref(qc[qo[b]:qo[b + 1]])
        some = some or want.max() > 0
        assert np.array_equal(got[b], want), b
    assert some
    n_docs = len(lens)
    cands = [np.array([5, 5, 0, 12, 3, 15]), np.array([], dtype=np.int64), np.arange(n_docs), np.array([9]),
             rng.integers(0, n_docs, 300), np.array([6, 0])]
    co = np.concatenate([[0], np.cumsum([len(c) for c in cands])])
    flat = np.concatenate(cands).astype(np.int64)
    empty = rng.random(flat.shape[0]) < 0.05
    flat_dev = torch.from_numpy(np.where(empty, 0xFFFFFFFF, flat).astype(np.uint32).view(np.int32)).to(DEV)
    got = dz.scores(ix, torch.from_numpy(Q).to(DEV), q_lens, cand_ids=flat_dev, cand_offsets=co).cpu().numpy()
    for b, c in enumerate(cands):
        want = ref(qc[qo[b]:qo[b + 1]], c) if len(c) else np.zeros(0, np.int32)
        want = np.where(empty[co[b]:co[b + 1]], -1, want)
        assert np.array_equal(got[co[b]:co[b + 1]], want), b
    # top-k through the same path
    ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), q_lens, 10)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    for b in range(len(q_lens)):
        want_ids, want_sc = orc.topk(ref(qc[qo[b]:qo[b + 1]]), 10)
        assert np.array_equal(ids[b], want_ids) and np.array_equal(sc[b], want_sc), b


@pytest.mark.parametrize("algo", [dz.SCORE_BYTECMP, dz.SCORE_MASKLUT])
@pytest.mark.parametrize("L,Cb", [(8, 9), (8, 10), (8, 11), (16, 9), (16, 10), (32, 9), (8, 2), (8, 5), (8, 7), (8, 8)])
def test_scores_wide_and_l8_shapes(algo, L, Cb):
    say(f"scores L={L} C={Cb} algo={algo}")
    scoring_case(np.random.default_rng(L * 100 + Cb), 64, L, Cb, algo)


@pytest.mark.parametrize("L,Cb", [(12, 13), (4, 16), (20, 9), (64, 9)])
def test_scores_wide_shapes_without_a_mask_table(L, Cb):
    say(f"scores (default kernel choice) L={L} C={Cb}")
    scoring_case(np.random.default_rng(L * 100 + Cb), 32, L, Cb, dz.SCORE_AUTO)


@pytest.mark.parametrize("L,Cb", [(8, 11), (8, 9), (16, 10), (8, 4), (12, 12)])
def test_scores_wide_eq1_transform(L, Cb):
    say(f"scores with Eq. 1 L={L} C={Cb}")
    scoring_case(np.random.default_rng(L * 1000 + Cb), 64, L, Cb, dz.SCORE_AUTO, eq1=True)


@pytest.mark.parametrize("m", [2, 4, 8, 16, 32, 64, 128, 256, 512, 1024])
def test_synthetic_experiment_shape(m):
    """Sec. 6.1: 1000 documents of m vectors, L = 8, C = log2(m) + 1, queries = documents with noise."""
    nq = 8 if m <= 256 else 3
    w = gen.make(gen.sweep_preset(m, nq))
    p = w.preset
    say(f"synthetic experiment m={m} L={p.L} C={p.C} N={w.n_docs} B={nq}")
    ix = dz.create(p.d, p.L, p.C, proj=w.proj.to(DEV))
    codes, offsets = dz.build_index(ix, w.docs.to(DEV), w.lengths)
    R = w.proj.numpy()
    dc, qc = orc.hash_i8(w.docs.numpy(), R, p.L, p.C), orc.hash_i8(w.queries.numpy(), R, p.L, p.C)
    assert np.array_equal(codes.cpu().numpy(), dc)
    ids, sc = dz.search(ix, w.queries.to(DEV), w.q_lengths, p.k)
    raw = dz.scores(ix, w.queries.to(DEV), w.q_lengths).cpu().numpy()
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    off = w.offsets.numpy()
    hits = 0
    for b in range(nq):
        want = orc.scores(dc, off, qc[b * m:(b + 1) * m])
        assert np.array_equal(raw[b], want), b
        want_ids, want_sc = orc.topk(want, p.k)
        assert np.array_equal(ids[b], want_ids) and np.array_equal(sc[b], want_sc), b
        hits += int(ids[b, 0] == int(w.planted[b, 0]))
    if m >= 8:
        assert hits == nq            # the paper's setting: the noisy copy of a document retrieves that document


@pytest.mark.parametrize("seed", range(8))
def test_random_wide_configuration_end_to_end(seed):
    rng = np.random.default_rng(5000 + seed)
    d = int(rng.choice([8, 50, 64, 128]))
    L = int(rng.choice([4, 8, 12, 16, 32]))
    Cb = int(rng.integers(9, 17))
    n_docs = int(rng.integers(1, 500))
    lens = rng.integers(0, int(rng.choice([3, 20, 90])), n_docs)
    if lens.sum() == 0:
        lens[0] = 2
    V = int(lens.sum())
    B = int(rng.integers(1, 5))
    q_lens = rng.integers(1, int(rng.choice([4, 33, 70])), B)
    k = int(rng.choice([1, 10, 64]))
    eq1 = bool(rng.integers(0, 2))
    say(f"random wide cfg seed={seed} d={d} L={L} C={Cb} N={n_docs} V={V} q_lens={q_lens.tolist()} k={k} eq1={eq1}")
    pool = rng.integers(-100, 101, (10, d))
    X = clustered(rng, V, d, pool, 6)
    nq = int(q_lens.sum())
    Q = clustered(rng, nq, d, pool, 4)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    if eq1:
        dz.set_score_transform(ix, dz.SCORE_EQ1_Q16)
    codes, _ = dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    assert np.array_equal(codes.cpu().numpy(), dc)
    off = np.concatenate([[0], np.cumsum(lens)])
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), q_lens, k)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    for b in range(B):
        q = qc[qo[b]:qo[b + 1]]
        s = orc.scores_eq1(dc, off, q, Cb) if eq1 else orc.scores(dc, off, q)
        want_ids, want_sc = orc.topk(s, k)
        assert np.array_equal(sc[b], want_sc) and np.array_equal(ids[b], want_ids), b
