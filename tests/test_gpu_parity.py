"""GPU parity: every call goes through the C ABI (via the thin binding) and is compared
element by element with the CPU oracle on the same seeded inputs.  Integer paths are bit-exact."""
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


def oracle_codes(w):
    p = w.preset
    R = w.proj.cpu().numpy()
    fn = orc.hash_i8 if p.dtype == "i8" else orc.hash_fp
    return fn(w.docs.cpu().numpy(), R, p.L, p.C), fn(w.queries.cpu().numpy(), R, p.L, p.C)


def make_index(w, hash_algo=dz.HASH_AUTO, score_algo=dz.SCORE_AUTO):
    p = w.preset
    ix = dz.create(p.d, p.L, p.C, dtype=dz.I8 if p.dtype == "i8" else dz.F16,
                   proj_kind=dz.PROJ_RADEMACHER_I8 if p.proj_kind == "rademacher" else dz.PROJ_GAUSSIAN_F32,
                   proj=w.proj.to(DEV))
    dz.set_algo(ix, hash_algo, score_algo)
    codes, offsets = dz.build_index(ix, w.docs.to(DEV), w.lengths)
    return ix, codes, offsets


# ------------------------------------------------------------------ hashing
@pytest.mark.parametrize("algo", [dz.HASH_SCALAR, dz.HASH_MFMA])
@pytest.mark.parametrize("n", [1, 31, 32, 33, 63, 64, 65, 127, 129, 1000, 4099])
def test_hash_i8_bit_exact_ragged_sizes(algo, n):
    say(f"hash algo={algo} n={n} d=128 L=32 C=7")
    rng = np.random.default_rng(n)
    X = rng.integers(-127, 128, (n, 128)).astype(np.int8)
    X[0] = 0                                   # all projections exactly zero -> every bit 1
    R = (rng.integers(0, 2, (224, 128)) * 2 - 1).astype(np.int8)
    ix = dz.create(128, 32, 7, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, algo, dz.SCORE_AUTO)
    got = dz.hash(ix, torch.from_numpy(X).to(DEV)).cpu().numpy()
    want = orc.hash_i8(X, R, 32, 7)
    assert np.array_equal(got, want)
    assert np.all(got[0] == 127)


@pytest.mark.parametrize("d,L,Cb", [(128, 16, 6), (64, 16, 1), (256, 32, 8), (128, 64, 5), (64, 64, 8), (256, 16, 4),
                                    # more than 64 bytes of code row: hashed in table groups, one launch per group
                                    (128, 128, 5), (64, 128, 8), (128, 128, 1), (256, 64, 8), (256, 128, 5)])
def test_hash_mfma_shapes(d, L, Cb):
    say(f"hash mfma d={d} L={L} C={Cb}")
    rng = np.random.default_rng(d + L + Cb)
    n = 777
    # small magnitudes make exact-zero projections frequent: exercises the sign(0) rule
    X = rng.integers(-2, 3, (n, d)).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, dz.HASH_MFMA, dz.SCORE_AUTO)
    got = dz.hash(ix, torch.from_numpy(X).to(DEV)).cpu().numpy()
    codes, proj = orc.hash_i8(X, R, L, Cb, want_proj=True)
    assert (proj == 0).mean() > 0.01
    assert np.array_equal(got, codes)


@pytest.mark.parametrize("L,Cb,n", [(32, 7, 1_200_001), (32, 3, 70_000), (64, 8, 140_003), (16, 12, 150_000), (32, 9, 140_003),
                                    (128, 7, 70_001), (64, 11, 70_001)])
def test_hash_long_runs_several_tiles_per_wave(L, Cb, n):
    """Runs long enough that a wave of the MFMA kernel loops over several tiles (more than 4096 workgroups x 4 waves x
    64 vectors in the first case), ragged tail, both code widths."""
    say(f"hash long run L={L} C={Cb} n={n}")
    rng = np.random.default_rng(L * 31 + Cb)
    d = 128
    X = rng.integers(-127, 128, (n, d)).astype(np.int8)
    X[::1001] = 0
    X[n - 1] = -X[0]
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, dz.HASH_MFMA, dz.SCORE_AUTO)
    got = dz.hash(ix, torch.from_numpy(X).to(DEV)).cpu().numpy()
    assert np.array_equal(got, orc.hash_i8(X, R, L, Cb))


def test_hash_scalar_odd_shapes_and_seed_rule():
    say("hash scalar d=50 L=12 C=3 seed-derived projection")
    rng = np.random.default_rng(1)
    d, L, Cb, n = 50, 12, 3, 301
    X = rng.integers(-127, 128, (n, d)).astype(np.int8)
    ix = dz.create(d, L, Cb, seed=987654321)
    R = dz.get_projection(ix).cpu().numpy()
    assert np.array_equal(R, orc.rademacher(987654321, L * Cb, d))
    got = dz.hash(ix, torch.from_numpy(X).to(DEV)).cpu().numpy()
    assert np.array_equal(got, orc.hash_i8(X, R, L, Cb))


@pytest.mark.parametrize("algo", [dz.HASH_SCALAR, dz.HASH_MFMA])
@pytest.mark.parametrize("d,L,Cb,n", [(256, 64, 8, 5000), (128, 32, 7, 1000), (64, 16, 3, 333),
                                      # L = 128: two groups of 64 tables; L = 8: a single dword of codes per lane half
                                      (128, 128, 8, 3000), (256, 128, 6, 2000), (64, 8, 5, 1000)])
def test_hash_fp16_gaussian_within_tolerance(algo, d, L, Cb, n):
    say(f"hash f16 x gaussian f32 algo={algo} d={d} L={L} C={Cb} n={n}")
    rng = np.random.default_rng(d + L + Cb)
    X = rng.standard_normal((n, d))
    X = (X / np.linalg.norm(X, axis=1, keepdims=True)).astype(np.float16)
    X[0] = 0                                   # zero vector: every projection is +0 -> every bit 1
    R = rng.standard_normal((L * Cb, d)).astype(np.float32)
    R[5, :] *= 1e-3                            # a row of small entries (lo part of the split underflows less gracefully)
    ix = dz.create(d, L, Cb, dtype=dz.F16, proj_kind=dz.PROJ_GAUSSIAN_F32, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, algo, dz.SCORE_AUTO)
    got = dz.hash(ix, torch.from_numpy(X).to(DEV)).cpu().numpy()
    want, proj = orc.hash_fp(X, R, L, Cb, want_proj=True)
    assert np.all(got[0] == (1 << Cb) - 1)
    bits_got = np.unpackbits(got[..., None], axis=2, bitorder="little")[:, :, :Cb]
    bits_want = np.unpackbits(want[..., None], axis=2, bitorder="little")[:, :, :Cb]
    diff = bits_got != bits_want
    assert diff.mean() <= 1e-4, diff.mean()
    norms = np.linalg.norm(X.astype(np.float64), axis=1)
    margins = np.abs(proj.reshape(n, L, Cb))
    rnorm = np.linalg.norm(R.astype(np.float64), axis=1).reshape(L, Cb) / np.sqrt(d)
    # a mismatch is allowed only where the projection is within 1e-3*||x|| of zero: the plain bound, and for a row of small
    # entries (rms below 1, whose projections are all small) that bound scaled down with the row, never up
    bound = 1e-3 * norms[:, None, None] * np.clip(rnorm[None], 1e-30, 1.0)
    assert np.all(margins[diff] < np.broadcast_to(bound, margins.shape)[diff])
    assert got.max() < (1 << Cb)


# ------------------------------------------------------------------ index build
def test_build_index_codes_and_offsets_cfg1():
    say("build_index cfg1")
    w = gen.make(1)
    ix, codes, offsets = make_index(w)
    dc, _ = oracle_codes(w)
    assert np.array_equal(codes.cpu().numpy(), dc)
    assert np.array_equal(offsets.cpu().numpy(), w.offsets.numpy())


# ------------------------------------------------------------------ scoring
def check_scores(w, score_algo, tag):
    p = w.preset
    say(f"scores {tag} algo={score_algo} N={w.n_docs} B={p.n_queries} |Q|={p.q_len} L={p.L} C={p.C} cand={p.n_cand}")
    ix, codes, _ = make_index(w, score_algo=score_algo)
    dc, qc = oracle_codes(w)
    assert np.array_equal(codes.cpu().numpy(), dc)
    got = dz.scores(ix, w.queries.to(DEV), w.q_lengths, cand_ids=None if w.cand_ids is None else w.cand_ids.to(DEV))
    got = got.cpu().numpy().reshape(p.n_queries, -1)
    off = w.offsets.numpy()
    qo = np.concatenate([[0], np.cumsum(w.q_lengths.numpy())])
    for b in range(p.n_queries):
        cand = None if w.cand_ids is None else w.cand_ids[b].cpu().numpy()
        want = orc.scores(dc, off, qc[qo[b]:qo[b + 1]], cand)
        assert np.array_equal(got[b], want), (tag, b)
    return ix, dc, qc


@pytest.mark.parametrize("algo", [dz.SCORE_BYTECMP, dz.SCORE_MASKLUT])
def test_scores_cfg1_full(algo):
    check_scores(gen.make(1), algo, "cfg1")


@pytest.mark.parametrize("algo", [dz.SCORE_BYTECMP, dz.SCORE_MASKLUT])
def test_scores_cfg2_reduced(algo):
    check_scores(gen.make(2, n_docs=3001, n_queries=5), algo, "cfg2-reduced")


@pytest.mark.parametrize("algo", [dz.SCORE_BYTECMP, dz.SCORE_MASKLUT])
def test_scores_cfg3_reduced_candidates(algo):
    check_scores(gen.make(3, n_docs=20000, n_queries=6, n_cand=777), algo, "cfg3-reduced")


@pytest.mark.parametrize("algo", [dz.SCORE_BYTECMP, dz.SCORE_MASKLUT])
def test_scores_edge_lengths_and_ragged_queries(algo):
    say(f"scores edge cases algo={algo}")
    rng = np.random.default_rng(77)
    d, L, Cb = 128, 32, 7
    lens = np.array([0, 1, 15, 16, 17, 180, 0, 31, 33, 64, 65, 2, 0], dtype=np.int64)
    V = int(lens.sum())
    # few distinct vectors so that collisions (and ties) are common
    pool = rng.integers(-127, 128, (12, d)).astype(np.int8)
    X = pool[rng.integers(0, 12, V)]
    fresh = rng.random(V) < 0.3
    X[fresh] = rng.integers(-127, 128, (int(fresh.sum()), d)).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    q_lens = np.array([1, 32, 33, 40, 7, 64], dtype=np.int64)
    Q = pool[rng.integers(0, 12, int(q_lens.sum()))]
    noise = rng.integers(-20, 21, Q.shape)
    Q = np.clip(Q.astype(np.int64) + noise, -127, 127).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, dz.HASH_AUTO, algo)
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    off = np.concatenate([[0], np.cumsum(lens)])
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    # exhaustive
    got = dz.scores(ix, torch.from_numpy(Q).to(DEV), q_lens).cpu().numpy()
    for b in range(len(q_lens)):
        assert np.array_equal(got[b], orc.scores(dc, off, qc[qo[b]:qo[b + 1]])), b
    # ragged candidate lists with duplicates and an empty list
    cands = [np.array([5, 5, 0, 12, 3]), np.array([], dtype=np.int64), np.arange(13), np.array([9]),
             rng.integers(0, 13, 300), np.array([6, 0])]
    co = np.concatenate([[0], np.cumsum([len(c) for c in cands])])
    flat = torch.from_numpy(np.concatenate(cands).astype(np.int32)).to(DEV)
    got = dz.scores(ix, torch.from_numpy(Q).to(DEV), q_lens, cand_ids=flat, cand_offsets=co).cpu().numpy()
    for b, c in enumerate(cands):
        assert np.array_equal(got[co[b]:co[b + 1]], orc.scores(dc, off, qc[qo[b]:qo[b + 1]], c)), b


@pytest.mark.parametrize("L,Cb,eq1,hash_algo", [(32, 7, False, dz.HASH_AUTO), (64, 8, True, dz.HASH_AUTO),
                                                 (8, 11, False, dz.HASH_AUTO),
                                                 (32, 7, False, dz.HASH_SCALAR),   # the grouping as a launch of its own
                                                 (16, 9, True, dz.HASH_SCALAR)])
def test_scores_long_candidate_lists_in_any_id_order(L, Cb, eq1, hash_algo):
    """Lists long enough for the mask-table kernel to take them grouped by document id range: uniform ids, ids all
    from one narrow range (one range gets nearly everything), descending ids, empty slots and repeats, lists of unequal
    length, one too short for the grouping.  Every score must land in its own slot."""
    say(f"long candidate lists L={L} C={Cb} eq1={eq1} hash_algo={hash_algo}")
    rng = np.random.default_rng(L + Cb)
    d, N = 64, 50_000
    lens = rng.integers(0, 6, N)
    V = int(lens.sum())
    pool = rng.integers(-127, 128, (30, d))
    X = np.clip(pool[rng.integers(0, 30, V)] + rng.integers(-40, 41, (V, d)), -127, 127).astype(np.int8)
    q_lens = np.array([5, 33, 2, 9, 4, 1, 12, 7], dtype=np.int64)  # eight lists or more are grouped
    nq = int(q_lens.sum())
    Q = np.clip(pool[rng.integers(0, 30, nq)] + rng.integers(-40, 41, (nq, d)), -127, 127).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, hash_algo, dz.SCORE_AUTO)
    if eq1:
        dz.set_score_transform(ix, dz.SCORE_EQ1_Q16)
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    EMPTY = 0xFFFFFFFF
    with_gaps = rng.integers(0, N, 3000).astype(np.int64)
    with_gaps[::7] = EMPTY
    cands = [rng.integers(0, N, 5000).astype(np.int64),                     # uniform, with repeats
             rng.integers(20_000, 20_040, 2500).astype(np.int64),           # one narrow range
             np.arange(N - 1, N - 1 - 1500, -1).astype(np.int64),           # descending
             with_gaps,                                                     # empty slots
             rng.integers(0, N, 700).astype(np.int64),                      # shorter than the others
             np.sort(rng.integers(0, N, 1024)).astype(np.int64),            # ascending
             np.full(1100, 31_337, dtype=np.int64),                         # one document over and over
             rng.integers(N - 300, N, 2048).astype(np.int64)]               # the top of the id range
    co = np.concatenate([[0], np.cumsum([len(c) for c in cands])])
    flat = torch.from_numpy(np.concatenate(cands).astype(np.uint32).view(np.int32)).to(DEV)
    got = dz.scores(ix, torch.from_numpy(Q).to(DEV), q_lens, cand_ids=flat, cand_offsets=co).cpu().numpy()
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    off = np.concatenate([[0], np.cumsum(lens)])
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    for b, c in enumerate(cands):
        real = c != EMPTY
        q = qc[qo[b]:qo[b + 1]]
        want_real = orc.scores_eq1(dc, off, q, Cb, c[real]) if eq1 else orc.scores(dc, off, q, c[real])
        want = np.full(len(c), -1, dtype=np.int64)
        want[real] = want_real
        assert np.array_equal(got[co[b]:co[b + 1]].astype(np.int64), want), b
    # the same lists through the top-k
    ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), q_lens, 50, cand_ids=flat, cand_offsets=co)
    for b, c in enumerate(cands):
        real = c != EMPTY
        w_ids, w_sc = orc.topk(got[co[b]:co[b + 1]][real], 50, c[real])
        assert np.array_equal(sc.cpu().numpy()[b], w_sc) and np.array_equal(ids.cpu().numpy()[b], w_ids), b


@pytest.mark.parametrize("L,Cb", [(16, 6), (64, 8), (128, 5), (16, 8)])
def test_scores_masklut_other_shapes(L, Cb):
    say(f"scores masklut L={L} C={Cb}")
    rng = np.random.default_rng(L * 10 + Cb)
    d = 64
    lens = rng.integers(1, 40, 300)
    V = int(lens.sum())
    pool = rng.integers(-127, 128, (40, d))
    X = np.clip(pool[rng.integers(0, 40, V)] + rng.integers(-30, 31, (V, d)), -127, 127).astype(np.int8)
    Q = np.clip(pool[rng.integers(0, 40, 50)] + rng.integers(-30, 31, (50, d)), -127, 127).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, dz.HASH_AUTO, dz.SCORE_MASKLUT)
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    off = np.concatenate([[0], np.cumsum(lens)])
    got = dz.scores(ix, torch.from_numpy(Q).to(DEV), [20, 30]).cpu().numpy()
    assert np.array_equal(got[0], orc.scores(dc, off, qc[:20]))
    assert np.array_equal(got[1], orc.scores(dc, off, qc[20:]))


@pytest.mark.parametrize("L,Cb", [(8, 7), (16, 6), (32, 7), (64, 8), (128, 6)])
def test_scores_short_documents_at_every_line_alignment(L, Cb):
    """The scoring rounds start on 128-byte lines of the code array: documents of 1..12 vectors placed so that
    every start position modulo a line occurs, first and last documents included, candidate lists and all documents."""
    say(f"scores short documents at every alignment L={L} C={Cb}")
    rng = np.random.default_rng(900 + L)
    d = 64
    lens = np.concatenate([np.arange(1, 13), rng.integers(1, 13, 400), [1, 1, 1, 2, 3, 5, 7, 11, 12, 1]]).astype(np.int64)
    V = int(lens.sum())
    off = np.concatenate([[0], np.cumsum(lens)])
    rows_per_line = max(1, 128 // L)
    assert len(set((off[:-1] % rows_per_line).tolist())) == rows_per_line
    pool = rng.integers(-127, 128, (30, d))
    X = np.clip(pool[rng.integers(0, 30, V)] + rng.integers(-25, 26, (V, d)), -127, 127).astype(np.int8)
    q_lens = np.array([32, 9, 40], dtype=np.int64)
    Q = np.clip(pool[rng.integers(0, 30, int(q_lens.sum()))] + rng.integers(-25, 26, (int(q_lens.sum()), d)), -127, 127).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, dz.HASH_AUTO, dz.SCORE_MASKLUT)
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    got = dz.scores(ix, torch.from_numpy(Q).to(DEV), q_lens).cpu().numpy()
    for b in range(len(q_lens)):
        assert np.array_equal(got[b], orc.scores(dc, off, qc[qo[b]:qo[b + 1]])), b
    n = len(lens)
    cands = [rng.permutation(n)[:137], np.array([0, n - 1, n - 2, 1]), rng.integers(0, n, 300)]
    co = np.concatenate([[0], np.cumsum([len(c) for c in cands])])
    flat = torch.from_numpy(np.concatenate(cands).astype(np.int32)).to(DEV)
    got = dz.scores(ix, torch.from_numpy(Q).to(DEV), q_lens, cand_ids=flat, cand_offsets=co).cpu().numpy()
    for b, c in enumerate(cands):
        assert np.array_equal(got[co[b]:co[b + 1]], orc.scores(dc, off, qc[qo[b]:qo[b + 1]], c)), b


def test_build_index_again_on_the_same_handle():
    """Two builds in a row on one handle (the offsets travel on the library's own stream beside the hash kernel),
    each searched straight away without a synchronisation in between."""
    say("build_index twice on one handle, search after each")
    rng = np.random.default_rng(4242)
    d, L, Cb = 128, 32, 7
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    Q = rng.integers(-127, 128, (32, d)).astype(np.int8)
    qc = orc.hash_i8(Q, R, L, Cb)
    codes = offsets = None
    for n_docs, lo, hi in [(5000, 1, 40), (1200, 8, 100), (7000, 1, 12)]:
        lens = rng.integers(lo, hi, n_docs).astype(np.int64)
        X = rng.integers(-127, 128, (int(lens.sum()), d)).astype(np.int8)
        X[rng.integers(0, len(X), 64)] = Q[rng.integers(0, 32, 64)]     # some exact copies of query vectors
        codes, offsets = dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
        ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), [32], 20)
        dc = orc.hash_i8(X, R, L, Cb)
        off = np.concatenate([[0], np.cumsum(lens)])
        assert np.array_equal(offsets.cpu().numpy(), off)
        want_ids, want_sc, _ = orc.search(dc, off, [qc], 20)
        assert np.array_equal(ids.cpu().numpy(), want_ids)
        assert np.array_equal(sc.cpu().numpy(), want_sc)


def test_attach_index_resumes_without_rehashing(tmp_path):
    """An index is its code array and offsets (Alg. 1's sketch): saved, reloaded and attached to a new handle made with the
    same projection matrix it answers exactly as the handle that built it, filter included."""
    say("attach_index: save codes / offsets / projection, attach to a fresh handle")
    w = gen.make(3, n_docs=5000, n_queries=9, n_cand=300)
    p = w.preset
    ix, codes, offsets = make_index(w)
    q, cand = w.queries.to(DEV), w.cand_ids.to(DEV)
    want = dz.search(ix, q, w.q_lengths, p.k, cand_ids=cand)
    want_all = dz.search(ix, q, w.q_lengths, 7)
    torch.save({"codes": codes.cpu(), "offsets": offsets.cpu(), "proj": dz.get_projection(ix).cpu()}, tmp_path / "index.pt")
    del ix
    saved = torch.load(tmp_path / "index.pt", weights_only=True)
    ix2 = dz.create(p.d, p.L, p.C, proj=saved["proj"].to(DEV))
    with pytest.raises(dz.DessertError) as e:
        dz.search(ix2, q, w.q_lengths, p.k, cand_ids=cand)
    assert e.value.status == dz.ESTATE
    dz.attach_index(ix2, saved["codes"].to(DEV), saved["offsets"].to(DEV))
    got = dz.search(ix2, q, w.q_lengths, p.k, cand_ids=cand)
    got_all = dz.search(ix2, q, w.q_lengths, 7)
    assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1])
    assert torch.equal(got_all[0], want_all[0]) and torch.equal(got_all[1], want_all[1])
    dc, qc = oracle_codes(w)
    qs = [qc[b * p.q_len:(b + 1) * p.q_len] for b in range(p.n_queries)]
    o_ids, o_sc, _ = orc.search(dc, w.offsets.numpy(), qs, 7)
    assert np.array_equal(got_all[0].cpu().numpy(), o_ids) and np.array_equal(got_all[1].cpu().numpy(), o_sc)
    l = dz.lib()
    assert l.dessert_attach_index(ix2.handle, None, ix2.offsets.data_ptr(), 5, 10, 3) == dz.EINVAL
    assert l.dessert_attach_index(ix2.handle, ix2.codes.data_ptr(), None, 5, 10, 3) == dz.EINVAL
    assert l.dessert_attach_index(ix2.handle, ix2.codes.data_ptr(), ix2.offsets.data_ptr(), 5, 10, 11) == dz.EINVAL
    assert l.dessert_attach_index(ix2.handle, ix2.codes.data_ptr(), ix2.offsets.data_ptr(), 5, 10, 0) == dz.EINVAL


def test_score_transform_switches_in_stream_order_without_waiting():
    """dessert_set_score_transform writes the new table in stream order: calls enqueued before the switch use the old
    table, calls after it the new one, with no synchronisation in between."""
    say("score transform switched between back-to-back calls")
    w = gen.make(2, n_docs=4000, n_queries=6)
    p = w.preset
    ix, codes, _ = make_index(w)
    q = w.queries.to(DEV)
    outs = []
    for t in (dz.SCORE_EQ1_Q16, dz.SCORE_MAX_EXPM1_Q16, dz.SCORE_RAW_COUNTS, dz.SCORE_MAX_SIGMOID_Q16, dz.SCORE_EQ1_Q16):
        dz.set_score_transform(ix, t)
        outs.append((t, dz.scores(ix, q, w.q_lengths)))          # no synchronisation between the calls
    torch.cuda.synchronize()
    dc, qc = oracle_codes(w)
    off = w.offsets.numpy()
    kinds = {dz.SCORE_EQ1_Q16: orc.PHI_EQ1, dz.SCORE_MAX_EXPM1_Q16: orc.PHI_EXPM1, dz.SCORE_MAX_SIGMOID_Q16: orc.PHI_SIGMOID}
    for t, got in outs:
        g = got.cpu().numpy()
        for b in (0, 5):
            qb = qc[b * p.q_len:(b + 1) * p.q_len]
            want = orc.scores(dc, off, qb) if t == dz.SCORE_RAW_COUNTS else orc.scores_general(dc, off, qb, kinds[t], orc.SIGMA_MAX, eq1_C=p.C)
            assert np.array_equal(g[b], want), (t, b)


# ------------------------------------------------------------------ top-k and whole search
def check_search(w, tag, score_algo=dz.SCORE_AUTO):
    p = w.preset
    say(f"search {tag} N={w.n_docs} B={p.n_queries} k={p.k} cand={p.n_cand}")
    ix, codes, _ = make_index(w, score_algo=score_algo)
    dc, qc = oracle_codes(w)
    cand = None if w.cand_ids is None else w.cand_ids.to(DEV)
    ids, sc = dz.search(ix, w.queries.to(DEV), w.q_lengths, p.k, cand_ids=cand)
    qo = np.concatenate([[0], np.cumsum(w.q_lengths.numpy())])
    qs = [qc[qo[b]:qo[b + 1]] for b in range(p.n_queries)]
    want_ids, want_sc, _ = orc.search(dc, w.offsets.numpy(), qs, p.k,
                                      None if w.cand_ids is None else w.cand_ids.cpu().numpy())
    assert np.array_equal(sc.cpu().numpy(), want_sc), tag
    assert np.array_equal(ids.cpu().numpy(), want_ids), tag
    return ids.cpu().numpy()


def test_search_cfg1_full():
    w = gen.make(1)
    ids = check_search(w, "cfg1")
    assert np.array_equal(ids[:, 0], w.planted[:, 0].numpy())


def test_search_cfg2_reduced():
    check_search(gen.make(2, n_docs=5000, n_queries=4), "cfg2-reduced")


def test_search_cfg3_reduced():
    w = gen.make(3, n_docs=30000, n_queries=5, n_cand=1024)
    ids = check_search(w, "cfg3-reduced")
    # each planted document contributed only 4 of the 32 query vectors; most still reach the top-10
    for b in range(5):
        assert len(set(w.planted[b].tolist()) & set(ids[b].tolist())) >= 4


def test_search_k_larger_than_scored_and_all_ties():
    say("search: k > n, all-equal scores, duplicate candidates")
    d, L, Cb = 128, 32, 7
    rng = np.random.default_rng(5)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    x = rng.integers(-127, 128, (1, d)).astype(np.int8)
    lens = np.full(50, 3)
    X = np.repeat(x, 150, axis=0)                        # every document identical: all scores tie
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    Q = np.repeat(x, 4, axis=0)
    ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), [4], 64)
    ids, sc = ids.cpu().numpy()[0], sc.cpu().numpy()[0]
    assert ids[:50].tolist() == list(range(50)) and np.all(sc[:50] == 4 * L)
    assert np.all(ids[50:] == 0xFFFFFFFF) and np.all(sc[50:] == -1)
    cand = torch.tensor([7, 3, 7, 49, 3, 0], dtype=torch.int32, device=DEV)
    ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), [4], 4, cand_ids=cand, cand_offsets=[0, 6])
    assert ids.cpu().numpy()[0].tolist() == [0, 3, 3, 7]


def test_search_two_level_topk_many_short_documents():
    say("search: 300000 one-to-three-vector documents, sliced top-k")
    rng = np.random.default_rng(21)
    d, L, Cb, N = 64, 16, 4, 300_000
    lens = rng.integers(1, 4, N)
    V = int(lens.sum())
    pool = rng.integers(-127, 128, (64, d))
    X = np.clip(pool[rng.integers(0, 64, V)] + rng.integers(-60, 61, (V, d)), -127, 127).astype(np.int8)
    Q = np.clip(pool[rng.integers(0, 64, 6)] + rng.integers(-60, 61, (6, d)), -127, 127).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), [2, 4], 100)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    off = np.concatenate([[0], np.cumsum(lens)])
    want_ids, want_sc, _ = orc.search(dc, off, [qc[:2], qc[2:]], 100)
    assert np.array_equal(sc.cpu().numpy(), want_sc)
    assert np.array_equal(ids.cpu().numpy(), want_ids)


def test_search_with_the_largest_number_of_query_sets():
    """65 535 query sets in one call (the limit the header states), exhaustive and with candidate lists; scores of a
    sample of the sets and every top-k against the oracle."""
    say("search: 65535 query sets of 1-2 vectors")
    rng = np.random.default_rng(77)
    d, L, Cb, N, B = 64, 16, 5, 300, 65535
    lens = rng.integers(0, 5, N)
    V = int(lens.sum())
    pool = rng.integers(-127, 128, (32, d))
    X = np.clip(pool[rng.integers(0, 32, V)] + rng.integers(-40, 41, (V, d)), -127, 127).astype(np.int8)
    q_lens = rng.integers(1, 3, B).astype(np.int64)
    nq = int(q_lens.sum())
    Q = np.clip(pool[rng.integers(0, 32, nq)] + rng.integers(-40, 41, (nq, d)), -127, 127).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    off = np.concatenate([[0], np.cumsum(lens)])
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    Qd = torch.from_numpy(Q).to(DEV)
    raw = dz.scores(ix, Qd, q_lens).cpu().numpy()
    ids, sc = dz.search(ix, Qd, q_lens, 5)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    sample = np.unique(np.concatenate([[0, 1, B - 2, B - 1], rng.integers(0, B, 1500)]))
    for b in sample:
        assert np.array_equal(raw[b], orc.scores(dc, off, qc[qo[b]:qo[b + 1]])), b
    for b in range(B):
        want_ids, want_sc = orc.topk(raw[b], 5)
        assert np.array_equal(ids[b], want_ids) and np.array_equal(sc[b], want_sc), b
    cand = rng.integers(0, N, (B, 6)).astype(np.int64)
    got = dz.scores(ix, Qd, q_lens, cand_ids=torch.from_numpy(cand.astype(np.int32)).to(DEV)).cpu().numpy().reshape(B, 6)
    for b in sample:
        assert np.array_equal(got[b], orc.scores(dc, off, qc[qo[b]:qo[b + 1]], cand[b])), b
    with pytest.raises(dz.DessertError) as e:
        dz.scores(ix, torch.cat([Qd, Qd[:1]]), np.concatenate([q_lens, [1]]))
    assert e.value.status == dz.EINVAL


@pytest.mark.parametrize("L,Cb", [(16, 6), (32, 7), (128, 8)])
def test_scores_one_very_long_document_among_short_ones(L, Cb):
    """A document of 200 000 vectors (longer than any 16-bit length field) between short and empty ones: every
    scoring form, exhaustive and as a candidate."""
    say(f"scores: a 200000-vector document, L={L} C={Cb}")
    rng = np.random.default_rng(L + Cb)
    d = 64
    lens = np.array([3, 0, 200_000, 1, 70, 0, 65_535, 65_536, 2], dtype=np.int64)
    V = int(lens.sum())
    pool = rng.integers(-127, 128, (40, d))
    X = np.clip(pool[rng.integers(0, 40, V)] + rng.integers(-50, 51, (V, d)), -127, 127).astype(np.int8)
    q_lens = np.array([32, 7, 40], dtype=np.int64)
    nq = int(q_lens.sum())
    Q = np.clip(pool[rng.integers(0, 40, nq)] + rng.integers(-50, 51, (nq, d)), -127, 127).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    off = np.concatenate([[0], np.cumsum(lens)])
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    Qd = torch.from_numpy(Q).to(DEV)
    cand = np.array([2, 7, 2, 0, 6, 1], dtype=np.int64)
    cand_dev = torch.from_numpy(np.tile(cand, (3, 1)).astype(np.int32)).to(DEV)
    forms = [(dz.SCORE_RAW_COUNTS, lambda q, sel: orc.scores(dc, off, q, sel)),
             (dz.SCORE_EQ1_Q16, lambda q, sel: orc.scores_eq1(dc, off, q, Cb, sel)),
             (dz.SCORE_MEAN_IDENTITY_Q16, lambda q, sel: orc.scores_general(dc, off, q, orc.PHI_IDENTITY, orc.SIGMA_MEAN, doc_ids=sel))]
    want = {t: [(ref(qc[qo[b]:qo[b + 1]], None), ref(qc[qo[b]:qo[b + 1]], cand)) for b in range(3)] for t, ref in forms}
    for algo in (dz.SCORE_MASKLUT, dz.SCORE_BYTECMP):
        dz.set_algo(ix, dz.HASH_AUTO, algo)
        for transform, _ in forms:
            if transform == dz.SCORE_MEAN_IDENTITY_Q16 and algo == dz.SCORE_MASKLUT:
                continue                        # documents over 65 535 vectors: the mean runs on the code-compare kernel
            dz.set_score_transform(ix, transform)
            got = dz.scores(ix, Qd, q_lens).cpu().numpy()
            gotc = dz.scores(ix, Qd, q_lens, cand_ids=cand_dev).cpu().numpy().reshape(3, len(cand))
            for b in range(3):
                assert np.array_equal(got[b], want[transform][b][0]), (algo, transform, b)
                assert np.array_equal(gotc[b], want[transform][b][1]), (algo, transform, b)
    dz.set_algo(ix, dz.HASH_AUTO, dz.SCORE_AUTO)
    dz.set_score_transform(ix, dz.SCORE_MEAN_IDENTITY_Q16)  # AUTO routes the mean to the kernel that takes such lengths
    got = dz.scores(ix, Qd, q_lens).cpu().numpy()
    assert np.array_equal(got[0], want[dz.SCORE_MEAN_IDENTITY_Q16][0][0])


def test_determinism_same_inputs_twice():
    say("determinism cfg3-reduced")
    w = gen.make(3, n_docs=20000, n_queries=4, n_cand=512)
    ix, _, _ = make_index(w)
    a = dz.search(ix, w.queries.to(DEV), w.q_lengths, 10, cand_ids=w.cand_ids.to(DEV))
    b = dz.search(ix, w.queries.to(DEV), w.q_lengths, 10, cand_ids=w.cand_ids.to(DEV))
    assert torch.equal(a[0].cpu(), b[0].cpu()) and torch.equal(a[1], b[1])


def test_search_before_build_is_a_state_error():
    ix = dz.create(128, 32, 7, seed=3)
    q = torch.zeros(4, 128, dtype=torch.int8, device=DEV)
    with pytest.raises(dz.DessertError) as e:
        dz.search(ix, q, [4], 3)
    assert e.value.status == dz.ESTATE


# ------------------------------------------------------------------ Eq. 1 score transform (Sec. 5)
@pytest.mark.parametrize("algo", [dz.SCORE_BYTECMP, dz.SCORE_MASKLUT])
@pytest.mark.parametrize("L,Cb,q_lens", [(32, 7, [32, 5, 33]), (64, 8, [40, 64]), (16, 1, [8, 8])])
def test_scores_eq1_transform_bit_exact(algo, L, Cb, q_lens):
    say(f"scores Eq.1 transform algo={algo} L={L} C={Cb} q_lens={q_lens}")
    rng = np.random.default_rng(L + Cb)
    d = 64
    lens = rng.integers(0, 50, 400)
    V = int(lens.sum())
    pool = rng.integers(-127, 128, (30, d))
    X = np.clip(pool[rng.integers(0, 30, V)] + rng.integers(-25, 26, (V, d)), -127, 127).astype(np.int8)
    nq = int(sum(q_lens))
    Q = np.clip(pool[rng.integers(0, 30, nq)] + rng.integers(-25, 26, (nq, d)), -127, 127).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.set_algo(ix, dz.HASH_AUTO, algo)
    dz.set_score_transform(ix, dz.SCORE_EQ1_Q16)
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    off = np.concatenate([[0], np.cumsum(lens)])
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    got = dz.scores(ix, torch.from_numpy(Q).to(DEV), q_lens).cpu().numpy()
    for b in range(len(q_lens)):
        assert np.array_equal(got[b], orc.scores_eq1(dc, off, qc[qo[b]:qo[b + 1]], Cb)), b
    # top-k on the transformed scores, candidate mode with duplicates
    cand = rng.integers(0, 400, (len(q_lens), 150))
    ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), q_lens, 20, cand_ids=torch.from_numpy(cand).to(DEV))
    for b in range(len(q_lens)):
        s = orc.scores_eq1(dc, off, qc[qo[b]:qo[b + 1]], Cb, cand[b])
        want_ids, want_sc = orc.topk(s, 20, cand[b])
        assert np.array_equal(ids[b].cpu().numpy(), want_ids) and np.array_equal(sc[b].cpu().numpy(), want_sc), b
    # back to raw counts
    dz.set_score_transform(ix, dz.SCORE_RAW_COUNTS)
    got = dz.scores(ix, torch.from_numpy(Q).to(DEV), q_lens).cpu().numpy()
    assert np.array_equal(got[0], orc.scores(dc, off, qc[qo[0]:qo[1]]))


def test_search_eq1_cfg3_reduced_changes_ranking_but_matches_oracle():
    w = gen.make(3, n_docs=30000, n_queries=6, n_cand=2048)
    p = w.preset
    say("search Eq.1 cfg3-reduced")
    ix, codes, _ = make_index(w)
    dz.set_score_transform(ix, dz.SCORE_EQ1_Q16)
    cand = w.cand_ids.to(DEV)
    ids, sc = dz.search(ix, w.queries.to(DEV), w.q_lengths, p.k, cand_ids=cand)
    dc, qc = oracle_codes(w)
    for b in range(p.n_queries):
        c = w.cand_ids[b].numpy()
        s = orc.scores_eq1(dc, w.offsets.numpy(), qc[b * p.q_len:(b + 1) * p.q_len], p.C, c)
        want_ids, want_sc = orc.topk(s, p.k, c)
        assert np.array_equal(ids[b].cpu().numpy(), want_ids) and np.array_equal(sc[b].cpu().numpy(), want_sc), b


# ------------------------------------------------------------------ randomized sweep over configurations
@pytest.mark.parametrize("k", [512, 1000, 3000, 8192, 16384])
def test_search_large_k_full_order(k):
    """k from one key per thread of the selecting workgroup up to the largest allowed: the whole result order."""
    say(f"search: large k={k}")
    rng = np.random.default_rng(77)
    d, L, Cb, N = 64, 16, 5, 20_000
    lens = rng.integers(1, 5, N)
    V = int(lens.sum())
    pool = rng.integers(-127, 128, (40, d))
    X = np.clip(pool[rng.integers(0, 40, V)] + rng.integers(-50, 51, (V, d)), -127, 127).astype(np.int8)
    Q = np.clip(pool[rng.integers(0, 40, 9)] + rng.integers(-50, 51, (9, d)), -127, 127).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    cand = rng.choice(N, 9000, replace=False).astype(np.int32)
    ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), [4, 5], k)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    off = np.concatenate([[0], np.cumsum(lens)])
    want_ids, want_sc, _ = orc.search(dc, off, [qc[:4], qc[4:]], k)
    assert np.array_equal(sc.cpu().numpy(), want_sc)
    assert np.array_equal(ids.cpu().numpy(), want_ids)
    # a candidate list shorter than k: the tail is padding
    ids, sc = dz.search(ix, torch.from_numpy(Q[:4]).to(DEV), [4], k, cand_ids=torch.from_numpy(cand).to(DEV), cand_offsets=[0, 9000])
    s_all = orc.scores(dc, off, qc[:4], cand)
    w_ids, w_sc = orc.topk(s_all, k, cand)
    assert np.array_equal(sc.cpu().numpy()[0], w_sc) and np.array_equal(ids.cpu().numpy()[0], w_ids)


@pytest.mark.parametrize("seed", range(10))
def test_search_random_list_lengths_and_k_with_heavy_ties(seed):
    """The selection alone under stress: few tables (scores tie in large groups), candidate lists of random length with
    repeated ids, k from 1 to the largest allowed, lists shorter than, equal to and longer than k."""
    rng = np.random.default_rng(4000 + seed)
    d, L, Cb, N = 64, 4, int(rng.integers(1, 4)), 30_000
    lens = rng.integers(1, 3, N)
    V = int(lens.sum())
    pool = rng.integers(-127, 128, (12, d))
    X = np.clip(pool[rng.integers(0, 12, V)] + rng.integers(-40, 41, (V, d)), -127, 127).astype(np.int8)
    B = int(rng.integers(1, 4))
    q_lens = rng.integers(1, 6, B)
    nq = int(q_lens.sum())
    Q = np.clip(pool[rng.integers(0, 12, nq)] + rng.integers(-40, 41, (nq, d)), -127, 127).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    k = int(rng.choice([1, 7, 64, 500, 512, 513, 2048, 5000, 16384]))
    n_cand = [int(rng.choice([1, 63, 500, 4096, 4097, 9000, 20_000])) for _ in range(B)]
    say(f"selection stress seed={seed} C={Cb} B={B} q_lens={q_lens.tolist()} k={k} lists={n_cand}")
    cands = [rng.integers(0, N, n).astype(np.int32) for n in n_cand]      # with replacement: repeated ids
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    c_off = np.concatenate([[0], np.cumsum(n_cand)])
    ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), q_lens, k, cand_ids=torch.from_numpy(np.concatenate(cands)).to(DEV),
                        cand_offsets=c_off)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    off = np.concatenate([[0], np.cumsum(lens)])
    q_off = np.concatenate([[0], np.cumsum(q_lens)])
    for b in range(B):
        s_all = orc.scores(dc, off, qc[q_off[b]:q_off[b + 1]], cands[b])
        w_ids, w_sc = orc.topk(s_all, k, cands[b])
        assert np.array_equal(sc[b], w_sc), f"scores differ for query set {b}"
        assert np.array_equal(ids[b], w_ids), f"ids differ for query set {b}"
    # every document for every query set, same k
    ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), q_lens, k)
    want_ids, want_sc, _ = orc.search(dc, off, [qc[q_off[b]:q_off[b + 1]] for b in range(B)], k)
    assert np.array_equal(sc.cpu().numpy(), want_sc) and np.array_equal(ids.cpu().numpy(), want_ids)


@pytest.mark.parametrize("seed", range(24))
def test_random_configuration_end_to_end(seed):
    """Random (d, L, C, lengths, query lengths, candidates, k, transform) through the default kernel choice."""
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([8, 24, 50, 64, 96, 128, 200, 256]))
    L = int(rng.choice([4, 8, 12, 16, 20, 32, 48, 64, 128]))
    Cb = int(rng.integers(1, 9))
    n_docs = int(rng.integers(1, 700))
    lens = rng.integers(0, int(rng.choice([3, 20, 90])), n_docs)
    if lens.sum() == 0:
        lens[0] = 2
    V = int(lens.sum())
    B = int(rng.integers(1, 5))
    q_lens = rng.integers(1, int(rng.choice([4, 33, 70])), B)
    k = int(rng.choice([1, 3, 10, 64, 300]))
    eq1 = bool(rng.integers(0, 2))
    use_cand = bool(rng.integers(0, 2))
    say(f"random cfg seed={seed} d={d} L={L} C={Cb} N={n_docs} V={V} q_lens={q_lens.tolist()} k={k} eq1={eq1} cand={use_cand}")
    pool = rng.integers(-127, 128, (25, d))
    X = np.clip(pool[rng.integers(0, 25, V)] + rng.integers(-30, 31, (V, d)), -127, 127).astype(np.int8)
    nq = int(q_lens.sum())
    Q = np.clip(pool[rng.integers(0, 25, nq)] + rng.integers(-30, 31, (nq, d)), -127, 127).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    if eq1:
        dz.set_score_transform(ix, dz.SCORE_EQ1_Q16)
    codes, offsets = dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    dc, qc = orc.hash_i8(X, R, L, Cb), orc.hash_i8(Q, R, L, Cb)
    assert np.array_equal(codes.cpu().numpy(), dc)
    off = np.concatenate([[0], np.cumsum(lens)])
    assert np.array_equal(offsets.cpu().numpy(), off)
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    if use_cand:
        cands = [rng.integers(0, n_docs, int(rng.integers(0, 400))) for _ in range(B)]
        co = np.concatenate([[0], np.cumsum([len(c) for c in cands])])
        flat = torch.from_numpy(np.concatenate(cands).astype(np.int32)).to(DEV) if co[-1] else \
            torch.zeros(1, dtype=torch.int32, device=DEV)[:0]
        if co[-1] == 0:
            return
        ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), q_lens, k, cand_ids=flat, cand_offsets=co)
    else:
        cands = [None] * B
        ids, sc = dz.search(ix, torch.from_numpy(Q).to(DEV), q_lens, k)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    for b in range(B):
        q = qc[qo[b]:qo[b + 1]]
        s = orc.scores_eq1(dc, off, q, Cb, cands[b]) if eq1 else orc.scores(dc, off, q, cands[b])
        want_ids, want_sc = orc.topk(s, k, cands[b])
        assert np.array_equal(sc[b], want_sc), b
        assert np.array_equal(ids[b], want_ids), b


def test_timing_of_every_call_and_of_every_third():
    """dessert_enable_timing: 1 = every call is timed, n = every n-th; dessert_get_timing reaches the timed calls only."""
    say("timing: every call, every third call, off")
    w = gen.make(1)
    p = w.preset
    ix = dz.create(p.d, p.L, p.C, proj=w.proj.to(DEV))
    dz.build_index(ix, w.docs.to(DEV), w.lengths)
    q, ql = w.queries.to(DEV), w.q_lengths
    want = dz.search(ix, q, ql, p.k)
    dz.enable_timing(ix, True)
    for _ in range(4):
        got = dz.search(ix, q, ql, p.k)
    for back in range(4):
        t = dz.get_timing(ix, back)
        assert t["total_ms"] > 0 and t["score_ms"] > 0 and t["hash_ms"] > 0 and t["topk_ms"] > 0
        assert t["total_ms"] >= t["score_ms"]
    with pytest.raises(dz.DessertError):
        dz.get_timing(ix, 4)
    dz.enable_timing(ix, 3)                      # calls 0, 3 and 6 of the next seven
    for _ in range(7):
        got = dz.search(ix, q, ql, p.k)
    for back in range(3):
        assert dz.get_timing(ix, back)["total_ms"] > 0
    with pytest.raises(dz.DessertError):
        dz.get_timing(ix, 3)
    dz.enable_timing(ix, False)
    dz.search(ix, q, ql, p.k)
    with pytest.raises(dz.DessertError):
        dz.get_timing(ix, 0)
    assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1])
