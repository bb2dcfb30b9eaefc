"""Pins for the CPU oracle: each test checks it against something other than itself.

P1  exact sum-of-max similarity by brute force (Sec. 1.1 problem statement, Sec. 2 ColBERT form)
P2  SRP collision probability closed form (Sec. 3 LSH property; Sec. 5 concatenation: sim^C)
P3  binomial model of the collision counts (proof of Lemma 3: count ~ Binomial(L, s))
P4  invariants of the score
P5  literal bucket form of Alg. 1 + Alg. 2
P6  top-k against numpy lexsort
P7  hand-computed example (tests/golden/hand_example.txt)
P8  published SplitMix64 test vector for the seed-derived Rademacher matrix
"""
import math
import os

import numpy as np
import pytest

from oracle import oracle as orc
from synth import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def unit(v):
    return v / np.linalg.norm(v, axis=-1, keepdims=True)


def pair_at_angle(rng, d, theta):
    a = unit(rng.standard_normal(d))
    b = rng.standard_normal(d)
    b = unit(b - a * (a @ b))
    return a, unit(math.cos(theta) * a + math.sin(theta) * b)


# ---------------------------------------------------------------- P7 hand example
def load_hand():
    R, X, P, Cd, S, E = [], [], [], [], [], []
    for line in open(os.path.join(GOLDEN, "hand_example.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tag, rest = line[0], line[1:]
        if tag == "G":          # other aggregations: read by tests/test_oracle_aggregation_pins.py
            continue
        parts = [[int(t) for t in p.split()] for p in rest.split("|")]
        if tag == "R":
            R.append(parts[0])
        elif tag == "X":
            X.append(parts[0]); P.append(parts[1]); Cd.append(parts[2])
        elif tag == "S":
            S.append((parts[0], parts[1], parts[2][0]))
        elif tag == "E":
            E.append((parts[0], parts[1], parts[2][0]))
    return (np.array(R, np.int8), np.array(X, np.int8), np.array(P, np.int32), np.array(Cd, np.uint8), S, E)


def test_p7_hand_example_codes_and_scores():
    R, X, P, Cd, S, E = load_hand()
    codes, proj = orc.hash_i8(X, R, 2, 2, want_proj=True)
    assert np.array_equal(proj, P)
    assert np.array_equal(codes, Cd)
    # the same values through the floating-point routine
    codes_fp, proj_fp = orc.hash_fp(X.astype(np.float32), R.astype(np.float32), 2, 2, want_proj=True)
    assert np.array_equal(codes_fp, Cd) and np.array_equal(proj_fp, P.astype(np.float64))
    for q_idx, s_idx, want in S:
        doc = codes[s_idx]
        got = orc.scores(doc, np.array([0, len(s_idx)]), codes[q_idx])
        assert got.tolist() == [want]
    for q_idx, s_idx, want in E:
        got = orc.scores_eq1(codes[s_idx], np.array([0, len(s_idx)]), codes[q_idx], 2)
        assert got.tolist() == [want]


# ---------------------------------------------------------------- P8 seed rule
def test_p8_rademacher_matches_published_splitmix64_vector():
    # SplitMix64 from state 1234567 emits 6457827717110365317, 3203168211198807973,
    # 9817491932198370423, 4593380528125082431, 16408922859458223821 (reference test vector);
    # entry k of the matrix takes the top bit of output k.
    outs = [6457827717110365317, 3203168211198807973, 9817491932198370423,
            4593380528125082431, 16408922859458223821]
    want = [1 if (o >> 63) else -1 for o in outs]
    assert orc.rademacher(1234567, 1, 5)[0].tolist() == want
    # row-major counter: a [2][3] matrix continues the same stream
    R = orc.rademacher(1234567, 2, 3)
    assert R.reshape(-1)[:5].tolist() == want
    big = orc.rademacher(42, 224, 128)
    assert set(np.unique(big)) == {-1, 1}
    assert abs(big.astype(np.float64).mean()) < 4 / math.sqrt(big.size)


# ---------------------------------------------------------------- P2 closed form
@pytest.mark.parametrize("Cbits", [1, 3, 7])
@pytest.mark.parametrize("theta", [0.2, 0.9, math.pi / 2, 2.4])
def test_p2_srp_collision_rate_gaussian(Cbits, theta):
    rng = np.random.default_rng(100 + Cbits)
    d, L = 32, 20000
    a, b = pair_at_angle(rng, d, theta)
    R = rng.standard_normal((L * Cbits, d)).astype(np.float32)
    codes = orc.hash_fp(np.stack([a, b]).astype(np.float32), R, L, Cbits)
    rate = float((codes[0] == codes[1]).mean())
    p = (1 - theta / math.pi) ** Cbits
    sd = math.sqrt(p * (1 - p) / L)
    assert abs(rate - p) < 4.5 * sd + 1e-3, (rate, p)


def test_p2_srp_collision_rate_rademacher_int8():
    # +-1 projections of int8 vectors: the same law up to a CLT-size deviation at d = 128
    rng = np.random.default_rng(7)
    d, L, Cbits = 128, 20000, 2
    for theta in (0.3, 1.0, 1.8):
        a, b = pair_at_angle(rng, d, theta)
        X = np.clip(np.rint(127 * np.stack([a, b])), -127, 127).astype(np.int8)
        xa, xb = X.astype(np.float64)
        th = math.acos(np.clip(xa @ xb / np.linalg.norm(xa) / np.linalg.norm(xb), -1, 1))
        R = rng.integers(0, 2, (L * Cbits, d)).astype(np.int8) * 2 - 1
        codes = orc.hash_i8(X, R, L, Cbits)
        rate = float((codes[0] == codes[1]).mean())
        p = (1 - th / math.pi) ** Cbits
        assert abs(rate - p) < 0.02, (theta, rate, p)


# ---------------------------------------------------------------- P3 binomial counts
def test_p3_counts_are_binomial():
    rng = np.random.default_rng(3)
    d, L, Cbits, trials = 24, 32, 2, 3000
    theta = 0.8
    p = (1 - theta / math.pi) ** Cbits
    a, b = pair_at_angle(rng, d, theta)
    X = np.stack([a, b]).astype(np.float32)
    cnt = np.empty(trials)
    for s in range(trials):
        R = rng.standard_normal((L * Cbits, d)).astype(np.float32)
        codes = orc.hash_fp(X, R, L, Cbits)
        cnt[s] = orc.scores(codes[1:2], np.array([0, 1]), codes[0:1])[0]   # one q, one x: score = count
    mean, var = cnt.mean(), cnt.var()
    assert abs(mean - L * p) < 5 * math.sqrt(L * p * (1 - p) / trials)
    assert abs(var - L * p * (1 - p)) < 0.15 * L * p * (1 - p)
    # Hoeffding tail of Lemma 3 (single vector, beta = 1): P[count/L <= p - D] <= exp(-2 L D^2)
    for D in (0.1, 0.2):
        emp = float((cnt / L <= p - D).mean())
        assert emp <= math.exp(-2 * L * D * D) + 3 / math.sqrt(trials)


# ---------------------------------------------------------------- P1 brute force
def exact_sum_max(Q, S, kind):
    sim = unit(Q) @ unit(S).T
    if kind == "angular":
        sim = 1 - np.arccos(np.clip(sim, -1, 1)) / math.pi
    return float(sim.max(axis=1).sum())


def test_p1_large_L_matches_exact_angular_sum_of_max():
    rng = np.random.default_rng(11)
    d, n_docs, m, mq, L = 16, 40, 6, 5, 8192
    docs = rng.standard_normal((n_docs, m, d))
    target = 17
    Q = docs[target, :mq] + 0.25 * rng.standard_normal((mq, d))
    R = rng.standard_normal((L, d)).astype(np.float32)           # C = 1: collision prob = 1 - theta/pi
    dcodes = orc.hash_fp(docs.reshape(-1, d).astype(np.float32), R, L, 1)
    qcodes = orc.hash_fp(Q.astype(np.float32), R, L, 1)
    offsets = np.arange(n_docs + 1) * m
    est = orc.scores(dcodes, offsets, qcodes) / L
    # hashing saw float32-rounded inputs; use the same values for the exact side
    docs32 = docs.astype(np.float32).astype(np.float64)
    Q32 = Q.astype(np.float32).astype(np.float64)
    exact = np.array([exact_sum_max(Q32, docs32[i], "angular") for i in range(n_docs)])
    # each of the mq maxima is a max of m estimates with sd <= 0.5/sqrt(L): small upward bias only
    assert np.all(est - exact > -4 * mq * 0.5 / math.sqrt(L))
    assert np.all(est - exact < mq * 0.5 / math.sqrt(L) * (3 + math.sqrt(2 * math.log(m))))
    assert int(np.argmax(est)) == target == int(np.argmax(exact))
    # rank agreement (Spearman) between estimate and exact
    ra, rb = np.argsort(np.argsort(est)), np.argsort(np.argsort(exact))
    rho = np.corrcoef(ra, rb)[0, 1]
    assert rho > 0.97, rho


def test_p1_planted_document_wins_under_cosine_brute_force_too():
    w = gen.make(1, n_docs=60, n_queries=6)
    p = w.preset
    X = w.docs.numpy(); Qv = w.queries.numpy(); R = w.proj.numpy()
    dcodes = orc.hash_i8(X, R, p.L, p.C)
    qcodes = orc.hash_i8(Qv, R, p.L, p.C)
    off = w.offsets.numpy()
    for b in range(p.n_queries):
        Qb = Qv[b * p.q_len:(b + 1) * p.q_len].astype(np.float64)
        exact = np.array([exact_sum_max(Qb, X[off[i]:off[i + 1]].astype(np.float64), "cosine")
                          for i in range(w.n_docs)])
        s = orc.scores(dcodes, off, qcodes[b * p.q_len:(b + 1) * p.q_len])
        assert int(np.argmax(exact)) == int(w.planted[b, 0])
        assert int(np.argmax(s)) == int(w.planted[b, 0])


# ---------------------------------------------------------------- P4 invariants
def test_p4_invariants():
    rng = np.random.default_rng(5)
    L, Cbits, d = 16, 6, 32
    R = rng.integers(0, 2, (L * Cbits, d)).astype(np.int8) * 2 - 1
    lens = rng.integers(0, 9, 50)
    lens[3] = 0
    off = np.concatenate([[0], np.cumsum(lens)])
    X = rng.integers(-127, 128, (off[-1], d)).astype(np.int8)
    Q = rng.integers(-127, 128, (7, d)).astype(np.int8)
    dc, qc = orc.hash_i8(X, R, L, Cbits), orc.hash_i8(Q, R, L, Cbits)
    s = orc.scores(dc, off, qc)
    assert s.min() >= 0 and s.max() <= 7 * L
    assert s[3] == 0                                             # empty document
    # a document that contains every query vector attains |Q| * L
    dc2 = np.concatenate([dc, qc]); off2 = np.concatenate([off, [off[-1] + 7]])
    assert orc.scores(dc2, off2, qc)[-1] == 7 * L
    # permutation of vectors inside a document / inside the query set
    i = int(np.argmax(lens))
    perm = rng.permutation(lens[i])
    one = dc[off[i]:off[i + 1]]
    assert orc.scores(one[perm], np.array([0, lens[i]]), qc[rng.permutation(7)])[0] == s[i]
    # duplicating a document vector changes nothing; a superset never scores lower
    dup = np.concatenate([one, one[:1]])
    assert orc.scores(dup, np.array([0, lens[i] + 1]), qc)[0] == s[i]
    sup = np.concatenate([one, dc[:5]])
    assert orc.scores(sup, np.array([0, lens[i] + 5]), qc)[0] >= s[i]
    # additivity over a split of the query set
    assert np.array_equal(orc.scores(dc, off, qc[:3]) + orc.scores(dc, off, qc[3:]), s)
    # duplicated query vectors count twice
    assert np.array_equal(orc.scores(dc, off, np.concatenate([qc, qc])), 2 * s)
    # candidate subset = the same documents' exhaustive scores, duplicates allowed
    ids = np.array([4, 4, 49, 0, 3])
    assert np.array_equal(orc.scores(dc, off, qc, ids), s[ids])
    # positive integer scaling keeps the code; negation complements it where no projection is 0
    small = rng.integers(-40, 41, (20, d)).astype(np.int8)
    c1, p1 = orc.hash_i8(small, R, L, Cbits, want_proj=True)
    assert np.array_equal(orc.hash_i8((small * 3).astype(np.int8), R, L, Cbits), c1)
    cneg = orc.hash_i8((-small).astype(np.int8), R, L, Cbits)
    nz = (p1.reshape(20, L, Cbits) != 0).all(axis=2)
    assert np.array_equal(cneg[nz], (2 ** Cbits - 1) - c1[nz])
    assert nz.sum() > 0 and (~nz).sum() >= 0


def test_p4_code_bits_match_independent_matmul():
    # the projection step is a plain matrix product; numpy's matmul is an independent routine
    rng = np.random.default_rng(9)
    L, Cbits, d = 32, 7, 128
    R = rng.integers(0, 2, (L * Cbits, d)).astype(np.int8) * 2 - 1
    X = rng.integers(-127, 128, (300, d)).astype(np.int8)
    codes, proj = orc.hash_i8(X, R, L, Cbits, want_proj=True)
    P = X.astype(np.int64) @ R.astype(np.int64).T
    assert np.array_equal(proj, P)
    bits = (P >= 0).reshape(300, L, Cbits).astype(np.int64)
    want = (bits << np.arange(Cbits)).sum(axis=2)
    assert np.array_equal(codes, want)
    assert codes.max() < 2 ** Cbits


# ---------------------------------------------------------------- P5 literal Alg. 1 + Alg. 2
def alg1_build(codes, offsets):
    """D[i] = dict (t, h) -> list of j, as in Alg. 1."""
    index = []
    for i in range(len(offsets) - 1):
        table = {}
        for j, row in enumerate(codes[offsets[i]:offsets[i + 1]]):
            for t, h in enumerate(row):
                table.setdefault((t, int(h)), []).append(j)
        index.append(table)
    return index


def alg2_scores(index, lengths, qcodes):
    out = np.zeros(len(index), dtype=np.int64)
    for i, table in enumerate(index):
        total = 0
        for hq in qcodes:
            s_hat = [0] * int(lengths[i])
            for t, h in enumerate(hq):
                for j in table.get((t, int(h)), ()):
                    s_hat[j] += 1
            total += max(s_hat) if s_hat else 0
        out[i] = total
    return out


def test_p5_bucket_form_equals_code_equality_on_cfg1():
    w = gen.make(1, n_docs=400)
    p = w.preset
    dc = orc.hash_i8(w.docs.numpy(), w.proj.numpy(), p.L, p.C)
    qc = orc.hash_i8(w.queries.numpy(), w.proj.numpy(), p.L, p.C)
    off = w.offsets.numpy()
    index = alg1_build(dc, off)
    for b in range(p.n_queries):
        q = qc[b * p.q_len:(b + 1) * p.q_len]
        assert np.array_equal(alg2_scores(index, w.lengths.numpy(), q), orc.scores(dc, off, q))


# ---------------------------------------------------------------- P6 top-k
@pytest.mark.parametrize("case", ["random", "all_equal", "two_valued", "short"])
def test_p6_topk_matches_lexsort(case):
    rng = np.random.default_rng(13)
    n, k = 500, 17
    if case == "random":
        s = rng.integers(0, 40, n)
    elif case == "all_equal":
        s = np.full(n, 5)
    elif case == "two_valued":
        s = rng.integers(0, 2, n) * 9
    else:
        n = 6
        s = rng.integers(0, 3, n)
    s = s.astype(np.int32)
    for ids in (None, rng.permutation(10 * n)[:n].astype(np.int64)):
        got_ids, got_sc = orc.topk(s, k, ids)
        idv = np.arange(n) if ids is None else ids
        order = np.lexsort((idv, -s.astype(np.int64)))[:k]
        m = len(order)
        assert np.array_equal(got_ids[:m], idv[order].astype(np.uint32))
        assert np.array_equal(got_sc[:m], s[order])
        assert np.all(got_ids[m:] == 0xFFFFFFFF) and np.all(got_sc[m:] == -1)


def test_search_chain_top1_is_planted_on_cfg1():
    w = gen.make(1)
    p = w.preset
    dc = orc.hash_i8(w.docs.numpy(), w.proj.numpy(), p.L, p.C)
    qc = orc.hash_i8(w.queries.numpy(), w.proj.numpy(), p.L, p.C)
    qs = [qc[b * p.q_len:(b + 1) * p.q_len] for b in range(p.n_queries)]
    ids, sc, raw = orc.search(dc, w.offsets.numpy(), qs, p.k)
    assert np.array_equal(ids[:, 0], w.planted[:, 0].numpy().astype(np.uint32))
    assert np.all(np.diff(sc.astype(np.int64), axis=1) <= 0)
    assert sc.max() <= p.q_len * p.L


# ---------------------------------------------------------------- Eq. 1 remap (Sec. 5)
def test_eq1_table_endpoints_monotone_and_identity_for_one_bit_tables():
    rng = np.random.default_rng(31)
    L, d = 32, 16
    X = rng.integers(-127, 128, (60, d)).astype(np.int8)
    off = np.arange(0, 61, 5)
    for Cbits in (1, 4, 7):
        R = (rng.integers(0, 2, (L * Cbits, d)) * 2 - 1).astype(np.int8)
        codes = orc.hash_i8(X, R, L, Cbits)
        s, table = orc.scores_eq1(codes, off, codes[:9], Cbits, want_table=True)
        assert table[0] == 0.0 and table[L] == 1.0 and np.all(np.diff(table) > 0)
        raw = orc.scores(codes, off, codes[:9])
        assert np.all(s >= 0) and np.all(s <= 9 * 65536)
        if Cbits == 1:
            # C = 1: Eq. 1 is the identity on count/L, and 65536/L is an integer for L = 32
            assert np.array_equal(s, raw * (65536 // L))
        else:
            # the remap is concave: per-vector similarities are at least count/L
            assert np.all(s >= raw * (65536 // L))
        # a document containing every query vector reaches similarity 1 for each of them
        assert orc.scores_eq1(codes[:9], np.array([0, 9]), codes[:9], Cbits)[0] == 9 * 65536


@pytest.mark.parametrize("Cbits", [2, 5])
@pytest.mark.parametrize("theta", [0.3, 1.0])
def test_eq1_recovers_the_angular_similarity(Cbits, theta):
    # Sec. 5: concatenating C hashes turns the collision probability into sim^C; Eq. 1 undoes it.
    rng = np.random.default_rng(200 + Cbits)
    d, L = 24, 40000
    a, b = pair_at_angle(rng, d, theta)
    R = rng.standard_normal((L * Cbits, d)).astype(np.float32)
    codes = orc.hash_fp(np.stack([a, b]).astype(np.float32), R, L, Cbits)
    est = orc.scores_eq1(codes[1:2], np.array([0, 1]), codes[0:1], Cbits)[0] / 65536.0
    sim = 1 - theta / math.pi
    p = sim ** Cbits
    # delta method: sd(p_hat^(1/C)) = sd(p_hat) * p^(1/C - 1) / C
    sd = math.sqrt(p * (1 - p) / L) * p ** (1.0 / Cbits - 1) / Cbits
    assert abs(est - sim) < 4.5 * sd + 2e-5, (est, sim, sd)
