"""Pins for the oracle's other aggregations: sigma = mean of phi(count / L) (Sec. 4.1, the lemma on
sigma(x) = (1/m) sum phi(x_i) with its three example phi) and the weighted outer sum of Sec. 4.2.

A1  hand-computed values (G lines of tests/golden/hand_example.txt)
A2  the paper's linear bounds on phi: x <= e^x - 1 <= (e - 1) x and 0.23 x <= sigmoid(x) - 1/2 <= 0.25 x on [0, 1]
A3  sigma = mean of the identity is the average collision fraction, counted through per-table buckets
A4  numpy counts + integer arithmetic written out for every (phi, sigma) with random weights
A5  reductions: weights all one = unweighted; sigma = max of the identity ranks like the raw counts; Eq. 1 with
    sigma = max equals the Eq. 1 routine; a document with every vector doubled keeps its mean; zero weights
"""
import math
import os
from collections import Counter

import numpy as np
import pytest

from oracle import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def hand():
    R, X, G = [], [], []
    for line in open(os.path.join(GOLDEN, "hand_example.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tag, fields = line[0], [f.split() for f in line[1:].split("|")]
        if tag == "R":
            R.append([int(t) for t in fields[0]])
        elif tag == "X":
            X.append([int(t) for t in fields[0]])
        elif tag == "G":
            w = None if fields[3] == ["-"] else [int(t) for t in fields[3]]
            G.append((int(fields[0][0]), int(fields[0][1]), [int(t) for t in fields[1]], [int(t) for t in fields[2]],
                      w, int(fields[4][0])))
    return np.array(R, np.int8), np.array(X, np.int8), G


def test_a1_hand_values():
    R, X, G = hand()
    codes = orc.hash_i8(X, R, 2, 2)
    assert len(G) == 5
    for phi, sigma, q_idx, s_idx, w, want in G:
        got = orc.scores_general(codes[s_idx], np.array([0, len(s_idx)]), codes[q_idx], phi, sigma, weights=w)
        assert got.tolist() == [want], (phi, sigma, w)


def test_a2_phi_tables_obey_the_papers_linear_bounds():
    L = 64
    dc = np.zeros((1, L), np.uint8)
    x = np.arange(L + 1) / L
    for phi, lo, hi in ((orc.PHI_IDENTITY, 1.0, 1.0), (orc.PHI_EXPM1, 1.0, math.e - 1), (orc.PHI_SIGMOID, 0.23, 0.25)):
        _, tab = orc.scores_general(dc, np.array([0, 1]), dc, phi, orc.SIGMA_MAX, want_table=True)
        assert tab[0] == 0.0
        assert np.all(tab >= lo * x - 1e-12) and np.all(tab <= hi * x + 1e-12), phi
        assert np.all(np.diff(tab) > 0)
    # end points by closed form
    _, tab = orc.scores_general(dc, np.array([0, 1]), dc, orc.PHI_EXPM1, orc.SIGMA_MAX, want_table=True)
    assert abs(tab[L] - (math.e - 1)) < 1e-15
    _, tab = orc.scores_general(dc, np.array([0, 1]), dc, orc.PHI_SIGMOID, orc.SIGMA_MAX, want_table=True)
    assert abs(tab[L] - (1 / (1 + 1 / math.e) - 0.5)) < 1e-15
    # a document equal to the one query vector: count L, score = round(65536 * phi(1))
    assert orc.scores_general(dc, np.array([0, 1]), dc, orc.PHI_EXPM1, orc.SIGMA_MEAN).tolist() == [112609]
    assert orc.scores_general(dc, np.array([0, 1]), dc, orc.PHI_SIGMOID, orc.SIGMA_MEAN).tolist() == [15143]


def random_case(rng, wide=False, n_docs=30, L=16):
    lens = rng.integers(0, 9, n_docs)
    off = np.concatenate([[0], np.cumsum(lens)])
    hi = 600 if wide else 4
    dt = np.uint16 if wide else np.uint8
    dc = rng.integers(0, 4, (off[-1], L)).astype(dt) * (hi // 4)
    qc = rng.integers(0, 4, (6, L)).astype(dt) * (hi // 4)
    return dc, qc, off, lens


def test_a3_mean_identity_is_the_average_collision_fraction():
    rng = np.random.default_rng(3)
    L = 16                                          # 65536 / L is an integer: the Q16 values are exact
    dc, qc, off, lens = random_case(rng, L=L)
    got = orc.scores_general(dc, off, qc, orc.PHI_IDENTITY, orc.SIGMA_MEAN)
    for i in range(len(lens)):
        rows = dc[off[i]:off[i + 1]]
        buckets = [Counter(rows[:, t].tolist()) for t in range(L)]        # table t: code -> number of vectors
        total = 0
        for q in qc:
            collisions = sum(buckets[t][int(q[t])] for t in range(L))     # sum over x of count(q, x)
            m = len(rows)
            total += (collisions * (65536 // L) + m // 2) // m if m else 0
        assert got[i] == total, i


@pytest.mark.parametrize("wide", [False, True])
@pytest.mark.parametrize("phi", [0, 1, 2, 3])
@pytest.mark.parametrize("sigma", [0, 1])
def test_a4_numpy_counts_and_integer_arithmetic(wide, phi, sigma):
    rng = np.random.default_rng(40 + phi * 2 + sigma)
    L, Cb = 12, 3
    dc, qc, off, lens = random_case(rng, wide=wide, L=L)
    w = rng.integers(0, 65537, qc.shape[0]).astype(np.uint32)
    w[0] = 65536
    x = np.arange(L + 1) / L
    f = [x, np.expm1(x), 0.5 * np.tanh(x / 2), x ** (1.0 / Cb)][phi]        # sigmoid(x) - 1/2 = tanh(x/2) / 2
    T = np.array([int(math.floor(65536 * v + 0.5)) for v in f], dtype=np.int64)
    sel = rng.integers(0, len(lens), 20)
    got = orc.scores_general(dc, off, qc, phi, sigma, weights=w, doc_ids=sel, eq1_C=Cb)
    for k, i in enumerate(sel):
        rows = dc[off[i]:off[i + 1]]
        cnt = (qc[:, None, :] == rows[None, :, :]).sum(axis=2)              # [q, x]
        y = T[cnt]
        m = rows.shape[0]
        if sigma == 0:
            sg = y.max(axis=1) if m else np.zeros(len(qc), np.int64)
        else:
            sg = (y.sum(axis=1) + m // 2) // m if m else np.zeros(len(qc), np.int64)
        want = int(((w.astype(np.int64) * sg + 32768) >> 16).sum())
        assert got[k] == want, (i, m)


def test_a5_reductions():
    rng = np.random.default_rng(5)
    L = 16
    dc, qc, off, lens = random_case(rng, L=L)
    ones = np.full(qc.shape[0], 65536, np.uint32)
    for phi in (0, 1, 2):
        for sigma in (0, 1):
            a = orc.scores_general(dc, off, qc, phi, sigma)
            assert np.array_equal(a, orc.scores_general(dc, off, qc, phi, sigma, weights=ones))
            assert np.all(orc.scores_general(dc, off, qc, phi, sigma, weights=0 * ones) == 0)
    # sigma = max of the identity = raw counts scaled by 65536 / L
    assert np.array_equal(orc.scores_general(dc, off, qc, orc.PHI_IDENTITY, orc.SIGMA_MAX), orc.scores(dc, off, qc) * (65536 // L))
    # Eq. 1 with sigma = max: the routine pinned in test_oracle_pins.py
    for Cb in (1, 2, 7):
        assert np.array_equal(orc.scores_general(dc, off, qc, orc.PHI_EQ1, orc.SIGMA_MAX, eq1_C=Cb), orc.scores_eq1(dc, off, qc, Cb))
    # doubling every vector of every document leaves the mean unchanged when no rounding is involved (identity, L | 65536,
    # even sums): compare on documents whose mean is exact
    dc2 = np.repeat(dc, 2, axis=0)
    a = orc.scores_general(dc, off, qc[:1], orc.PHI_IDENTITY, orc.SIGMA_MAX)
    assert np.array_equal(a, orc.scores_general(dc2, off * 2, qc[:1], orc.PHI_IDENTITY, orc.SIGMA_MAX))
    one_vec = lens == 1
    b = orc.scores_general(dc, off, qc, orc.PHI_EXPM1, orc.SIGMA_MEAN)
    b2 = orc.scores_general(dc2, off * 2, qc, orc.PHI_EXPM1, orc.SIGMA_MEAN)
    assert one_vec.any() and np.array_equal(b[one_vec], b2[one_vec])
    # a one-hot weight picks one query vector's sigma
    for j in range(qc.shape[0]):
        w = np.zeros(qc.shape[0], np.uint32); w[j] = 65536
        assert np.array_equal(orc.scores_general(dc, off, qc, orc.PHI_SIGMOID, orc.SIGMA_MEAN, weights=w),
                              orc.scores_general(dc, off, qc[j:j + 1], orc.PHI_SIGMOID, orc.SIGMA_MEAN))
