"""Pins for the oracle's wide codes (more than 8 one-bit hashes per table; Sec. 6.1 uses C = log2(m) + 1).

W1  hand-computed example with C = 9 (tests/golden/wide_hand_example.txt): bit 8 and the bit order
W2  numpy matmul + explicit bit packing at C = 11, L = 8; low 8 bits against the one-byte routine
W3  SRP collision probability (1 - theta/pi)^C at C = 11 (Sec. 3 LSH property, Sec. 5 concatenation)
W4  literal bucket form of Alg. 1 + Alg. 2 on 16-bit codes
W5  scoring: 16-bit routine on widened one-byte codes equals the one-byte routine; Eq. 1 values by closed form
"""
import math
import os

import numpy as np
import pytest

from oracle import oracle as orc
from tests.test_oracle_pins import alg1_build, alg2_scores, pair_at_angle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_w1_hand_example_nine_bits():
    R, X, P, Cd = [], [], [], []
    for line in open(os.path.join(GOLDEN, "wide_hand_example.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tag, rest = line[0], line[1:]
        parts = [[int(t) for t in p.split()] for p in rest.split("|")]
        if tag == "R":
            R.append(parts[0])
        else:
            X.append(parts[0]); P.append(parts[1]); Cd.append(parts[2])
    R, X = np.array(R, np.int8), np.array(X, np.int8)
    codes = orc.hash_i8(X, R, 1, 9)
    assert codes.dtype == np.uint16 and np.array_equal(codes, np.array(Cd, np.uint16))
    codes_fp, proj = orc.hash_fp(X.astype(np.float32), R.astype(np.float32), 1, 9, want_proj=True)
    assert np.array_equal(codes_fp, np.array(Cd, np.uint16)) and np.array_equal(proj, np.array(P, np.float64))


@pytest.mark.parametrize("L,Cbits", [(8, 11), (8, 9), (4, 16), (32, 10)])
def test_w2_code_bits_match_independent_matmul(L, Cbits):
    rng = np.random.default_rng(L * 100 + Cbits)
    d = 128
    R = rng.integers(0, 2, (L * Cbits, d)).astype(np.int8) * 2 - 1
    X = rng.integers(-127, 128, (200, d)).astype(np.int8)
    X[0] = 0                                                     # every projection 0 -> every bit 1
    codes = orc.hash_i8(X, R, L, Cbits)
    P = X.astype(np.int64) @ R.astype(np.int64).T
    bits = (P >= 0).reshape(200, L, Cbits).astype(np.int64)
    want = (bits << np.arange(Cbits)).sum(axis=2)
    assert np.array_equal(codes.astype(np.int64), want) and codes[0].tolist() == [2 ** Cbits - 1] * L
    # the low 8 bits are what the one-byte routine gives for the first 8 rows of every table
    rows = (np.arange(L)[:, None] * Cbits + np.arange(8)[None, :]).reshape(-1)
    assert np.array_equal(codes & 0xFF, orc.hash_i8(X, R[rows], L, 8))
    # floating-point routine on the same integers
    assert np.array_equal(orc.hash_fp(X.astype(np.float32), R.astype(np.float32), L, Cbits), codes)


@pytest.mark.parametrize("theta", [0.1, 0.25, 0.6])
def test_w3_srp_collision_rate_eleven_bits(theta):
    rng = np.random.default_rng(11)
    d, L, Cbits = 32, 20000, 11
    a, b = pair_at_angle(rng, d, theta)
    R = rng.standard_normal((L * Cbits, d)).astype(np.float32)
    codes = orc.hash_fp(np.stack([a, b]).astype(np.float32), R, L, Cbits)
    rate = float((codes[0] == codes[1]).mean())
    p = (1 - theta / math.pi) ** Cbits
    assert abs(rate - p) < 4.5 * math.sqrt(p * (1 - p) / L) + 1e-3, (rate, p)


def test_w4_bucket_form_equals_code_equality_on_wide_codes():
    rng = np.random.default_rng(4)
    d, L, Cbits, n_docs = 16, 8, 10, 60
    lens = rng.integers(0, 9, n_docs)
    off = np.concatenate([[0], np.cumsum(lens)])
    base = rng.integers(-100, 101, (12, d))
    X = np.clip(base[rng.integers(0, 12, off[-1])] + rng.integers(-25, 26, (off[-1], d)), -127, 127).astype(np.int8)
    R = rng.integers(0, 2, (L * Cbits, d)).astype(np.int8) * 2 - 1
    dc = orc.hash_i8(X, R, L, Cbits)
    assert dc.max() > 255
    index = alg1_build(dc, off)
    for b in range(5):
        Q = np.clip(X[rng.integers(0, off[-1], 6)].astype(np.int64) + rng.integers(-10, 11, (6, d)), -127, 127).astype(np.int8)
        qc = orc.hash_i8(Q, R, L, Cbits)
        got = orc.scores(dc, off, qc)
        assert np.array_equal(alg2_scores(index, lens, qc), got)
        assert got.max() > 0


def test_w5_wide_scoring_reduces_to_narrow_and_eq1_closed_form():
    rng = np.random.default_rng(5)
    L, n_docs = 8, 40
    lens = rng.integers(0, 7, n_docs)
    off = np.concatenate([[0], np.cumsum(lens)])
    dc = rng.integers(0, 4, (off[-1], L)).astype(np.uint8)        # few distinct codes: many collisions
    qc = rng.integers(0, 4, (5, L)).astype(np.uint8)
    sel = rng.integers(0, n_docs, 25)
    assert np.array_equal(orc.scores(dc.astype(np.uint16), off, qc.astype(np.uint16)), orc.scores(dc, off, qc))
    assert np.array_equal(orc.scores(dc.astype(np.uint16), off, qc.astype(np.uint16), sel), orc.scores(dc, off, qc, sel))
    # codes that differ only above bit 7 must not collide
    hi = dc.astype(np.uint16) + 256 * rng.integers(1, 8, dc.shape).astype(np.uint16)
    assert np.all(orc.scores(hi, off, qc.astype(np.uint16)) == 0)
    # Eq. 1 in Q16: a document equal to the query set scores mq * 65536; one matching table of L = 2 at C = 9
    # gives round(65536 * (1/2)^(1/9))
    q = np.array([[300, 7], [300, 9]], np.uint16)
    assert orc.scores_eq1(q, np.array([0, 2]), q, 9).tolist() == [2 * 65536]
    one = np.array([[300, 1000]], np.uint16)
    assert orc.scores_eq1(one, np.array([0, 1]), q[:1], 9).tolist() == [round(65536 * 0.5 ** (1 / 9))]
    for Cb in (9, 11):
        assert np.array_equal(orc.scores_eq1(dc.astype(np.uint16), off, qc.astype(np.uint16), Cb),
                              orc.scores_eq1(dc, off, qc, Cb))
