"""Pins for the oracle's k-means (Sec. 5 "Filtering": the filter's centroids come from k-means on a sample).

K1  one Lloyd iteration against scikit-learn's KMeans (lloyd, given initial centres, max_iter = 1), rounded
K2  K = 1 is the rounded mean of the sample; a centroid without vectors stays
K3  the assignment step's inertia never increases by more than the rounding allows, and well-separated
    clusters are recovered exactly
K4  rounding of means with a fractional part of exactly one half, on both sides of zero
"""
import numpy as np
import pytest

from oracle import oracle as orc


def round_half_up(x):
    return np.floor(x + 0.5).astype(np.int64)


def test_k1_one_iteration_matches_sklearn_lloyd():
    from sklearn.cluster import KMeans
    rng = np.random.default_rng(1)
    d, K, n = 8, 5, 400
    centres = rng.integers(-90, 91, (K, d))
    X = np.clip(centres[rng.integers(0, K, n)] + rng.integers(-20, 21, (n, d)), -127, 127).astype(np.int8)
    init = X[rng.choice(n, K, replace=False)].copy()
    km = KMeans(n_clusters=K, init=init.astype(np.float64), n_init=1, max_iter=1, algorithm="lloyd", tol=0.0).fit(X.astype(np.float64))
    means = km.cluster_centers_                                   # float means after the one update
    frac = np.abs(means - np.floor(means) - 0.5)
    got = orc.kmeans(X, init, 1)
    safe = frac > 1e-9                                            # away from exact halves the rounding is unambiguous
    assert safe.mean() > 0.9
    assert np.array_equal(got[safe].astype(np.int64), round_half_up(means)[safe])


def test_k2_single_centroid_and_empty_cluster():
    rng = np.random.default_rng(2)
    X = rng.integers(-127, 128, (301, 6)).astype(np.int8)
    got = orc.kmeans(X, np.zeros((1, 6), np.int8), 3)
    assert np.array_equal(got[0].astype(np.int64), round_half_up(X.astype(np.float64).mean(axis=0)))
    # a far-away second centroid receives nothing and must stay where it is
    X2 = rng.integers(-10, 11, (50, 6)).astype(np.int8)
    init = np.array([[0] * 6, [120] * 6], np.int8)
    got = orc.kmeans(X2, init, 4)
    assert got[1].tolist() == [120] * 6
    assert np.array_equal(got[0].astype(np.int64), round_half_up(X2.astype(np.float64).mean(axis=0)))


def test_k3_inertia_and_recovery_of_separated_clusters():
    rng = np.random.default_rng(3)
    d, K = 16, 6
    centres = rng.integers(-100, 101, (K, d))
    lab = rng.integers(0, K, 2000)
    X = np.clip(centres[lab] + rng.integers(-3, 4, (2000, d)), -127, 127).astype(np.int8)
    init = np.stack([X[np.nonzero(lab == k)[0][0]] for k in range(K)])      # one member of each cluster
    got, inertia = orc.kmeans(X, init, 6, want_inertia=True)
    # rounding moves a centroid by at most 1/2 per coordinate: allow n * d / 4 of slack per step
    assert np.all(np.diff(inertia) <= 2000 * d // 4)
    assert inertia[-1] <= inertia[0]
    assert np.array_equal(orc.assign_centroids(X, got), lab)
    for k in range(K):
        assert np.array_equal(got[k].astype(np.int64), round_half_up(X[lab == k].astype(np.float64).mean(axis=0)))
    # a fixed point stays fixed
    assert np.array_equal(orc.kmeans(X, got, 2), got)


def test_k4_half_rounds_up_on_both_sides_of_zero():
    X = np.array([[1, -1, 3, -3], [2, -2, 4, -4]], np.int8)                  # means 1.5, -1.5, 3.5, -3.5
    got = orc.kmeans(X, np.zeros((1, 4), np.int8), 1)
    assert got[0].tolist() == [2, -1, 4, -3]
    X = np.array([[5, -5], [5, -5], [6, -6]], np.int8)                        # means 5.33, -5.33
    assert orc.kmeans(X, np.zeros((1, 2), np.int8), 1)[0].tolist() == [5, -5]
