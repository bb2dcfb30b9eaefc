"""Pins for the oracle's candidate filter (Sec. 5 "Filtering"): numpy brute force, python sets and
dictionaries following the paper's description, a closed form at probe = K, tie rules, a hand example."""
import os

import numpy as np
import pytest

from oracle import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def make(rng, n_docs=60, d=12, K=17, max_len=9):
    lens = rng.integers(0, max_len, n_docs)
    off = np.concatenate([[0], np.cumsum(lens)])
    pool = rng.integers(-100, 101, (K, d))
    X = np.clip(pool[rng.integers(0, K, off[-1])] + rng.integers(-40, 41, (off[-1], d)), -127, 127).astype(np.int8)
    Cn = np.clip(pool + rng.integers(-5, 6, (K, d)), -127, 127).astype(np.int8)
    return X, Cn, off


def test_assign_matches_numpy_distance_matrix():
    rng = np.random.default_rng(1)
    X, Cn, _ = make(rng, n_docs=200)
    x, c = X.astype(np.int64), Cn.astype(np.int64)
    dist = (x * x).sum(1)[:, None] - 2 * x @ c.T + (c * c).sum(1)[None, :]
    assert np.array_equal(orc.assign_centroids(X, Cn), np.argmin(dist, axis=1))     # argmin takes the first minimum


def test_assign_ties_go_to_the_lower_id():
    Cn = np.array([[3, 3], [3, 3], [-3, 3], [3, -3]], np.int8)      # centroids 0 and 1 coincide
    X = np.array([[3, 3], [0, 3], [0, 0], [3, 0]], np.int8)           # (0,3): c0,c1,c2 tie; (0,0): all tie; (3,0): 0,1,3
    assert orc.assign_centroids(X, Cn).tolist() == [0, 0, 0, 0]
    X2 = np.array([[-3, 3], [3, -3], [-1, 3]], np.int8)
    assert orc.assign_centroids(X2, Cn).tolist() == [2, 3, 2]


def test_inverted_index_matches_python_sets():
    rng = np.random.default_rng(2)
    X, Cn, off = make(rng)
    K = Cn.shape[0]
    assign = orc.assign_centroids(X, Cn)
    bo, docs = orc.inverted_index(assign, off, K)
    want = [sorted({i for i in range(len(off) - 1) if k in set(assign[off[i]:off[i + 1]].tolist())}) for k in range(K)]
    for k in range(K):
        assert docs[bo[k]:bo[k + 1]].tolist() == want[k]
    assert bo[-1] == sum(len(w) for w in want) == docs.shape[0]


@pytest.mark.parametrize("probe,filter_k", [(1, 5), (3, 10), (17, 100), (2, 1)])
def test_filter_query_matches_dictionary_counting(probe, filter_k):
    rng = np.random.default_rng(3 + probe)
    X, Cn, off = make(rng)
    K, n_docs = Cn.shape[0], len(off) - 1
    assign = orc.assign_centroids(X, Cn)
    bo, docs = orc.inverted_index(assign, off, K)
    Q = np.clip(Cn[rng.integers(0, K, 6)] + rng.integers(-30, 31, (6, X.shape[1])), -127, 127).astype(np.int8)
    # the paper's description, literally: probe the closest centroids of each query vector, add up bucket hits
    counts = {}
    c = Cn.astype(np.int64)
    for q in Q.astype(np.int64):
        dist = ((q[None, :] - c) ** 2).sum(1)
        for k in np.lexsort((np.arange(K), dist))[:probe]:
            for doc in docs[bo[k]:bo[k + 1]]:
                counts[int(doc)] = counts.get(int(doc), 0) + 1
    ranked = sorted(counts.items(), key=lambda kv: (-kv[1], kv[0]))[:filter_k]
    ids, cnt = orc.filter_query(Q, Cn, bo, docs, n_docs, probe, filter_k)
    m = len(ranked)
    assert ids[:m].tolist() == [r[0] for r in ranked] and cnt[:m].tolist() == [r[1] for r in ranked]
    assert np.all(ids[m:] == 0xFFFFFFFF) and np.all(cnt[m:] == -1)
    if probe == K:
        # every bucket is probed by every query vector: count = |Q| * (distinct centroids of the document)
        for doc, n in counts.items():
            assert n == len(Q) * len(set(assign[off[doc]:off[doc + 1]].tolist()))


def test_filter_hand_example():
    Cn, docs, assigns, buckets, Q, F = [], {}, {}, {}, [], []
    for line in open(os.path.join(GOLDEN, "filter_hand_example.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tag, rest = line[0], line[1:]
        parts = [[int(t) for t in p.split()] for p in rest.split("|")]
        if tag == "C":
            Cn.append(parts[0])
        elif tag == "D":
            docs[parts[0][0]] = parts[1:]
        elif tag == "A":
            assigns[parts[0][0]] = parts[1]
        elif tag == "B":
            buckets[parts[0][0]] = parts[1]
        elif tag == "Q":
            Q.append(parts[0])
        elif tag == "F":
            F.append((parts[0][0], parts[0][1], parts[1], parts[2]))
    Cn = np.array(Cn, np.int8)
    order = sorted(docs)
    X = np.array([v for i in order for v in docs[i]], np.int8)
    off = np.concatenate([[0], np.cumsum([len(docs[i]) for i in order])])
    assign = orc.assign_centroids(X, Cn)
    assert assign.tolist() == [a for i in order for a in assigns[i]]
    bo, bd = orc.inverted_index(assign, off, len(Cn))
    for k in range(len(Cn)):
        assert bd[bo[k]:bo[k + 1]].tolist() == buckets[k]
    for probe, fk, want_ids, want_cnt in F:
        ids, cnt = orc.filter_query(np.array(Q, np.int8), Cn, bo, bd, len(order), probe, fk)
        assert ids.tolist() == want_ids and cnt.tolist() == want_cnt
