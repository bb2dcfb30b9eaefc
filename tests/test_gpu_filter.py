"""GPU parity of the candidate filter (Sec. 5 "Filtering") against the oracle: closest-centroid assignment,
buckets (as sets: the order inside a bucket is unspecified), probe-and-count selection, and the chain
filter -> scoring with empty candidate slots -> top-k."""
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


def setup(rng, d, K, n_docs, max_len, L=32, Cb=7, dup_centroids=False):
    lens = rng.integers(0, max_len, n_docs)
    lens[0] = max(lens[0], 1)
    off = np.concatenate([[0], np.cumsum(lens)])
    pool = rng.integers(-100, 101, (K, d))
    Cn = np.clip(pool + rng.integers(-4, 5, (K, d)), -127, 127).astype(np.int8)
    if dup_centroids:
        Cn[K // 2] = Cn[0]
        Cn[K - 1] = Cn[1]
    X = np.clip(pool[rng.integers(0, K, off[-1])] + rng.integers(-50, 51, (off[-1], d)), -127, 127).astype(np.int8)
    X[0] = 0
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    return ix, X, Cn, R, off, lens


def buckets_as_sets(bo, bd):
    return [sorted(bd[bo[k]:bo[k + 1]].tolist()) for k in range(len(bo) - 1)]


@pytest.mark.parametrize("d,K,n_docs,dup,max_len", [(128, 1000, 900, False, 40), (64, 37, 300, True, 40),
                                                    (256, 513, 400, True, 40), (128, 32, 50, False, 40),
                                                    (128, 5, 2000, True, 40),
                                                    (128, 7, 300, True, 200),      # documents of 65..199 vectors
                                                    (64, 150, 200, False, 300)])
def test_filter_build_assignments_and_buckets(d, K, n_docs, dup, max_len):
    say(f"filter build d={d} K={K} N={n_docs} dup={dup} max_len={max_len}")
    rng = np.random.default_rng(d + K)
    ix, X, Cn, R, off, lens = setup(rng, d, K, n_docs, max_len, dup_centroids=dup)
    assign, bo, bd = dz.filter_build(ix, torch.from_numpy(Cn).to(DEV), torch.from_numpy(X).to(DEV))
    want = orc.assign_centroids(X, Cn)
    assert np.array_equal(assign.cpu().numpy(), want)
    obo, obd = orc.inverted_index(want, off, K)
    bo, bd = bo.cpu().numpy().astype(np.int64), bd.cpu().numpy().astype(np.uint32)
    assert np.array_equal(bo, obo)
    assert buckets_as_sets(bo, bd) == buckets_as_sets(obo, obd)


@pytest.mark.parametrize("probe,filter_k,q_lens,n_docs,max_len", [
    (1, 64, [32, 32, 32], 1500, 12), (2, 300, [5, 40, 1], 1500, 12), (4, 16, [32], 1500, 12),
    (8, 4096, [12, 7], 1500, 12), (37, 50, [3, 3], 1500, 12), (8, 5000, [12, 7], 30_000, 3),
    (37, 200, [10, 2], 1500, 12),            # counts up to 370: 16-bit counters
    (37, 16384, [1800, 5], 1500, 12),        # counts up to 66600: 32-bit counters
    (2, 1000, [32, 9], 300_000, 3),          # ten document slabs of 8-bit counters, first-hit queues overflow
    (3, 777, [100, 30], 150_000, 3),         # document slabs of 16-bit counters
    (37, 2000, [1800, 5], 150_000, 3),       # 32-bit counters over several slabs; count and id fields pass 32 bits: 64-bit list keys
    (1, 4096, [32, 32], 200_000, 3),         # seven slabs, one probe: the k-th key is found inside one slab's run of the list
    (1, 50, [32], 200_000, 3),               # same lists, small k: few keys above the threshold count
    (3, 5000, [20, 32, 7], 100_000, 3)])     # counts up to 96: the widest per-slab histograms (128 bins)
def test_filter_query_matches_oracle(probe, filter_k, q_lens, n_docs, max_len):
    say(f"filter query probe={probe} filter_k={filter_k} q_lens={q_lens} N={n_docs}")
    rng = np.random.default_rng(100 + probe)
    d, K = 128, 37
    ix, X, Cn, R, off, lens = setup(rng, d, K, n_docs, max_len, dup_centroids=True)
    dz.filter_build(ix, torch.from_numpy(Cn).to(DEV), torch.from_numpy(X).to(DEV))
    nq = int(sum(q_lens))
    Q = np.clip(Cn[rng.integers(0, K, nq)].astype(np.int64) + rng.integers(-60, 61, (nq, d)), -127, 127).astype(np.int8)
    ids, cnt = dz.filter_query(ix, torch.from_numpy(Q).to(DEV), q_lens, probe, filter_k)
    ids, cnt = ids.cpu().numpy(), cnt.cpu().numpy()
    obo, obd = orc.inverted_index(orc.assign_centroids(X, Cn), off, K)
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    for b in range(len(q_lens)):
        want_ids, want_cnt = orc.filter_query(Q[qo[b]:qo[b + 1]], Cn, obo, obd, n_docs, probe, filter_k)
        assert np.array_equal(cnt[b], want_cnt), b
        assert np.array_equal(ids[b], want_ids), b


@pytest.mark.parametrize("d,K,probe,n_q", [(128, 3000, 1, 40), (128, 3000, 3, 40), (64, 2500, 5, 300),
                                           (256, 1200, 8, 70), (128, 3, 2, 10), (128, 3000, 9, 20),
                                           (128, 700, 4, 5000)])
def test_filter_probe_selection_over_tile_ranges(d, K, probe, n_q):
    """Many centroids: the probe selection runs over several centroid-tile ranges whose lists are merged;
    duplicated centroids sit in different ranges (ties must go to the lower id)."""
    say(f"filter probe ranges d={d} K={K} probe={probe} n_q={n_q}")
    rng = np.random.default_rng(7 * d + K + probe)
    n_docs = 400
    ix, X, Cn, R, off, lens = setup(rng, d, K, n_docs, 30, dup_centroids=K > 3)
    if K > 100:
        Cn[K - 7] = Cn[3]; Cn[K // 3] = Cn[3]; Cn[40] = Cn[K - 2]
    dz.filter_build(ix, torch.from_numpy(Cn).to(DEV), torch.from_numpy(X).to(DEV))
    Q = np.clip(Cn[rng.integers(0, K, n_q)].astype(np.int64) + rng.integers(-30, 31, (n_q, d)), -127, 127).astype(np.int8)
    Q[: min(n_q, 8)] = Cn[np.array([3, K - 2, 0, 1, 3, K - 1, K // 2, 2])[: min(n_q, 8)] % K]       # exact ties
    q_lens = [n_q // 2, n_q - n_q // 2]
    filter_k = 350
    ids, cnt = dz.filter_query(ix, torch.from_numpy(Q).to(DEV), q_lens, probe, filter_k)
    ids, cnt = ids.cpu().numpy(), cnt.cpu().numpy()
    obo, obd = orc.inverted_index(orc.assign_centroids(X, Cn), off, K)
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    for b in range(2):
        want_ids, want_cnt = orc.filter_query(Q[qo[b]:qo[b + 1]], Cn, obo, obd, n_docs, probe, filter_k)
        assert np.array_equal(cnt[b], want_cnt), b
        assert np.array_equal(ids[b], want_ids), b


def test_filter_then_search_chain_with_empty_slots():
    say("filter -> search chain, cfg3-like reduced")
    w = gen.make(3, n_docs=20000, n_queries=6)
    p = w.preset
    Cn = gen.filter_centroids(w)                       # the 1024 mixture centres
    ix = dz.create(p.d, p.L, p.C, proj=w.proj.to(DEV))
    dz.build_index(ix, w.docs.to(DEV), w.lengths)
    dz.filter_build(ix, Cn.to(DEV), w.docs.to(DEV))
    filter_k, probe = 512, 1
    cand, cnt = dz.filter_query(ix, w.queries.to(DEV), w.q_lengths, probe, filter_k)
    ids, sc = dz.search(ix, w.queries.to(DEV), w.q_lengths, p.k, cand_ids=cand)
    raw = dz.scores(ix, w.queries.to(DEV), w.q_lengths, cand_ids=cand).cpu().numpy().reshape(p.n_queries, filter_k)
    cand, ids, sc = cand.cpu().numpy(), ids.cpu().numpy(), sc.cpu().numpy()
    # oracle pipeline
    X, Q, R = w.docs.numpy(), w.queries.numpy(), w.proj.numpy()
    off = w.offsets.numpy()
    obo, obd = orc.inverted_index(orc.assign_centroids(X, Cn.numpy()), off, Cn.shape[0])
    dc, qc = orc.hash_i8(X, R, p.L, p.C), orc.hash_i8(Q, R, p.L, p.C)
    hits = 0
    for b in range(p.n_queries):
        q = slice(b * p.q_len, (b + 1) * p.q_len)
        want_cand, _ = orc.filter_query(Q[q], Cn.numpy(), obo, obd, w.n_docs, probe, filter_k)
        assert np.array_equal(cand[b], want_cand), b
        real = want_cand != 0xFFFFFFFF
        s = orc.scores(dc, off, qc[q], want_cand[real].astype(np.int64))
        assert np.array_equal(raw[b][real], s) and np.all(raw[b][~real] == -1)
        want_ids, want_sc = orc.topk(s, p.k, want_cand[real].astype(np.int64))
        assert np.array_equal(ids[b], want_ids) and np.array_equal(sc[b], want_sc), b
        hits += len(set(w.planted[b].tolist()) & set(cand[b].tolist()))
    # Each planted document supplied 4 of the 32 query vectors and documents here spread their ~70 vectors over
    # random centres, so an unrelated document already collects ~2 hits: about half of the planted ones make the
    # cut of 512.  A uniformly random cut would keep 512/20000 of them (about 1 of 48).
    assert hits >= 12, hits


@pytest.mark.parametrize("probe,filter_k,k,q_lens,n_docs,max_len", [
    (1, 512, 10, [32] * 6, 20_000, 40),        # equal lengths, lists filled
    (1, 4096, 10, [32], 200_000, 3),           # one query set: the single-query form of the chain
    (1, 4096, 4096, [32], 200_000, 3),         # the same with k = filter_k: every selected candidate is compared
    (2, 1000, 1000, [9] * 40, 60_000, 3),      # 40 lists: still the two-launch selection; k = filter_k
    (1, 700, 700, [16] * 70, 60_000, 3),       # 70 lists: one workgroup per list
    (2, 300, 50, [5, 40, 1, 33], 1500, 12),    # unequal query sets
    (4, 16, 16, [32, 7], 1500, 12),            # k = filter_k
    (8, 4096, 100, [12, 7], 1500, 12),         # fewer hit documents than filter_k: empty slots reach the scoring
    (37, 2000, 20, [1800, 5], 150_000, 3),     # 64-bit list keys
    (37, 2000, 2000, [1800, 5], 150_000, 3),   # the same with k = filter_k: the selected set itself is compared
    (3, 5000, 5000, [20, 32, 7], 100_000, 3)])
def test_filter_search_equals_filter_then_search_and_the_oracle(probe, filter_k, k, q_lens, n_docs, max_len):
    """dessert_filter_search (one call, candidates unordered in between) against dessert_filter_query + dessert_search
    and against the oracle's pipeline: the filter's set of documents, their scores, the k best."""
    say(f"filter_search probe={probe} filter_k={filter_k} k={k} q_lens={q_lens[:4]} N={n_docs}")
    rng = np.random.default_rng(500 + probe)
    d, K = 128, 37
    ix, X, Cn, R, off, lens = setup(rng, d, K, n_docs, max_len, dup_centroids=True)
    dz.filter_build(ix, torch.from_numpy(Cn).to(DEV), torch.from_numpy(X).to(DEV))
    nq = int(sum(q_lens))
    Q = np.clip(Cn[rng.integers(0, K, nq)].astype(np.int64) + rng.integers(-60, 61, (nq, d)), -127, 127).astype(np.int8)
    Qd = torch.from_numpy(Q).to(DEV)
    ids, sc = dz.filter_search(ix, Qd, q_lens, probe, filter_k, k)
    cand, _ = dz.filter_query(ix, Qd, q_lens, probe, filter_k)
    ids2, sc2 = dz.search(ix, Qd, q_lens, k, cand_ids=cand)
    assert torch.equal(ids, ids2) and torch.equal(sc, sc2)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    obo, obd = orc.inverted_index(orc.assign_centroids(X, Cn), off, K)
    dc, qc = orc.hash_i8(X, R, 32, 7), orc.hash_i8(Q, R, 32, 7)
    qo = np.concatenate([[0], np.cumsum(q_lens)])
    for b in range(len(q_lens)):
        want_cand, _ = orc.filter_query(Q[qo[b]:qo[b + 1]], Cn, obo, obd, n_docs, probe, filter_k)
        real = want_cand[want_cand != 0xFFFFFFFF].astype(np.int64)
        want_ids, want_sc = orc.topk(orc.scores(dc, off, qc[qo[b]:qo[b + 1]], real), k, real)
        assert np.array_equal(ids[b], want_ids) and np.array_equal(sc[b], want_sc), b
    # twice more on the same workspace: same answer (the unordered candidate lists may differ from call to call)
    ws = torch.empty(int(dz.lib().dessert_filter_search_workspace_bytes(ix.handle, len(q_lens), nq, max(q_lens), probe, filter_k, k)),
                     dtype=torch.uint8, device=DEV)
    for _ in range(2):
        a, b_ = dz.filter_search(ix, Qd, q_lens, probe, filter_k, k, workspace=ws)
        assert np.array_equal(a.cpu().numpy(), ids) and np.array_equal(b_.cpu().numpy(), sc)


def test_filter_search_argument_errors():
    rng = np.random.default_rng(77)
    ix, X, Cn, R, off, lens = setup(rng, 128, 9, 300, 10)
    Qd = torch.from_numpy(X[:40].copy()).to(DEV)
    with pytest.raises(dz.DessertError, match="dessert_filter_build has not been called") as e:
        dz.filter_search(ix, Qd, [8, 32], 1, 10, 5)
    assert e.value.status == dz.ESTATE
    dz.filter_build(ix, torch.from_numpy(Cn).to(DEV), torch.from_numpy(X).to(DEV))
    for args, msg in [((0, 10, 5), "filter_probe must be"), ((10, 10, 5), "filter_probe must be"), ((1, 16385, 5), "filter_k must be"),
                      ((1, 10, 0), "k must be")]:
        with pytest.raises(dz.DessertError, match=msg) as e:
            dz.filter_search(ix, Qd, [8, 32], *args)
        assert e.value.status == dz.EINVAL
    with pytest.raises(dz.DessertError, match="workspace too small"):
        dz.filter_search(ix, Qd, [8, 32], 1, 10, 5, workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    ids, sc = dz.filter_search(ix, Qd, [8, 32], 1, 10, 5)
    cand, _ = dz.filter_query(ix, Qd, [8, 32], 1, 10)
    ids2, sc2 = dz.search(ix, Qd, [8, 32], 5, cand_ids=cand)
    assert torch.equal(ids, ids2) and torch.equal(sc, sc2)


def test_search_all_slots_empty_and_k_larger_than_real_candidates():
    say("search with mostly empty candidate slots")
    rng = np.random.default_rng(9)
    ix, X, Cn, R, off, lens = setup(rng, 128, 16, 100, 10)
    q = torch.from_numpy(X[:8]).to(DEV)
    cand = torch.full((2, 6), 0xFFFFFFFF, dtype=torch.int64).to(torch.int32).to(DEV)
    cand[1, 2] = 7
    cand[1, 4] = 3
    ids, sc = dz.search(ix, q, [4, 4], 4, cand_ids=cand)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    assert np.all(ids[0] == 0xFFFFFFFF) and np.all(sc[0] == -1)
    assert set(ids[1, :2].tolist()) == {3, 7} and np.all(ids[1, 2:] == 0xFFFFFFFF) and np.all(sc[1, 2:] == -1)


@pytest.mark.parametrize("d,K,n,iters", [(128, 7, 500, 3), (64, 1, 301, 2), (256, 300, 5000, 4), (128, 40, 3000, 6),
                                         (128, 5, 0, 2), (64, 33, 64, 1)])
def test_filter_kmeans_matches_oracle(d, K, n, iters):
    say(f"filter kmeans d={d} K={K} n={n} iters={iters}")
    rng = np.random.default_rng(d + K + n)
    pool = rng.integers(-110, 111, (max(K // 2, 1), d))
    X = np.clip(pool[rng.integers(0, len(pool), n)] + rng.integers(-30, 31, (n, d)), -127, 127).astype(np.int8)
    if n >= K:
        init = X[rng.choice(n, K, replace=False)].copy()
    else:
        init = rng.integers(-127, 128, (K, d)).astype(np.int8)
    if K > 3:
        init[K - 1] = 127                      # far from everything: stays empty
        init[K - 2] = init[0]                  # duplicate: ties go to the lower id, so this one stays empty too
    ix = dz.create(d, 32, 7, seed=1)
    Xd = torch.from_numpy(X).to(DEV) if n else torch.zeros(0, d, dtype=torch.int8, device=DEV)
    got = dz.filter_kmeans(ix, Xd, torch.from_numpy(init).to(DEV), iters).cpu().numpy()
    want = orc.kmeans(X, init, iters)
    assert np.array_equal(got, want)
    if K > 3:
        assert np.array_equal(got[K - 1], init[K - 1])


def test_filter_kmeans_then_filter_chain():
    say("kmeans -> filter_build -> filter_query, cfg3-like reduced")
    w = gen.make(3, n_docs=4000, n_queries=4)
    p = w.preset
    K, iters, probe, filter_k = 500, 3, 2, 256
    rng = np.random.default_rng(0)
    sample_rows = rng.choice(w.n_vectors, 20000, replace=False)
    sample = w.docs.numpy()[sample_rows]
    init = sample[:K].copy()
    ix = dz.create(p.d, p.L, p.C, proj=w.proj.to(DEV))
    dz.build_index(ix, w.docs.to(DEV), w.lengths)
    cent = dz.filter_kmeans(ix, torch.from_numpy(sample).to(DEV), torch.from_numpy(init).to(DEV), iters)
    want_cent = orc.kmeans(sample, init, iters)
    assert np.array_equal(cent.cpu().numpy(), want_cent)
    dz.filter_build(ix, cent, w.docs.to(DEV))
    ids, cnt = dz.filter_query(ix, w.queries.to(DEV), w.q_lengths, probe, filter_k)
    obo, obd = orc.inverted_index(orc.assign_centroids(w.docs.numpy(), want_cent), w.offsets.numpy(), K)
    for b in range(p.n_queries):
        q = w.queries.numpy()[b * p.q_len:(b + 1) * p.q_len]
        want_ids, want_cnt = orc.filter_query(q, want_cent, obo, obd, w.n_docs, probe, filter_k)
        assert np.array_equal(ids[b].cpu().numpy(), want_ids) and np.array_equal(cnt[b].cpu().numpy(), want_cnt), b
