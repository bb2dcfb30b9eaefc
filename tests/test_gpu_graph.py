"""dessert_search under HIP graph capture: with equal-length query sets and candidate lists a search is a fixed
sequence of kernel launches on the index's stream (no allocation, no copy, no synchronisation, no memset node),
so a caller can capture it once and replay it.  Every replay is checked against an eager call and the oracle,
with eager work and synchronisation between the replays."""
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


@pytest.mark.parametrize("case", ["cfg3_candidates", "cfg1_exhaustive", "sweep_m256_split_chunks", "eq1"])
def test_search_replays_from_a_captured_graph(case):
    say(f"graph capture {case}")
    if case == "cfg3_candidates":
        w = gen.make(3, n_docs=3000, n_queries=6, n_cand=512)
    elif case == "sweep_m256_split_chunks":
        w = gen.make(gen.sweep_preset(256, 3), n_docs=200)
    else:
        w = gen.make(1)
    p = w.preset
    stream = torch.cuda.Stream(device=DEV)
    B, k = p.n_queries, p.k
    n_scored = B * (p.n_cand if p.n_cand else w.n_docs)
    with torch.cuda.stream(stream):
        ix = dz.create(p.d, p.L, p.C, proj=w.proj.to(DEV), stream=stream)
        if case == "eq1":
            dz.set_score_transform(ix, dz.SCORE_EQ1_Q16)
        dz.build_index(ix, w.docs.to(DEV), w.lengths)
        q_buf = w.queries.to(DEV).clone()
        cand = None if w.cand_ids is None else w.cand_ids.to(torch.int32).to(DEV).contiguous()
        co = None if cand is None else np.arange(B + 1, dtype=np.uint64) * p.n_cand
        ws = torch.empty(dz.workspace_bytes(ix, B, q_buf.shape[0], n_scored, k), dtype=torch.uint8, device=DEV)
        out_ids = torch.empty(B, k, dtype=torch.uint32, device=DEV)
        out_sc = torch.empty(B, k, dtype=torch.int32, device=DEV)
        ql = w.q_lengths.numpy().astype(np.uint32)
        run = lambda: dz.search(ix, q_buf, ql, k, cand_ids=cand, cand_offsets=co, workspace=ws, out_ids=out_ids, out_scores=out_sc)
        run()                                   # warm-up outside the capture (one-time function attributes)
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        run()
    R = w.proj.numpy()
    dc = orc.hash_i8(w.docs.numpy(), R, p.L, p.C)
    off = w.offsets.numpy()
    rng = np.random.default_rng(1)
    for rep in range(4):
        # new query vectors each time: rows of the documents with fresh noise (eager work between the replays)
        rows = rng.integers(0, w.n_vectors, q_buf.shape[0])
        Q = np.clip(w.docs.numpy()[rows].astype(np.int64) + rng.integers(-9, 10, (q_buf.shape[0], p.d)), -127, 127).astype(np.int8)
        q_buf.copy_(torch.from_numpy(Q).to(DEV))
        out_ids.zero_(); out_sc.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        g_ids, g_sc = out_ids.cpu().numpy().copy(), out_sc.cpu().numpy().copy()
        with torch.cuda.stream(stream):
            run()
        stream.synchronize()
        assert np.array_equal(g_ids, out_ids.cpu().numpy()) and np.array_equal(g_sc, out_sc.cpu().numpy()), rep
        qc = orc.hash_i8(Q, R, p.L, p.C)
        for b in range(B):
            q = qc[b * p.q_len:(b + 1) * p.q_len]
            sel = None if w.cand_ids is None else w.cand_ids[b].numpy()
            s = orc.scores_eq1(dc, off, q, p.C, sel) if case == "eq1" else orc.scores(dc, off, q, sel)
            want_ids, want_sc = orc.topk(s, k, sel)
            assert np.array_equal(g_ids[b], want_ids) and np.array_equal(g_sc[b], want_sc), (rep, b)


def test_filter_then_search_replays_from_a_captured_graph():
    """dessert_filter_query followed by dessert_search on its ids, captured as one graph (equal-length query sets:
    kernel launches only).  Every replay is checked against eager calls and, for the filter, against the oracle."""
    say("graph capture: filter query + search on the filter's candidates")
    rng = np.random.default_rng(11)
    d, L, Cb, K, N, B, q_len, probe, filter_k, k = 128, 32, 7, 200, 60_000, 3, 16, 1, 512, 10
    lens = rng.integers(1, 4, N)
    V = int(lens.sum())
    pool = rng.integers(-127, 128, (300, d))
    X = np.clip(pool[rng.integers(0, 300, V)] + rng.integers(-25, 26, (V, d)), -127, 127).astype(np.int8)
    Cn = np.clip(pool[rng.choice(300, K, replace=False)] + rng.integers(-5, 6, (K, d)), -127, 127).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    off = np.concatenate([[0], np.cumsum(lens)])
    stream = torch.cuda.Stream(device=DEV)
    with torch.cuda.stream(stream):
        ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV), stream=stream)
        Xd = torch.from_numpy(X).to(DEV)
        dz.build_index(ix, Xd, lens)
        assign, bo, bd = dz.filter_build(ix, torch.from_numpy(Cn).to(DEV), Xd)
        q_buf = torch.zeros(B * q_len, d, dtype=torch.int8, device=DEV)
        ql = np.full(B, q_len, dtype=np.uint32)
        co = np.arange(B + 1, dtype=np.uint64) * filter_k
        f_ws = torch.empty(int(dz.lib().dessert_filter_workspace_bytes(ix.handle, B, B * q_len, q_len, probe)), dtype=torch.uint8, device=DEV)
        s_ws = torch.empty(dz.workspace_bytes(ix, B, B * q_len, B * filter_k, k), dtype=torch.uint8, device=DEV)
        out_ids = torch.empty(B, k, dtype=torch.uint32, device=DEV)
        out_sc = torch.empty(B, k, dtype=torch.int32, device=DEV)

        def run():
            f_ids, f_cnt = dz.filter_query(ix, q_buf, ql, probe, filter_k, workspace=f_ws)
            dz.search(ix, q_buf, ql, k, cand_ids=f_ids.view(torch.int32), cand_offsets=co, workspace=s_ws, out_ids=out_ids,
                      out_scores=out_sc)
            return f_ids, f_cnt
        run()                                   # warm-up outside the capture (one-time function attributes)
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        g_fids, g_fcnt = run()                  # allocated from the graph's pool: the replays write them again
    obo, obd = orc.inverted_index(orc.assign_centroids(X, Cn), off, K)
    for rep in range(4):
        rows = rng.integers(0, V, B * q_len)
        Q = np.clip(X[rows].astype(np.int64) + rng.integers(-9, 10, (B * q_len, d)), -127, 127).astype(np.int8)
        q_buf.copy_(torch.from_numpy(Q).to(DEV))
        out_ids.zero_(); out_sc.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        r_fids, r_fcnt = g_fids.cpu().numpy().copy(), g_fcnt.cpu().numpy().copy()
        r_ids, r_sc = out_ids.cpu().numpy().copy(), out_sc.cpu().numpy().copy()
        with torch.cuda.stream(stream):
            e_fids, e_fcnt = run()
        stream.synchronize()
        assert np.array_equal(r_fids, e_fids.cpu().numpy()) and np.array_equal(r_fcnt, e_fcnt.cpu().numpy()), rep
        assert np.array_equal(r_ids, out_ids.cpu().numpy()) and np.array_equal(r_sc, out_sc.cpu().numpy()), rep
        for b in range(B):
            w_ids, w_cnt = orc.filter_query(Q[b * q_len:(b + 1) * q_len], Cn, obo, obd, N, probe, filter_k)
            assert np.array_equal(r_fids[b], w_ids) and np.array_equal(r_fcnt[b], w_cnt), (rep, b)
