"""Error paths of the C ABI that need a built index on a GPU: every one must come back as a status with a message
(DESSERT_EINVAL / DESSERT_ESTATE), never as a device fault.  Also the debug mode's range check of candidate ids
(Sec. 1.1: candidates are ids of the N sets), the state of the candidate filter across index rebuilds (Sec. 5
"Filtering"), and the timing ring when only every n-th call is timed."""
import ctypes as C
import sys

import numpy as np
import pytest
import torch

import paper_2210_15748_amd as dz
from oracle import oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print("[case]", msg, flush=True)
    sys.stdout.flush()


def small_index(seed=5, n_docs=400, d=128, L=32, Cb=7, max_len=12):
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, max_len, n_docs).astype(np.int64)
    X = rng.integers(-127, 128, (int(lens.sum()), d)).astype(np.int8)
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    Xd = torch.from_numpy(X).to(DEV)
    dz.build_index(ix, Xd, lens)
    Q = rng.integers(-127, 128, (40, d)).astype(np.int8)
    return rng, ix, X, Xd, lens, R, Q


def expect(status, match, fn):
    with pytest.raises(dz.DessertError, match=match) as e:
        fn()
    assert e.value.status == status, (e.value.status, str(e.value))


def test_search_argument_errors_with_a_built_index():
    say("search/scores argument errors (bad offsets, workspace, lengths, k)")
    rng, ix, X, Xd, lens, R, Q = small_index()
    Qd = torch.from_numpy(Q).to(DEV)
    ql = np.array([8, 32], dtype=np.uint32)
    ids = torch.from_numpy(rng.integers(0, len(lens), 30).astype(np.int32)).to(DEV)
    l = dz.lib()
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    out_i = torch.empty(2, 5, dtype=torch.uint32, device=DEV)
    out_s = torch.empty(2, 5, dtype=torch.int32, device=DEV)

    def search(co=None, q_lengths=ql, k=5, wsp=ws.data_ptr(), wsn=ws.numel(), cand=ids.data_ptr()):
        coa = None if co is None else np.asarray(co, dtype=np.uint64)
        st = l.dessert_search(ix.handle, Qd.data_ptr(), q_lengths.ctypes.data, len(q_lengths), cand,
                              None if coa is None else coa.ctypes.data, k, wsp, wsn, out_i.data_ptr(), out_s.data_ptr())
        if st != dz.OK:
            raise dz.DessertError(st, dz.last_error())

    search(co=[0, 10, 30])                                                    # the valid call
    expect(dz.EINVAL, "non-decreasing", lambda: search(co=[0, 20, 10]))
    expect(dz.EINVAL, r"cand_offsets_host\[0\]", lambda: search(co=[1, 10, 30]))
    expect(dz.EINVAL, "cand_offsets_host is NULL", lambda: search(co=None))
    expect(dz.EINVAL, "workspace too small", lambda: search(co=[0, 10, 30], wsn=64))
    expect(dz.EINVAL, "256-byte aligned", lambda: search(co=[0, 10, 30], wsp=ws.data_ptr() + 16))
    expect(dz.EINVAL, "workspace_dev is NULL", lambda: search(co=[0, 10, 30], wsp=None))
    expect(dz.EINVAL, r"q_lengths_host\[1\] = 0", lambda: search(co=[0, 10, 30], q_lengths=np.array([8, 0], dtype=np.uint32)))
    expect(dz.EINVAL, "k must be", lambda: search(co=[0, 10, 30], k=0))
    expect(dz.EINVAL, "k must be", lambda: search(co=[0, 10, 30], k=16385))
    expect(dz.EINVAL, "exceed 65535 bytes", lambda: search(co=[0, 10, 30], q_lengths=np.array([8, 4000], dtype=np.uint32)))
    # after all those refusals the handle still works
    got_i, got_s = dz.search(ix, Qd, ql, 5, cand_ids=ids, cand_offsets=[0, 10, 30])
    dc, qc = orc.hash_i8(X, R, 32, 7), orc.hash_i8(Q, R, 32, 7)
    off = np.concatenate([[0], np.cumsum(lens)])
    c = ids.cpu().numpy().astype(np.int64)
    for b, (lo, hi, q0, q1) in enumerate([(0, 10, 0, 8), (10, 30, 8, 40)]):
        w_i, w_s = orc.topk(orc.scores(dc, off, qc[q0:q1], c[lo:hi]), 5, c[lo:hi])
        assert np.array_equal(got_i.cpu().numpy()[b], w_i) and np.array_equal(got_s.cpu().numpy()[b], w_s)


def test_build_index_argument_errors():
    say("build_index argument errors")
    rng, ix, X, Xd, lens, R, Q = small_index()
    codes = torch.empty(X.shape[0], 32, dtype=torch.uint8, device=DEV)
    offs = torch.empty(len(lens) + 1, dtype=torch.int64, device=DEV)
    l = dz.lib()
    lens32 = lens.astype(np.uint32)

    def build(n_vectors=X.shape[0], lp=lens32.ctypes.data, vec=Xd.data_ptr(), cd=codes.data_ptr(), od=offs.data_ptr()):
        st = l.dessert_build_index(ix.handle, vec, n_vectors, lp, len(lens32), cd, od)
        if st != dz.OK:
            raise dz.DessertError(st, dz.last_error())

    expect(dz.EINVAL, "sum of lengths_host", lambda: build(n_vectors=X.shape[0] - 1))
    expect(dz.EINVAL, "lengths_host is NULL", lambda: build(lp=None))
    expect(dz.EINVAL, "offsets_dev is NULL", lambda: build(od=None))
    expect(dz.EINVAL, "vectors_dev / codes_dev is NULL", lambda: build(cd=None))
    build()
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), orc.hash_i8(X, R, 32, 7))


def test_filter_argument_and_state_errors():
    say("filter: query before build, probe > K, filter_k too large, misaligned workspace")
    rng, ix, X, Xd, lens, R, Q = small_index()
    Qd = torch.from_numpy(Q).to(DEV)
    ql = [8, 32]
    expect(dz.ESTATE, "dessert_filter_build has not been called", lambda: dz.filter_query(ix, Qd, ql, 1, 10))
    K = 9
    Cn = torch.from_numpy(X[:K].copy()).to(DEV)
    dz.filter_build(ix, Cn, Xd)
    expect(dz.EINVAL, "filter_probe must be", lambda: dz.filter_query(ix, Qd, ql, K + 1, 10))
    expect(dz.EINVAL, "filter_probe must be", lambda: dz.filter_query(ix, Qd, ql, 0, 10))
    expect(dz.EINVAL, "filter_k must be", lambda: dz.filter_query(ix, Qd, ql, 1, 16385))
    expect(dz.EINVAL, "filter_k must be|NULL argument", lambda: dz.filter_query(ix, Qd, ql, 1, 0))
    ws = torch.empty(1 << 22, dtype=torch.uint8, device=DEV)
    expect(dz.EINVAL, "aligned", lambda: dz.filter_query(ix, Qd, ql, 1, 10, workspace=ws[16:]))
    expect(dz.EINVAL, "workspace too small", lambda: dz.filter_query(ix, Qd, ql, 1, 10, workspace=ws[:256]))
    expect(dz.EINVAL, r"q_lengths_host\[0\] = 0", lambda: dz.filter_query(ix, Qd[:32], [0, 32], 1, 10))
    expect(dz.EINVAL, "n_centroids must be|NULL argument", lambda: dz.filter_build(ix, Cn[:0], Xd))
    ids, cnt = dz.filter_query(ix, Qd, ql, 2, 10)
    off = np.concatenate([[0], np.cumsum(lens)])
    obo, obd = orc.inverted_index(orc.assign_centroids(X, X[:K]), off, K)
    w_ids, w_cnt = orc.filter_query(Q[:8], X[:K], obo, obd, len(lens), 2, 10)
    assert np.array_equal(ids.cpu().numpy()[0], w_ids) and np.array_equal(cnt.cpu().numpy()[0], w_cnt)


def test_rebuilding_the_index_drops_the_filter():
    """build, filter_build, then build_index over ANOTHER collection: the filter of the first collection must not
    answer for the second one; after a new filter_build the results are those of the oracle on the new collection."""
    say("filter state across index rebuilds")
    rng, ix, X, Xd, lens, R, Q = small_index(seed=8, n_docs=500)
    Qd = torch.from_numpy(Q).to(DEV)
    K = 12
    dz.filter_build(ix, torch.from_numpy(X[:K].copy()).to(DEV), Xd)
    dz.filter_query(ix, Qd, [8, 32], 2, 20)
    lens2 = rng.integers(1, 30, 211).astype(np.int64)              # a different number of documents
    X2 = rng.integers(-127, 128, (int(lens2.sum()), 128)).astype(np.int8)
    X2d = torch.from_numpy(X2).to(DEV)
    dz.build_index(ix, X2d, lens2)
    expect(dz.ESTATE, "dessert_filter_build has not been called", lambda: dz.filter_query(ix, Qd, [8, 32], 2, 20))
    assert dz.lib().dessert_filter_workspace_bytes(ix.handle, 2, 40, 32, 2) == 0
    Cn2 = X2[5:5 + K].copy()
    dz.filter_build(ix, torch.from_numpy(Cn2).to(DEV), X2d)
    ids, cnt = dz.filter_query(ix, Qd, [8, 32], 2, 20)
    off2 = np.concatenate([[0], np.cumsum(lens2)])
    obo, obd = orc.inverted_index(orc.assign_centroids(X2, Cn2), off2, K)
    for b, (q0, q1) in enumerate([(0, 8), (8, 40)]):
        w_ids, w_cnt = orc.filter_query(Q[q0:q1], Cn2, obo, obd, len(lens2), 2, 20)
        assert np.array_equal(ids.cpu().numpy()[b], w_ids) and np.array_equal(cnt.cpu().numpy()[b], w_cnt), b
    # once more on the same collection: first with the same number of centroids (the library keeps its buffers), then
    # with another number (it allocates them again)
    for K3, first in ((K, 40), (20, 90)):
        Cn3 = X2[first:first + K3].copy()
        dz.filter_build(ix, torch.from_numpy(Cn3).to(DEV), X2d)
        ids, cnt = dz.filter_query(ix, Qd, [8, 32], 2, 20)
        obo, obd = orc.inverted_index(orc.assign_centroids(X2, Cn3), off2, K3)
        for b, (q0, q1) in enumerate([(0, 8), (8, 40)]):
            w_ids, w_cnt = orc.filter_query(Q[q0:q1], Cn3, obo, obd, len(lens2), 2, 20)
            assert np.array_equal(ids.cpu().numpy()[b], w_ids) and np.array_equal(cnt.cpu().numpy()[b], w_cnt), (K3, b)


def test_debug_mode_catches_a_candidate_id_out_of_range():
    say("debug mode: candidate id = n_docs is an error, not a fault")
    rng, ix, X, Xd, lens, R, Q = small_index()
    N = len(lens)
    Qd = torch.from_numpy(Q[:32].copy()).to(DEV)
    good = rng.integers(0, N, 64).astype(np.int64)
    good[3] = 0xFFFFFFFF                                            # an empty slot is fine
    bad = good.copy()
    bad[17] = N                                                     # one past the last document
    bad[40] = N + 5
    as_dev = lambda a: torch.from_numpy(a.astype(np.uint32).view(np.int32)).to(DEV)
    dz.set_debug(ix, True)
    expect(dz.EINVAL, r"cand_ids_dev\[17\]", lambda: dz.search(ix, Qd, [32], 5, cand_ids=as_dev(bad), cand_offsets=[0, 64]))
    expect(dz.EINVAL, r"cand_ids_dev\[17\]", lambda: dz.scores(ix, Qd, [32], cand_ids=as_dev(bad), cand_offsets=[0, 64]))
    expect(dz.EINVAL, r"cand_ids_dev\[17\]", lambda: dz.search_noalloc(ix, Qd, 32, 5, cand_ids=as_dev(bad).view(1, 64)))
    got = dz.scores(ix, Qd, [32], cand_ids=as_dev(good), cand_offsets=[0, 64]).cpu().numpy()
    dz.set_debug(ix, False)
    again = dz.scores(ix, Qd, [32], cand_ids=as_dev(good), cand_offsets=[0, 64]).cpu().numpy()
    dc, qc = orc.hash_i8(X, R, 32, 7), orc.hash_i8(Q[:32], R, 32, 7)
    off = np.concatenate([[0], np.cumsum(lens)])
    real = good != 0xFFFFFFFF
    want = np.full(64, -1, dtype=np.int64)
    want[real] = orc.scores(dc, off, qc, good[real])
    assert np.array_equal(got, want) and np.array_equal(again, want)


def test_capture_refuses_what_it_cannot_record():
    """Unequal query-set or candidate-list lengths need an offsets upload, which a graph would replay from a staging
    buffer that later calls overwrite: the call must refuse while the stream is capturing, and work again afterwards."""
    say("graph capture with unequal lengths / build_index -> DESSERT_ESTATE")
    rng, ix0, X, Xd, lens, R, Q = small_index()
    del ix0
    side = torch.cuda.Stream(device=DEV)
    with torch.cuda.stream(side):
        ix = dz.create(128, 32, 7, proj=torch.from_numpy(R).to(DEV))      # the handle works on the side stream
        codes, offs = dz.build_index(ix, Xd, lens)
        Qd = torch.from_numpy(Q).to(DEV)
        ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
        out_i = torch.empty(2, 5, dtype=torch.uint32, device=DEV)
        out_s = torch.empty(2, 5, dtype=torch.int32, device=DEV)
        eager = dz.search(ix, Qd, [20, 20], 5)
        side.synchronize()
        seen = []
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for fn in (lambda: dz.search(ix, Qd, [8, 32], 5, workspace=ws, out_ids=out_i, out_scores=out_s),
                       lambda: dz.build_index(ix, Xd, lens, codes, offs)):
                try:
                    fn()
                    seen.append(None)
                except dz.DessertError as e:
                    seen.append((e.status, str(e)))
            dz.search(ix, Qd, [20, 20], 5, workspace=ws, out_ids=out_i, out_scores=out_s)   # equal lengths: recorded
        assert seen[0] is not None and seen[0][0] == dz.ESTATE and "equal length" in seen[0][1], seen
        assert seen[1] is not None and seen[1][0] == dz.ESTATE and "captured" in seen[1][1], seen
        out_i.zero_(); out_s.zero_()
        g.replay()
        side.synchronize()
        assert torch.equal(out_i, eager[0]) and torch.equal(out_s, eager[1])
        got = dz.search(ix, Qd, [8, 32], 5)                                  # unequal lengths work again when not capturing
        side.synchronize()
    dc, qc = orc.hash_i8(X, R, 32, 7), orc.hash_i8(Q, R, 32, 7)
    off = np.concatenate([[0], np.cumsum(lens)])
    w_i, w_s, _ = orc.search(dc, off, [qc[:8], qc[8:]], 5)
    assert np.array_equal(got[0].cpu().numpy(), w_i) and np.array_equal(got[1].cpu().numpy(), w_s)


def test_timing_ring_keeps_64_records_when_every_third_call_is_timed():
    say("timing: 64 records readable with period 3 (untimed calls must not wipe live records)")
    rng, ix, X, Xd, lens, R, Q = small_index()
    Qd = torch.from_numpy(Q).to(DEV)
    dz.enable_timing(ix, 3)
    for _ in range(3 * 70):
        dz.search(ix, Qd, [8, 32], 5)
    torch.cuda.synchronize()
    for back in range(64):
        t = dz.get_timing(ix, back)
        assert t["total_ms"] > 0 and t["score_ms"] > 0, back
    expect(dz.ESTATE, "no timed call", lambda: dz.get_timing(ix, 64))
