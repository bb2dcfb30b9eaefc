"""The allocation-free entry point (dessert_search_noalloc) against dessert_search: same ids and scores, bit for bit,
on two calls in a row, the second with a smaller input (the built-in scratch array keeps the first call's contents),
then the oracle on top; sizes beyond the array are refused with a message."""
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


def test_noalloc_matches_search_on_two_calls_second_smaller():
    say("search_noalloc vs search: candidate lists (grouped by id range), then a smaller batch, then every document")
    w = gen.make(3, n_docs=30_000, n_queries=24, n_cand=2048)
    p = w.preset
    ix = dz.create(p.d, p.L, p.C, proj=w.proj.to(DEV))
    dz.build_index(ix, w.docs.to(DEV), w.lengths)
    Q = w.queries.to(DEV)
    cand = w.cand_ids.to(DEV).to(torch.int32).contiguous()
    B, k = p.n_queries, p.k
    # reference results through the workspace-taking entry point
    ref1 = dz.search(ix, Q, w.q_lengths, k, cand_ids=cand)
    b2, c2 = 5, 700                                              # second call: fewer query sets, shorter lists
    Q2 = Q[: b2 * p.q_len].contiguous()
    cand2 = cand[:b2, :c2].contiguous()
    ref2 = dz.search(ix, Q2, w.q_lengths[:b2], k, cand_ids=cand2)
    ref3 = dz.search(ix, Q2, w.q_lengths[:b2], 7)                # every document
    torch.cuda.synchronize()
    out_i = torch.empty(B, k, dtype=torch.uint32, device=DEV)
    out_s = torch.empty(B, k, dtype=torch.int32, device=DEV)
    out_i2 = torch.empty(b2, k, dtype=torch.uint32, device=DEV)
    out_s2 = torch.empty(b2, k, dtype=torch.int32, device=DEV)
    out_i3 = torch.empty(b2, 7, dtype=torch.uint32, device=DEV)
    out_s3 = torch.empty(b2, 7, dtype=torch.int32, device=DEV)
    dz.search_noalloc(ix, Q, p.q_len, k, cand_ids=cand, out_ids=out_i, out_scores=out_s)
    dz.search_noalloc(ix, Q2, p.q_len, k, cand_ids=cand2, out_ids=out_i2, out_scores=out_s2)
    dz.search_noalloc(ix, Q2, p.q_len, 7, out_ids=out_i3, out_scores=out_s3)
    torch.cuda.synchronize()
    assert torch.equal(out_i, ref1[0]) and torch.equal(out_s, ref1[1])
    assert torch.equal(out_i2, ref2[0]) and torch.equal(out_s2, ref2[1])
    assert torch.equal(out_i3, ref3[0]) and torch.equal(out_s3, ref3[1])
    # and the oracle on the second (smaller) call
    R = w.proj.numpy()
    dc = orc.hash_i8(w.docs.numpy(), R, p.L, p.C)
    qc = orc.hash_i8(w.queries.numpy()[: b2 * p.q_len], R, p.L, p.C)
    qs = [qc[b * p.q_len:(b + 1) * p.q_len] for b in range(b2)]
    want_ids, want_sc, _ = orc.search(dc, w.offsets.numpy(), qs, k, cand_ids=cand2.cpu().numpy())
    assert np.array_equal(out_i2.cpu().numpy(), want_ids) and np.array_equal(out_s2.cpu().numpy(), want_sc)


def test_noalloc_long_query_sets_split_over_workgroups_start_from_zero():
    """Query sets of 70 vectors on a small grid: partial sums are added into the scores with atomics, so the score
    region of the shared array must be cleared by the call itself; run after a call that left other values there."""
    say("search_noalloc: chunks split over workgroups (scores accumulated) after a call that filled the array")
    rng = np.random.default_rng(31)
    d, L, Cb = 64, 16, 6
    lens = rng.integers(0, 30, 500).astype(np.int64)
    X = rng.integers(-127, 128, (int(lens.sum()), d)).astype(np.int8)
    X[::3] = X[0]
    R = (rng.integers(0, 2, (L * Cb, d)) * 2 - 1).astype(np.int8)
    ix = dz.create(d, L, Cb, proj=torch.from_numpy(R).to(DEV))
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    Q = torch.from_numpy(np.concatenate([X[:100], X[40:180]])[:210].copy()).to(DEV)     # 3 sets of 70
    for _ in range(2):
        got = dz.search_noalloc(ix, Q, 70, 9)
        ref = dz.search(ix, Q, [70, 70, 70], 9)
        assert dz.last_score_kernel(ix).endswith("true>")
        torch.cuda.synchronize()
        assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1])


def test_noalloc_refuses_what_does_not_fit():
    say("search_noalloc: sizes beyond the scratch array, empty arguments")
    rng = np.random.default_rng(3)
    d, L, Cb, N = 64, 16, 6, 70_000
    lens = np.ones(N, dtype=np.int64)
    X = rng.integers(-127, 128, (N, d)).astype(np.int8)
    ix = dz.create(d, L, Cb, seed=11)
    dz.build_index(ix, torch.from_numpy(X).to(DEV), lens)
    assert dz.noalloc_scratch_bytes() == 16 << 20
    Q = torch.from_numpy(X[:64 * 8].copy()).to(DEV)
    with pytest.raises(dz.DessertError, match="scratch array holds") as e:
        dz.search_noalloc(ix, Q, 8, 10)                         # 64 query sets x 70 000 documents x 4 bytes > 16 MiB
    assert e.value.status == dz.EINVAL
    out = torch.empty(64, dtype=torch.int32, device=DEV)
    st = dz.lib().dessert_search_noalloc(ix.handle, Q.data_ptr(), 0, 4, None, 0, 10, out.data_ptr(), out.data_ptr())
    assert st == dz.EINVAL and "q_length = 0" in dz.last_error()
    st = dz.lib().dessert_search_noalloc(ix.handle, Q.data_ptr(), 8, 4, None, 0, 0, out.data_ptr(), out.data_ptr())
    assert st == dz.EINVAL and "k must be" in dz.last_error()
    ids, sc = dz.search_noalloc(ix, Q[:32].contiguous(), 8, 10)   # 4 x 70 000: fits
    ref = dz.search(ix, Q[:32].contiguous(), [8] * 4, 10)
    torch.cuda.synchronize()
    assert torch.equal(ids, ref[0]) and torch.equal(sc, ref[1])
