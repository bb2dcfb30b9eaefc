#!/usr/bin/env python3
"""Benchmark of the hashed set-to-set scoring hot path on one MI355X.

A "step" is one batched search through the C ABI: hash the query vectors, score every
(query set, candidate document) pair, select the top-k (rows S1-S5 of the hot path).  The index
(rows H1-H3: hashing of all document vectors and the code layout) is built before the timed
region, as in the paper's split between Alg. 1 and Alg. 2, and its own throughput is timed in the
same run and reported under "index_build".

Workload: the candidate-rerank preset (1M documents in HBM, lengths ~ truncated normal(70, 25),
d=128 int8, L=32, C=7, 256 query sets x 32 vectors, 4096 candidates each, top-10), all synthetic and
generated on the device from fixed seeds.

Prints ONE JSON line.  "value" = doc-set scores per second of the whole step with inputs resident in HBM;
"roofline" = the scoring kernel's algorithmic code bytes per launch over its measured duration, against the
published HBM peak (plus the HBM traffic read from the rocprofv3 counter summary under profiles/ and what a plain
streaming read achieves in the same run); "index_build" and "candidate_filter" = the build and the pre-filter timed
on their own; "cpu_baseline" = the CPU oracle on a bounded sample of the same workload; "exhaustive_mid_scale" = the
same metric on the exhaustive mid-scale preset (100 000 documents, 64 query sets, every document scored), measured by
a child process after the timed regions of this one.

Other presets (--config 2, 4, 5: every document scored for every query set) are parity-test workloads, not the
metric; there the codes are shared by the query sets of a batch, the scoring kernel is bound by the vector ALU and
"roofline" is in lane-operations per second ("bound": "alu"); with fp16 vectors the index build is priced against
the fp16 matrix cores ("bound": "mfma").
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


VALU_PEAK_TLOPS = 256 * 4 * 16 * 2.4e9 / 1e12   # 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T 32-bit lane-operations/s
MFMA_F16_PEAK_TFLOPS = 2500.0


def masklut_lane_ops(L: int, paired: bool) -> int:
    """Lane-operations the mask-table method needs per (document vector, 32 query vectors): table addresses, the
    carry-save adder tree that sums L one-bit-per-query masks into bit planes, and the bit-sliced running maximum."""
    fa = ha = 0
    n = L
    while n > 1:          # one weight of the tree: (n-1)//2 full adders, one half adder if n is even
        fa += (n - 1) // 2
        ha += 1 if n % 2 == 0 else 0
        n //= 2
    planes = L.bit_length()           # counts 0..L
    return (L // 2 if paired else L) + 2 * fa + 2 * ha + 2 * planes


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_roofline(p, n_vectors: int, hash_kernel_ms, mix_gbs=None):
    """int8 vectors: the hash kernel is bound by HBM (d bytes read + L code bytes written per vector); `mix_gbs` is what
    a kernel with the same 4 : 1 read : write traffic and no arithmetic gets on this GPU in this run.  fp16 vectors with
    a Gaussian matrix: bound by the fp16 matrix cores.  The method's work is 2 * d * L * C flops per vector (Sec. 3
    SRP, the m L d hashing term of Thm 2): that is `achieved`.  The kernel issues 2 * 2 * d * 8L (the fp32 matrix is
    split into two fp16 parts and a table's C bit rows are padded to 8 per tile): reported as `kernel_issued`."""
    if not hash_kernel_ms:
        return None
    if p.dtype == "i8":
        a = n_vectors * (p.d + p.L) / (hash_kernel_ms * 1e-3) / 1e9
        r = {"bound": "hbm", "kernel": "hash_mfma_i8_kernel", "achieved": round(a, 2), "peak": HBM_PEAK_GBS,
             "unit": "GB/s", "frac": round(a / HBM_PEAK_GBS, 4), "traffic": None,
             "algorithmic_bytes_per_launch": n_vectors * (p.d + p.L), "kernel_ms": round(hash_kernel_ms, 5)}
        if mix_gbs:
            r["measured_read_write_mix_GBs"] = round(mix_gbs, 1)
            r["frac_of_measured_mix"] = round(a / mix_gbs, 4)
        return r
    method = n_vectors * 2 * p.d * p.L * p.C / (hash_kernel_ms * 1e-3) / 1e12
    issued = n_vectors * 2 * 2 * p.d * 8 * p.L / (hash_kernel_ms * 1e-3) / 1e12
    return {"bound": "mfma", "kernel": "hash_mfma_f16_kernel", "achieved": round(method, 2), "peak": MFMA_F16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": round(method / MFMA_F16_PEAK_TFLOPS, 4), "traffic": None,
            "flops": "the method's 2*d*L*C per vector", "kernel_ms": round(hash_kernel_ms, 5),
            "kernel_issued": {"achieved": round(issued, 2), "frac": round(issued / MFMA_F16_PEAK_TFLOPS, 4),
                              "flops": "2*2*d*8L per vector: hi + lo fp16 parts of the fp32 matrix, 8 bit rows per table"}}


def traffic_from_profile(kernel: str):
    """HBM bytes per launch of the scoring kernel from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE in KiB per dispatch, scaled by the copy-kernel calibration factors 2.0 and 1.0 stated there).
    `kernel` is the instantiation this run launched, spelled as the profiler prints it: the summary's lines must be
    about exactly that instantiation, else None (a summary made for an older kernel says nothing about this one).
    Valid for the full candidate-rerank preset only."""
    path = os.path.join(ROOT, "profiles", "cfg3_search_and_build_kernels.txt")
    try:
        text = open(path).read()
    except OSError:
        return None
    if not kernel:
        return None
    vals = {}
    section = None
    for line in text.splitlines():
        if line.startswith("## --pmc FETCH_SIZE"):
            section = "fetch"
        elif line.startswith("## --pmc WRITE_SIZE"):
            section = "write"
        elif line.startswith("## "):
            section = None
        elif section and "mean=" in line:
            name = line.split("grid=")[0].strip()
            # the summary keeps the tail of long names: from "score_" on it must be exactly the launched instantiation
            if "score_" in name and name[name.index("score_"):] == kernel:
                vals.setdefault(section, float(line.split("mean=")[1]))
    if "fetch" not in vals or "write" not in vals:
        return None
    return int((vals["fetch"] * 2.0 + vals["write"] * 1.0) * 1024)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--settle-ms", type=float, default=60.0,
                    help="untimed search steps run for about this long BEFORE the warm-up steps (reported as settle_steps): "
                         "after a change of load this GPU runs 10-30 %% slower for some 25 ms while its power "
                         "management settles (DESIGN.md, measurement), which at 0.4 ms per step is longer than any "
                         "reasonable count of warm-up steps; 0 = none")
    ap.add_argument("--config", type=int, default=3, help="preset number (3 = candidate rerank, the metric's workload)")
    ap.add_argument("--sweep-m", type=int, default=None,
                    help="run the synthetic-experiment shape instead of a preset: 1000 documents of m vectors, L = 8, "
                         "C = log2(m) + 1, queries = noisy documents (not the metric's workload)")
    ap.add_argument("--L", type=int, default=None, help="override the preset's number of tables (the paper's App. B grid: 16..128; not the metric)")
    ap.add_argument("--C", type=int, default=None, help="override the preset's hashes per table (App. B grid: 4..8; not the metric)")
    ap.add_argument("--n-cand", type=int, default=None, help="override the candidates per query set (App. B: filter_k 4096..16384; not the metric)")
    ap.add_argument("--n-docs", type=int, default=None, help="shrink the preset (for quick trials; not the metric)")
    ap.add_argument("--n-queries", type=int, default=None)
    ap.add_argument("--build-reps", type=int, default=20)
    ap.add_argument("--build-warmup", type=int, default=10)
    ap.add_argument("--score-algo", type=int, default=0)
    ap.add_argument("--hash-algo", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--transform", type=int, default=0,
                    help="score transform (0 raw counts: the metric; 1 = the paper's Eq. 1 remap before the sum; "
                         "2-4 max of the other phi of Sec. 4.1); implies --no-cpu-baseline")
    ap.add_argument("--cpu-sample-queries", type=int, default=32)
    ap.add_argument("--graph", action="store_true",
                    help="capture the search step in a HIP graph and time replays (per-kernel times are then taken from "
                         "a few eager calls before the capture)")
    ap.add_argument("--no-filter", action="store_true", help="skip the candidate-filter section (config 3 only)")
    ap.add_argument("--filter-centroids", type=int, default=65536)
    ap.add_argument("--kmeans-iters", type=int, default=4, help="Lloyd iterations for the filter's centroids (0: sampled vectors)")
    ap.add_argument("--kmeans-sample", type=int, default=1 << 20)
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the exhaustive mid-scale preset that the default run also measures (in a child process)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference point for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on exactly one GPU (no sharding, no collectives); --gpus must be 1")
        return 2

    import numpy as np
    import torch
    import paper_2210_15748_amd as dz
    from synth import gen

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the library has no CPU path")
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.graph:      # capture needs a stream other than the default one; the index is created on it
        side = torch.cuda.Stream(device=dev)
        torch.cuda.set_stream(side)

    t0 = time.time()
    which = gen.sweep_preset(args.sweep_m) if args.sweep_m else args.config
    overridden = args.L is not None or args.C is not None or args.n_cand is not None
    if overridden and not args.sweep_m:
        import dataclasses
        base = gen.PRESETS[args.config]
        which = dataclasses.replace(base, L=args.L or base.L, C=args.C or base.C, n_cand=base.n_cand if args.n_cand is None else args.n_cand)
        which.name = f"{base.name}_L{which.L}_C{which.C}_cand{which.n_cand}"
        args.no_secondary = True
    w = gen.make(which, device=dev, n_docs=args.n_docs, n_queries=args.n_queries)
    p = w.preset
    torch.cuda.synchronize()
    log(f"[bench] generated {p.name}: N={w.n_docs} V={w.n_vectors} B={p.n_queries} in {time.time() - t0:.1f}s")

    ix = dz.create(p.d, p.L, p.C, dtype=dz.I8 if p.dtype == "i8" else dz.F16,
                   proj_kind=dz.PROJ_RADEMACHER_I8 if p.proj_kind == "rademacher" else dz.PROJ_GAUSSIAN_F32,
                   proj=w.proj)
    dz.set_algo(ix, args.hash_algo, args.score_algo)
    if args.transform:
        dz.set_score_transform(ix, args.transform)
        args.no_cpu_baseline = True
        args.no_filter = True
    dz.enable_timing(ix, True)

    # ---- index build (H1-H3), timed on its own
    codes = torch.empty(w.n_vectors, p.L, dtype=dz.code_dtype(ix), device=dev)
    offsets = torch.empty(w.n_docs + 1, dtype=torch.int64, device=dev)
    lengths = w.lengths.numpy().astype(np.uint32)
    for _ in range(max(1, args.build_warmup)):                   # warm-up + the index used below
        dz.build_index(ix, w.docs, lengths, codes, offsets)
    torch.cuda.synchronize()
    tb = time.perf_counter()
    for _ in range(args.build_reps):
        dz.build_index(ix, w.docs, lengths, codes, offsets)
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - tb) * 1e3 / max(1, args.build_reps)
    hash_kernel_ms = float(np.mean([dz.get_timing(ix, i)["hash_ms"] for i in range(min(args.build_reps, 64))])) \
        if args.build_reps else 0.0
    log(f"[bench] build_index: {build_ms:.3f} ms/call, hash kernel {hash_kernel_ms:.3f} ms  per call: "
        + " ".join(f"{dz.get_timing(ix, i)['hash_ms']:.3f}" for i in reversed(range(min(args.build_reps, 64)))))

    # ---- search (S1-S5)
    B, k = p.n_queries, p.k
    cand = None if w.cand_ids is None else w.cand_ids.to(torch.int32).contiguous()
    n_scored = B * (p.n_cand if p.n_cand else w.n_docs)
    ws = torch.empty(dz.workspace_bytes(ix, B, w.queries.shape[0], n_scored, k), dtype=torch.uint8, device=dev)
    out_ids = torch.empty(B, k, dtype=torch.uint32, device=dev)
    out_sc = torch.empty(B, k, dtype=torch.int32, device=dev)
    ql = w.q_lengths.numpy().astype(np.uint32)
    co = None if cand is None else np.arange(B + 1, dtype=np.uint64) * p.n_cand

    def step():
        dz.search(ix, w.queries, ql, k, cand_ids=cand, cand_offsets=co, workspace=ws, out_ids=out_ids, out_scores=out_sc)

    # settle phase (see --settle-ms): the same step, untimed, until the clocks have settled; then the W warm-up steps
    settle_steps = 0
    if args.settle_ms > 0:
        t_s = time.perf_counter()
        while (time.perf_counter() - t_s) * 1e3 < args.settle_ms:
            for _ in range(8):
                step()
            torch.cuda.synchronize()
            settle_steps += 8
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Per-kernel durations come from HIP events that the library records around its launches on a sample of the
    # timed steps (every period-th: at least 8 of them); on every step the records themselves cost 4 % of a 0.45 ms step.
    period = 1 if args.graph else max(1, args.steps // 8)
    dz.enable_timing(ix, period)
    n_t = min((args.steps + period - 1) // period, 64)
    timed_step = step
    if args.graph:
        for _ in range(n_t):
            step()
        torch.cuda.synchronize()
        tim = [dz.get_timing(ix, i) for i in range(n_t)]
        dz.enable_timing(ix, False)             # no event records inside the captured step
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.current_stream()):
            step()
        timed_step = graph.replay
        for _ in range(args.warmup):
            timed_step()
        torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        timed_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    ms_per_step = elapsed * 1e3 / args.steps
    if not args.graph:
        tim = [dz.get_timing(ix, i) for i in range(n_t)]
    score_kernel = dz.last_score_kernel(ix)
    score_ms = float(np.mean([t["score_ms"] for t in tim]))
    qhash_ms = float(np.mean([t["hash_ms"] for t in tim]))
    topk_ms = float(np.mean([t["topk_ms"] for t in tim]))
    value = n_scored / (ms_per_step * 1e-3)
    log(f"[bench] search: {ms_per_step:.4f} ms/step  (hash {qhash_ms:.4f}  score {score_ms:.4f}  topk {topk_ms:.4f})")

    # ---- candidate filter (Sec. 5 "Filtering") in front of the same search: reported beside the metric, not part of it
    filt = None
    if args.config == 3 and not args.sweep_m and p.dtype == "i8" and not args.no_filter and not overridden:
        def ev_ms(fn, reps):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                r = fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps, r
        Kc = min(args.filter_centroids, w.n_vectors)
        Cn = gen.filter_centroids(w, Kc)                    # K document vectors drawn without replacement
        kmeans_ms = None
        if args.kmeans_iters:
            gs = torch.Generator(device=dev)
            gs.manual_seed(1000 * p.cfg + 77)
            n_s = min(args.kmeans_sample, w.n_vectors)
            sample = w.docs[torch.randint(0, w.n_vectors, (n_s,), generator=gs, device=dev)].contiguous()
            kmeans_ms, Cn = ev_ms(lambda: dz.filter_kmeans(ix, sample, Cn, args.kmeans_iters), 1)
            del sample
        f_build_ms, (assign, b_off, b_docs) = ev_ms(lambda: dz.filter_build(ix, Cn, w.docs), 1)
        f_probe, f_k = 1, p.n_cand
        f_query_ms, (f_ids, f_cnt) = ev_ms(lambda: dz.filter_query(ix, w.queries, ql, f_probe, f_k), 10)
        f_cand = f_ids.view(torch.int32)

        def chain(qv, qlen):   # filter, then search among the filter's ids, in one call; workspace and outputs allocated once, as a serving loop would
            nb = len(qlen)
            c_ws = torch.empty(int(dz.lib().dessert_filter_search_workspace_bytes(ix.handle, nb, qv.shape[0], int(max(qlen)), f_probe, f_k, k)),
                               dtype=torch.uint8, device=dev)
            o_ids = torch.empty(nb, k, dtype=torch.uint32, device=dev)
            o_sc = torch.empty(nb, k, dtype=torch.int32, device=dev)
            return lambda: dz.filter_search(ix, qv, qlen, f_probe, f_k, k, workspace=c_ws, out_ids=o_ids, out_scores=o_sc)
        chain_ms, _ = ev_ms(chain(w.queries, ql), 10)
        # one query set at a time (the paper's tables quote latency per query): same chain, batch of 1
        q1, ql1 = w.queries[: p.q_len].contiguous(), ql[:1]
        one_ms, _ = ev_ms(chain(q1, ql1), 200)
        kept = float(np.mean([len(set(w.planted[b].tolist()) & set(f_ids[b].cpu().tolist())) for b in range(0, B, 8)]))
        gemm_ops = 2.0 * w.n_vectors * Kc * p.d
        filt = {"n_centroids": Kc,
                "centroids": (f"{args.kmeans_iters} Lloyd iterations on {min(args.kmeans_sample, w.n_vectors)} sampled vectors, "
                              "started from document vectors drawn without replacement") if args.kmeans_iters
                else "document vectors drawn without replacement",
                "kmeans_ms": None if kmeans_ms is None else round(kmeans_ms, 2),
                "bucket_entries": int(b_off[-1].item()), "build_ms": round(f_build_ms, 2),
                "build_roofline": {"bound": "mfma", "kernel": "filter_gemm_kernel (vectors x centroids, int8)",
                                   "achieved": round(gemm_ops / (f_build_ms * 1e-3) / 1e12, 1), "peak": 5000.0,
                                   "unit": "TOP/s", "frac": round(gemm_ops / (f_build_ms * 1e-3) / 1e12 / 5000.0, 4),
                                   "note": "whole dessert_filter_build call (GEMM + argmin + bucket build) over the GEMM's operations"},
                "filter_probe": f_probe, "filter_k": f_k, "query_ms_per_batch": round(f_query_ms, 4),
                "queries_per_s": round(B / (f_query_ms * 1e-3), 1),
                "filter_then_search_ms_per_batch": round(chain_ms, 4),
                "filter_then_search_ms_single_query": round(one_ms, 4),
                "planted_docs_kept_of_%d" % p.planted_per_query: round(kept, 2)}
        log(f"[bench] filter: {filt}")
        del assign, b_off, b_docs, f_ids, f_cnt, f_cand

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- what a kernel that only reads gets out of HBM on this GPU (context for the roofline fraction)
    probe = torch.empty(1 << 30, dtype=torch.int32, device=dev).zero_()     # 4 GiB
    read_gbs = dz.probe_read_bandwidth(probe, reps=10)
    del probe
    log(f"[bench] plain streaming read: {read_gbs:.0f} GB/s")
    # ---- and a kernel with the index build's traffic (128 bytes read, 32 written per vector) and no arithmetic
    mix_gbs = None
    if p.dtype == "i8":
        mix_src = torch.empty(1 << 30, dtype=torch.int32, device=dev).zero_()   # 4 GiB read
        mix_dst = torch.empty(1 << 28, dtype=torch.int32, device=dev)           # 1 GiB written
        mix_gbs = dz.probe_mix_bandwidth(mix_src, mix_dst, reps=10)
        del mix_src, mix_dst
        log(f"[bench] read-write mix 4:1 without arithmetic: {mix_gbs:.0f} GB/s")

    # ---- roofline of the dominant kernel (scoring): algorithmic bytes = code bytes of every scored document
    if cand is not None:
        doc_len = w.lengths.to(dev)[w.cand_ids.reshape(-1)]
        code_bytes = int(doc_len.sum().item()) * p.L * codes.element_size()
    else:
        code_bytes = w.n_vectors * p.L * codes.element_size() * B      # each query set reads every document's codes once
    if cand is not None:
        achieved = code_bytes / (score_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "score_masklut_kernel", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "kernel_launched": score_kernel,
                    "traffic": traffic_from_profile(score_kernel)
                    if (args.config == 3 and not args.sweep_m and args.n_docs is None and args.n_queries is None and not overridden) else None,
                    "algorithmic_bytes_per_launch": code_bytes, "kernel_ms": round(score_ms, 5),
                    "measured_stream_read_GBs": round(read_gbs, 1), "frac_of_measured_stream": round(achieved / read_gbs, 4)}
    else:
        # every document for every query set: the codes are shared by the query sets of a batch (HBM is idle) and
        # the kernel is bound by the vector ALU.  Algorithmic work = lane-operations of the bit-sliced count per
        # (document vector, chunk of 32 query vectors): one address per table (half when two query sets share the
        # lookups), two per full/half adder of the carry-save tree, two per plane of the running maximum.
        # (whether two query sets shared the lookups is read off the instantiation the launch picked: its fifth parameter)
        inst = score_kernel[score_kernel.find("<") + 1:score_kernel.rfind(">")].split(",") if "masklut" in score_kernel else []
        ops_unit = masklut_lane_ops(p.L, paired=(len(inst) == 6 and inst[4].strip() == "2"))
        chunks = (p.q_len + 31) // 32
        lane_ops = w.n_vectors * B * chunks * ops_unit
        achieved = lane_ops / (score_ms * 1e-3) / 1e12
        roofline = {"bound": "alu", "kernel": "score_masklut_kernel", "achieved": round(achieved, 3), "peak": VALU_PEAK_TLOPS,
                    "unit": "T lane-op/s", "frac": round(achieved / VALU_PEAK_TLOPS, 4), "traffic": None,
                    "kernel_launched": score_kernel,
                    "lane_ops_per_vector_and_32_queries": ops_unit, "algorithmic_lane_ops_per_launch": lane_ops,
                    "kernel_ms": round(score_ms, 5), "code_bytes_streamed_once": w.n_vectors * p.L * codes.element_size(),
                    # the same work in the method's own unit: table-code comparisons (document vector x query vector x table)
                    "equality_tests_per_s": round(w.n_vectors * B * p.q_len * p.L / (score_ms * 1e-3), 1)}

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        nb = max(1, min(args.cpu_sample_queries, B))
        R = w.proj.cpu().numpy()
        off_all = w.offsets.numpy()
        if cand is not None:
            ids = w.cand_ids[:nb].cpu().numpy()
            uniq, inv = np.unique(ids.reshape(-1), return_inverse=True)
        else:
            # bound the oracle's hashing work (about 2e10 multiply-adds)
            mean_len = max(1.0, w.n_vectors / max(1, w.n_docs))
            cap = int(2e10 / (mean_len * p.L * p.C * p.d))
            uniq = np.arange(min(w.n_docs, 8192, max(64, cap)))
            inv = None
        rows = np.concatenate([np.arange(off_all[i], off_all[i + 1]) for i in uniq])
        sub_docs = w.docs[torch.from_numpy(rows).to(dev)].cpu().numpy()
        sub_len = (off_all[uniq + 1] - off_all[uniq])
        sub_off = np.concatenate([[0], np.cumsum(sub_len)])
        qv = w.queries[: nb * p.q_len].cpu().numpy()
        th = time.perf_counter()
        fn = orc.hash_i8 if p.dtype == "i8" else orc.hash_fp
        dc = fn(sub_docs, R, p.L, p.C)
        qc = fn(qv, R, p.L, p.C)
        hash_s = time.perf_counter() - th
        ts = time.perf_counter()
        total = 0
        if cand is not None:
            got = dz.scores(ix, w.queries[: nb * p.q_len].contiguous(), ql[:nb],
                            cand_ids=cand[:nb].contiguous()).cpu().numpy().reshape(nb, -1)
        else:   # exhaustive: score the sampled documents as an explicit candidate list
            sel_ids = torch.from_numpy(np.tile(uniq, nb).astype(np.int32)).to(dev)
            got = dz.scores(ix, w.queries[: nb * p.q_len].contiguous(), ql[:nb], cand_ids=sel_ids,
                            cand_offsets=np.arange(nb + 1, dtype=np.uint64) * len(uniq)).cpu().numpy().reshape(nb, -1)
        ok, n_diff, max_diff = True, 0, 0
        ts = time.perf_counter()
        for b in range(nb):
            sel = inv.reshape(nb, -1)[b] if inv is not None else None
            s = orc.scores(dc, sub_off, qc[b * p.q_len:(b + 1) * p.q_len], sel)
            total += s.shape[0]
            ok = ok and bool(np.array_equal(s, got[b][: s.shape[0]]))
            n_diff += int(np.count_nonzero(s != got[b][: s.shape[0]]))
            max_diff = max(max_diff, int(np.abs(s.astype(np.int64) - got[b][: s.shape[0]]).max(initial=0)))
        score_s = time.perf_counter() - ts
        cpu = {"value": round(total / score_s, 1), "unit": "doc-set scores/s", "cores": orc.num_threads(), "kind": "oracle",
               "sample": f"{nb} query sets x {total // nb} documents each ({rows.shape[0]} vectors hashed by the oracle)",
               "seconds": round(score_s, 3), "hash_vectors_per_s": round((rows.shape[0] + qv.shape[0]) / hash_s, 1),
               "hash_seconds": round(hash_s, 3), "matches_gpu_on_sample": ok}
        if p.dtype != "i8":  # tolerance path: codes may differ where a projection is within rounding of zero
            cpu["scores_differing_on_sample"] = n_diff
            cpu["max_abs_score_difference"] = max_diff
        log(f"[bench] oracle: {cpu}")

    line = {
        "metric": "doc-set scores/sec (|Q|=32, m~70, L=32, C=7)",
        "value": round(value, 1),
        "unit": "doc-set scores/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_steps": settle_steps,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": p.name, "n_docs": w.n_docs, "n_vectors": w.n_vectors, "d": p.d, "L": p.L, "C": p.C,
                   "query_sets": B, "q_len": p.q_len, "candidates_per_query": p.n_cand, "k": k,
                   "score_transform": args.transform,
                   "step": "dessert_search: query hashing + scoring + top-k (index built once, before the timed region)"
                           + (", replayed from a captured HIP graph" if args.graph else "")},
        "kernel_ms": {"query_hash": round(qhash_ms, 5), "score": round(score_ms, 5), "topk": round(topk_ms, 5)},
        # the scoring launches the means above are taken over (HIP events on a sample of the timed steps)
        "score_kernel_ms_samples": {"n": len(tim), "median": round(float(np.median([t["score_ms"] for t in tim])), 5),
                                    "min": round(float(np.min([t["score_ms"] for t in tim])), 5),
                                    "max": round(float(np.max([t["score_ms"] for t in tim])), 5)},
        "index_build": {"metric": "index-build vectors/sec", "value": round(w.n_vectors / (build_ms * 1e-3), 1),
                        "unit": "vectors/s", "ms_per_call": round(build_ms, 4), "hash_kernel_ms": round(hash_kernel_ms, 4),
                        "reps": args.build_reps, "warmup": max(1, args.build_warmup),
                        "roofline": build_roofline(p, w.n_vectors, hash_kernel_ms, mix_gbs)},
        "candidate_filter": filt,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    # The default run also measures the other presets that score every document for every query set, each in a child
    # process after this one's timed regions (not part of "value"): the exhaustive mid-scale preset (the same metric,
    # ALU-bound instead of HBM-bound), the large preset (8M documents: the index build over 563M vectors and a batch of
    # 32 query sets) and the fp16 / Gaussian stress preset (tolerance path, checked against the oracle on a sample).
    if (args.config == 3 and not args.sweep_m and args.n_docs is None and args.n_queries is None and not args.graph
            and not args.transform and not args.no_cpu_baseline and not args.no_secondary):
        import subprocess
        torch.cuda.synchronize()
        torch.cuda.empty_cache()

        def child(name, argv, timeout):
            try:
                r = subprocess.run([sys.executable, os.path.abspath(__file__)] + argv, capture_output=True, text=True,
                                   timeout=timeout)
                sub = json.loads(r.stdout.strip().splitlines()[-1])
                out = {"workload": sub["config"]["workload"], "value": sub["value"], "unit": sub["unit"],
                       "ms_per_step": sub["ms_per_step"], "kernel_ms": sub["kernel_ms"], "config": sub["config"],
                       "roofline": sub["roofline"], "index_build": sub["index_build"]}
                if sub.get("cpu_baseline"):
                    out["cpu_baseline"] = sub["cpu_baseline"]
                line[name] = out
            except Exception as e:  # the metric line must come out whatever happens to an extra measurement
                line[name] = {"error": repr(e)}
            log(f"[bench] {name}: {json.dumps(line[name])[:400]}")

        child("exhaustive_mid_scale", ["--config", "2", "--no-cpu-baseline", "--steps", "20", "--warmup", "3", "--build-reps", "20"], 240)
        child("large_exhaustive_index_build", ["--config", "4", "--no-cpu-baseline", "--steps", "10", "--warmup", "2", "--build-reps", "5"], 300)
        child("fp16_stress", ["--config", "5", "--steps", "5", "--warmup", "2", "--build-reps", "3", "--cpu-sample-queries", "8"], 300)
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
