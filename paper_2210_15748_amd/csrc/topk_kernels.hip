// Stand-alone top-k kernels for gfx950 (the selection itself is in topk_select.hpp).
// One workgroup per (query set, slice) selects the k best keys of its slice; a single slice
// gives the final result directly, otherwise a second launch selects among the slices' keys.
#include "kernels.hpp"
#include "topk_select.hpp"

namespace dessert {

constexpr uint32_t TOPK_THREADS = 512;
constexpr uint64_t TOPK_SLICE = 1u << 16;

// Slices per query set: long lists are cut into 65536-element slices; shorter ones are still cut
// (down to 8192 elements per slice) when the batch alone would leave most CUs without a workgroup.
// Non-decreasing in max_scored, so a bound on the list length bounds the slice count.
uint32_t topk_slices(uint64_t max_scored, uint32_t n_queries) {
    uint64_t by_size = max_scored <= 2 * TOPK_SLICE ? 1 : (max_scored + TOPK_SLICE - 1) / TOPK_SLICE;
    uint64_t want = n_queries ? (1024 + n_queries - 1) / n_queries : 1;
    uint64_t by_fill = max_scored / 8192 < want ? max_scored / 8192 : want;
    uint64_t s = by_size > by_fill ? by_size : by_fill;
    return (uint32_t)(s ? s : 1);
}

// grid (slices, B).  slices == 1: final results; else per-slice keys to a.partial.
// KT: the width the keys are computed in (uint32_t when keys_fit_32).  T threads with U loads in flight each; a slice of
// at most T * U = 4096 scores stays in registers for all passes.  T = 512, U = 8 in general; T = 1024, U = 4 when no
// slice is longer than that (candidate lists): the phases of such a selection are short chains of LDS round trips and
// barriers, which sixteen waves get through sooner than eight (17 -> 14 us for 256 lists of 4096); on long slices the
// wider workgroup is slower (0.90 -> 1.20 ms on 8M documents).
constexpr uint32_t TOPK_THREADS_SHORT = 1024;
template <typename KT, int T, int U>
__global__ __launch_bounds__(T) void topk_scores_kernel(TopkArgs a, KeyPlan plan, uint32_t slices, uint32_t kpad) {
    extern __shared__ uint64_t sorted[];
    __shared__ SelectShared sh;
    const uint32_t b = blockIdx.y, s = blockIdx.x;
    uint64_t base, count;
    if (a.cand_ids) {
        base = a.cand_uniform ? (uint64_t)b * a.cand_uniform : a.cand_off[b];
        count = a.cand_uniform ? a.cand_uniform : a.cand_off[b + 1] - base;
    } else {
        base = (uint64_t)b * a.n_docs;
        count = a.n_docs;
    }
    const uint64_t per = (count + slices - 1) / slices;
    const uint64_t lo = (uint64_t)s * per < count ? (uint64_t)s * per : count;
    const uint64_t hi = lo + per < count ? lo + per : count;
    ScoreKeysT<KT> keys{a.scores + base + lo, a.cand_ids ? a.cand_ids + base + lo : nullptr, lo, plan.id_bits};
    block_select<T, ScoreKeysT<KT>, U, true>(keys, hi - lo, a.k, kpad, sorted, sh, plan);
    if (slices == 1) {
        for (uint32_t i = threadIdx.x; i < a.k; i += T)
            write_result(sorted[i], plan.id_bits, a.out_ids + (size_t)b * a.k + i, a.out_scores + (size_t)b * a.k + i);
    } else {
        uint64_t* dst = a.partial + ((size_t)b * slices + s) * a.k;
        for (uint32_t i = threadIdx.x; i < a.k; i += T) dst[i] = sorted[i];
    }
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_merge_kernel(TopkArgs a, KeyPlan plan, uint32_t slices,
                                                                  uint32_t kpad) {
    extern __shared__ uint64_t sorted[];
    __shared__ SelectShared sh;
    const uint32_t b = blockIdx.x;
    StoredKeys keys{a.partial + (size_t)b * slices * a.k};
    block_select<TOPK_THREADS>(keys, (uint64_t)slices * a.k, a.k, kpad, sorted, sh, plan);
    for (uint32_t i = threadIdx.x; i < a.k; i += TOPK_THREADS)
        write_result(sorted[i], plan.id_bits, a.out_ids + (size_t)b * a.k + i, a.out_scores + (size_t)b * a.k + i);
}

// one workgroup per stored list whose length is read from device memory.  There are only as many workgroups
// as lists, so each is wide and keeps many loads in flight: a pass over a list is a few round trips.
constexpr uint32_t TOPK_LIST_THREADS = 1024;
template <typename KT, bool ORDERED>  // stored key type: uint64_t, or uint32_t when keys_fit_32; ORDERED: best first, else any order
__global__ __launch_bounds__(TOPK_LIST_THREADS) void topk_lists_kernel(const KT* __restrict__ lists, uint64_t list_stride,
                                                                       const uint32_t* __restrict__ counts, uint32_t k,
                                                                       KeyPlan plan, uint32_t kpad, uint32_t* __restrict__ out_ids,
                                                                       int32_t* __restrict__ out_scores,
                                                                       const uint32_t* __restrict__ hist0, uint32_t hist_bins,
                                                                       const uint32_t* __restrict__ segs, uint32_t slabs) {
    extern __shared__ uint64_t sorted[];
    __shared__ SelectShared sh;
    const uint32_t b = blockIdx.x;
    // segs != nullptr: hist0 holds rows per slab (see SlabDirectory); else one histogram per list, or nothing
    const uint32_t* first_hist = (hist0 && !segs) ? hist0 + (size_t)b * hist_bins : nullptr;
    SlabDirectory directory{nullptr, nullptr, 0, 0};
    if (segs) directory = SlabDirectory{hist0 + (size_t)b * slabs * hist_bins, segs + (size_t)b * slabs * 2, slabs, hist_bins};
    const SlabDirectory* dir = segs ? &directory : nullptr;
    if constexpr (sizeof(KT) == 8) {
        StoredKeysPairs keys{lists + (size_t)b * list_stride};
        block_select<TOPK_LIST_THREADS, StoredKeysPairs, 8, false, ORDERED>(keys, counts[b], k, kpad, sorted, sh, plan, first_hist, dir);
    } else {
        StoredKeys32 keys{lists + (size_t)b * list_stride};
        block_select<TOPK_LIST_THREADS, StoredKeys32, 8, false, ORDERED>(keys, counts[b], k, kpad, sorted, sh, plan, first_hist, dir);
    }
    for (uint32_t i = threadIdx.x; i < k; i += TOPK_LIST_THREADS)
        write_result(sorted[i], plan.id_bits, out_ids + (size_t)b * k + i, out_scores + (size_t)b * k + i);
}

// The same selection for a few long lists, in two launches: one workgroup per list finds the k-th key (everything
// block_select does short of its last pass over the list) and leaves it in emit_plan[b]; topk_lists_emit_kernel then
// copies the keys at or above it with many workgroups per list.  With one workgroup per list that last pass is the
// longest part of the selection, and with a handful of lists the rest of the chip idles meanwhile.  Unordered results.
// emit_plan[b] = {k-th key (low, high word), copies of it to take, done flag, output cursor, copies taken, -, -}.
constexpr uint32_t TOPK_EMIT_WORDS = TOPK_LISTS_EMIT_WORDS;
constexpr uint32_t TOPK_EMIT_PARTS = 32;   // workgroups per list in the second launch
template <typename KT>
__global__ __launch_bounds__(TOPK_LIST_THREADS) void topk_lists_plan_kernel(const KT* __restrict__ lists, uint64_t list_stride,
                                                                            const uint32_t* __restrict__ counts, uint32_t k,
                                                                            KeyPlan plan, uint32_t kpad, uint32_t* __restrict__ out_ids,
                                                                            int32_t* __restrict__ out_scores,
                                                                            const uint32_t* __restrict__ hist0, uint32_t hist_bins,
                                                                            const uint32_t* __restrict__ segs, uint32_t slabs,
                                                                            uint32_t* __restrict__ emit_plan) {
    extern __shared__ uint64_t sorted[];
    __shared__ SelectShared sh;
    const uint32_t b = blockIdx.x;
    const uint32_t* first_hist = (hist0 && !segs) ? hist0 + (size_t)b * hist_bins : nullptr;
    SlabDirectory directory{nullptr, nullptr, 0, 0};
    if (segs) directory = SlabDirectory{hist0 + (size_t)b * slabs * hist_bins, segs + (size_t)b * slabs * 2, slabs, hist_bins};
    const SlabDirectory* dir = segs ? &directory : nullptr;
    bool done;
    if constexpr (sizeof(KT) == 8) {
        StoredKeysPairs keys{lists + (size_t)b * list_stride};
        done = block_select<TOPK_LIST_THREADS, StoredKeysPairs, 8, false, false, false>(keys, counts[b], k, kpad, sorted, sh, plan, first_hist, dir);
    } else {
        StoredKeys32 keys{lists + (size_t)b * list_stride};
        done = block_select<TOPK_LIST_THREADS, StoredKeys32, 8, false, false, false>(keys, counts[b], k, kpad, sorted, sh, plan, first_hist, dir);
    }
    uint32_t* p = emit_plan + (size_t)b * TOPK_EMIT_WORDS;
    if (done) {  // a short list, or few keys at the top: the result is complete
        for (uint32_t i = threadIdx.x; i < k; i += TOPK_LIST_THREADS)
            write_result(sorted[i], plan.id_bits, out_ids + (size_t)b * k + i, out_scores + (size_t)b * k + i);
        if (threadIdx.x == 0) p[3] = 1;
    } else if (threadIdx.x == 0) {
        p[0] = (uint32_t)sh.prefix;
        p[1] = (uint32_t)(sh.prefix >> 32);
        p[2] = sh.need;
        p[3] = 0;
        p[4] = 0;
        p[5] = 0;
    }
}

// grid (parts, B): workgroup (x, b) copies, of its part of list b, the keys above the k-th key and as many copies of the
// k-th key itself as the plan says; output slots are taken with one atomic per wave and trip.
constexpr uint32_t TOPK_EMIT_THREADS = 256;
template <typename KT>
__global__ __launch_bounds__(TOPK_EMIT_THREADS) void topk_lists_emit_kernel(const KT* __restrict__ lists, uint64_t list_stride,
                                                                            const uint32_t* __restrict__ counts, uint32_t k,
                                                                            uint32_t id_bits, uint32_t* __restrict__ emit_plan,
                                                                            uint32_t* __restrict__ out_ids,
                                                                            int32_t* __restrict__ out_scores) {
    constexpr uint32_t V = 16 / sizeof(KT), U = 4, T = TOPK_EMIT_THREADS;
    const uint32_t b = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
    uint32_t* p = emit_plan + (size_t)b * TOPK_EMIT_WORDS;
    if (p[3]) return;
    const uint64_t n = counts[b];
    const KT kth = (KT)((uint64_t)p[0] | ((uint64_t)p[1] << 32));
    const uint32_t need_eq = p[2];
    const KT* keys = lists + (size_t)b * list_stride;
    uint64_t part = (n + gridDim.x - 1) / gridDim.x;
    part = (part + V - 1) / V * V;  // parts start on 16-byte boundaries
    const uint64_t lo = (uint64_t)blockIdx.x * part < n ? (uint64_t)blockIdx.x * part : n;
    const uint64_t hi = lo + part < n ? lo + part : n;
    for (uint64_t t0 = lo; t0 < hi; t0 += (uint64_t)U * T * V) {
        KT key[U][V];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint64_t i = t0 + ((uint64_t)u * T + tid) * V;
#pragma unroll
            for (uint32_t v = 0; v < V; ++v) key[u][v] = 0;
            if (i < hi) {  // a vector that starts below the list's end stays inside its allocation
                if constexpr (sizeof(KT) == 8) {
                    const ulonglong2 x = *(const ulonglong2*)(keys + i);
                    key[u][0] = x.x;
                    key[u][1] = x.y;
                } else {
                    const uint4 x = *(const uint4*)(keys + i);
                    key[u][0] = x.x;
                    key[u][1] = x.y;
                    key[u][2] = x.z;
                    key[u][3] = x.w;
                }
            }
        }
        uint32_t flags = 0;
#pragma unroll
        for (uint32_t u = 0; u < U; ++u)
#pragma unroll
            for (uint32_t v = 0; v < V; ++v) {
                const uint64_t i = t0 + ((uint64_t)u * T + tid) * V + v;
                bool take = i < hi && key[u][v] > kth;
                if (i < hi && key[u][v] == kth) take = atomicAdd(&p[5], 1u) < need_eq;
                flags |= (take ? 1u : 0u) << (u * V + v);
            }
        const uint32_t cnt = (uint32_t)__builtin_popcount(flags);
        uint32_t incl = cnt;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t o = __shfl_up(incl, off, 64);
            if ((int)lane >= off) incl += o;
        }
        uint32_t base = 0;
        if (lane == 63 && incl) base = atomicAdd(&p[4], incl);
        base = __shfl(base, 63, 64);
        uint32_t pos = base + incl - cnt;
#pragma unroll
        for (uint32_t u = 0; u < U; ++u)
#pragma unroll
            for (uint32_t v = 0; v < V; ++v)
                if ((flags >> (u * V + v)) & 1u) {
                    if (pos < k) write_result((uint64_t)key[u][v], id_bits, out_ids + (size_t)b * k + pos, out_scores + (size_t)b * k + pos);
                    ++pos;
                }
    }
}

static hipError_t allow_large_k() {  // large k: opt in to more dynamic LDS (the selection state is another 8.3 KB)
    static hipError_t a0 = hipFuncSetAttribute((const void*)topk_scores_kernel<uint32_t, TOPK_THREADS, 8>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, TOPK_KMAX * 8);
    static hipError_t a1 = hipFuncSetAttribute((const void*)topk_scores_kernel<uint64_t, TOPK_THREADS, 8>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, TOPK_KMAX * 8);
    static hipError_t a9 = hipFuncSetAttribute((const void*)topk_scores_kernel<uint32_t, TOPK_THREADS_SHORT, 4>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, TOPK_KMAX * 8);
    static hipError_t a10 = hipFuncSetAttribute((const void*)topk_scores_kernel<uint64_t, TOPK_THREADS_SHORT, 4>,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, TOPK_KMAX * 8);
    static hipError_t a2 = hipFuncSetAttribute((const void*)topk_merge_kernel,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, TOPK_KMAX * 8);
    static hipError_t a3 = hipFuncSetAttribute((const void*)topk_lists_kernel<uint64_t, true>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, TOPK_KMAX * 8);
    static hipError_t a4 = hipFuncSetAttribute((const void*)topk_lists_kernel<uint32_t, true>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, TOPK_KMAX * 8);
    static hipError_t a5 = hipFuncSetAttribute((const void*)topk_lists_kernel<uint64_t, false>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, TOPK_KMAX * 8);
    static hipError_t a6 = hipFuncSetAttribute((const void*)topk_lists_kernel<uint32_t, false>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, TOPK_KMAX * 8);
    static hipError_t a7 = hipFuncSetAttribute((const void*)topk_lists_plan_kernel<uint64_t>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, TOPK_KMAX * 8);
    static hipError_t a8 = hipFuncSetAttribute((const void*)topk_lists_plan_kernel<uint32_t>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, TOPK_KMAX * 8);
    return a0 != hipSuccess ? a0 : a1 != hipSuccess ? a1 : a2 != hipSuccess ? a2 : a3 != hipSuccess ? a3 : a4 != hipSuccess ? a4
           : a5 != hipSuccess ? a5 : a6 != hipSuccess ? a6 : a7 != hipSuccess ? a7 : a8 != hipSuccess ? a8 : a9 != hipSuccess ? a9 : a10;
}

hipError_t launch_topk_lists(const uint64_t* lists, uint64_t list_stride, const uint32_t* counts, uint32_t n_queries,
                             uint32_t k, uint32_t max_score, uint64_t max_id, const FilterHistPlan* hp, uint32_t* out_ids,
                             int32_t* out_scores, bool ordered, hipStream_t stream, uint32_t* emit_plan) {
    if (n_queries == 0 || k == 0) return hipSuccess;
    if (emit_plan && ordered) return hipErrorInvalidValue;  // the two-launch form leaves the result unordered
    if (k > TOPK_KMAX) return hipErrorInvalidValue;
    // the lists are read 16 bytes at a time
    if ((uintptr_t)lists % 16 || list_stride % 4) return hipErrorInvalidValue;
    uint32_t kpad = 2;
    while (kpad < k) kpad <<= 1;
    const KeyPlan plan = make_key_plan(max_score, max_id);
    const size_t lds = (size_t)kpad * 8;
    if (lds > 48 * 1024) {
        hipError_t e = allow_large_k();
        if (e != hipSuccess) return e;
    }
    const uint32_t hist_bins = (hp && hp->bins) ? hp->bins : 0;
    if (hist_bins && hist_bins != leading_score_bins(max_score, max_id)) return hipErrorInvalidValue;
    if (hist_bins && hp->rows && hp->slabs > TOPK_LIST_THREADS) return hipErrorInvalidValue;
    const uint32_t* hist0 = hist_bins ? counts + hp->hist_off : nullptr;
    const uint32_t* segs = (hist_bins && hp->rows) ? counts + hp->seg_off : nullptr;
    const uint32_t slabs = hist_bins ? hp->slabs : 0;
    const dim3 grid(n_queries), block(TOPK_LIST_THREADS);
    if (emit_plan) {
        const dim3 egrid(TOPK_EMIT_PARTS, n_queries), eblock(TOPK_EMIT_THREADS);
        if (keys_fit_32(max_score, max_id)) {
            hipLaunchKernelGGL(topk_lists_plan_kernel<uint32_t>, grid, block, lds, stream, (const uint32_t*)lists, list_stride, counts,
                               k, plan, kpad, out_ids, out_scores, hist0, hist_bins, segs, slabs, emit_plan);
            hipLaunchKernelGGL(topk_lists_emit_kernel<uint32_t>, egrid, eblock, 0, stream, (const uint32_t*)lists, list_stride,
                               counts, k, plan.id_bits, emit_plan, out_ids, out_scores);
        } else {
            hipLaunchKernelGGL(topk_lists_plan_kernel<uint64_t>, grid, block, lds, stream, lists, list_stride, counts, k, plan, kpad,
                               out_ids, out_scores, hist0, hist_bins, segs, slabs, emit_plan);
            hipLaunchKernelGGL(topk_lists_emit_kernel<uint64_t>, egrid, eblock, 0, stream, lists, list_stride, counts, k,
                               plan.id_bits, emit_plan, out_ids, out_scores);
        }
        return hipGetLastError();
    }
    if (keys_fit_32(max_score, max_id)) {
        auto kern = ordered ? topk_lists_kernel<uint32_t, true> : topk_lists_kernel<uint32_t, false>;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, (const uint32_t*)lists, list_stride, counts, k, plan, kpad, out_ids,
                           out_scores, hist0, hist_bins, segs, slabs);
    } else {
        auto kern = ordered ? topk_lists_kernel<uint64_t, true> : topk_lists_kernel<uint64_t, false>;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, lists, list_stride, counts, k, plan, kpad, out_ids, out_scores, hist0,
                           hist_bins, segs, slabs);
    }
    return hipGetLastError();
}

hipError_t launch_topk(const TopkArgs& a, hipStream_t stream) {
    if (a.n_queries == 0 || a.k == 0) return hipSuccess;
    if (a.k > TOPK_KMAX || a.n_queries > 65535) return hipErrorInvalidValue;
    uint32_t kpad = 2;
    while (kpad < a.k) kpad <<= 1;
    const KeyPlan plan = make_key_plan(a.max_score, a.n_docs ? a.n_docs - 1 : 0);
    const uint32_t slices = topk_slices(a.max_scored, a.n_queries);
    const size_t lds = (size_t)kpad * 8;
    if (lds > 48 * 1024) {
        hipError_t e = allow_large_k();
        if (e != hipSuccess) return e;
    }
    const bool fit32 = keys_fit_32(a.max_score, a.n_docs ? a.n_docs - 1 : 0);
    const dim3 grid(slices, a.n_queries);
    // every slice short enough to stay in the registers of the wider workgroup (see topk_scores_kernel)
    if ((a.max_scored + slices - 1) / slices <= (uint64_t)TOPK_THREADS_SHORT * 4) {
        if (fit32)
            hipLaunchKernelGGL((topk_scores_kernel<uint32_t, TOPK_THREADS_SHORT, 4>), grid, dim3(TOPK_THREADS_SHORT), lds, stream, a, plan,
                               slices, kpad);
        else
            hipLaunchKernelGGL((topk_scores_kernel<uint64_t, TOPK_THREADS_SHORT, 4>), grid, dim3(TOPK_THREADS_SHORT), lds, stream, a, plan,
                               slices, kpad);
    } else {
        if (fit32)
            hipLaunchKernelGGL((topk_scores_kernel<uint32_t, TOPK_THREADS, 8>), grid, dim3(TOPK_THREADS), lds, stream, a, plan, slices, kpad);
        else
            hipLaunchKernelGGL((topk_scores_kernel<uint64_t, TOPK_THREADS, 8>), grid, dim3(TOPK_THREADS), lds, stream, a, plan, slices, kpad);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || slices == 1) return e;
    hipLaunchKernelGGL(topk_merge_kernel, dim3(a.n_queries), dim3(TOPK_THREADS), lds, stream, a, plan, slices, kpad);
    return hipGetLastError();
}

}  // namespace dessert
