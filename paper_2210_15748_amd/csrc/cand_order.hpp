// Grouping of candidate lists by range of document id (device code shared by the stand-alone kernel and by the
// query-hashing launch that carries it along).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dessert {

struct CandOrderArgs {
    const uint32_t* cand_ids;   // dev, the lists of all query sets concatenated
    const uint64_t* cand_off;   // dev [n_lists+1]; unused when cand_uniform != 0
    uint64_t cand_uniform;      // != 0: every list has this many ids
    uint32_t n_lists;
    uint32_t shift, ranges;     // range of an id = id >> shift, clamped to ranges - 1
    uint32_t* order;            // dev out, [total ids]: per list, its slots grouped by range
};

// Counting sort of list b's slots by range of document id: one workgroup of T threads, two passes over the ids
// (eight loads in flight per thread; a list of up to 8*T ids stays in registers for the second pass).
// bin: a.ranges words of LDS; wave_sum: T/64 words of LDS.  Every thread of the workgroup calls this.
template <int T>
__device__ inline void cand_order_body(const CandOrderArgs& a, uint32_t b, uint32_t* bin, uint32_t* wave_sum) {
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t shift = a.shift, ranges = a.ranges;
    const uint64_t base = a.cand_uniform ? (uint64_t)b * a.cand_uniform : a.cand_off[b];
    const uint64_t n = a.cand_uniform ? a.cand_uniform : a.cand_off[b + 1] - base;
    const uint32_t* ids = a.cand_ids + base;
    uint32_t* out = a.order + base;
    auto range_of = [&](uint32_t id) {  // empty slots (id 0xFFFFFFFF) and anything past the end go to the last range
        const uint32_t r = shift < 32 ? id >> shift : 0;
        return r < ranges ? r : ranges - 1;
    };
    for (uint32_t i = tid; i < ranges; i += T) bin[i] = 0;
    __syncthreads();
    constexpr int U = 8;
    const bool cached = n <= (uint64_t)U * T;
    uint32_t held[U];
    for (uint64_t i0 = 0; i0 < n; i0 += (uint64_t)U * T) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t i = i0 + tid + (uint64_t)u * T;
            held[u] = i < n ? ids[i] : 0;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (i0 + tid + (uint64_t)u * T < n) atomicAdd(&bin[range_of(held[u])], 1u);
    }
    __syncthreads();
    // exclusive prefix sum of the bins: thread t owns bins [t*per, (t+1)*per)
    const uint32_t per = (ranges + T - 1) / T;
    uint32_t mine = 0;
    for (uint32_t j = 0; j < per; ++j)
        if (tid * per + j < ranges) mine += bin[tid * per + j];
    uint32_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_up(incl, off, 64);
        if ((int)lane >= off) incl += o;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    uint32_t run = incl - mine;
    for (uint32_t w2 = 0; w2 < wave; ++w2) run += wave_sum[w2];
    for (uint32_t j = 0; j < per; ++j)
        if (tid * per + j < ranges) {
            const uint32_t c = bin[tid * per + j];
            bin[tid * per + j] = run;
            run += c;
        }
    __syncthreads();
    for (uint64_t i0 = 0; i0 < n; i0 += (uint64_t)U * T) {
        if (!cached) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint64_t i = i0 + tid + (uint64_t)u * T;
                held[u] = i < n ? ids[i] : 0;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t i = i0 + tid + (uint64_t)u * T;
            if (i < n) out[atomicAdd(&bin[range_of(held[u])], 1u)] = (uint32_t)i;
        }
    }
}

}  // namespace dessert
