// Exact top-k over integer scores for gfx950 (Alg. 2's last line returns the
// argmax; this returns the k best, ordered by score descending and, among
// equal scores, by ascending document id).
//
// Every scored document becomes one 64-bit key
//     key = (score + 1) << 32 | (0xFFFFFFFF - id)
// so "larger key" is exactly "ranks earlier", and key 0 never occurs (it pads).
// A workgroup selects the k largest keys of its input by most-significant-
// digit radix selection (8-bit digits over the 48 significant bits: six
// histogram passes that fix the k-th largest key digit by digit), then emits
// the keys above it plus as many copies of it as are still needed, and sorts
// those k keys in LDS with a bitonic network.  Long inputs are cut into slices:
// one workgroup per (query set, slice) writes its k best keys, and a second
// launch selects among the slices' keys.
#include "kernels.hpp"

namespace dessert {

constexpr uint32_t TOPK_THREADS = 512;
constexpr uint32_t TOPK_KMAX = 4096;
constexpr uint64_t TOPK_SLICE = 1u << 16;

uint32_t topk_slices(uint64_t max_scored) {
    if (max_scored <= 2 * TOPK_SLICE) return 1;
    return (uint32_t)((max_scored + TOPK_SLICE - 1) / TOPK_SLICE);
}

struct ScoreKeys {  // keys computed from a score array (+ optional candidate ids)
    const int32_t* scores;
    const uint32_t* ids;  // nullptr: id = first_id + i
    uint64_t first_id;
    __device__ uint64_t operator()(uint64_t i) const {
        uint32_t id = ids ? ids[i] : (uint32_t)(first_id + i);
        return ((uint64_t)(uint32_t)(scores[i] + 1) << 32) | (uint64_t)(0xFFFFFFFFu - id);
    }
};

struct StoredKeys {
    const uint64_t* keys;
    __device__ uint64_t operator()(uint64_t i) const { return keys[i]; }
};

// Select the k largest of keys(0..n-1) into sorted[0..k) (descending, zero padded).
// sorted: LDS array of kpad = next power of two >= k entries.  Whole workgroup calls this.
template <typename Keys>
__device__ void block_select(const Keys& keys, uint64_t n, uint32_t k, uint32_t kpad, uint64_t* sorted,
                             uint32_t* hist /*[256]*/, uint64_t* sh_prefix, uint32_t* sh_need, uint32_t* sh_count) {
    const uint32_t tid = threadIdx.x;
    for (uint32_t i = tid; i < kpad; i += TOPK_THREADS) sorted[i] = 0;
    if (tid == 0) {
        *sh_count = 0;
        *sh_prefix = 0;
        *sh_need = k;
    }
    __syncthreads();
    if (n <= k) {
        for (uint64_t i = tid; i < n; i += TOPK_THREADS) sorted[i] = keys(i);
    } else {
        // fix the k-th largest key digit by digit; keys use bits 0..47
        for (int shift = 40; shift >= 0; shift -= 8) {
            for (uint32_t i = tid; i < 256; i += TOPK_THREADS) hist[i] = 0;
            __syncthreads();
            const uint64_t prefix = *sh_prefix;
            for (uint64_t i = tid; i < n; i += TOPK_THREADS) {
                uint64_t key = keys(i);
                if ((key >> (shift + 8)) == prefix) atomicAdd(&hist[(key >> shift) & 0xFF], 1u);
            }
            __syncthreads();
            if (tid == 0) {
                uint32_t need = *sh_need, above = 0;
                int dgt = 255;
                for (; dgt > 0; --dgt) {
                    if (above + hist[dgt] >= need) break;
                    above += hist[dgt];
                }
                *sh_need = need - above;  // still needed from inside the chosen digit
                *sh_prefix = (prefix << 8) | (uint64_t)dgt;
            }
            __syncthreads();
        }
        const uint64_t kth = *sh_prefix;   // the k-th largest key
        const uint32_t need_eq = *sh_need;  // copies of it that belong to the result
        __syncthreads();
        if (tid == 0) *sh_need = 0;  // now counts emitted copies of kth
        __syncthreads();
        for (uint64_t i = tid; i < n; i += TOPK_THREADS) {
            uint64_t key = keys(i);
            if (key > kth) {
                sorted[atomicAdd(sh_count, 1u)] = key;
            } else if (key == kth) {
                if (atomicAdd(sh_need, 1u) < need_eq) sorted[atomicAdd(sh_count, 1u)] = key;
            }
        }
    }
    __syncthreads();
    // bitonic sort, descending
    for (uint32_t size = 2; size <= kpad; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            for (uint32_t i = tid; i < kpad / 2; i += TOPK_THREADS) {
                uint32_t lo = 2 * i - (i & (stride - 1));
                uint32_t hi = lo + stride;
                bool desc = ((lo & size) == 0);
                uint64_t x = sorted[lo], y = sorted[hi];
                if ((x < y) == desc) {
                    sorted[lo] = y;
                    sorted[hi] = x;
                }
            }
            __syncthreads();
        }
    }
}

__device__ inline void write_result(uint64_t key, uint32_t* id, int32_t* score) {
    if (key == 0) {
        *id = 0xFFFFFFFFu;
        *score = -1;
    } else {
        *id = 0xFFFFFFFFu - (uint32_t)key;
        *score = (int32_t)(key >> 32) - 1;
    }
}

struct TopkShared {
    uint32_t hist[256];
    uint64_t prefix;
    uint32_t need;
    uint32_t count;
};

// grid (slices, B).  slices == 1: final results; else per-slice keys to a.partial.
__global__ __launch_bounds__(TOPK_THREADS) void topk_scores_kernel(TopkArgs a, uint32_t slices, uint32_t kpad) {
    extern __shared__ uint64_t sorted[];
    __shared__ TopkShared sh;
    const uint32_t b = blockIdx.y, s = blockIdx.x;
    uint64_t base, count;
    if (a.cand_ids) {
        base = a.cand_off[b];
        count = a.cand_off[b + 1] - base;
    } else {
        base = (uint64_t)b * a.n_docs;
        count = a.n_docs;
    }
    const uint64_t per = (count + slices - 1) / slices;
    const uint64_t lo = (uint64_t)s * per < count ? (uint64_t)s * per : count;
    const uint64_t hi = lo + per < count ? lo + per : count;
    ScoreKeys keys{a.scores + base + lo, a.cand_ids ? a.cand_ids + base + lo : nullptr, lo};
    block_select(keys, hi - lo, a.k, kpad, sorted, sh.hist, &sh.prefix, &sh.need, &sh.count);
    if (slices == 1) {
        for (uint32_t i = threadIdx.x; i < a.k; i += TOPK_THREADS)
            write_result(sorted[i], a.out_ids + (size_t)b * a.k + i, a.out_scores + (size_t)b * a.k + i);
    } else {
        uint64_t* dst = a.partial + ((size_t)b * slices + s) * a.k;
        for (uint32_t i = threadIdx.x; i < a.k; i += TOPK_THREADS) dst[i] = sorted[i];
    }
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_merge_kernel(TopkArgs a, uint32_t slices, uint32_t kpad) {
    extern __shared__ uint64_t sorted[];
    __shared__ TopkShared sh;
    const uint32_t b = blockIdx.x;
    StoredKeys keys{a.partial + (size_t)b * slices * a.k};
    block_select(keys, (uint64_t)slices * a.k, a.k, kpad, sorted, sh.hist, &sh.prefix, &sh.need, &sh.count);
    for (uint32_t i = threadIdx.x; i < a.k; i += TOPK_THREADS)
        write_result(sorted[i], a.out_ids + (size_t)b * a.k + i, a.out_scores + (size_t)b * a.k + i);
}

hipError_t launch_topk(const TopkArgs& a, hipStream_t stream) {
    if (a.n_queries == 0 || a.k == 0) return hipSuccess;
    if (a.k > TOPK_KMAX || a.n_queries > 65535) return hipErrorInvalidValue;
    uint32_t kpad = 2;
    while (kpad < a.k) kpad <<= 1;
    const uint32_t slices = topk_slices(a.max_scored);
    const size_t lds = (size_t)kpad * 8;
    hipLaunchKernelGGL(topk_scores_kernel, dim3(slices, a.n_queries), dim3(TOPK_THREADS), lds, stream, a, slices, kpad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || slices == 1) return e;
    hipLaunchKernelGGL(topk_merge_kernel, dim3(a.n_queries), dim3(TOPK_THREADS), lds, stream, a, slices, kpad);
    return hipGetLastError();
}

}  // namespace dessert
