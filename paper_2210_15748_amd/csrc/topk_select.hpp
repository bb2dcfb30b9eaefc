// Exact block-level top-k selection for gfx950 (device code shared by the stand-alone
// top-k kernels and by the scoring kernel's fused finish).
//
// Alg. 2's last line returns the argmax; here the k best are returned, ordered by score
// descending and, among equal scores, by ascending document id.  Every scored document
// becomes one dense integer key
//     key = (score + 1) << id_bits | (2^id_bits - 1 - id)
// so "larger key" is exactly "ranks earlier" and key 0 never occurs (it pads).  A workgroup
// fixes the k-th largest key by most-significant-digit radix selection (digits of up to 11
// bits, one histogram pass each, the digit chosen by a parallel suffix scan of the
// histogram), emits the keys above it plus as many copies of it as are still needed, and
// sorts those k keys in LDS with a bitonic network.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dessert {

constexpr uint32_t TOPK_KMAX = 16384;
constexpr uint32_t TOPK_DIGIT_BITS = 11;
constexpr uint32_t TOPK_HIST = 1u << TOPK_DIGIT_BITS;

struct KeyPlan {
    uint8_t id_bits;     // bits that hold 2^id_bits-1-id
    uint8_t n_digits;    // radix passes, most significant digit first
    uint8_t shift[6];
    uint8_t width[6];
};

inline uint32_t bits_for(uint64_t max_value) {
    uint32_t b = 1;
    while (b < 64 && (max_value >> b)) ++b;
    return b;
}

// max_score: largest possible score; max_id: largest document id that can occur.
// The leading digit is exactly the score field when that is at most one digit wide (its histogram then has
// few occupied bins and block_select merges the adds per wave); the id bits are spread evenly over the rest.
inline KeyPlan make_key_plan(uint32_t max_score, uint64_t max_id) {
    KeyPlan p{};
    p.id_bits = (uint8_t)bits_for(max_id);
    const uint32_t score_bits = bits_for((uint64_t)max_score + 1);
    uint32_t hi = p.id_bits + score_bits;
    uint32_t i = 0;
    if (score_bits <= TOPK_DIGIT_BITS) {
        p.width[0] = (uint8_t)score_bits;
        p.shift[0] = p.id_bits;
        hi = p.id_bits;
        i = 1;
    }
    const uint32_t n = i + (hi + TOPK_DIGIT_BITS - 1) / TOPK_DIGIT_BITS;
    for (; i < n; ++i) {
        uint32_t w = (hi + (n - i) - 1) / (n - i);  // spread the bits evenly over the remaining digits
        p.width[i] = (uint8_t)w;
        p.shift[i] = (uint8_t)(hi - w);
        hi -= w;
    }
    p.n_digits = (uint8_t)n;
    return p;
}

// stored key lists use 32-bit keys when the score and id fields fit
inline bool keys_fit_32(uint32_t max_score, uint64_t max_id) {
    return bits_for(max_id) + bits_for((uint64_t)max_score + 1) <= 32;
}

__device__ inline uint64_t make_key(int32_t score, uint32_t id, uint32_t id_bits) {
    if (score < 0) return 0;  // an empty candidate slot (scored -1) is padding
    const uint64_t idmask = (1ull << id_bits) - 1;
    return ((uint64_t)(uint32_t)(score + 1) << id_bits) | (idmask - (uint64_t)id);
}

__device__ inline void write_result(uint64_t key, uint32_t id_bits, uint32_t* id, int32_t* score) {
    if (key == 0) {
        *id = 0xFFFFFFFFu;
        *score = -1;
    } else {
        const uint64_t idmask = (1ull << id_bits) - 1;
        *id = (uint32_t)(idmask - (key & idmask));
        *score = (int32_t)(key >> id_bits) - 1;
    }
}

struct SelectShared {
    uint32_t hist[TOPK_HIST];
    uint32_t wave_sum[16];
    uint64_t prefix;
    uint32_t need;
    uint32_t count;
    uint32_t eq_taken;
};

// Select the k largest of keys(0..n-1) into sorted[0..kpad) (descending, zero padded).
// T = workgroup size (multiple of 64, at most 1024); every thread of the workgroup calls this.
// U = key loads a thread keeps in flight while it scans the list (a pass over n keys is n / (T*U) round trips).
// sorted: kpad = next power of two >= max(k, 2) entries of LDS.
template <int T, typename Keys, int U = 4>
__device__ void block_select(const Keys& keys, uint64_t n, uint32_t k, uint32_t kpad, uint64_t* sorted,
                             SelectShared& sh, const KeyPlan& plan) {
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63, wave = tid >> 6;
    constexpr int WAVES = T / 64;
    for (uint32_t i = tid; i < kpad; i += T) sorted[i] = 0;
    if (tid == 0) {
        sh.count = 0;
        sh.prefix = 0;
        sh.need = k;
        sh.eq_taken = 0;
    }
    __syncthreads();
    if (n <= k) {
        for (uint64_t i = tid; i < n; i += T) sorted[i] = keys(i);
    } else {
        for (uint32_t d = 0; d < plan.n_digits; ++d) {
            const uint32_t shift = plan.shift[d], width = plan.width[d];
            const uint32_t nbins = 1u << width, dmask = nbins - 1;
            for (uint32_t i = tid; i < nbins; i += T) sh.hist[i] = 0;
            __syncthreads();
            const uint64_t prefix = sh.prefix;
            const uint32_t need = sh.need;
            uint32_t run_bin = 0xFFFFFFFFu, run_len = 0;
            for (uint64_t i = tid; i < n; i += U * T) {  // U loads in flight per thread
                uint64_t key[U];
#pragma unroll
                for (int u = 0; u < U; ++u) key[u] = i + u * T < n ? keys(i + u * T) : 0;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const bool in = i + u * T < n && (key[u] >> (shift + width)) == prefix;
                    const uint32_t bin = (uint32_t)(key[u] >> shift) & dmask;
                    if (d == 0) {
                        // the leading digit holds the score's top bits and few values occur, mostly in runs: a thread
                        // counts a run of equal bins in a register and adds it once
                        if (in) {
                            if (bin == run_bin) {
                                ++run_len;
                            } else {
                                if (run_len) atomicAdd(&sh.hist[run_bin], run_len);
                                run_bin = bin;
                                run_len = 1;
                            }
                        }
                    } else if (in) {
                        atomicAdd(&sh.hist[bin], 1u);
                    }
                }
            }
            if (run_len) atomicAdd(&sh.hist[run_bin], run_len);
            __syncthreads();
            // digit D with  count(digits > D) < need <= count(digits >= D):
            // thread t owns bins [t*per, (t+1)*per); suffix sums over threads, then a short scan
            const uint32_t per = (nbins + T - 1) / T;
            const uint32_t b0 = tid * per;
            uint32_t mine = 0;
            for (uint32_t j = 0; j < per; ++j)
                if (b0 + j < nbins) mine += sh.hist[b0 + j];
            uint32_t incl = mine;  // inclusive suffix sum within the wave (lanes above contribute)
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                uint32_t o = __shfl_down(incl, off, 64);
                if ((int)lane + off < 64) incl += o;
            }
            if (lane == 0) sh.wave_sum[wave] = incl;
            __syncthreads();
            uint32_t above = incl - mine;  // bins owned by higher threads
            for (int w2 = (int)wave + 1; w2 < WAVES; ++w2) above += sh.wave_sum[w2];
            if (above < need && need <= above + mine) {  // exactly one thread
                for (int j = (int)per - 1; j >= 0; --j) {
                    if (b0 + j >= nbins) continue;
                    uint32_t c = sh.hist[b0 + j];
                    if (above + c >= need) {
                        sh.need = need - above;
                        sh.prefix = (prefix << width) | (uint64_t)(b0 + j);
                        break;
                    }
                    above += c;
                }
            }
            __syncthreads();
        }
        const uint64_t kth = sh.prefix;   // the k-th largest key
        const uint32_t need_eq = sh.need;  // copies of it that belong to the result
        for (uint64_t i = tid; i < n; i += U * T) {
            uint64_t key[U];
#pragma unroll
            for (int u = 0; u < U; ++u) key[u] = i + u * T < n ? keys(i + u * T) : 0;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (i + u * T >= n) continue;
                if (key[u] > kth) {
                    sorted[atomicAdd(&sh.count, 1u)] = key[u];
                } else if (key[u] == kth) {
                    if (atomicAdd(&sh.eq_taken, 1u) < need_eq) sorted[atomicAdd(&sh.count, 1u)] = key[u];
                }
            }
        }
    }
    __syncthreads();
    // bitonic sort, descending.  Two steps (strides s and s/2) per trip through LDS: a thread takes the four keys
    // base, base+s/2, base+s, base+3s/2, which both steps pair among themselves, so the array is read and written
    // once per two steps.  Wave w owns the groups of the run [w*seg, (w+1)*seg) of the array (seg = kpad / WAVES);
    // a trip whose groups stay inside such a run touches only keys the same wave wrote, and a wave's LDS operations
    // execute in order, so two such trips in a row need no workgroup barrier between them.
    auto order = [](uint64_t& x, uint64_t& y, bool desc) {
        if ((x < y) == desc) {
            const uint64_t t = x;
            x = y;
            y = t;
        }
    };
    const bool by_wave = kpad >= 256u * WAVES;   // every lane has at least one group of four in its wave's run
    const uint32_t seg = by_wave ? kpad / WAVES : kpad;
    bool prev_local = false;
    for (uint32_t size = 2; size <= kpad; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0;) {
            const bool local = by_wave && 2 * stride <= seg;
            if (!(local && prev_local)) {
                __syncthreads();
            } else {
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
            prev_local = local;
            if (stride >= 2) {  // strides `stride` and `stride / 2` together
                const uint32_t h = stride >> 1;
                const uint32_t groups = kpad / 4;
                const uint32_t g_lo = by_wave ? wave * (seg / 4) : 0, g_n = by_wave ? seg / 4 : groups;
                for (uint32_t m = by_wave ? lane : tid; m < g_n; m += by_wave ? 64 : T) {
                    const uint32_t g = g_lo + m;
                    const uint32_t base = (g / h) * (2 * stride) + (g % h);
                    const bool desc = ((base & size) == 0);
                    uint64_t k0 = sorted[base], k1 = sorted[base + h], k2 = sorted[base + stride], k3 = sorted[base + stride + h];
                    order(k0, k2, desc);
                    order(k1, k3, desc);
                    order(k0, k1, desc);
                    order(k2, k3, desc);
                    sorted[base] = k0;
                    sorted[base + h] = k1;
                    sorted[base + stride] = k2;
                    sorted[base + stride + h] = k3;
                }
                stride >>= 2;
            } else {  // stride 1 alone
                const uint32_t p_lo = by_wave ? wave * (seg / 2) : 0, p_n = by_wave ? seg / 2 : kpad / 2;
                for (uint32_t m = by_wave ? lane : tid; m < p_n; m += by_wave ? 64 : T) {
                    const uint32_t lo = 2 * (p_lo + m);
                    const bool desc = ((lo & size) == 0);
                    uint64_t x = sorted[lo], y = sorted[lo + 1];
                    order(x, y, desc);
                    sorted[lo] = x;
                    sorted[lo + 1] = y;
                }
                stride = 0;
            }
        }
    }
    __syncthreads();
}

struct ScoreKeys {  // keys computed from a score array (+ optional candidate ids)
    const int32_t* scores;
    const uint32_t* ids;  // nullptr: id = first_id + i
    uint64_t first_id;
    uint32_t id_bits;
    __device__ uint64_t operator()(uint64_t i) const {
        uint32_t id = ids ? ids[i] : (uint32_t)(first_id + i);
        return make_key(scores[i], id, id_bits);
    }
};

struct StoredKeys {
    const uint64_t* keys;
    __device__ uint64_t operator()(uint64_t i) const { return keys[i]; }
};

struct StoredKeys32 {  // keys of at most 32 bits (score and id fields together), stored as u32
    const uint32_t* keys;
    __device__ uint64_t operator()(uint64_t i) const { return keys[i]; }
};

}  // namespace dessert
