// Exact block-level top-k selection for gfx950 (device code shared by the stand-alone
// top-k kernels and the candidate filter's probe and list selections).
//
// Alg. 2's last line returns the argmax; here the k best are returned, ordered by score
// descending and, among equal scores, by ascending document id.  Every scored document
// becomes one dense integer key
//     key = (score + 1) << id_bits | (2^id_bits - 1 - id)
// so "larger key" is exactly "ranks earlier" and key 0 never occurs (it pads).  A workgroup
// fixes the k-th largest key by most-significant-digit radix selection (digits of up to 11
// bits, one histogram pass each, the digit chosen by a parallel suffix scan of the
// histogram), emits the keys above it plus as many copies of it as are still needed, and
// sorts those k keys with a bitonic network (in registers when a thread holds 1 to 16 of them, else in LDS).
// Shortcut after the first digit: when at most 1024 keys lie at or above its threshold bin they are gathered
// and sorted in LDS, and the remaining passes are skipped.
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

// Bins of the leading digit when that digit is exactly the score field (bin = score + 1), else 0.  A producer of
// stored key lists that knows the scores can then hand block_select the leading digit's histogram (first_hist)
// and save it the first pass over the list.
inline uint32_t leading_score_bins(uint32_t max_score, uint64_t max_id) {
    const KeyPlan p = make_key_plan(max_score, max_id);
    return (p.n_digits > 1 && p.shift[0] == p.id_bits && p.width[0] == bits_for((uint64_t)max_score + 1)) ? 1u << p.width[0] : 0;
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

// Optional description of a stored key list whose producer wrote its keys slab by slab: slab s holds the keys of an
// id range below that of slab s+1 (so, for equal scores, all its keys rank before those of later slabs) as one
// run of the list.  With the leading digit = the score field, block_select then finds the k-th key inside one slab's
// run instead of scanning the whole list once per id digit.
struct SlabDirectory {
    const uint32_t* rows;      // [slabs][bins]: per slab the histogram of its keys' leading digit (bin = score + 1)
    const uint32_t* segments;  // [slabs][2]: start and length of the slab's run within the list
    uint32_t slabs, bins;      // bins = leading_score_bins(); at most T slabs
};

struct SelectShared {
    uint32_t hist[TOPK_HIST];
    uint32_t wave_sum[16];
    uint64_t prefix;
    uint32_t need;
    uint32_t count;
    uint32_t eq_taken;
    uint32_t sub_slab;
};

constexpr int ilog2_floor(int x) { return x <= 1 ? 0 : 1 + ilog2_floor(x / 2); }

// Bitonic sort (descending) of sorted[0 .. R*T) with the keys in registers: thread `tid` holds elements
// R*tid .. R*tid+R-1, so a compare-exchange at stride < R pairs two of a thread's own registers, at stride < 64*R
// two lanes of a wave (one shuffle per key, no barrier), and only strides >= 64*R cross waves.  Those go through
// LDS, all strides >= 64*R of a merge in one trip: the T/64 elements that differ only in the wave bits form a
// column which one thread loads, orders over all those strides, and stores.  A sort of 4096 keys by 1024 threads
// makes 4 trips through LDS with a barrier pair each (sizes 512 .. 4096) instead of one per stride.
// KS = uint32_t when every key is below 2^32: half the shuffles, and an exchange is one or two v_med3_u32.
template <int T, int R, typename KS>
__device__ void bitonic_sort_regs(uint64_t* sorted) {
    constexpr int WAVES = T / 64, LOG_WAVES = ilog2_floor(WAVES);
    constexpr uint32_t KPAD = (uint32_t)R * T, COLS = 64u * R;
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    // 32-bit keys: the median of (x, y, 0) is their minimum and the median of (x, y, 2^32-1) their maximum, so one
    // v_med3_u32 with a per-lane third operand picks the side a lane keeps
    auto med3 = [](uint32_t x, uint32_t y, uint32_t z) {
        uint32_t r;
        asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(y), "v"(z));
        return r;
    };
    auto order = [&](KS& x, KS& y, bool desc) {  // desc: larger first
        if constexpr (sizeof(KS) == 4) {
            const uint32_t top = desc ? 0xFFFFFFFFu : 0u;
            const uint32_t nx = med3(x, y, top), ny = med3(x, y, ~top);
            x = nx;
            y = ny;
        } else {
            const KS lo = x < y ? x : y, hi = x < y ? y : x;
            x = desc ? hi : lo;
            y = desc ? lo : hi;
        }
    };
    KS key[R];
#pragma unroll
    for (int r = 0; r < R; ++r) key[r] = (KS)sorted[R * tid + r];
    for (uint32_t size = 2; size <= KPAD; size <<= 1) {
        uint32_t stride = size >> 1;
        if (stride >= COLS) {  // strides that cross waves
            // (a thread's own slots: nobody else reads them between the trips)
#pragma unroll
            for (int r = 0; r < R; ++r) sorted[R * tid + r] = key[r];
            __syncthreads();
            for (uint32_t c = tid; c < COLS; c += T) {
                KS col[WAVES];
#pragma unroll
                for (int w = 0; w < WAVES; ++w) col[w] = (KS)sorted[c + COLS * w];
#pragma unroll
                for (int sb = LOG_WAVES - 1; sb >= 0; --sb) {
                    if ((COLS << sb) > stride) continue;
#pragma unroll
                    for (int w = 0; w < WAVES; ++w)
                        if ((w & (1 << sb)) == 0) order(col[w], col[w | (1 << sb)], ((COLS * w) & size) == 0);
                }
#pragma unroll
                for (int w = 0; w < WAVES; ++w) sorted[c + COLS * w] = col[w];
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < R; ++r) key[r] = (KS)sorted[R * tid + r];
            stride = COLS >> 1;
        }
        for (; stride >= (uint32_t)R; stride >>= 1) {  // strides between lanes of a wave
            const uint32_t lx = stride / R;
            // this thread keeps the larger key of a pair when it holds the pair's lower element in a descending run
            const bool keep_max = ((lane & lx) == 0) == (((R * tid) & size) == 0);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if constexpr (sizeof(KS) == 8) {
                    const KS o = __shfl_xor((unsigned long long)key[r], (int)lx, 64);
                    const KS lo = key[r] < o ? key[r] : o, hi = key[r] < o ? o : key[r];
                    key[r] = keep_max ? hi : lo;
                } else {
                    const uint32_t o = __shfl_xor((unsigned int)key[r], (int)lx, 64);
                    key[r] = med3(key[r], o, keep_max ? 0xFFFFFFFFu : 0u);
                }
            }
        }
#pragma unroll
        for (int st = R / 2; st >= 1; st >>= 1) {  // strides inside a thread
            if ((uint32_t)st > stride) continue;
#pragma unroll
            for (int r = 0; r < R; ++r)
                if ((r & st) == 0) order(key[r], key[r | st], ((R * tid + r) & size) == 0);
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) sorted[R * tid + r] = key[r];
    __syncthreads();
}

// Bitonic sort (descending) of a[0 .. npad) in LDS, npad a power of two >= 2; the array must be complete (a workgroup
// barrier behind its last write) on entry and is complete on return.  Two steps (strides s and s/2) per trip through
// LDS: a thread takes the four keys base, base+s/2, base+s, base+3s/2, which both steps pair among themselves, so the
// array is read and written once per two steps.  Wave w owns the groups of the run [w*seg, (w+1)*seg) of the array
// (seg = npad / WAVES); a trip whose groups stay inside such a run touches only keys the same wave wrote, and a wave's
// LDS operations execute in order, so two such trips in a row need no workgroup barrier between them.
template <int T>
__device__ void bitonic_sort_lds(uint64_t* a, uint32_t npad) {
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int WAVES = T / 64;
    auto order = [](uint64_t& x, uint64_t& y, bool desc) {
        if ((x < y) == desc) {
            const uint64_t t = x;
            x = y;
            y = t;
        }
    };
    const bool by_wave = npad >= 256u * WAVES;   // every lane has at least one group of four in its wave's run
    const uint32_t seg = by_wave ? npad / WAVES : npad;
    bool prev_local = false;
    for (uint32_t size = 2; size <= npad; size <<= 1) {
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
                const uint32_t groups = npad / 4;
                const uint32_t g_lo = by_wave ? wave * (seg / 4) : 0, g_n = by_wave ? seg / 4 : groups;
                for (uint32_t m = by_wave ? lane : tid; m < g_n; m += by_wave ? 64 : T) {
                    const uint32_t g = g_lo + m;
                    const uint32_t base = (g / h) * (2 * stride) + (g % h);
                    const bool desc = ((base & size) == 0);
                    uint64_t k0 = a[base], k1 = a[base + h], k2 = a[base + stride], k3 = a[base + stride + h];
                    order(k0, k2, desc);
                    order(k1, k3, desc);
                    order(k0, k1, desc);
                    order(k2, k3, desc);
                    a[base] = k0;
                    a[base + h] = k1;
                    a[base + stride] = k2;
                    a[base + stride + h] = k3;
                }
                stride >>= 2;
            } else {  // stride 1 alone
                const uint32_t p_lo = by_wave ? wave * (seg / 2) : 0, p_n = by_wave ? seg / 2 : npad / 2;
                for (uint32_t m = by_wave ? lane : tid; m < p_n; m += by_wave ? 64 : T) {
                    const uint32_t lo = 2 * (p_lo + m);
                    const bool desc = ((lo & size) == 0);
                    uint64_t x = a[lo], y = a[lo + 1];
                    order(x, y, desc);
                    a[lo] = x;
                    a[lo + 1] = y;
                }
                stride = 0;
            }
        }
    }
    __syncthreads();
}

// Select the k largest of keys(0..n-1) into sorted[0..kpad) (descending, zero padded).
// T = workgroup size (multiple of 64, at most 1024); every thread of the workgroup calls this.
// U = key loads a thread keeps in flight while it scans the list; a load brings Keys::VEC consecutive keys (stored
// lists: 16 bytes), so a pass over n keys is n / (T * U * VEC) round trips.  CACHE: see below.
// sorted: kpad = next power of two >= max(k, 2) entries of LDS.
// first_hist: optional, leading_score_bins() counters (see there).  dir: optional, see SlabDirectory (key sources
// with SEGMENTS only); it replaces first_hist.
// ORDERED = false: the k best keys are left in `sorted` in no particular order (callers that only need the set).
// EMIT = false: when the selection ends in a pass over the whole list that copies the keys at or above the k-th one,
// that pass is left to the caller: the function returns false with the k-th key in sh.prefix and the number of its
// copies that belong to the result in sh.need (`sorted` then holds nothing).  It returns true when `sorted` holds the
// result (always with EMIT = true); the value is the same for every thread.
template <int T, typename Keys, int U = 4, bool CACHE = false, bool ORDERED = true, bool EMIT = true>
__device__ bool block_select(const Keys& keys, uint64_t n, uint32_t k, uint32_t kpad, uint64_t* sorted,
                             SelectShared& sh, const KeyPlan& plan, const uint32_t* first_hist = nullptr,
                             const SlabDirectory* dir = nullptr) {
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63, wave = tid >> 6;
    constexpr int WAVES = T / 64;
    constexpr int V = Keys::VEC;
    using K = typename Keys::key_t;  // arithmetic on the keys of a pass is done in the stored width
    for (uint32_t i = tid; i < kpad; i += T) sorted[i] = 0;
    if (tid == 0) {
        sh.count = 0;
        sh.prefix = 0;
        sh.need = k;
        sh.eq_taken = 0;
    }
    __syncthreads();
    // CACHE: a list of at most T*U*V keys is loaded once and kept in registers for all passes (U*V more live
    // registers: for kernels whose lists are usually that short).
    const bool cached = CACHE && n <= (uint64_t)T * U * V;
    K cache[CACHE ? U : 1][CACHE ? V : 1];
    if constexpr (CACHE) {
        if (cached) {
#pragma unroll
            for (int u = 0; u < U; ++u) keys.load((uint64_t)tid * V + (uint64_t)u * T * V, n, cache[u]);
        }
    }
    // f(key) for every key of the list.  Only a thread's last, partial trip checks indices key by key.
    auto scan = [&](auto&& f) {
        if constexpr (CACHE) {
            if (cached) {
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int v = 0; v < V; ++v)
                        if ((uint64_t)tid * V + (uint64_t)u * T * V + v < n) f(cache[u][v]);
                return;
            }
        }
        for (uint64_t i = (uint64_t)tid * V; i < n; i += (uint64_t)U * T * V) {  // U loads in flight per thread
            K key[U][V];
#pragma unroll
            for (int u = 0; u < U; ++u) keys.load(i + (uint64_t)u * T * V, n, key[u]);
            if (i + (uint64_t)(U - 1) * T * V + V <= n) {
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int v = 0; v < V; ++v) f(key[u][v]);
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int v = 0; v < V; ++v)
                        if (i + (uint64_t)u * T * V + v < n) f(key[u][v]);
            }
        }
    };
    // the digits after the first may be decided on one slab's run of the list (see SlabDirectory)
    uint64_t sub_start = 0, n_sub = 0;
    bool use_sub = false;
    auto scan_sub = [&](auto&& f) {
        if constexpr (Keys::SEGMENTS) {
            for (uint64_t i = tid; i < n_sub; i += 4 * T) {
                K key[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) key[u] = i + (uint64_t)u * T < n_sub ? (K)keys(sub_start + i + (uint64_t)u * T) : K(0);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (i + (uint64_t)u * T < n_sub) f(key[u]);
            }
        }
    };
    // dst[sh.count++] = key for every key of the list with take(key).  Per trip a thread marks which of its keys go
    // out, the wave adds the counts up (prefix sum over lanes) and takes its slots with one atomic: a few round trips
    // per pass instead of one per key.  Every lane of the workgroup makes every trip.
    static_assert(U * V <= 32, "one flag bit per key of a trip");
    auto append_pass = [&](uint64_t* dst, auto&& take) {
        const uint64_t per_trip = (uint64_t)U * T * V;
        for (uint64_t t0 = 0; t0 < n; t0 += per_trip) {
            const uint64_t i = t0 + (uint64_t)tid * V;
            K key[U][V];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if constexpr (CACHE) {
                    if (cached) {
#pragma unroll
                        for (int v = 0; v < V; ++v) key[u][v] = cache[u][v];
                        continue;
                    }
                }
                keys.load(i + (uint64_t)u * T * V, n, key[u]);
            }
            uint32_t flags = 0;
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const bool have = i + (uint64_t)u * T * V + v < n;
                    flags |= ((have && take(key[u][v])) ? 1u : 0u) << (u * V + v);
                }
            const uint32_t cnt = (uint32_t)__builtin_popcount(flags);
            uint32_t incl = cnt;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t o = __shfl_up(incl, off, 64);
                if ((int)lane >= off) incl += o;
            }
            uint32_t base = 0;
            if (lane == 63 && incl) base = atomicAdd(&sh.count, incl);
            base = __shfl(base, 63, 64);
            uint32_t pos = base + incl - cnt;
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int v = 0; v < V; ++v)
                    if ((flags >> (u * V + v)) & 1u) dst[pos++] = key[u][v];
        }
    };
    if (n <= k) {
        for (uint64_t i = tid; i < n; i += T) sorted[i] = keys(i);
    } else {
        for (uint32_t d = 0; d < plan.n_digits; ++d) {
            const uint32_t shift = plan.shift[d], width = plan.width[d];
            const uint32_t nbins = 1u << width, dmask = nbins - 1;
            // first_hist: the leading digit's histogram over all n keys, counted by whoever wrote the list
            const bool by_dir = Keys::SEGMENTS && dir != nullptr && dir->bins == nbins && dir->slabs <= (uint32_t)T;
            const bool given = d == 0 && (first_hist != nullptr || by_dir);
            if (d == 0 && by_dir) {  // the list's histogram is the sum of its slabs' rows (all loads in flight together)
                for (uint32_t i = tid; i < nbins; i += T) sh.hist[i] = 0;
                __syncthreads();
                const uint32_t cells = dir->slabs * nbins;
                for (uint32_t i = tid; i < cells; i += T) {
                    const uint32_t c = dir->rows[i];
                    if (c) atomicAdd(&sh.hist[i & dmask], c);
                }
            } else {
                for (uint32_t i = tid; i < nbins; i += T) sh.hist[i] = given ? first_hist[i] : 0;
            }
            __syncthreads();
            const uint64_t prefix = sh.prefix;
            const uint32_t need = sh.need;
            // a key takes part in this pass when its bits above the digit equal the digits fixed so far
            const uint32_t above_bits = shift + width;
            const K hi_mask = above_bits >= 8 * sizeof(K) ? K(0) : (K)(~K(0) << above_bits);
            const K hi_value = above_bits >= 8 * sizeof(K) ? K(0) : (K)((K)prefix << above_bits);
            if (given) {
            } else if (d == 0) {
                // the leading digit holds the score's top bits and few values occur, mostly in runs: a thread
                // counts a run of equal bins in a register and adds it once
                uint32_t run_bin = 0xFFFFFFFFu, run_len = 0;
                scan([&](K key) {
                    if ((key & hi_mask) != hi_value) return;
                    const uint32_t bin = (uint32_t)(key >> shift) & dmask;
                    if (bin == run_bin) {
                        ++run_len;
                    } else {
                        if (run_len) atomicAdd(&sh.hist[run_bin], run_len);
                        run_bin = bin;
                        run_len = 1;
                    }
                });
                if (run_len) atomicAdd(&sh.hist[run_bin], run_len);
            } else if (use_sub) {
                scan_sub([&](K key) {
                    if ((key & hi_mask) == hi_value) atomicAdd(&sh.hist[(uint32_t)(key >> shift) & dmask], 1u);
                });
            } else {
                scan([&](K key) {
                    if ((key & hi_mask) == hi_value) atomicAdd(&sh.hist[(uint32_t)(key >> shift) & dmask], 1u);
                });
            }
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
            // Few keys left at or above the threshold bin of the leading digit (the usual case when that digit is
            // the score and k is small): gather them in LDS (the histogram's space), sort them there and take the
            // first k, instead of one more pass over the list per remaining digit plus the emit.
            if (d == 0 && plan.n_digits > 1) {
                constexpr uint32_t CAP = TOPK_HIST / 2;  // 64-bit keys that fit the histogram
                const uint32_t bin0 = (uint32_t)sh.prefix;
                const uint32_t at_or_above = (k - sh.need) + sh.hist[bin0];  // >= k
                __syncthreads();  // everyone has read the histogram
                if (at_or_above <= CAP) {
                    uint64_t* gathered = reinterpret_cast<uint64_t*>(sh.hist);
                    const K lowest = (K)((K)bin0 << shift);
                    append_pass(gathered, [&](K key) { return key >= lowest; });
                    uint32_t gpad = 2;
                    while (gpad < at_or_above) gpad <<= 1;
                    for (uint32_t i = at_or_above + tid; i < gpad; i += T) gathered[i] = 0;
                    __syncthreads();
                    // (sorted even when the order is not asked for: more keys than k were gathered)
                    bitonic_sort_lds<T>(gathered, gpad);
                    for (uint32_t i = tid; i < k; i += T) sorted[i] = gathered[i];
                    __syncthreads();
                    return true;
                }
                if (by_dir) {
                    // The keys of the threshold bin rank slab by slab: thread s takes slab s's count of them, an
                    // inclusive prefix sum over the slabs finds the slab that holds the need-th, and the remaining
                    // digits are decided among that slab's keys alone.
                    const uint32_t need0 = sh.need;
                    const uint32_t mine = tid < dir->slabs ? dir->rows[(size_t)tid * nbins + bin0] : 0;
                    uint32_t incl = mine;
#pragma unroll
                    for (int off = 1; off < 64; off <<= 1) {
                        const uint32_t o = __shfl_up(incl, off, 64);
                        if ((int)lane >= off) incl += o;
                    }
                    if (lane == 63) sh.wave_sum[wave] = incl;
                    __syncthreads();
                    uint32_t before = 0;
                    for (uint32_t w2 = 0; w2 < wave; ++w2) before += sh.wave_sum[w2];
                    incl += before;
                    __syncthreads();  // wave_sum is reused by the digit loop
                    if (incl - mine < need0 && need0 <= incl) {  // exactly one thread
                        sh.sub_slab = tid;
                        sh.need = need0 - (incl - mine);
                    }
                    __syncthreads();
                    sub_start = dir->segments[2 * sh.sub_slab];
                    n_sub = dir->segments[2 * sh.sub_slab + 1];
                    use_sub = true;
                }
            }
        }
        if constexpr (!EMIT) return false;
        const K kth = (K)sh.prefix;        // the k-th largest key
        const uint32_t need_eq = sh.need;  // copies of it that belong to the result
        append_pass(sorted, [&](K key) {
            bool take = key > kth;
            if (key == kth) take = atomicAdd(&sh.eq_taken, 1u) < need_eq;
            return take;
        });
    }
    __syncthreads();
    if constexpr (!ORDERED) return true;
    // 1 to 16 keys per thread: sort in registers
    if (kpad >= (uint32_t)T && kpad <= 16u * T) {
        switch (kpad / T) {
            case 1: bitonic_sort_regs<T, 1, K>(sorted); break;
            case 2: bitonic_sort_regs<T, 2, K>(sorted); break;
            case 4: bitonic_sort_regs<T, 4, K>(sorted); break;
            case 8: bitonic_sort_regs<T, 8, K>(sorted); break;
            default: bitonic_sort_regs<T, 16, K>(sorted); break;
        }
        return true;
    }
    bitonic_sort_lds<T>(sorted, kpad);
    return true;
}

// Key sources.  operator()(i) = key i; load(i, n, out) = the VEC keys i .. i+VEC-1 (i a multiple of VEC; entries at or
// past n are unspecified and the caller ignores them; nothing is read when i >= n).
template <typename KT>  // uint64_t, or uint32_t when keys_fit_32
struct ScoreKeysT {  // keys computed from a score array (+ optional candidate ids)
    static constexpr int VEC = 1;
    static constexpr bool SEGMENTS = false;
    using key_t = KT;
    const int32_t* scores;
    const uint32_t* ids;  // nullptr: id = first_id + i
    uint64_t first_id;
    uint32_t id_bits;
    __device__ uint64_t operator()(uint64_t i) const {
        uint32_t id = ids ? ids[i] : (uint32_t)(first_id + i);
        return make_key(scores[i], id, id_bits);
    }
    __device__ void load(uint64_t i, uint64_t n, KT (&out)[1]) const { out[0] = i < n ? (KT)(*this)(i) : KT(0); }
};
using ScoreKeys = ScoreKeysT<uint64_t>;

struct StoredKeys {  // 64-bit keys at any 8-byte aligned address
    static constexpr int VEC = 1;
    static constexpr bool SEGMENTS = false;
    using key_t = uint64_t;
    const uint64_t* keys;
    __device__ uint64_t operator()(uint64_t i) const { return keys[i]; }
    __device__ void load(uint64_t i, uint64_t n, uint64_t (&out)[1]) const { out[0] = i < n ? keys[i] : 0; }
};

// The two list forms below need lists that start 16-byte aligned and are allocated up to a multiple of 16 bytes, so
// that a vector load which begins below n stays inside the list's allocation.
struct StoredKeysPairs {
    static constexpr int VEC = 2;
    static constexpr bool SEGMENTS = true;
    using key_t = uint64_t;
    const uint64_t* keys;
    __device__ uint64_t operator()(uint64_t i) const { return keys[i]; }
    __device__ void load(uint64_t i, uint64_t n, uint64_t (&out)[2]) const {
        out[0] = out[1] = 0;
        if (i < n) {
            const ulonglong2 v = *(const ulonglong2*)(keys + i);
            out[0] = v.x;
            out[1] = v.y;
        }
    }
};

struct StoredKeys32 {  // keys of at most 32 bits (score and id fields together), stored as u32
    static constexpr int VEC = 4;
    static constexpr bool SEGMENTS = true;
    using key_t = uint32_t;
    const uint32_t* keys;
    __device__ uint64_t operator()(uint64_t i) const { return keys[i]; }
    __device__ void load(uint64_t i, uint64_t n, uint32_t (&out)[4]) const {
        out[0] = out[1] = out[2] = out[3] = 0;
        if (i < n) {
            const uint4 v = *(const uint4*)(keys + i);
            out[0] = v.x;
            out[1] = v.y;
            out[2] = v.z;
            out[3] = v.w;
        }
    }
};

}  // namespace dessert
