// Candidate filter for gfx950 (Sec. 5 "Filtering"): an inverted index from centroid ids to
// document ids, built from the closest centroid of every document vector, and the query-side
// probe-and-count that keeps the filter_k documents whose buckets are hit most often.
//
// "Closest" is the squared Euclidean distance with ties to the lower centroid id.  Since
// |x|^2 is common to all centroids, argmin_k |x - c_k|^2 = argmax_k (2 x.c_k - |c_k|^2): the
// dense part is an int8 GEMM (vectors x centroids) on v_mfma_i32_32x32x32_i8, exact in int32.
#include "kernels.hpp"
#include "topk_select.hpp"

namespace dessert {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int FILTER_TG = 8;           // centroid tiles per LDS group (the kernel may take half of it)
constexpr int32_t FILTER_BIAS = 1 << 24;  // 2 x.c - |c|^2 lies in (-2^24, 2^24) for int8 vectors up to d = 256

// accumulator register r of lane half g holds tile row 8*(r/4) + 4*g + r%4
__host__ __device__ inline uint32_t tile_row(uint32_t r, uint32_t g) { return 8 * (r / 4) + 4 * g + (r % 4); }

// ---------------------------------------------------------------------------
// Centroids in MFMA operand order, [tiles][KS][64 lanes][16 B] (tile = 32 centroids, rows past K
// are zero), and the per-row constants, for accumulator register r of lane half g:
//   H[tiles][2][16]  -ceil(|c|^2 / 2): the accumulators start from it, so that after the MFMAs
//                    acc = x.c - ceil(|c|^2 / 2) =: h  and  2 x.c - |c|^2 = 2 h + (|c|^2 & 1);
//                    rows past K start from -2^25, below every real value (> -2^24 / 2)
//   PAR[tiles][2]    bit r = |c|^2 & 1
// A lane's largest h bounds its largest value (<= 2 h + 1): most tiles are dismissed by a max
// over the raw accumulators, without building any per-row key.
constexpr int32_t FILTER_PAD_INIT = -(1 << 25);

__global__ void filter_prep_kernel(const int8_t* __restrict__ Cn, uint32_t K, uint32_t d, int8_t* __restrict__ Cp,
                                   int32_t* __restrict__ H, uint32_t tiles) {
    const uint32_t KS = d / 32;
    const uint32_t total = tiles * KS * 1024;
    uint32_t* PAR = (uint32_t*)H + (size_t)tiles * 32;
    for (uint32_t idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
        uint32_t e = idx & 15, l = (idx >> 4) & 63;
        uint32_t ks = (idx >> 10) % KS, tile = (idx >> 10) / KS;
        uint32_t c = tile * 32 + (l & 31);
        uint32_t kk = ks * 32 + 16 * (l >> 5) + e;
        Cp[idx] = c < K ? Cn[(size_t)c * d + kk] : (int8_t)0;
    }
    for (uint32_t idx = blockIdx.x * blockDim.x + threadIdx.x; idx < tiles * 2; idx += gridDim.x * blockDim.x) {
        const uint32_t g = idx & 1, tile = idx >> 1;
        uint32_t par = 0;
        for (uint32_t r = 0; r < 16; ++r) {
            const uint32_t c = tile * 32 + tile_row(r, g);
            int32_t h = FILTER_PAD_INIT;
            if (c < K) {
                int32_t nrm = 0;
                for (uint32_t i = 0; i < d; ++i) nrm += (int32_t)Cn[(size_t)c * d + i] * (int32_t)Cn[(size_t)c * d + i];
                h = -((nrm + 1) >> 1);
                par |= (uint32_t)(nrm & 1) << r;
            }
            H[(size_t)idx * 16 + r] = h;
        }
        PAR[idx] = par;
    }
}

// ---------------------------------------------------------------------------
// vectors x centroids.  Each wave keeps 32*NT vectors as MFMA B fragments in registers and walks
// over a range of centroid tiles (blockIdx.y selects the range); the workgroup keeps two groups of TG
// tiles of centroids (and their key constants) in LDS, one being multiplied, one being filled.  Three epilogues:
//   MODE = 0      closest centroid of every vector (running max of the keys; the two lane halves
//                 of a column are merged at the end); one tile range only.
//   MODE = P > 0  the P best centroids each lane has seen, as sorted lists of 64-bit entries
//                 (value in the high word, ~id in the low word: larger = closer, then lower id),
//                 lists[v][range][half][P]; filter_merge_kernel joins the lists of a vector.
//   MODE = -1     the values 2 x.c - |c|^2 themselves, out[v][tiles*32] (any probe count).
constexpr int64_t LIST_EMPTY = INT64_MIN;

template <int P>
__device__ __forceinline__ void list_insert(int64_t (&best)[P], int64_t x) {
#pragma unroll
    for (int i = 0; i < P; ++i) {
        const bool gt = x > best[i];
        const int64_t lo = gt ? best[i] : x;
        best[i] = gt ? x : best[i];
        x = lo;
    }
}

__device__ __forceinline__ int32_t max3(int32_t a, int32_t b, int32_t c) {  // one v_max3_i32
    const int32_t ab = a > b ? a : b;
    return ab > c ? ab : c;
}

template <int KS, int NT, int MODE>
__global__ __launch_bounds__(256) void filter_gemm_kernel(const int8_t* __restrict__ X, uint64_t n,
                                                          const v4i* __restrict__ Cp, const v4i* __restrict__ T2,
                                                          uint32_t tiles, uint32_t K, uint32_t tiles_per_range,
                                                          uint32_t* __restrict__ assign, int32_t* __restrict__ out,
                                                          int64_t* __restrict__ lists, uint32_t zero_words) {
    constexpr int D = KS * 32;
    constexpr int P = MODE > 0 ? MODE : 1;
    // list modes do not write `assign`: there it names zero_words words that the first workgroup clears for the kernel
    // that follows (the counting kernel's list lengths), which saves a launch on the single-query path
    if constexpr (MODE > 0) {
        if (zero_words && blockIdx.x == 0 && blockIdx.y == 0)
            for (uint32_t i = threadIdx.x; i < zero_words; i += 256) assign[i] = 0;
    }
    // a list of one entry is an argmax: MODE = 1 keeps the 32-bit running key of MODE = 0 (no 64-bit list
    // inserts in the loop) and forms its list entry at the end
    constexpr bool ARGMAX = MODE == 0 || MODE == 1;
    // centroid tiles per group: 8 for the build's assignment (long ranges, d <= 128), 4 on the query side and for
    // d = 256, where two buffers of 8 tiles would leave a CU with fewer workgroups than the registers allow
    constexpr int TG = (MODE == 0 && KS <= 4) ? FILTER_TG : FILTER_TG / 2;
    // two groups of centroid tiles in LDS: while the waves multiply one, the next is copied from global memory
    // straight into the other buffer (global_load ... lds: no staging registers; a wave's 64 lanes fill
    // consecutive LDS), one barrier per group
    __shared__ v4i sA[2][TG * KS * 64];
    __shared__ v4i sT[2][TG * 8];  // 32 ints per tile
    __shared__ uint32_t sP[2][64];        // TG * 2 in use; a wave's copy lands at lane * 4 bytes
    const uint32_t* PAR = (const uint32_t*)T2 + (size_t)tiles * 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, g = lane >> 5;
    const uint64_t v0 = ((uint64_t)blockIdx.x * 4 + wave) * (32 * NT);
    const uint32_t t_begin = blockIdx.y * tiles_per_range;
    const uint32_t t_end = tiles - t_begin < tiles_per_range ? tiles : t_begin + tiles_per_range;

    v4i b[NT][KS];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        uint64_t v = v0 + nt * 32 + col;
        if (v >= n) v = n - 1;
        const v4i* src = (const v4i*)(X + v * D + g * 16);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) b[nt][ks] = src[ks * 2];
    }
    // MODE 0: best_key = 16 * value + (15 - register) of the best row so far, best_tile its tile
    int32_t best_key[NT];
    uint32_t best_tile[NT];
    int64_t best[NT][P];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        best_key[nt] = (int32_t)0x80000000;
        best_tile[nt] = 0;
#pragma unroll
        for (int i = 0; i < P; ++i) best[nt][i] = LIST_EMPTY;
    }

    static_assert(TG * 8 <= 64 && TG * 2 <= 64, "the key constants of a group are one wave's copy");
    auto stage = [&](uint32_t t0, int buf) {  // every copy instruction is issued by whole waves (exec masks the tail)
        const uint32_t tg = t_end - t0 < TG ? t_end - t0 : TG;
        for (uint32_t i = threadIdx.x; i < tg * KS * 64; i += 256)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Cp + (size_t)t0 * KS * 64 + i),
                                             (__attribute__((address_space(3))) void*)&sA[buf][i - lane], 16, 0, 0);
        if (wave == 0 && (uint32_t)lane < tg * 8)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(T2 + (size_t)t0 * 8 + lane),
                                             (__attribute__((address_space(3))) void*)&sT[buf][0], 16, 0, 0);
        if (wave == 1 && (uint32_t)lane < tg * 2)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(PAR + (size_t)t0 * 2 + lane),
                                             (__attribute__((address_space(3))) void*)&sP[buf][0], 4, 0, 0);
    };
    if (t_begin < t_end) stage(t_begin, 0);
    int buf = 0;
    for (uint32_t t0 = t_begin; t0 < t_end; t0 += TG, buf ^= 1) {
        const uint32_t tg = t_end - t0 < TG ? t_end - t0 : TG;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this thread's copies into sA[buf] have landed
        __syncthreads();                                   // everyone's have, and everyone is done with the other buffer
        if (t0 + TG < t_end) stage(t0 + TG, buf ^ 1);
#pragma unroll 1
        for (uint32_t tt = 0; tt < tg; ++tt) {
            v16i init;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                v4i t = sT[buf][tt * 8 + g * 4 + q];
                init[4 * q] = t.x; init[4 * q + 1] = t.y; init[4 * q + 2] = t.z; init[4 * q + 3] = t.w;
            }
            const uint32_t par = sP[buf][tt * 2 + g];
            v16i acc[NT];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                v4i a = sA[buf][(tt * KS + ks) * 64 + lane];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[nt][ks], ks == 0 ? init : acc[nt], 0, 0, 0);
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                if constexpr (MODE < 0) {
                    const uint64_t v = v0 + nt * 32 + col;
                    if (v < n) {
                        int32_t* dst = out + v * ((uint64_t)tiles * 32) + (uint64_t)(t0 + tt) * 32 + 4 * g;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            v4i o;
#pragma unroll
                            for (int j = 0; j < 4; ++j) o[j] = 2 * acc[nt][4 * q + j] + (int32_t)((par >> (4 * q + j)) & 1);
                            *(v4i*)(dst + 8 * q) = o;
                        }
                    }
                } else {
                    int32_t m = max3(acc[nt][0], acc[nt][1], acc[nt][2]);
#pragma unroll
                    for (int r = 3; r < 15; r += 2) m = max3(m, acc[nt][r], acc[nt][r + 1]);
                    m = acc[nt][15] > m ? acc[nt][15] : m;
                    // a lane meets centroid ids in increasing tile order, so only a strictly larger value can
                    // replace what it holds, and no value of this tile exceeds 2 m + 1
                    const int32_t bound = ARGMAX ? best_key[nt] >> 4 : (int32_t)(best[nt][P - 1] >> 32);
                    if (2 * m + 1 > bound) {
                        if constexpr (ARGMAX) {
                            int32_t km = (int32_t)0x80000000;
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int32_t val = 2 * acc[nt][r] + (int32_t)((par >> r) & 1);
                                const int32_t key = val * 16 + (15 - r);  // equal values: the lower register = lower row
                                km = key > km ? key : km;
                            }
                            if ((km >> 4) > bound) {
                                best_key[nt] = km;
                                best_tile[nt] = t0 + tt;
                            }
                        } else {
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int32_t val = 2 * acc[nt][r] + (int32_t)((par >> r) & 1);
                                const uint32_t cid = (t0 + tt) * 32 + tile_row(r, g);
                                const int64_t e = (int64_t)(((uint64_t)(uint32_t)val << 32) | (uint32_t)~cid);
                                if (cid < K && e > best[nt][P - 1]) list_insert<P>(best[nt], e);
                            }
                        }
                    }
                }
            }
        }
    }
    if constexpr (MODE == 0) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            int32_t val = best_key[nt] >> 4;
            uint32_t c = best_tile[nt] * 32 + tile_row(15 - (best_key[nt] & 15), g);
            int32_t oval = __shfl_xor(val, 32, 64);
            uint32_t oc = (uint32_t)__shfl_xor((int)c, 32, 64);
            if (oval > val || (oval == val && oc < c)) c = oc;
            const uint64_t v = v0 + nt * 32 + col;
            if (g == 0 && v < n) assign[v] = c;
        }
    } else if constexpr (MODE > 0) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if constexpr (MODE == 1) {
                const uint32_t cid = best_tile[nt] * 32 + tile_row(15 - (best_key[nt] & 15), g);
                const int32_t val = best_key[nt] >> 4;
                best[nt][0] = (best_key[nt] != (int32_t)0x80000000 && cid < K)
                                  ? (int64_t)(((uint64_t)(uint32_t)val << 32) | (uint32_t)~cid)
                                  : LIST_EMPTY;
            }
            const uint64_t v = v0 + nt * 32 + col;
            if (v < n) {
                int64_t* dst = lists + ((v * gridDim.y + blockIdx.y) * 2 + g) * P;
#pragma unroll
                for (int i = 0; i < P; ++i) dst[i] = best[nt][i];
            }
        }
    }
}

// one probe per vector: one wave per vector, lanes stride over its per_vec entries, wave maximum
__global__ __launch_bounds__(256) void filter_merge1_kernel(const int64_t* __restrict__ lists, uint64_t n,
                                                            uint32_t per_vec, uint32_t* __restrict__ probe_ids) {
    const uint32_t lane = threadIdx.x & 63;
    const uint64_t v = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= n) return;
    const int64_t* src = lists + v * per_vec;
    int64_t best = LIST_EMPTY;
    for (uint32_t i = lane; i < per_vec; i += 64) {
        const int64_t e = src[i];
        best = e > best ? e : best;
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const int64_t other = __shfl_xor((long long)best, o, 64);
        best = other > best ? other : best;
    }
    if (lane == 0) probe_ids[v] = best == LIST_EMPTY ? 0xFFFFFFFFu : ~(uint32_t)best;
}

// one thread per vector: the `probe` best entries of its per_vec list entries, closest first
template <int P>
__global__ __launch_bounds__(256) void filter_merge_kernel(const int64_t* __restrict__ lists, uint64_t n,
                                                           uint32_t per_vec, uint32_t probe,
                                                           uint32_t* __restrict__ probe_ids) {
    const uint64_t v = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= n) return;
    int64_t best[P];
#pragma unroll
    for (int i = 0; i < P; ++i) best[i] = LIST_EMPTY;
    const int64_t* src = lists + v * per_vec;
    for (uint32_t i = 0; i < per_vec; ++i) {
        const int64_t e = src[i];
        if (e > best[P - 1]) list_insert<P>(best, e);
    }
#pragma unroll
    for (int i = 0; i < P; ++i)
        if ((uint32_t)i < probe) probe_ids[v * probe + i] = best[i] == LIST_EMPTY ? 0xFFFFFFFFu : ~(uint32_t)best[i];
}

// ---------------------------------------------------------------------------
// Inverted index.  One wave per document; a vector is the first of its document with its
// centroid if no earlier vector of the document has the same one (a bucket holds a document
// once).  A document goes to sub-bucket c*S + (doc >> sub_shift) of its centroid c.  FILL = false counts
// sub-bucket sizes; FILL = true writes document ids at sub_off[...] + (atomic cursor), so the order inside
// a sub-bucket is unspecified.
template <bool FILL>
__global__ __launch_bounds__(256) void filter_bucket_kernel(const uint32_t* __restrict__ assign,
                                                            const uint64_t* __restrict__ doc_off, uint64_t n_docs,
                                                            uint32_t S, uint32_t sub_shift,
                                                            uint32_t* __restrict__ size_or_cursor,
                                                            const uint32_t* __restrict__ sub_off,
                                                            uint32_t* __restrict__ bucket_docs) {
    const uint32_t lane = threadIdx.x & 63;
    for (uint64_t doc = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6); doc < n_docs; doc += (uint64_t)gridDim.x * 4) {
        const uint64_t lo = doc_off[doc], hi = doc_off[doc + 1];
        for (uint64_t j0 = lo; j0 < hi; j0 += 64) {  // 64 vectors of the document per pass, one per lane
            const bool valid = j0 + lane < hi;
            const uint32_t c = valid ? assign[j0 + lane] : 0xFFFFFFFFu;
            bool first = valid;
            for (uint64_t e0 = lo; e0 <= j0; e0 += 64) {  // against every earlier vector, 64 at a time
                const uint32_t ce = e0 == j0 ? c : assign[e0 + lane];  // e0 < j0: a full chunk
                const uint32_t cnt = e0 == j0 ? (uint32_t)(hi - j0 < 64 ? hi - j0 : 64) : 64u;
                for (uint32_t e = 0; e < cnt; ++e) {
                    const uint32_t v = (uint32_t)__builtin_amdgcn_readlane((int)ce, (int)e);
                    if (v == c && (e0 < j0 || e < lane)) first = false;
                }
            }
            if (first) {
                const uint32_t sub = c * S + (uint32_t)(doc >> sub_shift);
                uint32_t pos = atomicAdd(&size_or_cursor[sub], 1u);
                if constexpr (FILL) bucket_docs[sub_off[sub] + pos] = (uint32_t)doc;
            }
        }
    }
}

// exclusive scan of size[0..K) into off[0..K], one workgroup; size is zeroed for reuse as cursors
__global__ __launch_bounds__(1024) void filter_scan_kernel(uint32_t* __restrict__ size, uint32_t K,
                                                           uint32_t* __restrict__ off) {
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t carry;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (uint32_t base = 0; base < K; base += 1024) {
        const uint32_t i = base + tid;
        const uint32_t x = i < K ? size[i] : 0;
        uint32_t incl = x;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            uint32_t y = __shfl_up(incl, o, 64);
            if ((int)lane >= o) incl += y;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        uint32_t before = carry;
        for (uint32_t w = 0; w < wave; ++w) before += wsum[w];
        if (i < K) {
            off[i] = before + incl - x;
            size[i] = 0;
        }
        __syncthreads();
        if (tid == 1023) carry = before + incl;
        __syncthreads();
    }
    if (tid == 0) off[K] = carry;
}

// bucket_off[c] = sub_off[c*S] for c = 0..K: the caller-visible bucket starts
__global__ void filter_bucket_starts_kernel(const uint32_t* __restrict__ sub_off, uint32_t K, uint32_t S,
                                            uint32_t* __restrict__ bucket_off) {
    const uint32_t c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c <= K) bucket_off[c] = sub_off[(size_t)c * S];
}

// ---------------------------------------------------------------------------
// Query side.
struct DistKeys {  // key = (value + bias) above the centroid id: closest first, lower id first
    const int32_t* row;
    uint32_t id_bits;
    static constexpr int VEC = 1;
    static constexpr bool SEGMENTS = false;
    using key_t = uint64_t;
    __device__ uint64_t operator()(uint64_t i) const { return make_key(row[i] + FILTER_BIAS, (uint32_t)i, id_bits); }
    __device__ void load(uint64_t i, uint64_t n, uint64_t (&out)[1]) const { out[0] = i < n ? (*this)(i) : 0; }
};

// one workgroup per query vector: its `probe` closest centroids, closest first
__global__ __launch_bounds__(256) void filter_probe_kernel(const int32_t* __restrict__ dist, uint32_t row_stride,
                                                           uint32_t K, uint32_t probe, uint32_t kpad, KeyPlan plan,
                                                           uint32_t* __restrict__ probe_ids) {
    extern __shared__ uint64_t sorted[];
    __shared__ SelectShared sh;
    const uint32_t q = blockIdx.x;
    DistKeys keys{dist + (size_t)q * row_stride, plan.id_bits};
    block_select<256>(keys, K, probe, kpad, sorted, sh, plan);
    const uint64_t idmask = (1ull << plan.id_bits) - 1;
    for (uint32_t i = threadIdx.x; i < probe; i += 256)
        probe_ids[(size_t)q * probe + i] = sorted[i] ? (uint32_t)(idmask - (sorted[i] & idmask)) : 0xFFFFFFFFu;
}

__global__ void filter_zero_kernel(int32_t* __restrict__ p, uint64_t n) {
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

// Bucket counting without global atomics.  Workgroup (slab, query set) owns the documents
// [slab * slab_docs, +slab_docs) and keeps one counter per document in LDS (W bytes each, packed into
// 32-bit words; a count never exceeds the number of probed buckets, which the host bounds by the
// counter range).  It reads, of every bucket its query set probes, the sub-buckets that overlap its slab
// (a wave takes its buckets' ranges as one concatenated run, so all its loads are in flight together),
// counts the ids that fall into the slab, and remembers each document at its first hit in a queue.  Then
// one key (count, id) in the top-k key format per queued document goes to the query set's list;
// cursor[b] ends as the number of distinct documents hit.  The order inside a list is unspecified.
// Only if the queue overflows (more than FILTER_QUEUE distinct documents of one slab hit) are the counters
// scanned instead.
// first-hit queue entries per workgroup (positions within the slab: QT = u16, or u32 for slabs over 65536 documents).
// 3712: with a slab of 32768 one-byte counters and the 128-bin histogram the workgroup then needs just under 40 KB
// of LDS and four fit a CU.
constexpr uint32_t FILTER_QUEUE = 3712;
constexpr uint32_t FILTER_HSMALL = 128;  // bins of the per-workgroup histogram of counts

template <int W, int T, typename QT, typename KT>
__global__ __launch_bounds__(T) void filter_count_kernel(const uint32_t* __restrict__ probe_ids, uint32_t probe,
                                                            const uint32_t* __restrict__ q_off, uint32_t q_uniform,
                                                            const uint32_t* __restrict__ sub_off, uint32_t S,
                                                            uint32_t sub_shift,
                                                            const uint32_t* __restrict__ bucket_docs, uint64_t n_docs,
                                                            uint32_t slab_docs, uint32_t id_bits,
                                                            KT* __restrict__ lists, uint64_t list_stride,
                                                            uint32_t* __restrict__ cursor, uint32_t* __restrict__ hist,
                                                            uint32_t hist_bins, uint32_t* __restrict__ segs) {
    extern __shared__ uint32_t cnt[];
    __shared__ QT queue[FILTER_QUEUE];
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t base_sh, q_count;
    constexpr uint32_t PER = 4 / W, BITS = 8 * W, WAVES = T / 64;
    constexpr uint32_t MASK = W == 4 ? 0xFFFFFFFFu : (1u << (BITS % 32)) - 1;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t b = blockIdx.y;
    const uint32_t doc0 = blockIdx.x * slab_docs;
    const uint32_t here = n_docs - doc0 < slab_docs ? (uint32_t)(n_docs - doc0) : slab_docs;
    const uint32_t words = (here + PER - 1) / PER;
    const uint32_t q_lo = q_uniform ? b * q_uniform : q_off[b];
    const uint32_t q_hi = q_uniform ? q_lo + q_uniform : q_off[b + 1];
    const uint32_t pairs = (q_hi - q_lo) * probe;
    const uint32_t* mine = probe_ids + (uint64_t)q_lo * probe;
    // the sub-buckets that overlap this slab's document range (whole sub-buckets: ids outside the slab are skipped below)
    const uint32_t s_lo = doc0 >> sub_shift;
    uint32_t s_hi = (uint32_t)(((uint64_t)doc0 + here + ((1u << sub_shift) - 1)) >> sub_shift);
    s_hi = s_hi < S ? s_hi : S;
    // first batch of this wave's buckets: lane l takes pair wave + l*WAVES; its bounds are requested before the
    // counters are cleared
    auto bounds = [&](uint32_t p0, uint32_t& lo_l, uint32_t& n_l) {
        const uint32_t myp = p0 + lane * WAVES;
        lo_l = n_l = 0;
        if (myp < pairs) {
            const uint32_t c = mine[myp];
            if (c != 0xFFFFFFFFu) {
                lo_l = sub_off[(size_t)c * S + s_lo];
                n_l = sub_off[(size_t)c * S + s_hi] - lo_l;
            }
        }
    };
    // Histogram of the emitted keys' score fields (bin = count + 1) for the selection that follows.  Nearly every
    // document is hit once: a thread counts those in a register; the workgroup gathers its counts in a small LDS
    // histogram.  segs != nullptr: this workgroup's histogram and the run of the list it writes are stored as they
    // are, hist[b][slab][bins] and segs[b][slab][2] (at most FILTER_HSMALL bins).  Else the occupied bins are added to
    // the query set's histogram hist[b][bins] (a handful of global atomics per workgroup; one per key made this kernel
    // four times slower: they all go to the same few addresses).
    __shared__ uint32_t hsmall[FILTER_HSMALL];
    const bool tallying = hist_bins != 0;
    uint32_t* my_hist = !tallying ? nullptr
                        : segs    ? hist + ((size_t)b * gridDim.x + blockIdx.x) * hist_bins
                                  : hist + (size_t)b * hist_bins;
    uint32_t ones = 0;
    if (tid < FILTER_HSMALL) hsmall[tid] = 0;  // ordered before the first tally by the barriers of the counting phase
    auto tally = [&](uint32_t c) {
        if (!tallying) return;
        if (c == 1) ++ones;
        else if (c + 1 < FILTER_HSMALL) atomicAdd(&hsmall[c + 1], 1u);
        else atomicAdd(&my_hist[c + 1], 1u);  // not with segs: the host gives rows only to histograms that fit hsmall
    };
    auto flush_tally = [&](uint32_t list_start, uint32_t list_len) {  // called by every thread of the workgroup
        if (!tallying) return;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) ones += __shfl_down(ones, o, 64);
        if (lane == 0 && ones) atomicAdd(&hsmall[2], ones);
        __syncthreads();
        if (segs) {
            if (tid < hist_bins) my_hist[tid] = hsmall[tid];
            if (tid == 0) {
                uint32_t* sg = segs + ((size_t)b * gridDim.x + blockIdx.x) * 2;
                sg[0] = list_start;
                sg[1] = list_len;
            }
        } else if (tid < FILTER_HSMALL && tid < hist_bins && hsmall[tid]) {
            atomicAdd(&my_hist[tid], hsmall[tid]);
        }
    };
    uint32_t lo_l, n_l;
    bounds(wave, lo_l, n_l);
    for (uint32_t i = tid; i < words; i += T) cnt[i] = 0;
    if (tid == 0) q_count = 0;
    __syncthreads();
    for (uint32_t p0 = wave; p0 < pairs; p0 += WAVES * 64) {
        if (p0 != wave) bounds(p0, lo_l, n_l);
        // concatenate the ranges: inclusive prefix of the sizes over the lanes
        uint32_t incl = n_l;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            uint32_t y = __shfl_up(incl, o, 64);
            if ((int)lane >= o) incl += y;
        }
        const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        const uint32_t left = (pairs - p0 + WAVES - 1) / WAVES;
        const uint32_t n_ranges = left < 64 ? left : 64;
        constexpr int U = 8;  // elements per lane per trip
        for (uint32_t f0 = 0; f0 < total; f0 += 64 * U) {
            uint32_t id[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                // element f of the concatenated run: the range j with excl_j <= f < incl_j
                const uint32_t f = f0 + u * 64 + lane;
                uint32_t addr = 0xFFFFFFFFu;
                if (f < total) {
                    for (uint32_t j = 0; j < n_ranges; ++j) {
                        const uint32_t in_j = (uint32_t)__builtin_amdgcn_readlane((int)incl, (int)j);
                        const uint32_t n_j = (uint32_t)__builtin_amdgcn_readlane((int)n_l, (int)j);
                        if (addr == 0xFFFFFFFFu && f < in_j)
                            addr = (uint32_t)__builtin_amdgcn_readlane((int)lo_l, (int)j) + (f - (in_j - n_j));
                    }
                }
                id[u] = addr != 0xFFFFFFFFu ? bucket_docs[addr] : 0xFFFFFFFFu;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t local = id[u] - doc0;  // wraps to a large value for ids below the slab
                const bool hit = id[u] != 0xFFFFFFFFu && local < here;
                bool first = false;
                if (hit) {
                    const uint32_t sh = (local % PER) * BITS;
                    const uint32_t old = atomicAdd(&cnt[local / PER], 1u << sh);
                    first = ((old >> sh) & MASK) == 0;
                }
                // documents hit for the first time go to the queue: one LDS atomic per wave
                const uint64_t fm = __ballot(first);
                if (fm) {
                    uint32_t base = 0;
                    if (lane == (uint32_t)__builtin_ctzll(fm)) base = atomicAdd(&q_count, (uint32_t)__builtin_popcountll(fm));
                    base = (uint32_t)__builtin_amdgcn_readlane((int)base, __builtin_ctzll(fm));
                    const uint32_t pos = base + (uint32_t)__builtin_popcountll(fm & ((1ull << lane) - 1));
                    if (first && pos < FILTER_QUEUE) queue[pos] = (QT)local;
                }
            }
        }
    }
    __syncthreads();
    const uint32_t hits = q_count;
    if (hits <= FILTER_QUEUE) {
        if (tid == 0) base_sh = hits ? atomicAdd(&cursor[b], hits) : 0;
        __syncthreads();
        KT* dst = lists + (uint64_t)b * list_stride + base_sh;
        for (uint32_t i = tid; i < hits; i += T) {
            const uint32_t local = queue[i];
            const uint32_t c = (cnt[local / PER] >> ((local % PER) * BITS)) & MASK;
            dst[i] = (KT)make_key((int32_t)c, doc0 + local, id_bits);
            tally(c);
        }
        flush_tally(base_sh, hits);
        return;
    }
    // queue overflow: scan the counters
    uint32_t nz = 0;
    for (uint32_t i = tid; i < words; i += T) {
        const uint32_t x = cnt[i];
        if (x) {
#pragma unroll
            for (uint32_t j = 0; j < PER; ++j) nz += ((x >> (j * BITS)) & MASK) != 0;
        }
    }
    uint32_t incl = nz;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t y = __shfl_up(incl, o, 64);
        if ((int)lane >= o) incl += y;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    if (tid == 0) {
        uint32_t total = 0;
        for (int w = 0; w < (int)WAVES; ++w) total += wsum[w];
        base_sh = total ? atomicAdd(&cursor[b], total) : 0;
    }
    uint32_t before = 0;
    for (uint32_t w = 0; w < wave; ++w) before += wsum[w];
    __syncthreads();
    KT* dst = lists + (uint64_t)b * list_stride + base_sh + before + incl - nz;
    for (uint32_t i = tid; i < words; i += T) {
        const uint32_t x = cnt[i];
        if (x) {
#pragma unroll
            for (uint32_t j = 0; j < PER; ++j) {
                const uint32_t c = (x >> (j * BITS)) & MASK;
                if (c) {
                    *dst++ = (KT)make_key((int32_t)c, doc0 + i * PER + j, id_bits);
                    tally(c);
                }
            }
        }
    }
    flush_tally(base_sh, hits);  // as many keys as first hits
}

// ---------------------------------------------------------------------------
// k-means for the centroids (Sec. 5 "Filtering": k-means on a sample of the vectors): Lloyd's iteration
// in integers.  The assignment step is the GEMM above; these two kernels are the update step.
// One thread per (vector, 4 coordinates): sums[c][i] += x[i]; the thread of the first coordinates counts the vector.
__global__ __launch_bounds__(256) void kmeans_accumulate_kernel(const int8_t* __restrict__ X, uint64_t n, uint32_t d,
                                                                const uint32_t* __restrict__ assign,
                                                                int32_t* __restrict__ sums, uint32_t* __restrict__ counts) {
    const uint32_t parts = d / 4;
    const uint64_t idx = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * parts) return;
    const uint64_t v = idx / parts;
    const uint32_t part = (uint32_t)(idx - v * parts);
    const uint32_t c = assign[v];
    const uint32_t x = *(const uint32_t*)(X + v * d + part * 4);
    int32_t* dst = sums + (size_t)c * d + part * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int32_t xi = (int32_t)(int8_t)(x >> (8 * i));
        if (xi) atomicAdd(dst + i, xi);
    }
    if (part == 0) atomicAdd(counts + c, 1u);
}

// centroid = coordinate-wise mean rounded to the nearest integer, half up: floor((2 sum + n) / (2 n));
// a centroid that received no vector stays
__global__ __launch_bounds__(256) void kmeans_update_kernel(const int32_t* __restrict__ sums,
                                                            const uint32_t* __restrict__ counts, uint32_t K, uint32_t d,
                                                            int8_t* __restrict__ Cn) {
    const uint32_t idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= K * d) return;
    const int64_t cnt = counts[idx / d];
    if (cnt == 0) return;
    const int64_t a = 2 * (int64_t)sums[idx] + cnt, b = 2 * cnt;
    int64_t q = a / b;
    if (a % b != 0 && a < 0) --q;  // floor division
    Cn[idx] = (int8_t)q;
}

hipError_t launch_kmeans_update(const int8_t* X, uint64_t n, uint32_t d, const uint32_t* assign, uint32_t K,
                                int32_t* sums, uint32_t* counts, int8_t* Cn, hipStream_t stream) {
    if (d % 4 || K == 0 || (uint64_t)K * d > 0x7fffffffull) return hipErrorInvalidValue;
    const uint64_t cells = (uint64_t)K * d;
    hipLaunchKernelGGL(filter_zero_kernel, dim3((unsigned)((cells + 2047) / 2048)), dim3(256), 0, stream, sums, cells);
    hipLaunchKernelGGL(filter_zero_kernel, dim3((K + 255) / 256), dim3(256), 0, stream, (int32_t*)counts, (uint64_t)K);
    if (n) {
        const uint64_t blocks = (n * (d / 4) + 255) / 256;
        if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
        hipLaunchKernelGGL(kmeans_accumulate_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, X, n, d, assign, sums,
                           counts);
    }
    hipLaunchKernelGGL(kmeans_update_kernel, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, stream, sums, counts, K,
                       d, Cn);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
static bool filter_shape(uint32_t d) { return d == 64 || d == 128 || d == 256; }
bool filter_supported(uint32_t d) { return filter_shape(d); }
uint32_t filter_tiles(uint32_t K) { return (K + 31) / 32; }
size_t filter_centroid_bytes(uint32_t K, uint32_t d) { return (size_t)filter_tiles(K) * (d / 32) * 1024; }
size_t filter_table_bytes(uint32_t K) { return (size_t)filter_tiles(K) * (32 + 2) * 4; }

hipError_t launch_filter_prep(const int8_t* Cn, uint32_t K, uint32_t d, void* Cp, void* T2, hipStream_t stream) {
    if (!filter_shape(d) || K == 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(filter_prep_kernel, dim3(1024), dim3(256), 0, stream, Cn, K, d, (int8_t*)Cp, (int32_t*)T2,
                       filter_tiles(K));
    return hipGetLastError();
}

template <int NT, int MODE>
static hipError_t launch_gemm(const int8_t* X, uint64_t n, uint32_t d, uint32_t K, const void* Cp, const void* T2,
                              uint32_t ranges, uint32_t tiles_per_range, uint32_t* assign, int32_t* out, int64_t* lists,
                              hipStream_t stream, uint32_t zero_words = 0) {
    if (n == 0) return hipSuccess;
    uint64_t blocks = (n + 4 * 32 * NT - 1) / (4 * 32 * NT);
    if (blocks > 0x7fffffffull || ranges == 0 || ranges > 65535) return hipErrorInvalidValue;
    const uint32_t tiles = filter_tiles(K);
    if ((uint64_t)ranges * tiles_per_range < tiles || (uint64_t)(ranges - 1) * tiles_per_range >= tiles)
        return hipErrorInvalidValue;  // every range must hold at least one tile and together they cover all
    dim3 grid((unsigned)blocks, ranges), block(256);
    if (d == 64)
        hipLaunchKernelGGL((filter_gemm_kernel<2, NT, MODE>), grid, block, 0, stream, X, n, (const v4i*)Cp, (const v4i*)T2, tiles, K, tiles_per_range, assign, out, lists, zero_words);
    else if (d == 128)
        hipLaunchKernelGGL((filter_gemm_kernel<4, NT, MODE>), grid, block, 0, stream, X, n, (const v4i*)Cp, (const v4i*)T2, tiles, K, tiles_per_range, assign, out, lists, zero_words);
    else if (d == 256)
        hipLaunchKernelGGL((filter_gemm_kernel<8, NT, MODE>), grid, block, 0, stream, X, n, (const v4i*)Cp, (const v4i*)T2, tiles, K, tiles_per_range, assign, out, lists, zero_words);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_filter_assign(const int8_t* X, uint64_t n, uint32_t d, uint32_t K, const void* Cp, const void* T2,
                                uint32_t* assign, hipStream_t stream) {
    return launch_gemm<4, 0>(X, n, d, K, Cp, T2, 1, filter_tiles(K), assign, nullptr, nullptr, stream);
}

hipError_t launch_filter_distances(const int8_t* X, uint64_t n, uint32_t d, uint32_t K, const void* Cp, const void* T2,
                                   int32_t* out, hipStream_t stream) {
    return launch_gemm<2, -1>(X, n, d, K, Cp, T2, 1, filter_tiles(K), nullptr, out, nullptr, stream);
}

// Query side with a small probe count: the centroid tiles are split into ranges so that the few query
// vectors of a batch still fill the chip, and every range keeps its best P = 2^ceil(log2 probe) in registers.
static uint32_t list_width(uint32_t probe) { return probe <= 1 ? 1 : probe <= 2 ? 2 : probe <= 4 ? 4 : 8; }

FilterProbePlan filter_probe_plan(uint64_t n, uint32_t K, uint32_t probe) {
    FilterProbePlan pl{};
    if (probe == 0 || probe > FILTER_LIST_MAX || n == 0) return pl;  // ranges = 0: use the distance matrix
    const uint32_t tiles = filter_tiles(K);
    const uint32_t groups = (tiles + FILTER_TG - 1) / FILTER_TG;
    // more vectors per workgroup halve the centroid bytes staged through LDS per vector
    pl.nt = n >= 4096 ? 2 : 1;
    const uint64_t blocks = (n + 128 * pl.nt - 1) / (128 * pl.nt);
    uint64_t want = (2048 + blocks - 1) / blocks;  // aim at ~2048 workgroups
    if (want > groups) want = groups;
    // a few query vectors alone (one query set): the launch is a chain of global -> LDS stages per workgroup, so more,
    // shorter ranges cut its latency; the merge of a vector's lists is wave-wide for one probe, a thread's loop otherwise
    const uint64_t cap = blocks <= 4 ? (probe == 1 ? 512 : 128) : 64;
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    const uint32_t per = (groups + (uint32_t)want - 1) / (uint32_t)want;
    pl.tiles_per_range = per * FILTER_TG;
    pl.ranges = (tiles + pl.tiles_per_range - 1) / pl.tiles_per_range;
    pl.width = list_width(probe);
    pl.list_bytes = (size_t)n * pl.ranges * 2 * pl.width * 8;
    return pl;
}

hipError_t launch_filter_probe_lists(const int8_t* X, uint64_t n, uint32_t d, uint32_t K, const void* Cp, const void* T2,
                                     uint32_t probe, const FilterProbePlan& pl, int64_t* lists, uint32_t* probe_ids,
                                     hipStream_t stream, uint32_t* zero, uint32_t zero_words) {
    if (n == 0) return hipSuccess;
    if (pl.ranges == 0 || probe > K || pl.width != list_width(probe)) return hipErrorInvalidValue;
    hipError_t e;
    const uint32_t per_vec = pl.ranges * 2 * pl.width;
    const dim3 mgrid((unsigned)((n + 255) / 256)), mblock(256);
    switch (pl.width) {
        case 1:
            e = pl.nt == 2 ? launch_gemm<2, 1>(X, n, d, K, Cp, T2, pl.ranges, pl.tiles_per_range, zero, nullptr, lists, stream, zero_words)
                           : launch_gemm<1, 1>(X, n, d, K, Cp, T2, pl.ranges, pl.tiles_per_range, zero, nullptr, lists, stream, zero_words);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(filter_merge1_kernel, dim3((unsigned)((n + 3) / 4)), mblock, 0, stream, lists, n, per_vec, probe_ids);
            break;
        case 2:
            e = pl.nt == 2 ? launch_gemm<2, 2>(X, n, d, K, Cp, T2, pl.ranges, pl.tiles_per_range, zero, nullptr, lists, stream, zero_words)
                           : launch_gemm<1, 2>(X, n, d, K, Cp, T2, pl.ranges, pl.tiles_per_range, zero, nullptr, lists, stream, zero_words);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(filter_merge_kernel<2>, mgrid, mblock, 0, stream, lists, n, per_vec, probe, probe_ids);
            break;
        case 4:
            e = pl.nt == 2 ? launch_gemm<2, 4>(X, n, d, K, Cp, T2, pl.ranges, pl.tiles_per_range, zero, nullptr, lists, stream, zero_words)
                           : launch_gemm<1, 4>(X, n, d, K, Cp, T2, pl.ranges, pl.tiles_per_range, zero, nullptr, lists, stream, zero_words);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(filter_merge_kernel<4>, mgrid, mblock, 0, stream, lists, n, per_vec, probe, probe_ids);
            break;
        default:
            e = pl.nt == 2 ? launch_gemm<2, 8>(X, n, d, K, Cp, T2, pl.ranges, pl.tiles_per_range, zero, nullptr, lists, stream, zero_words)
                           : launch_gemm<1, 8>(X, n, d, K, Cp, T2, pl.ranges, pl.tiles_per_range, zero, nullptr, lists, stream, zero_words);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(filter_merge_kernel<8>, mgrid, mblock, 0, stream, lists, n, per_vec, probe, probe_ids);
            break;
    }
    return hipGetLastError();
}

FilterSubPlan filter_sub_plan(uint64_t n_docs, uint32_t K) {
    // ranges of 32768 documents (the smallest slab of the counting kernel), wider while K*S would pass 2^22 entries
    FilterSubPlan sp{1, 15};
    for (;;) {
        const uint64_t S = n_docs ? ((n_docs - 1) >> sp.sub_shift) + 1 : 1;
        if (S * K <= (1ull << 22) || sp.sub_shift >= 31) {
            sp.S = (uint32_t)S;
            return sp;
        }
        ++sp.sub_shift;
    }
}

hipError_t launch_filter_buckets(const uint32_t* assign, const uint64_t* doc_off, uint64_t n_docs, uint32_t K,
                                 FilterSubPlan sp, uint32_t* cursor, uint32_t* sub_off, uint32_t* bucket_off,
                                 uint32_t* bucket_docs, hipStream_t stream) {
    uint64_t blocks = (n_docs + 3) / 4;
    if (blocks > 65536) blocks = 65536;
    if (blocks == 0) blocks = 1;
    const uint64_t KS = (uint64_t)K * sp.S;
    if (KS > 0x7fffffffull) return hipErrorInvalidValue;
    uint64_t zb = (KS + 255) / 256;
    if (zb > 65536) zb = 65536;
    hipLaunchKernelGGL(filter_zero_kernel, dim3((unsigned)zb), dim3(256), 0, stream, (int32_t*)cursor, KS);
    hipLaunchKernelGGL(filter_bucket_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, assign, doc_off, n_docs,
                       sp.S, sp.sub_shift, cursor, sub_off, bucket_docs);
    hipLaunchKernelGGL(filter_scan_kernel, dim3(1), dim3(1024), 0, stream, cursor, (uint32_t)KS, sub_off);
    hipLaunchKernelGGL(filter_bucket_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, assign, doc_off, n_docs,
                       sp.S, sp.sub_shift, cursor, sub_off, bucket_docs);
    hipLaunchKernelGGL(filter_bucket_starts_kernel, dim3(K / 256 + 1), dim3(256), 0, stream, sub_off, K, sp.S, bucket_off);
    return hipGetLastError();
}

hipError_t launch_filter_probe(const int32_t* dist, uint64_t total_q, uint32_t K, uint32_t probe, uint32_t* probe_ids,
                               hipStream_t stream) {
    if (total_q == 0) return hipSuccess;
    if (total_q > 0x7fffffffull || probe == 0 || probe > K || probe > 1024) return hipErrorInvalidValue;
    uint32_t kpad = 2;
    while (kpad < probe) kpad <<= 1;
    KeyPlan plan = make_key_plan((uint32_t)(2 * FILTER_BIAS), K - 1);
    hipLaunchKernelGGL(filter_probe_kernel, dim3((unsigned)total_q), dim3(256), (size_t)kpad * 8, stream, dist,
                       filter_tiles(K) * 32, K, probe, kpad, plan, probe_ids);
    return hipGetLastError();
}

constexpr uint32_t FILTER_SLAB_BYTES = 128 * 1024;  // most LDS counters one workgroup may hold (the queue takes up to 16 KB more)

template <int W, int T, typename QT, typename KT>
static hipError_t launch_filter_count_t(dim3 grid, size_t lds, hipStream_t stream, const uint32_t* probe_ids, uint32_t probe,
                                        const uint32_t* q_off, uint32_t q_uniform, const uint32_t* sub_off, FilterSubPlan sp,
                                        const uint32_t* bucket_docs, uint64_t n_docs, uint32_t slab_docs, uint32_t id_bits,
                                        uint64_t* lists, uint64_t list_stride, uint32_t* cursor, uint32_t* hist,
                                        uint32_t hist_bins, uint32_t* segs) {
    static hipError_t attr = hipFuncSetAttribute((const void*)filter_count_kernel<W, T, QT, KT>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, FILTER_SLAB_BYTES);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((filter_count_kernel<W, T, QT, KT>), grid, dim3(T), lds, stream, probe_ids, probe, q_off, q_uniform, sub_off,
                       sp.S, sp.sub_shift, bucket_docs, n_docs, slab_docs, id_bits, (KT*)lists, list_stride, cursor, hist, hist_bins, segs);
    return hipGetLastError();
}

FilterHistPlan filter_hist_plan(uint32_t n_queries, uint32_t max_pairs, uint64_t n_docs, FilterSubPlan sp) {
    FilterHistPlan hp{};
    hp.counter_bytes = max_pairs <= 255 ? 1 : max_pairs <= 65535 ? 2 : 4;  // a count is at most the number of probed buckets
    // A slab is one sub-bucket range of documents when its counters fit (32768 documents: 32 KB of LDS with
    // one-byte counters; four workgroups of 512 threads per CU overlap their phases), else as many documents as fit.
    uint64_t slab_docs = 1ull << sp.sub_shift;
    if (slab_docs * hp.counter_bytes > FILTER_SLAB_BYTES) slab_docs = FILTER_SLAB_BYTES / hp.counter_bytes;
    if (slab_docs > n_docs) slab_docs = (n_docs + 3) & ~3ull;
    hp.slab_docs = (uint32_t)slab_docs;
    const uint64_t slabs = slab_docs ? (n_docs + slab_docs - 1) / slab_docs : 0;
    hp.slabs = slabs > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)slabs;
    hp.bins = n_docs ? leading_score_bins(max_pairs, n_docs - 1) : 0;
    hp.rows = hp.bins != 0 && hp.bins <= FILTER_HSMALL && hp.slabs <= 1024;  // one thread per slab in the selection
    hp.hist_off = ((size_t)n_queries + 63) / 64 * 64;
    const size_t hist_words = hp.rows ? (size_t)n_queries * hp.slabs * hp.bins : (size_t)n_queries * hp.bins;
    hp.seg_off = hp.hist_off + hist_words;
    hp.words = hp.seg_off + (hp.rows ? (size_t)n_queries * hp.slabs * 2 : 0);
    return hp;
}

uint64_t filter_count_zero_words(const FilterHistPlan& hp, uint32_t n_queries) { return hp.rows ? n_queries : hp.seg_off; }

hipError_t launch_filter_count(const uint32_t* probe_ids, uint64_t total_q, uint32_t probe, uint32_t max_pairs,
                               const uint32_t* q_off, uint32_t q_uniform, uint32_t n_queries, const uint32_t* sub_off,
                               FilterSubPlan sp, const uint32_t* bucket_docs, uint64_t n_docs, uint64_t* lists,
                               uint64_t list_stride, uint32_t* cursor, hipStream_t stream, bool zeroed) {
    if (n_queries == 0) return hipSuccess;
    if (n_queries > 65535 || n_docs > 0xFFFFFFFEull) return hipErrorInvalidValue;
    const FilterHistPlan hp = filter_hist_plan(n_queries, max_pairs, n_docs, sp);
    const uint32_t hist_bins = hp.bins;
    uint32_t* hist = hist_bins ? cursor + hp.hist_off : nullptr;
    uint32_t* segs = hp.rows ? cursor + hp.seg_off : nullptr;
    // the list lengths start from zero, and so does a histogram that is added up with atomics (rows are stored)
    const uint64_t zero_words = filter_count_zero_words(hp, n_queries);
    uint64_t zb = (zero_words + 1023) / 1024;
    if (!zeroed)
        hipLaunchKernelGGL(filter_zero_kernel, dim3((unsigned)(zb > 4096 ? 4096 : zb)), dim3(256), 0, stream, (int32_t*)cursor,
                           zero_words);
    if (n_docs == 0 || total_q == 0) return hipGetLastError();
    const uint32_t W = hp.counter_bytes;
    const uint64_t slab_docs = hp.slab_docs;
    const uint64_t slabs = hp.slabs;
    if (slabs > 0x7fffffffull) return hipErrorInvalidValue;
    const size_t lds = (size_t)slab_docs * W;
    const uint32_t id_bits = bits_for(n_docs - 1);
    const dim3 grid((unsigned)slabs, n_queries);
#define DESSERT_COUNT_ARGS grid, lds, stream, probe_ids, probe, q_off, q_uniform, sub_off, sp, bucket_docs, n_docs, \
                           (uint32_t)slab_docs, id_bits, lists, list_stride, cursor, hist, hist_bins, segs
#define DESSERT_COUNT_CASE(W_, T_)                                                                              \
    do {                                                                                                        \
        if (slab_docs <= 65536)                                                                                 \
            return k32 ? launch_filter_count_t<W_, T_, uint16_t, uint32_t>(DESSERT_COUNT_ARGS)                    \
                       : launch_filter_count_t<W_, T_, uint16_t, uint64_t>(DESSERT_COUNT_ARGS);                   \
        return k32 ? launch_filter_count_t<W_, T_, uint32_t, uint32_t>(DESSERT_COUNT_ARGS)                        \
                   : launch_filter_count_t<W_, T_, uint32_t, uint64_t>(DESSERT_COUNT_ARGS);                       \
    } while (0)
    const bool k32 = keys_fit_32(max_pairs, n_docs - 1);  // the lists hold u32 keys then (launch_topk_lists reads them so)
    if (W == 1) DESSERT_COUNT_CASE(1, 512);
    if (W == 2) DESSERT_COUNT_CASE(2, 512);
    DESSERT_COUNT_CASE(4, 512);
#undef DESSERT_COUNT_ARGS
#undef DESSERT_COUNT_CASE
}

}  // namespace dessert
