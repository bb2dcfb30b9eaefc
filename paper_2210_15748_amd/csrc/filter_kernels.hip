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

constexpr int FILTER_TG = 8;           // centroid tiles staged in LDS per step
constexpr int32_t FILTER_BIAS = 1 << 24;  // 2 x.c - |c|^2 lies in (-2^24, 2^24) for int8 vectors up to d = 256

// accumulator register r of lane half g holds tile row 8*(r/4) + 4*g + r%4
__host__ __device__ inline uint32_t tile_row(uint32_t r, uint32_t g) { return 8 * (r / 4) + 4 * g + (r % 4); }

// ---------------------------------------------------------------------------
// Centroids in MFMA operand order, [tiles][KS][64 lanes][16 B] (tile = 32 centroids, rows past K
// are zero), and the per-row constants of the comparison key, [tiles][2 halves][16 registers]:
//   key(r) = (dot << 5) + T  with  T = (15 - r) - (|c|^2 << 4)
//          = 16 * (2 dot - |c|^2) + (15 - r),
// so a plain signed max over a lane's 16 keys picks the largest 2 x.c - |c|^2 and, among equal
// ones, the lowest register = lowest row.  Rows past K get a constant that can never win.
__global__ void filter_prep_kernel(const int8_t* __restrict__ Cn, uint32_t K, uint32_t d, int8_t* __restrict__ Cp,
                                   int32_t* __restrict__ T2, uint32_t tiles) {
    const uint32_t KS = d / 32;
    const uint32_t total = tiles * KS * 1024;
    for (uint32_t idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
        uint32_t e = idx & 15, l = (idx >> 4) & 63;
        uint32_t ks = (idx >> 10) % KS, tile = (idx >> 10) / KS;
        uint32_t c = tile * 32 + (l & 31);
        uint32_t kk = ks * 32 + 16 * (l >> 5) + e;
        Cp[idx] = c < K ? Cn[(size_t)c * d + kk] : (int8_t)0;
    }
    for (uint32_t idx = blockIdx.x * blockDim.x + threadIdx.x; idx < tiles * 32; idx += gridDim.x * blockDim.x) {
        uint32_t r = idx & 15, g = (idx >> 4) & 1, tile = idx >> 5;
        uint32_t c = tile * 32 + tile_row(r, g);
        int32_t t;
        if (c < K) {
            int32_t nrm = 0;
            for (uint32_t i = 0; i < d; ++i) nrm += (int32_t)Cn[(size_t)c * d + i] * (int32_t)Cn[(size_t)c * d + i];
            t = (int32_t)(15 - r) - (nrm << 4);
        } else {
            t = -(1 << 30);
        }
        T2[idx] = t;
    }
}

// ---------------------------------------------------------------------------
// vectors x centroids.  Each wave keeps 32*NT vectors as MFMA B fragments in registers and walks
// over all centroid tiles; the workgroup stages FILTER_TG tiles of centroids (and their key
// constants) in LDS at a time.  STORE = false: closest centroid of every vector (running max of
// the keys; the two lane halves of a column are merged at the end).  STORE = true: the values
// 2 x.c - |c|^2 themselves, out[v][tiles*32] (for the query-side probe selection).
template <int KS, int NT, bool STORE>
__global__ __launch_bounds__(256) void filter_gemm_kernel(const int8_t* __restrict__ X, uint64_t n,
                                                          const v4i* __restrict__ Cp, const v4i* __restrict__ T2,
                                                          uint32_t tiles, uint32_t* __restrict__ assign,
                                                          int32_t* __restrict__ out) {
    constexpr int D = KS * 32;
    __shared__ v4i sA[FILTER_TG * KS * 64];
    __shared__ v4i sT[FILTER_TG * 8];  // 32 ints per tile
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, g = lane >> 5;
    const uint64_t v0 = ((uint64_t)blockIdx.x * 4 + wave) * (32 * NT);

    v4i b[NT][KS];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        uint64_t v = v0 + nt * 32 + col;
        if (v >= n) v = n - 1;
        const v4i* src = (const v4i*)(X + v * D + g * 16);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) b[nt][ks] = src[ks * 2];
    }
    int32_t best_key[NT];
    uint32_t best_tile[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        best_key[nt] = (int32_t)0x80000000;
        best_tile[nt] = 0;
    }

    for (uint32_t t0 = 0; t0 < tiles; t0 += FILTER_TG) {
        const uint32_t tg = tiles - t0 < FILTER_TG ? tiles - t0 : FILTER_TG;
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < tg * KS * 64; i += 256) sA[i] = Cp[(size_t)t0 * KS * 64 + i];
        for (uint32_t i = threadIdx.x; i < tg * 8; i += 256) sT[i] = T2[(size_t)t0 * 8 + i];
        __syncthreads();
#pragma unroll 1
        for (uint32_t tt = 0; tt < tg; ++tt) {
            v16i acc[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[nt][r] = 0;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                v4i a = sA[(tt * KS + ks) * 64 + lane];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[nt][ks], acc[nt], 0, 0, 0);
            }
            int32_t tc[16];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                v4i t = sT[tt * 8 + g * 4 + q];
                tc[4 * q] = t.x; tc[4 * q + 1] = t.y; tc[4 * q + 2] = t.z; tc[4 * q + 3] = t.w;
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                int32_t key[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) key[r] = (int32_t)(((uint32_t)acc[nt][r] << 5) + (uint32_t)tc[r]);
                if constexpr (STORE) {
                    const uint64_t v = v0 + nt * 32 + col;
                    if (v < n) {
                        int32_t* dst = out + v * ((uint64_t)tiles * 32) + (uint64_t)(t0 + tt) * 32 + 4 * g;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            v4i o = {key[4 * q] >> 4, key[4 * q + 1] >> 4, key[4 * q + 2] >> 4, key[4 * q + 3] >> 4};
                            *(v4i*)(dst + 8 * q) = o;
                        }
                    }
                } else {
                    int32_t m = key[0];
#pragma unroll
                    for (int r = 1; r < 16; ++r) m = key[r] > m ? key[r] : m;
                    // across tiles only the value counts (the low 4 bits rank rows inside one tile); strict,
                    // because an equal value in a later tile is a higher centroid id
                    if ((m | 15) > (best_key[nt] | 15)) {
                        best_key[nt] = m;
                        best_tile[nt] = t0 + tt;
                    }
                }
            }
        }
    }
    if constexpr (!STORE) {
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
    }
}

// ---------------------------------------------------------------------------
// Inverted index.  One wave per document; a vector is the first of its document with its
// centroid if no earlier vector of the document has the same one (a bucket holds a document
// once).  FILL = false counts bucket sizes; FILL = true writes document ids at
// offsets[c] + (atomic cursor), so the order inside a bucket is unspecified.
template <bool FILL>
__global__ __launch_bounds__(256) void filter_bucket_kernel(const uint32_t* __restrict__ assign,
                                                            const uint64_t* __restrict__ doc_off, uint64_t n_docs,
                                                            uint32_t* __restrict__ size_or_cursor,
                                                            const uint32_t* __restrict__ bucket_off,
                                                            uint32_t* __restrict__ bucket_docs) {
    const uint32_t lane = threadIdx.x & 63;
    for (uint64_t doc = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6); doc < n_docs; doc += (uint64_t)gridDim.x * 4) {
        const uint64_t lo = doc_off[doc], hi = doc_off[doc + 1];
        for (uint64_t j = lo + lane; j < hi; j += 64) {
            const uint32_t c = assign[j];
            bool first = true;
            for (uint64_t e = lo; e < j; ++e)
                if (assign[e] == c) {
                    first = false;
                    break;
                }
            if (first) {
                uint32_t pos = atomicAdd(&size_or_cursor[c], 1u);
                if constexpr (FILL) bucket_docs[bucket_off[c] + pos] = (uint32_t)doc;
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

// ---------------------------------------------------------------------------
// Query side.
struct DistKeys {  // key = (value + bias) above the centroid id: closest first, lower id first
    const int32_t* row;
    uint32_t id_bits;
    __device__ uint64_t operator()(uint64_t i) const { return make_key(row[i] + FILTER_BIAS, (uint32_t)i, id_bits); }
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

// one workgroup per (query vector, probe rank): every document of the probed bucket gets +1 in
// its query set's row of counts [B][n_docs]
__global__ __launch_bounds__(256) void filter_count_kernel(const uint32_t* __restrict__ probe_ids, uint32_t probe,
                                                           const uint32_t* __restrict__ q_off, uint32_t q_uniform,
                                                           uint32_t n_queries, const uint32_t* __restrict__ bucket_off,
                                                           const uint32_t* __restrict__ bucket_docs, uint64_t n_docs,
                                                           int32_t* __restrict__ counts) {
    const uint32_t q = blockIdx.x / probe;
    const uint32_t c = probe_ids[blockIdx.x];
    if (c == 0xFFFFFFFFu) return;
    uint32_t b;
    if (q_uniform) {
        b = q / q_uniform;
    } else {  // last query set starting at or before q
        uint32_t lo = 0, hi = n_queries;
        while (hi - lo > 1) {
            uint32_t mid = (lo + hi) / 2;
            if (q_off[mid] <= q) lo = mid; else hi = mid;
        }
        b = lo;
    }
    int32_t* row = counts + (uint64_t)b * n_docs;
    for (uint32_t e = bucket_off[c] + threadIdx.x; e < bucket_off[c + 1]; e += 256) atomicAdd(&row[bucket_docs[e]], 1);
}

// ---------------------------------------------------------------------------
static bool filter_shape(uint32_t d) { return d == 64 || d == 128 || d == 256; }
bool filter_supported(uint32_t d) { return filter_shape(d); }
uint32_t filter_tiles(uint32_t K) { return (K + 31) / 32; }
size_t filter_centroid_bytes(uint32_t K, uint32_t d) { return (size_t)filter_tiles(K) * (d / 32) * 1024; }
size_t filter_table_bytes(uint32_t K) { return (size_t)filter_tiles(K) * 32 * 4; }

hipError_t launch_filter_prep(const int8_t* Cn, uint32_t K, uint32_t d, void* Cp, void* T2, hipStream_t stream) {
    if (!filter_shape(d) || K == 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(filter_prep_kernel, dim3(1024), dim3(256), 0, stream, Cn, K, d, (int8_t*)Cp, (int32_t*)T2,
                       filter_tiles(K));
    return hipGetLastError();
}

template <bool STORE>
static hipError_t launch_gemm(const int8_t* X, uint64_t n, uint32_t d, uint32_t K, const void* Cp, const void* T2,
                              uint32_t* assign, int32_t* out, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    constexpr int NT = 2;
    uint64_t blocks = (n + 4 * 32 * NT - 1) / (4 * 32 * NT);
    if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
    const uint32_t tiles = filter_tiles(K);
    dim3 grid((unsigned)blocks), block(256);
    if (d == 64)
        hipLaunchKernelGGL((filter_gemm_kernel<2, NT, STORE>), grid, block, 0, stream, X, n, (const v4i*)Cp, (const v4i*)T2, tiles, assign, out);
    else if (d == 128)
        hipLaunchKernelGGL((filter_gemm_kernel<4, NT, STORE>), grid, block, 0, stream, X, n, (const v4i*)Cp, (const v4i*)T2, tiles, assign, out);
    else if (d == 256)
        hipLaunchKernelGGL((filter_gemm_kernel<8, NT, STORE>), grid, block, 0, stream, X, n, (const v4i*)Cp, (const v4i*)T2, tiles, assign, out);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_filter_assign(const int8_t* X, uint64_t n, uint32_t d, uint32_t K, const void* Cp, const void* T2,
                                uint32_t* assign, hipStream_t stream) {
    return launch_gemm<false>(X, n, d, K, Cp, T2, assign, nullptr, stream);
}

hipError_t launch_filter_distances(const int8_t* X, uint64_t n, uint32_t d, uint32_t K, const void* Cp, const void* T2,
                                   int32_t* out, hipStream_t stream) {
    return launch_gemm<true>(X, n, d, K, Cp, T2, nullptr, out, stream);
}

hipError_t launch_filter_buckets(const uint32_t* assign, const uint64_t* doc_off, uint64_t n_docs, uint32_t K,
                                 uint32_t* cursor, uint32_t* bucket_off, uint32_t* bucket_docs, hipStream_t stream) {
    uint64_t blocks = (n_docs + 3) / 4;
    if (blocks > 65536) blocks = 65536;
    if (blocks == 0) blocks = 1;
    hipLaunchKernelGGL(filter_zero_kernel, dim3((K + 255) / 256), dim3(256), 0, stream, (int32_t*)cursor, (uint64_t)K);
    hipLaunchKernelGGL(filter_bucket_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, assign, doc_off, n_docs,
                       cursor, bucket_off, bucket_docs);
    hipLaunchKernelGGL(filter_scan_kernel, dim3(1), dim3(1024), 0, stream, cursor, K, bucket_off);
    hipLaunchKernelGGL(filter_bucket_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, assign, doc_off, n_docs,
                       cursor, bucket_off, bucket_docs);
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

hipError_t launch_filter_count(const uint32_t* probe_ids, uint64_t total_q, uint32_t probe, const uint32_t* q_off,
                               uint32_t q_uniform, uint32_t n_queries, const uint32_t* bucket_off,
                               const uint32_t* bucket_docs, uint64_t n_docs, int32_t* counts, hipStream_t stream) {
    const uint64_t cells = (uint64_t)n_queries * n_docs;
    if (cells == 0 || total_q == 0) return hipSuccess;
    if (total_q * probe > 0x7fffffffull) return hipErrorInvalidValue;
    uint64_t zb = (cells + 256 * 8 - 1) / (256 * 8);
    if (zb > 1u << 20) zb = 1u << 20;
    hipLaunchKernelGGL(filter_zero_kernel, dim3((unsigned)zb), dim3(256), 0, stream, counts, cells);
    hipLaunchKernelGGL(filter_count_kernel, dim3((unsigned)(total_q * probe)), dim3(256), 0, stream, probe_ids, probe,
                       q_off, q_uniform, n_queries, bucket_off, bucket_docs, n_docs, counts);
    return hipGetLastError();
}

}  // namespace dessert
