// C ABI of the library (declared in include/dessert.h): argument validation,
// workspace carving and kernel sequencing.  Host-side arithmetic is limited to
// the exclusive scan of the document lengths in dessert_build_index, the L+1
// fixed-point table entries of a score transform (phi or Eq. 1 of the count / L
// values, host libm, in dessert_set_score_transform) and launch-shape planning.
#include "../../include/dessert.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "kernels.hpp"

using namespace dessert;

namespace {

thread_local char g_err[512] = "";

dessert_status_t fail(dessert_status_t st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

#define HIP_TRY(expr)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) return fail(DESSERT_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        ok = hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard() {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

// Workspace of dessert_search_noalloc: one array per GPU, held until the process ends.  In host code the name
// `scratch` is only a handle for hipGetSymbolAddress; the device address it yields (one per device) is what kernels
// and copies get.
constexpr size_t kScratchBytes = DESSERT_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

}  // namespace

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
// Device address of this device's copy of `scratch`; looked up once per device, with that device current.
dessert_status_t scratch_address(int device, void** out) {
    if (device < 0 || device >= kMaxDevices) return fail(DESSERT_EINVAL, "device %d out of range", device);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(DESSERT_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", device, hipGetErrorString(e));
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return DESSERT_OK;
}
}  // namespace

struct dessert_index {
    dessert_config_t cfg{};
    hipStream_t stream = nullptr;
    void* proj = nullptr;       // device, [L*C][d] int8 or float (library-owned copy)
    void* proj_mfma = nullptr;  // device, MFMA-ordered int8 copy (or null)
    uint32_t* remap = nullptr;  // device, [L+1] table of the current score transform in Q16 (library-owned)
    uint32_t remap_max = 0;     // its largest entry
    const uint32_t* q_weights = nullptr;  // caller's, Q16 weights of the query vectors (Sec. 4.2)
    uint64_t n_weights = 0;
    // candidate filter (library-owned: MFMA-ordered centroids, key constants, bucket cursors)
    void* f_cent = nullptr;
    void* f_table = nullptr;
    uint32_t* f_cursor = nullptr;
    uint32_t* f_sub_off = nullptr;   // [K*S+1] sub-bucket starts (library-owned)
    FilterSubPlan f_sub{1, 15};
    uint32_t f_K = 0;
    const uint32_t* f_bucket_off = nullptr;   // caller's
    const uint32_t* f_bucket_docs = nullptr;  // caller's
    uint32_t f_max_bucket = 0;                // most documents in one bucket
    uint32_t f_alloc_K = 0;                   // sizes the filter buffers above were allocated for
    size_t f_alloc_sub = 0;
    bool f_built = false;
    int transform = DESSERT_SCORE_RAW_COUNTS;
    char last_score_kernel[128] = "";  // instantiation launched by the last scoring step (dessert_last_score_kernel)
    bool debug = false;            // dessert_set_debug: candidate ids are range-checked before they are used
    unsigned long long* dbg_flag = nullptr;  // device, the first offending slot found by the checking kernel (library-owned)
    int hash_algo = DESSERT_HASH_AUTO;
    int score_algo = DESSERT_SCORE_AUTO;
    // index state
    const uint8_t* codes = nullptr;
    const uint64_t* offsets = nullptr;
    uint64_t n_docs = 0, n_vectors = 0;
    uint64_t max_len = 0;   // longest document of the index, in vectors
    bool built = false;
    // pinned staging for the offsets upload
    uint64_t* h_offsets = nullptr;
    size_t h_offsets_cap = 0;
    hipEvent_t upload_done = nullptr;  // recorded after each offsets upload
    hipStream_t copy_stream = nullptr; // library-owned: carries the offsets upload beside the hash kernel
    hipEvent_t build_entry = nullptr;  // recorded on the caller's stream when dessert_build_index starts
    bool upload_pending = false;
    // pinned staging ring for the per-batch offset arrays of a search (keeps the uploads asynchronous)
    static constexpr unsigned kMetaSlots = 8;
    struct MetaSlot {
        char* host = nullptr;
        size_t cap = 0;
        hipEvent_t done = nullptr;
        bool pending = false;
    };
    MetaSlot meta[kMetaSlots];
    unsigned meta_next = 0;
    // timing: a ring of event sets so that a run of calls can be timed without synchronising
    struct TimingSlot {
        hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
        bool hash = false, score = false, topk = false, any = false;
    };
    static constexpr unsigned kTimingSlots = 64;
    bool timing = false;
    uint32_t timing_period = 1;   // events are recorded on every timing_period-th call
    uint64_t timing_seen = 0;     // calls since timing was enabled
    TimingSlot slots[kTimingSlots];
    uint64_t timed_calls = 0;
    bool timed_now() { return timing && (timing_seen++ % timing_period) == 0; }
    TimingSlot& begin_timed() {
        TimingSlot& s = slots[timed_calls % kTimingSlots];
        s.hash = s.score = s.topk = s.any = false;
        return s;
    }
};

namespace {

size_t proj_elem_bytes(uint32_t kind) { return kind == DESSERT_PROJ_RADEMACHER_I8 ? 1 : 4; }
// bytes of one table's code: C one-bit hashes packed into one byte, or two when C > 8
uint32_t code_width(const dessert_config_t& c) { return c.C > 8 ? 2u : 1u; }

bool is_i8_mfma(const dessert_config_t& c) {
    return c.dtype == DESSERT_I8 && c.proj_kind == DESSERT_PROJ_RADEMACHER_I8 && hash_mfma_supported(c.d, c.L, c.C);
}
bool is_f16_mfma(const dessert_config_t& c) {
    return c.dtype == DESSERT_F16 && c.proj_kind == DESSERT_PROJ_GAUSSIAN_F32 && hash_mfma_f16_supported(c.d, c.L, c.C);
}
bool use_mfma(const dessert_index* ix) { return ix->proj_mfma && (is_i8_mfma(ix->cfg) || is_f16_mfma(ix->cfg)); }

// fused / fused_done: a candidate grouping to carry along in the hashing launch when that is the int8 MFMA kernel;
// *fused_done tells whether it was.
dessert_status_t run_hash(const dessert_index* ix, const void* X, uint64_t n, uint8_t* codes,
                          const CandOrderArgs* fused = nullptr, bool* fused_done = nullptr) {
    if (fused_done) *fused_done = false;
    if (n == 0) return DESSERT_OK;
    int algo = ix->hash_algo;
    bool aligned = ((uintptr_t)X % 16 == 0) && ((uintptr_t)codes % 16 == 0);
    if (algo == DESSERT_HASH_AUTO) algo = (use_mfma(ix) && aligned) ? DESSERT_HASH_MFMA : DESSERT_HASH_SCALAR;
    if (algo == DESSERT_HASH_MFMA) {
        if (!use_mfma(ix))
            return fail(DESSERT_EINVAL, "MFMA hashing needs int8 vectors with +-1 projections or fp16 vectors with "
                                        "Gaussian projections, d in {64,128,256}, L in {16,32,64} (int8 also L = 8, and 16-bit codes with "
                                        "L in {8,16,32})");
        if (!aligned) return fail(DESSERT_EINVAL, "MFMA hashing needs 16-byte aligned vectors and codes");
        if (ix->cfg.dtype == DESSERT_I8) {
            const bool fuse = fused && fused->ranges <= hash_mfma_fused_ranges(ix->cfg.d, ix->cfg.L, ix->cfg.C);
            HIP_TRY(launch_hash_mfma_i8((const int8_t*)X, n, ix->cfg.d, ix->cfg.L, ix->cfg.C, ix->proj_mfma, codes,
                                        fuse ? fused : nullptr, ix->stream));
            if (fuse && fused_done) *fused_done = true;
        }
        else
            HIP_TRY(launch_hash_mfma_f16(X, n, ix->cfg.d, ix->cfg.L, ix->cfg.C, ix->proj_mfma, codes, ix->stream));
    } else if (algo == DESSERT_HASH_SCALAR) {
        HIP_TRY(launch_hash_scalar(X, ix->cfg.dtype, n, ix->cfg.d, ix->proj, ix->cfg.proj_kind, ix->cfg.L, ix->cfg.C, codes,
                                   ix->stream));
    } else {
        return fail(DESSERT_EINVAL, "unknown hash algorithm %d", algo);
    }
    return DESSERT_OK;
}

// Workspace layout for a search batch (all regions 256-byte aligned).
struct Workspace {
    size_t qcodes, q_off, cand_off, scores, order, partial, total;
};

// The workspace holds room for the id-range order of the candidate slots unless the batch scores as many pairs as
// "every document for every query set" (then there are no candidate lists, or lists that cover everything).
bool order_space(const dessert_index* ix, uint32_t B, uint64_t total_scored) {
    return total_scored < (uint64_t)B * ix->n_docs;
}

Workspace carve(const dessert_index* ix, uint32_t B, uint64_t total_q, uint64_t total_scored, uint64_t max_scored, uint32_t k,
                bool own_scores) {
    Workspace w{};
    size_t p = 0;
    w.qcodes = p;   p += align_up((size_t)total_q * ix->cfg.L * code_width(ix->cfg), 256);
    w.q_off = p;    p += align_up(((size_t)B + 1) * 4, 256);
    w.cand_off = p; p += align_up(((size_t)B + 1) * 8, 256);
    w.scores = p;   if (own_scores) p += align_up((size_t)total_scored * 4, 256);
    // candidate slots by id range (see order_space)
    w.order = p;    if (order_space(ix, B, total_scored)) p += align_up((size_t)total_scored * 4, 256);
    w.partial = p;
    uint32_t slices = topk_slices(max_scored, B);
    if (k && slices > 1) p += align_up((size_t)B * slices * k * 8, 256);
    w.total = p;
    return w;
}

struct Batch {
    std::vector<uint32_t> q_off;
    uint64_t total_q = 0, total_scored = 0, max_scored = 0;
    uint32_t max_q_len = 0;
    uint32_t q_uniform = 0;      // common query-set length, 0 if they differ
    uint64_t cand_uniform = 0;   // common candidate-list length, 0 if they differ (or no candidates)
};

// Asynchronous upload of a small host array through one of the handle's pinned staging slots (a slot is reused
// only after the copy that read it has finished).
dessert_status_t upload_small(dessert_index* ix, const void* src, size_t bytes, void* dst_dev) {
    dessert_index::MetaSlot& ms = ix->meta[ix->meta_next++ % dessert_index::kMetaSlots];
    if (ms.pending) {
        HIP_TRY(hipEventSynchronize(ms.done));
        ms.pending = false;
    }
    if (ms.cap < bytes) {
        if (ms.host) (void)hipHostFree(ms.host);
        ms.host = nullptr;
        ms.cap = 0;
        hipError_t e = hipHostMalloc((void**)&ms.host, 2 * bytes, hipHostMallocDefault);
        if (e != hipSuccess) return fail(DESSERT_ENOMEM, "hipHostMalloc(batch offsets): %s", hipGetErrorString(e));
        ms.cap = 2 * bytes;
    }
    if (!ms.done) HIP_TRY(hipEventCreateWithFlags(&ms.done, hipEventDisableTiming));
    memcpy(ms.host, src, bytes);
    HIP_TRY(hipMemcpyAsync(dst_dev, ms.host, bytes, hipMemcpyHostToDevice, ix->stream));
    HIP_TRY(hipEventRecord(ms.done, ix->stream));
    ms.pending = true;
    return DESSERT_OK;
}

dessert_status_t check_batch(const dessert_index* ix, const void* q_vectors, const uint32_t* q_lengths, uint32_t B,
                             const uint32_t* cand_ids, const uint64_t* cand_off, Batch* out) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (!ix->built) return fail(DESSERT_ESTATE, "dessert_build_index has not been called");
    if (B == 0) return DESSERT_OK;
    if (B > 65535) return fail(DESSERT_EINVAL, "n_queries > 65535");
    if (!q_vectors || !q_lengths) return fail(DESSERT_EINVAL, "q_vectors_dev / q_lengths_host is NULL");
    out->q_off.assign(B + 1, 0);
    for (uint32_t b = 0; b < B; ++b) {
        if (q_lengths[b] == 0) return fail(DESSERT_EINVAL, "q_lengths_host[%u] = 0", b);
        if ((uint64_t)q_lengths[b] * ix->cfg.L * code_width(ix->cfg) > 65535)
            return fail(DESSERT_EINVAL, "q_lengths_host[%u]: the query set's codes (%llu bytes) exceed 65535 bytes", b,
                        (unsigned long long)q_lengths[b] * ix->cfg.L * code_width(ix->cfg));
        uint64_t nxt = (uint64_t)out->q_off[b] + q_lengths[b];
        if (nxt > 0xFFFFFFFFull) return fail(DESSERT_EINVAL, "more than 2^32-1 query vectors");
        out->q_off[b + 1] = (uint32_t)nxt;
        if (q_lengths[b] > out->max_q_len) out->max_q_len = q_lengths[b];
    }
    out->total_q = out->q_off[B];
    out->q_uniform = q_lengths[0];
    for (uint32_t b = 1; b < B; ++b)
        if (q_lengths[b] != q_lengths[0]) out->q_uniform = 0;
    if (cand_ids) {
        if (!cand_off) return fail(DESSERT_EINVAL, "cand_offsets_host is NULL with candidate ids given");
        if (cand_off[0] != 0) return fail(DESSERT_EINVAL, "cand_offsets_host[0] must be 0");
        for (uint32_t b = 0; b < B; ++b) {
            if (cand_off[b + 1] < cand_off[b]) return fail(DESSERT_EINVAL, "cand_offsets_host not non-decreasing at %u", b);
            uint64_t c = cand_off[b + 1] - cand_off[b];
            if (c > out->max_scored) out->max_scored = c;
        }
        out->total_scored = cand_off[B];
        out->cand_uniform = cand_off[1];
        for (uint32_t b = 1; b < B; ++b)
            if (cand_off[b + 1] - cand_off[b] != cand_off[1]) out->cand_uniform = 0;
    } else {
        out->max_scored = ix->n_docs;
        out->total_scored = (uint64_t)B * ix->n_docs;
    }
    if (out->max_scored > 0x7FFFFFFFull * 64) return fail(DESSERT_EINVAL, "too many documents per query set");
    return DESSERT_OK;
}

// The same checks for a batch whose query sets all have q_len vectors and whose candidate lists all have cand_len
// ids: nothing is read from host arrays and nothing is allocated.
dessert_status_t check_uniform_batch(const dessert_index* ix, const void* q_vectors, uint32_t q_len, uint32_t B,
                                     const uint32_t* cand_ids, uint64_t cand_len, Batch* out) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (!ix->built) return fail(DESSERT_ESTATE, "dessert_build_index has not been called");
    if (B == 0) return DESSERT_OK;
    if (B > 65535) return fail(DESSERT_EINVAL, "n_queries > 65535");
    if (!q_vectors) return fail(DESSERT_EINVAL, "q_vectors_dev is NULL");
    if (q_len == 0) return fail(DESSERT_EINVAL, "q_length = 0");
    if ((uint64_t)q_len * ix->cfg.L * code_width(ix->cfg) > 65535)
        return fail(DESSERT_EINVAL, "q_length: the query set's codes (%llu bytes) exceed 65535 bytes",
                    (unsigned long long)q_len * ix->cfg.L * code_width(ix->cfg));
    if ((uint64_t)q_len * B > 0xFFFFFFFFull) return fail(DESSERT_EINVAL, "more than 2^32-1 query vectors");
    out->total_q = (uint64_t)q_len * B;
    out->max_q_len = out->q_uniform = q_len;
    if (cand_ids) {
        if (cand_len == 0) return fail(DESSERT_EINVAL, "cand_length = 0 with candidate ids given");
        out->max_scored = out->cand_uniform = cand_len;
        out->total_scored = cand_len * B;
    } else {
        out->max_scored = ix->n_docs;
        out->total_scored = (uint64_t)B * ix->n_docs;
    }
    if (out->max_scored > 0x7FFFFFFFull * 64) return fail(DESSERT_EINVAL, "too many documents per query set");
    return DESSERT_OK;
}

// Is the handle's stream being captured into a HIP graph?  (A failed query counts as "no".)
bool stream_capturing(const dessert_index* ix) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(ix->stream, &cs) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return cs != hipStreamCaptureStatusNone;
}

// Shared body of dessert_search (k > 0), dessert_scores (k == 0) and dessert_search_noalloc, after the batch has
// been checked.  cand_off: host offsets, read only when the candidate lists have unequal lengths.
dessert_status_t search_impl(dessert_index* ix, const Batch& bt, const void* q_vectors, uint32_t B,
                             const uint32_t* cand_ids, const uint64_t* cand_off, uint32_t k, void* workspace,
                             size_t workspace_bytes, int32_t* scores_out, uint32_t* out_ids, int32_t* out_scores) {
    dessert_status_t st = DESSERT_OK;
    if (B == 0) return DESSERT_OK;
    if (ix->transform != DESSERT_SCORE_RAW_COUNTS && bt.max_q_len > 16383)
        return fail(DESSERT_EINVAL, "the fixed-point score transforms need query sets of at most 16383 vectors");
    if (ix->q_weights && ix->transform == DESSERT_SCORE_RAW_COUNTS)
        return fail(DESSERT_EINVAL, "query weights need a fixed-point (*_Q16) score transform");
    if (ix->q_weights && ix->n_weights != bt.total_q)
        return fail(DESSERT_EINVAL, "%llu query weights set, the batch has %llu query vectors",
                    (unsigned long long)ix->n_weights, (unsigned long long)bt.total_q);
    if (!workspace) return fail(DESSERT_EINVAL, "workspace_dev is NULL");
    if ((uintptr_t)workspace % 256) return fail(DESSERT_EINVAL, "workspace_dev must be 256-byte aligned");
    const bool own_scores = scores_out == nullptr;
    Workspace w = carve(ix, B, bt.total_q, bt.total_scored, bt.max_scored, k, own_scores);
    if (workspace_bytes < w.total)
        return fail(DESSERT_EINVAL, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, w.total);
    DeviceGuard guard(ix->cfg.device);
    if (!guard.ok) return fail(DESSERT_EHIP, "hipSetDevice(%d) failed", ix->cfg.device);

    char* ws = (char*)workspace;
    uint8_t* qcodes = (uint8_t*)(ws + w.qcodes);
    uint32_t* d_q_off = (uint32_t*)(ws + w.q_off);
    uint64_t* d_cand_off = (uint64_t*)(ws + w.cand_off);
    int32_t* scores = own_scores ? (int32_t*)(ws + w.scores) : scores_out;

    // Offset arrays are uploaded only when the lengths differ (equal lengths travel as kernel
    // arguments); they go through a pinned slot so that the uploads never block the host.
    const bool need_q = bt.q_uniform == 0, need_c = cand_ids && bt.cand_uniform == 0;
    // Under graph capture only a fixed sequence of kernel launches can be recorded: an offsets upload would replay
    // whatever a later call left in the pinned slot, and event records or a read-back cannot be captured at all.
    const bool capturing = stream_capturing(ix);
    if (capturing && (need_q || need_c))
        return fail(DESSERT_ESTATE, "graph capture needs query sets of equal length and candidate lists of equal length");
    if (capturing && ix->debug && cand_ids)
        return fail(DESSERT_ESTATE, "graph capture is not possible in debug mode (the id check reads a flag back)");
    if (ix->debug && cand_ids) {  // range-check the ids before any kernel uses them as indices
        unsigned long long bad_slot = 0;
        HIP_TRY(launch_check_cand_ids(cand_ids, bt.total_scored, ix->n_docs, ix->dbg_flag, ix->stream));
        HIP_TRY(hipMemcpyAsync(&bad_slot, ix->dbg_flag, sizeof(bad_slot), hipMemcpyDeviceToHost, ix->stream));
        HIP_TRY(hipStreamSynchronize(ix->stream));
        if (bad_slot != ~0ull)
            return fail(DESSERT_EINVAL, "cand_ids_dev[%llu] is neither below n_docs = %llu nor the empty-slot value 0xFFFFFFFF",
                        bad_slot, (unsigned long long)ix->n_docs);
    }
    const bool timed = !capturing && ix->timed_now();
    dessert_index::TimingSlot* tsp = timed ? &ix->begin_timed() : nullptr;
    if (timed) HIP_TRY(hipEventRecord(tsp->ev[0], ix->stream));
    if (need_q || need_c) {
        dessert_index::MetaSlot& ms = ix->meta[ix->meta_next++ % dessert_index::kMetaSlots];
        if (ms.pending) {
            HIP_TRY(hipEventSynchronize(ms.done));
            ms.pending = false;
        }
        const size_t qb = align_up(((size_t)B + 1) * 4, 256), cb = ((size_t)B + 1) * 8;
        if (ms.cap < qb + cb) {
            if (ms.host) (void)hipHostFree(ms.host);
            ms.host = nullptr;
            ms.cap = 0;
            hipError_t e = hipHostMalloc((void**)&ms.host, 2 * (qb + cb), hipHostMallocDefault);
            if (e != hipSuccess) return fail(DESSERT_ENOMEM, "hipHostMalloc(batch offsets): %s", hipGetErrorString(e));
            ms.cap = 2 * (qb + cb);
        }
        if (!ms.done) HIP_TRY(hipEventCreateWithFlags(&ms.done, hipEventDisableTiming));
        if (need_q) {
            memcpy(ms.host, bt.q_off.data(), ((size_t)B + 1) * 4);
            HIP_TRY(hipMemcpyAsync(d_q_off, ms.host, ((size_t)B + 1) * 4, hipMemcpyHostToDevice, ix->stream));
        }
        if (need_c) {
            memcpy(ms.host + qb, cand_off, cb);
            HIP_TRY(hipMemcpyAsync(d_cand_off, ms.host + qb, cb, hipMemcpyHostToDevice, ix->stream));
        }
        HIP_TRY(hipEventRecord(ms.done, ix->stream));
        ms.pending = true;
    }

    ScoreArgs sa{};
    sa.codes = ix->codes; sa.offsets = ix->offsets; sa.n_docs = ix->n_docs;
    sa.L = ix->cfg.L; sa.C = ix->cfg.C; sa.code_bytes = code_width(ix->cfg);
    sa.qcodes = qcodes; sa.q_off = d_q_off; sa.q_uniform = bt.q_uniform; sa.n_queries = B; sa.max_q_len = bt.max_q_len;
    sa.cand_ids = cand_ids; sa.cand_off = cand_ids ? d_cand_off : nullptr; sa.cand_uniform = cand_ids ? bt.cand_uniform : 0;
    sa.max_scored = bt.max_scored; sa.total_scored = bt.total_scored; sa.n_vectors = ix->n_vectors; sa.scores = scores;
    sa.remap = ix->transform != DESSERT_SCORE_RAW_COUNTS ? ix->remap : nullptr;
    sa.sigma_mean = ix->transform >= DESSERT_SCORE_MEAN_IDENTITY_Q16 ? 1u : 0u;
    // phi = identity with L a power of two: the table is 65536 / L * count exactly
    sa.phi_identity = ((ix->transform == DESSERT_SCORE_MEAN_IDENTITY_Q16 || ix->transform == DESSERT_SCORE_MAX_IDENTITY_Q16) &&
                       (ix->cfg.L & (ix->cfg.L - 1)) == 0) ? 1u : 0u;
    sa.q_weights = ix->q_weights;
    int algo = ix->score_algo;
    // sigma = mean has a mask-table form for phi = identity only (sums of counts), and for documents short enough
    const bool mean_on_masklut = sa.sigma_mean && sa.phi_identity && ix->max_len <= MASKLUT_MEAN_MAX_LEN;
    if (algo == DESSERT_SCORE_AUTO && sa.sigma_mean && !mean_on_masklut) algo = DESSERT_SCORE_BYTECMP;
    // the mask-table kernel lets idle lanes read code row 0, so it needs a non-empty code array
    if (algo == DESSERT_SCORE_AUTO || ix->n_vectors == 0)
        algo = (score_masklut_supported(ix->cfg.L, ix->cfg.C) && ix->n_vectors) ? DESSERT_SCORE_MASKLUT
                                                                                : DESSERT_SCORE_BYTECMP;
    // Query preparation: the query codes and, for the mask-table kernel with long candidate lists, each list's slots
    // grouped by document id range (with fewer than 8 lists the one workgroup per list of the grouping costs more
    // than the scoring gains).  The grouping rides in the hashing launch when that is the int8 MFMA kernel.
    CandOrderArgs oa{};
    bool grouping = algo == DESSERT_SCORE_MASKLUT && score_masklut_supported(ix->cfg.L, ix->cfg.C) &&
                    cand_ids && B >= 8 && bt.max_scored >= score_order_min() && order_space(ix, B, bt.total_scored);
    if (grouping) {
        const uint32_t fused_ranges = hash_mfma_fused_ranges(ix->cfg.d, ix->cfg.L, ix->cfg.C);
        grouping = cand_order_plan(cand_ids, sa.cand_off, sa.cand_uniform, B, bt.max_scored, ix->n_docs,
                                   fused_ranges >= 32 ? fused_ranges : 4096, (uint32_t*)(ws + w.order), &oa);
    }
    bool grouped = false;
    st = run_hash(ix, q_vectors, bt.total_q, qcodes, grouping ? &oa : nullptr, &grouped);
    if (st != DESSERT_OK) return st;
    if (grouping && !grouped) HIP_TRY(launch_cand_order(oa, ix->stream));
    if (grouping) sa.order = oa.order;
    if (timed) { HIP_TRY(hipEventRecord(tsp->ev[1], ix->stream)); tsp->hash = true; }
    if (algo == DESSERT_SCORE_MASKLUT) {
        if (sa.sigma_mean && !mean_on_masklut)
            return fail(DESSERT_EINVAL, "of the MEAN score transforms only MEAN_IDENTITY has a mask-table form (documents of at "
                                        "most 65535 vectors); the others run on the code-compare kernel only");
        if (!score_masklut_supported(ix->cfg.L, ix->cfg.C))
            return fail(DESSERT_EINVAL, "mask-table scoring needs L in {8,16,32,64,128} (C <= 8), or L = 8 with C <= 11, "
                                        "L = 16 with C <= 10, L = 32 with C = 9");
        HIP_TRY(launch_score_masklut(sa, ix->stream, ix->last_score_kernel, sizeof(ix->last_score_kernel)));
    } else if (algo == DESSERT_SCORE_BYTECMP) {
        HIP_TRY(launch_score_bytecmp(sa, ix->stream, ix->last_score_kernel, sizeof(ix->last_score_kernel)));
    } else {
        return fail(DESSERT_EINVAL, "unknown scoring algorithm %d", algo);
    }
    if (timed) { HIP_TRY(hipEventRecord(tsp->ev[2], ix->stream)); tsp->score = true; }

    if (k) {
        TopkArgs ta{};
        ta.scores = scores; ta.cand_ids = cand_ids; ta.cand_off = sa.cand_off; ta.cand_uniform = sa.cand_uniform; ta.n_docs = ix->n_docs;
        ta.n_queries = B; ta.max_scored = bt.max_scored; ta.k = k; ta.max_score = sa.remap ? bt.max_q_len * ix->remap_max : bt.max_q_len * ix->cfg.L;
        ta.partial = (uint64_t*)(ws + w.partial); ta.out_ids = out_ids; ta.out_scores = out_scores;
        HIP_TRY(launch_topk(ta, ix->stream));
        if (timed) { HIP_TRY(hipEventRecord(tsp->ev[3], ix->stream)); tsp->topk = true; }
    }
    if (timed) { HIP_TRY(hipEventRecord(tsp->ev[4], ix->stream)); tsp->any = true; ++ix->timed_calls; }
    return DESSERT_OK;
}

}  // namespace

extern "C" {

const char* dessert_last_error(void) { return g_err; }

dessert_status_t dessert_probe_read_bandwidth(const void* buf_dev, size_t bytes, int device, void* stream, int reps,
                                              float* ms_per_pass) {
    if (!buf_dev || !ms_per_pass || bytes < 16 || reps < 1) return fail(DESSERT_EINVAL, "bad probe arguments");
    if ((uintptr_t)buf_dev % 16) return fail(DESSERT_EINVAL, "probe buffer must be 16-byte aligned");
    DeviceGuard guard(device);
    if (!guard.ok) return fail(DESSERT_EHIP, "hipSetDevice(%d) failed", device);
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    if (hipError_t ec = hipEventCreate(&e1); ec != hipSuccess) {
        (void)hipEventDestroy(e0);
        return fail(DESSERT_EHIP, "hipEventCreate: %s", hipGetErrorString(ec));
    }
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = launch_read_probe(buf_dev, bytes, st);  // warm-up
    if (e == hipSuccess) e = hipEventRecord(e0, st);
    for (int r = 0; r < reps && e == hipSuccess; ++r) e = launch_read_probe(buf_dev, bytes, st);
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return fail(DESSERT_EHIP, "read probe: %s", hipGetErrorString(e));
    *ms_per_pass = ms / (float)reps;
    return DESSERT_OK;
}
dessert_status_t dessert_probe_mix_bandwidth(const void* in_dev, void* out_dev, size_t out_bytes, int device, void* stream,
                                            int reps, float* ms_per_pass) {
    if (!in_dev || !out_dev || !ms_per_pass || out_bytes < 16 || reps < 1) return fail(DESSERT_EINVAL, "bad probe arguments");
    if ((uintptr_t)in_dev % 16 || (uintptr_t)out_dev % 16) return fail(DESSERT_EINVAL, "probe buffers must be 16-byte aligned");
    DeviceGuard guard(device);
    if (!guard.ok) return fail(DESSERT_EHIP, "hipSetDevice(%d) failed", device);
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    if (hipError_t ec = hipEventCreate(&e1); ec != hipSuccess) {
        (void)hipEventDestroy(e0);
        return fail(DESSERT_EHIP, "hipEventCreate: %s", hipGetErrorString(ec));
    }
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = launch_mix_probe(in_dev, out_dev, out_bytes, st);  // warm-up
    if (e == hipSuccess) e = hipEventRecord(e0, st);
    for (int r = 0; r < reps && e == hipSuccess; ++r) e = launch_mix_probe(in_dev, out_dev, out_bytes, st);
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return fail(DESSERT_EHIP, "mix probe: %s", hipGetErrorString(e));
    *ms_per_pass = ms / (float)reps;
    return DESSERT_OK;
}
const char* dessert_version(void) { return "dessert-gfx950 0.2"; }

dessert_status_t dessert_create(const dessert_config_t* c, dessert_index_t** out) {
    if (!c || !out) return fail(DESSERT_EINVAL, "config or out is NULL");
    *out = nullptr;
    if (c->d == 0) return fail(DESSERT_EINVAL, "d must be >= 1");
    if (c->C < 1 || c->C > 16) return fail(DESSERT_EINVAL, "C must be in 1..16, got %u", c->C);
    if (c->L < 4 || c->L > 128 || c->L % 4) return fail(DESSERT_EINVAL, "L must be a multiple of 4 in 4..128, got %u", c->L);
    if (c->dtype != DESSERT_I8 && c->dtype != DESSERT_F16) return fail(DESSERT_EINVAL, "unknown dtype %u", c->dtype);
    if (c->proj_kind != DESSERT_PROJ_RADEMACHER_I8 && c->proj_kind != DESSERT_PROJ_GAUSSIAN_F32)
        return fail(DESSERT_EINVAL, "unknown proj_kind %u", c->proj_kind);
    if (!c->proj_dev && c->proj_kind == DESSERT_PROJ_GAUSSIAN_F32)
        return fail(DESSERT_EINVAL, "a Gaussian projection matrix must be passed in proj_dev");
    if ((uint64_t)c->d * c->L * c->C > (1ull << 31)) return fail(DESSERT_EINVAL, "projection matrix too large");
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0)
        return fail(DESSERT_EHIP, "no HIP device available: this library has no CPU path");
    if (c->device < 0 || c->device >= ndev) return fail(DESSERT_EINVAL, "device %d out of range (0..%d)", c->device, ndev - 1);

    DeviceGuard guard(c->device);
    if (!guard.ok) return fail(DESSERT_EHIP, "hipSetDevice(%d) failed", c->device);
    {   // the allocation-free entry point works in this device's copy of the scratch array
        void* sp = nullptr;
        dessert_status_t st = scratch_address(c->device, &sp);
        if (st != DESSERT_OK) return st;
    }
    dessert_index* ix = new (std::nothrow) dessert_index();
    if (!ix) return fail(DESSERT_ENOMEM, "out of host memory");
    ix->cfg = *c;
    ix->cfg.proj_dev = nullptr;
    ix->stream = (hipStream_t)c->stream;
    const size_t P = (size_t)c->L * c->C;
    const size_t pbytes = P * c->d * proj_elem_bytes(c->proj_kind);
    hipError_t e = hipMalloc(&ix->proj, pbytes);
    if (e != hipSuccess) {
        delete ix;
        return fail(DESSERT_ENOMEM, "hipMalloc(projection, %zu): %s", pbytes, hipGetErrorString(e));
    }
    if (c->proj_dev)
        e = hipMemcpyAsync(ix->proj, c->proj_dev, pbytes, hipMemcpyDeviceToDevice, ix->stream);
    else
        e = launch_rademacher(c->seed, (uint32_t)P, c->d, (int8_t*)ix->proj, ix->stream);
    if (e == hipSuccess && is_i8_mfma(*c)) {
        e = hipMalloc(&ix->proj_mfma, mfma_proj_bytes(c->d, c->L, c->C));
        if (e == hipSuccess) e = launch_repack_proj_i8((const int8_t*)ix->proj, c->d, c->L, c->C, ix->proj_mfma, ix->stream);
    } else if (e == hipSuccess && is_f16_mfma(*c)) {
        e = hipMalloc(&ix->proj_mfma, mfma_f16_proj_bytes(c->d, c->L));
        if (e == hipSuccess) e = launch_repack_proj_f16((const float*)ix->proj, c->d, c->L, c->C, ix->proj_mfma, ix->stream);
    }
    if (e == hipSuccess) e = hipMalloc((void**)&ix->remap, SCORE_TABLE_MAX * sizeof(uint32_t));
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ix->upload_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ix->build_entry, hipEventDisableTiming);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&ix->copy_stream, hipStreamNonBlocking);
    if (e != hipSuccess) {
        dessert_destroy(ix);
        return fail(DESSERT_EHIP, "projection setup: %s", hipGetErrorString(e));
    }
    *out = ix;
    return DESSERT_OK;
}

void dessert_destroy(dessert_index_t* ix) {
    if (!ix) return;
    DeviceGuard guard(ix->cfg.device);
    (void)hipStreamSynchronize(ix->stream);
    if (ix->copy_stream) {
        (void)hipStreamSynchronize(ix->copy_stream);
        (void)hipStreamDestroy(ix->copy_stream);
    }
    if (ix->upload_done) (void)hipEventDestroy(ix->upload_done);
    if (ix->build_entry) (void)hipEventDestroy(ix->build_entry);
    if (ix->proj) (void)hipFree(ix->proj);
    if (ix->proj_mfma) (void)hipFree(ix->proj_mfma);
    if (ix->remap) (void)hipFree(ix->remap);
    if (ix->dbg_flag) (void)hipFree(ix->dbg_flag);
    if (ix->f_cent) (void)hipFree(ix->f_cent);
    if (ix->f_table) (void)hipFree(ix->f_table);
    if (ix->f_cursor) (void)hipFree(ix->f_cursor);
    if (ix->f_sub_off) (void)hipFree(ix->f_sub_off);
    if (ix->h_offsets) (void)hipHostFree(ix->h_offsets);
    for (auto& slot : ix->slots)
        for (auto& ev : slot.ev)
            if (ev) (void)hipEventDestroy(ev);
    for (auto& m : ix->meta) {
        if (m.host) (void)hipHostFree(m.host);
        if (m.done) (void)hipEventDestroy(m.done);
    }
    delete ix;
}

dessert_status_t dessert_get_projection(const dessert_index_t* ix, void* proj_out_dev) {
    if (!ix || !proj_out_dev) return fail(DESSERT_EINVAL, "NULL argument");
    DeviceGuard guard(ix->cfg.device);
    size_t bytes = (size_t)ix->cfg.L * ix->cfg.C * ix->cfg.d * proj_elem_bytes(ix->cfg.proj_kind);
    HIP_TRY(hipMemcpyAsync(proj_out_dev, ix->proj, bytes, hipMemcpyDeviceToDevice, ix->stream));
    return DESSERT_OK;
}

dessert_status_t dessert_set_algo(dessert_index_t* ix, int hash_algo, int score_algo) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (hash_algo < 0 || hash_algo > DESSERT_HASH_MFMA) return fail(DESSERT_EINVAL, "unknown hash algorithm %d", hash_algo);
    if (score_algo < 0 || score_algo > DESSERT_SCORE_MASKLUT)
        return fail(DESSERT_EINVAL, "unknown scoring algorithm %d", score_algo);
    ix->hash_algo = hash_algo;
    ix->score_algo = score_algo;
    return DESSERT_OK;
}

dessert_status_t dessert_set_score_transform(dessert_index_t* ix, int transform) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (transform < DESSERT_SCORE_RAW_COUNTS || transform > DESSERT_SCORE_MEAN_SIGMOID_Q16)
        return fail(DESSERT_EINVAL, "unknown score transform %d", transform);
    if (transform != DESSERT_SCORE_RAW_COUNTS && transform != ix->transform) {
        // phi(count / L) for the L+1 possible collision counts, in Q16
        DeviceGuard guard(ix->cfg.device);
        const uint32_t L = ix->cfg.L, C = ix->cfg.C;
        std::vector<uint32_t> tab(L + 1, 0);
        uint32_t mx = 0;
        for (uint32_t c = 1; c <= L; ++c) {
            const double s = (double)c / (double)L;
            double y;
            switch (transform) {
                case DESSERT_SCORE_EQ1_Q16: y = std::exp(std::log(s) / (double)C); break;  // Eq. 1: s^(1/C)
                case DESSERT_SCORE_MAX_IDENTITY_Q16:
                case DESSERT_SCORE_MEAN_IDENTITY_Q16: y = s; break;
                case DESSERT_SCORE_MAX_EXPM1_Q16:
                case DESSERT_SCORE_MEAN_EXPM1_Q16: y = std::exp(s) - 1.0; break;
                default: y = 1.0 / (1.0 + std::exp(-s)) - 0.5; break;
            }
            tab[c] = (uint32_t)std::llround(65536.0 * y);
            mx = std::max(mx, tab[c]);
        }
        // written by a launch that carries the values as its argument: behind the searches in flight that still read the
        // old table, before those that follow; nothing to wait for
        HIP_TRY(launch_write_table(tab.data(), L + 1, ix->remap, ix->stream));
        ix->remap_max = mx;
    }
    ix->transform = transform;
    return DESSERT_OK;
}

dessert_status_t dessert_set_query_weights(dessert_index_t* ix, const uint32_t* weights_dev, uint64_t n_weights) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (weights_dev && n_weights == 0) return fail(DESSERT_EINVAL, "n_weights is 0");
    ix->q_weights = weights_dev;
    ix->n_weights = weights_dev ? n_weights : 0;
    return DESSERT_OK;
}

size_t dessert_code_bytes(const dessert_index_t* ix, uint64_t n_vectors) {
    return ix ? (size_t)n_vectors * ix->cfg.L * code_width(ix->cfg) : 0;
}

dessert_status_t dessert_hash(const dessert_index_t* ix, const void* vectors_dev, uint64_t n, uint8_t* codes_dev) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (n == 0) return DESSERT_OK;
    if (!vectors_dev || !codes_dev) return fail(DESSERT_EINVAL, "vectors_dev / codes_dev is NULL");
    if (n > (1ull << 40)) return fail(DESSERT_EINVAL, "n too large");
    DeviceGuard guard(ix->cfg.device);
    if (!guard.ok) return fail(DESSERT_EHIP, "hipSetDevice(%d) failed", ix->cfg.device);
    return run_hash(ix, vectors_dev, n, codes_dev);
}

dessert_status_t dessert_build_index(dessert_index_t* ix, const void* vectors_dev, uint64_t n_vectors,
                                     const uint32_t* lengths_host, uint64_t n_docs, uint8_t* codes_dev,
                                     uint64_t* offsets_dev) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (!offsets_dev) return fail(DESSERT_EINVAL, "offsets_dev is NULL");
    if (n_docs && !lengths_host) return fail(DESSERT_EINVAL, "lengths_host is NULL");
    if (n_vectors && (!vectors_dev || !codes_dev)) return fail(DESSERT_EINVAL, "vectors_dev / codes_dev is NULL");
    if (n_docs > 0xFFFFFFFEull) return fail(DESSERT_EINVAL, "document ids are 32-bit: n_docs too large");
    uint64_t sum = 0, longest = 0;
    for (uint64_t i = 0; i < n_docs; ++i) {
        sum += lengths_host[i];
        if (lengths_host[i] > longest) longest = lengths_host[i];
    }
    if (sum != n_vectors)
        return fail(DESSERT_EINVAL, "sum of lengths_host (%llu) != n_vectors (%llu)", (unsigned long long)sum,
                    (unsigned long long)n_vectors);
    DeviceGuard guard(ix->cfg.device);
    if (!guard.ok) return fail(DESSERT_EHIP, "hipSetDevice(%d) failed", ix->cfg.device);
    if (stream_capturing(ix))
        return fail(DESSERT_ESTATE, "dessert_build_index cannot be captured into a graph (it uploads the offsets from a "
                                    "staging buffer that later calls reuse)");
    // a new collection: the old index and any candidate filter built over it are gone
    ix->built = false;
    ix->f_built = false;
    ix->f_K = 0;
    const bool timed = ix->timed_now();
    dessert_index::TimingSlot* tsp = timed ? &ix->begin_timed() : nullptr;
    if (timed) HIP_TRY(hipEventRecord(tsp->ev[0], ix->stream));
    // The code layout does not depend on document boundaries, so hashing starts first, the host
    // scans the lengths while the GPU works, and the offsets go up on the library's own stream
    // beside the hash kernel: after whatever the caller's stream held at entry (it may still read
    // offsets_dev), and the caller's stream waits for the upload at the end.
    HIP_TRY(hipEventRecord(ix->build_entry, ix->stream));
    dessert_status_t st = run_hash(ix, vectors_dev, n_vectors, codes_dev);
    if (st != DESSERT_OK) return st;
    if (timed) { HIP_TRY(hipEventRecord(tsp->ev[1], ix->stream)); tsp->hash = true; }
    // the staging buffer may still feed the previous build's upload (enqueued before this hash launch)
    if (ix->upload_pending) {
        HIP_TRY(hipEventSynchronize(ix->upload_done));
        ix->upload_pending = false;
    }
    if (ix->h_offsets_cap < n_docs + 1) {
        if (ix->h_offsets) (void)hipHostFree(ix->h_offsets);
        ix->h_offsets = nullptr;
        ix->h_offsets_cap = 0;
        hipError_t e = hipHostMalloc((void**)&ix->h_offsets, (n_docs + 1) * 8, hipHostMallocDefault);
        if (e != hipSuccess) return fail(DESSERT_ENOMEM, "hipHostMalloc(offsets): %s", hipGetErrorString(e));
        ix->h_offsets_cap = n_docs + 1;
    }
    uint64_t run = 0;
    for (uint64_t i = 0; i < n_docs; ++i) {
        ix->h_offsets[i] = run;
        run += lengths_host[i];
    }
    ix->h_offsets[n_docs] = run;
    HIP_TRY(hipStreamWaitEvent(ix->copy_stream, ix->build_entry, 0));
    HIP_TRY(hipMemcpyAsync(offsets_dev, ix->h_offsets, (n_docs + 1) * 8, hipMemcpyHostToDevice, ix->copy_stream));
    HIP_TRY(hipEventRecord(ix->upload_done, ix->copy_stream));
    HIP_TRY(hipStreamWaitEvent(ix->stream, ix->upload_done, 0));
    ix->upload_pending = true;
    if (timed) { HIP_TRY(hipEventRecord(tsp->ev[4], ix->stream)); tsp->any = true; ++ix->timed_calls; }
    ix->codes = codes_dev;
    ix->offsets = offsets_dev;
    ix->n_docs = n_docs;
    ix->n_vectors = n_vectors;
    ix->max_len = longest;
    ix->built = true;
    return DESSERT_OK;
}

dessert_status_t dessert_attach_index(dessert_index_t* ix, const uint8_t* codes_dev, const uint64_t* offsets_dev, uint64_t n_docs,
                                      uint64_t n_vectors, uint64_t max_length) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (!offsets_dev) return fail(DESSERT_EINVAL, "offsets_dev is NULL");
    if (n_vectors && !codes_dev) return fail(DESSERT_EINVAL, "codes_dev is NULL");
    if (n_docs > 0xFFFFFFFEull) return fail(DESSERT_EINVAL, "document ids are 32-bit: n_docs too large");
    if (max_length > n_vectors) return fail(DESSERT_EINVAL, "max_length (%llu) exceeds n_vectors (%llu)",
                                            (unsigned long long)max_length, (unsigned long long)n_vectors);
    if (n_vectors && max_length == 0) return fail(DESSERT_EINVAL, "max_length is 0 with n_vectors > 0");
    // a new collection: any candidate filter built over the previous one is gone
    ix->f_built = false;
    ix->f_K = 0;
    ix->codes = codes_dev;
    ix->offsets = offsets_dev;
    ix->n_docs = n_docs;
    ix->n_vectors = n_vectors;
    ix->max_len = max_length;
    ix->built = true;
    return DESSERT_OK;
}

size_t dessert_search_workspace_bytes(const dessert_index_t* ix, uint32_t n_queries, uint64_t total_q_vectors,
                                      uint64_t total_scored, uint32_t k) {
    if (!ix) return 0;
    // the slice count depends on the longest list; total_scored bounds it from above
    Workspace w = carve(ix, n_queries, total_q_vectors, total_scored, total_scored, k, true);
    return w.total;
}

dessert_status_t dessert_search(const dessert_index_t* ix, const void* q_vectors_dev, const uint32_t* q_lengths_host,
                                uint32_t n_queries, const uint32_t* cand_ids_dev, const uint64_t* cand_offsets_host,
                                uint32_t k, void* workspace_dev, size_t workspace_bytes, uint32_t* out_ids_dev,
                                int32_t* out_scores_dev) {
    if (k == 0 || k > 16384) return fail(DESSERT_EINVAL, "k must be in 1..16384, got %u", k);
    if (n_queries && (!out_ids_dev || !out_scores_dev)) return fail(DESSERT_EINVAL, "output pointer is NULL");
    Batch bt;
    dessert_status_t st = check_batch(ix, q_vectors_dev, q_lengths_host, n_queries, cand_ids_dev, cand_offsets_host, &bt);
    if (st != DESSERT_OK) return st;
    return search_impl(const_cast<dessert_index*>(ix), bt, q_vectors_dev, n_queries, cand_ids_dev, cand_offsets_host, k,
                       workspace_dev, workspace_bytes, nullptr, out_ids_dev, out_scores_dev);
}

dessert_status_t dessert_scores(const dessert_index_t* ix, const void* q_vectors_dev, const uint32_t* q_lengths_host,
                                uint32_t n_queries, const uint32_t* cand_ids_dev, const uint64_t* cand_offsets_host,
                                void* workspace_dev, size_t workspace_bytes, int32_t* out_scores_dev) {
    if (n_queries && !out_scores_dev) return fail(DESSERT_EINVAL, "out_scores_dev is NULL");
    Batch bt;
    dessert_status_t st = check_batch(ix, q_vectors_dev, q_lengths_host, n_queries, cand_ids_dev, cand_offsets_host, &bt);
    if (st != DESSERT_OK) return st;
    return search_impl(const_cast<dessert_index*>(ix), bt, q_vectors_dev, n_queries, cand_ids_dev, cand_offsets_host, 0,
                       workspace_dev, workspace_bytes, out_scores_dev, nullptr, nullptr);
}

size_t dessert_noalloc_scratch_bytes(void) { return kScratchBytes; }

dessert_status_t dessert_search_noalloc(const dessert_index_t* ix, const void* q_vectors_dev, uint32_t q_length,
                                        uint32_t n_queries, const uint32_t* cand_ids_dev, uint64_t cand_length,
                                        uint32_t k, uint32_t* out_ids_dev, int32_t* out_scores_dev) {
    if (k == 0 || k > 16384) return fail(DESSERT_EINVAL, "k must be in 1..16384, got %u", k);
    if (n_queries && (!out_ids_dev || !out_scores_dev)) return fail(DESSERT_EINVAL, "output pointer is NULL");
    Batch bt;
    dessert_status_t st = check_uniform_batch(ix, q_vectors_dev, q_length, n_queries, cand_ids_dev, cand_length, &bt);
    if (st != DESSERT_OK) return st;
    if (n_queries == 0) return DESSERT_OK;
    const size_t need = carve(ix, n_queries, bt.total_q, bt.total_scored, bt.max_scored, k, true).total;
    if (need > kScratchBytes)
        return fail(DESSERT_EINVAL, "this batch needs %zu bytes of workspace, the built-in scratch array holds %zu: "
                                    "use dessert_search with a workspace of the caller's", need, kScratchBytes);
    void* ws = g_scratch_ptr[(ix->cfg.device >= 0 && ix->cfg.device < kMaxDevices) ? ix->cfg.device : 0];
    if (!ws) return fail(DESSERT_ESTATE, "no scratch address recorded for device %d", ix->cfg.device);
    return search_impl(const_cast<dessert_index*>(ix), bt, q_vectors_dev, n_queries, cand_ids_dev, nullptr, k, ws,
                       kScratchBytes, nullptr, out_ids_dev, out_scores_dev);
}

const char* dessert_last_score_kernel(const dessert_index_t* ix) { return ix ? ix->last_score_kernel : ""; }

dessert_status_t dessert_set_debug(dessert_index_t* ix, int enable) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (enable && !ix->dbg_flag) {
        DeviceGuard guard(ix->cfg.device);
        if (!guard.ok) return fail(DESSERT_EHIP, "hipSetDevice(%d) failed", ix->cfg.device);
        hipError_t e = hipMalloc((void**)&ix->dbg_flag, sizeof(unsigned long long));
        if (e != hipSuccess) return fail(DESSERT_ENOMEM, "hipMalloc(debug flag): %s", hipGetErrorString(e));
    }
    ix->debug = enable != 0;
    return DESSERT_OK;
}

dessert_status_t dessert_filter_build(dessert_index_t* ix, const int8_t* centroids_dev, uint32_t n_centroids,
                                      const void* vectors_dev, uint32_t* assign_dev, uint32_t* bucket_offsets_dev,
                                      uint32_t* bucket_docs_dev) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (!ix->built) return fail(DESSERT_ESTATE, "dessert_build_index has not been called");
    if (ix->cfg.dtype != DESSERT_I8 || !filter_supported(ix->cfg.d))
        return fail(DESSERT_EINVAL, "the candidate filter needs int8 vectors with d in {64,128,256}");
    if (!centroids_dev || !assign_dev || !bucket_offsets_dev || !bucket_docs_dev || (ix->n_vectors && !vectors_dev))
        return fail(DESSERT_EINVAL, "NULL argument");
    if (n_centroids == 0 || n_centroids > (1u << 20)) return fail(DESSERT_EINVAL, "n_centroids must be in 1..2^20");
    if (ix->n_vectors > 0xFFFFFFFFull) return fail(DESSERT_EINVAL, "more than 2^32-1 vectors");
    if ((uintptr_t)vectors_dev % 16) return fail(DESSERT_EINVAL, "vectors_dev must be 16-byte aligned");
    DeviceGuard guard(ix->cfg.device);
    if (!guard.ok) return fail(DESSERT_EHIP, "hipSetDevice(%d) failed", ix->cfg.device);
    ix->f_built = false;
    const FilterSubPlan sub = filter_sub_plan(ix->n_docs, n_centroids);
    const size_t n_sub = (size_t)n_centroids * sub.S;
    // the filter's own buffers are kept from one build to the next while their sizes stay the same (same number of
    // centroids and of sub-bucket ranges): such a rebuild frees and allocates nothing and runs in stream order
    if (!ix->f_cent || ix->f_alloc_K != n_centroids || ix->f_alloc_sub != n_sub) {
        HIP_TRY(hipStreamSynchronize(ix->stream));  // earlier filter work may still read the buffers freed below
        if (ix->f_cent) (void)hipFree(ix->f_cent);
        if (ix->f_table) (void)hipFree(ix->f_table);
        if (ix->f_cursor) (void)hipFree(ix->f_cursor);
        if (ix->f_sub_off) (void)hipFree(ix->f_sub_off);
        ix->f_cent = ix->f_table = nullptr;
        ix->f_cursor = ix->f_sub_off = nullptr;
        ix->f_alloc_K = 0;
        ix->f_alloc_sub = 0;
        hipError_t e = hipMalloc(&ix->f_cent, filter_centroid_bytes(n_centroids, ix->cfg.d));
        if (e == hipSuccess) e = hipMalloc(&ix->f_table, filter_table_bytes(n_centroids));
        if (e == hipSuccess) e = hipMalloc((void**)&ix->f_cursor, n_sub * 4);
        if (e == hipSuccess) e = hipMalloc((void**)&ix->f_sub_off, (n_sub + 1) * 4);
        if (e != hipSuccess) return fail(DESSERT_ENOMEM, "hipMalloc(filter state): %s", hipGetErrorString(e));
        ix->f_alloc_K = n_centroids;
        ix->f_alloc_sub = n_sub;
    }
    ix->f_sub = sub;
    HIP_TRY(launch_filter_prep(centroids_dev, n_centroids, ix->cfg.d, ix->f_cent, ix->f_table, ix->stream));
    HIP_TRY(launch_filter_assign((const int8_t*)vectors_dev, ix->n_vectors, ix->cfg.d, n_centroids, ix->f_cent,
                                 ix->f_table, assign_dev, ix->stream));
    HIP_TRY(launch_filter_buckets(assign_dev, ix->offsets, ix->n_docs, n_centroids, ix->f_sub, ix->f_cursor, ix->f_sub_off,
                                  bucket_offsets_dev, bucket_docs_dev, ix->stream));
    {   // the largest bucket bounds how many documents one query set can hit (sizes the query workspace)
        std::vector<uint32_t> off((size_t)n_centroids + 1);
        HIP_TRY(hipMemcpyAsync(off.data(), bucket_offsets_dev, off.size() * 4, hipMemcpyDeviceToHost, ix->stream));
        HIP_TRY(hipStreamSynchronize(ix->stream));
        uint32_t mx = 0;
        for (uint32_t c = 0; c < n_centroids; ++c) mx = std::max(mx, off[c + 1] - off[c]);
        ix->f_max_bucket = mx;
    }
    ix->f_K = n_centroids;
    ix->f_bucket_off = bucket_offsets_dev;
    ix->f_bucket_docs = bucket_docs_dev;
    ix->f_built = true;
    return DESSERT_OK;
}

namespace {
struct KmeansWorkspace {
    size_t assign, sums, counts, cent, table, total;
};
KmeansWorkspace carve_kmeans(uint32_t d, uint64_t n, uint32_t K) {
    KmeansWorkspace w{};
    size_t p = 0;
    w.assign = p; p += align_up((size_t)(n ? n : 1) * 4, 256);
    w.sums = p;   p += align_up((size_t)K * d * 4, 256);
    w.counts = p; p += align_up((size_t)K * 4, 256);
    w.cent = p;   p += align_up(filter_centroid_bytes(K, d), 256);
    w.table = p;  p += align_up(filter_table_bytes(K), 256);
    w.total = p;
    return w;
}
}  // namespace

size_t dessert_filter_kmeans_workspace_bytes(const dessert_index_t* ix, uint64_t n_sample, uint32_t n_centroids) {
    if (!ix || n_centroids == 0) return 0;
    return carve_kmeans(ix->cfg.d, n_sample, n_centroids).total;
}

dessert_status_t dessert_filter_kmeans(const dessert_index_t* ix, const int8_t* sample_dev, uint64_t n_sample,
                                       int8_t* centroids_dev, uint32_t n_centroids, uint32_t iterations,
                                       void* workspace_dev, size_t workspace_bytes) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (ix->cfg.dtype != DESSERT_I8 || !filter_supported(ix->cfg.d))
        return fail(DESSERT_EINVAL, "the candidate filter needs int8 vectors with d in {64,128,256}");
    if (!centroids_dev || !workspace_dev || (n_sample && !sample_dev)) return fail(DESSERT_EINVAL, "NULL argument");
    if (n_centroids == 0 || n_centroids > (1u << 20)) return fail(DESSERT_EINVAL, "n_centroids must be in 1..2^20");
    if (n_sample > (1ull << 23)) return fail(DESSERT_EINVAL, "at most 2^23 sample vectors (32-bit coordinate sums)");
    if ((uintptr_t)sample_dev % 16 || (uintptr_t)workspace_dev % 256)
        return fail(DESSERT_EINVAL, "sample_dev must be 16-byte and workspace_dev 256-byte aligned");
    const KmeansWorkspace w = carve_kmeans(ix->cfg.d, n_sample, n_centroids);
    if (workspace_bytes < w.total)
        return fail(DESSERT_EINVAL, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, w.total);
    DeviceGuard guard(ix->cfg.device);
    if (!guard.ok) return fail(DESSERT_EHIP, "hipSetDevice(%d) failed", ix->cfg.device);
    char* ws = (char*)workspace_dev;
    uint32_t* assign = (uint32_t*)(ws + w.assign);
    for (uint32_t it = 0; it < iterations; ++it) {
        HIP_TRY(launch_filter_prep(centroids_dev, n_centroids, ix->cfg.d, ws + w.cent, ws + w.table, ix->stream));
        HIP_TRY(launch_filter_assign(sample_dev, n_sample, ix->cfg.d, n_centroids, ws + w.cent, ws + w.table, assign,
                                     ix->stream));
        HIP_TRY(launch_kmeans_update(sample_dev, n_sample, ix->cfg.d, assign, n_centroids, (int32_t*)(ws + w.sums),
                                     (uint32_t*)(ws + w.counts), centroids_dev, ix->stream));
    }
    return DESSERT_OK;
}

namespace {
struct FilterWorkspace {
    size_t dist, probe_ids, q_off, cursor, emit_plan, lists, list_stride, total;
};
// At most this many query sets in a call: the list selection runs in its two-launch form (launch_topk_lists)
constexpr uint32_t FILTER_FEW_LISTS = 64;
// max_q: vectors of the longest query set
FilterWorkspace carve_filter(const dessert_index* ix, uint32_t B, uint64_t total_q, uint32_t max_q, uint32_t probe) {
    FilterWorkspace w{};
    size_t p = 0;
    // probe selection: per-range lists for small probe counts, else the full distance matrix
    const FilterProbePlan pl = filter_probe_plan(total_q, ix->f_K, probe);
    w.dist = p;      p += align_up(pl.ranges ? pl.list_bytes : (size_t)total_q * filter_tiles(ix->f_K) * 32 * 4, 256);
    w.probe_ids = p; p += align_up((size_t)total_q * probe * 4, 256);
    w.q_off = p;     p += align_up(((size_t)B + 1) * 4, 256);
    w.cursor = p;    p += align_up(filter_hist_plan(B, max_q * probe, ix->n_docs, ix->f_sub).words * 4, 256);  // list lengths + count histograms
    w.emit_plan = p; p += align_up((size_t)FILTER_FEW_LISTS * TOPK_LISTS_EMIT_WORDS * 4, 256);
    // a query set hits at most (its vectors * probe) buckets of at most f_max_bucket documents each
    uint64_t hit = (uint64_t)max_q * probe * ix->f_max_bucket;
    if (hit > ix->n_docs) hit = ix->n_docs;
    w.list_stride = (size_t)((hit + 31) & ~31ull);
    w.lists = p;     p += align_up((size_t)B * w.list_stride * 8, 256);
    w.total = p;
    return w;
}
}  // namespace

size_t dessert_filter_workspace_bytes(const dessert_index_t* ix, uint32_t n_queries, uint64_t total_q_vectors,
                                      uint32_t max_q_len, uint32_t filter_probe) {
    if (!ix || !ix->f_built) return 0;
    return carve_filter(ix, n_queries, total_q_vectors, max_q_len, filter_probe).total;
}

namespace {
// Body of dessert_filter_query.  ordered = false: the filter_k documents of a query set are written in no particular
// order (dessert_filter_search only needs the set).
dessert_status_t filter_query_impl(const dessert_index_t* cix, const void* q_vectors_dev,
                                   const uint32_t* q_lengths_host, uint32_t n_queries, uint32_t filter_probe,
                                   uint32_t filter_k, void* workspace_dev, size_t workspace_bytes,
                                   uint32_t* out_ids_dev, int32_t* out_counts_dev, bool ordered) {
    dessert_index* ix = const_cast<dessert_index*>(cix);
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (!ix->f_built) return fail(DESSERT_ESTATE, "dessert_filter_build has not been called");
    if (n_queries == 0) return DESSERT_OK;
    if (n_queries > 65535) return fail(DESSERT_EINVAL, "n_queries > 65535");
    if (!q_vectors_dev || !q_lengths_host || !workspace_dev || !out_ids_dev || !out_counts_dev)
        return fail(DESSERT_EINVAL, "NULL argument");
    if (filter_probe == 0 || filter_probe > ix->f_K || filter_probe > 1024)
        return fail(DESSERT_EINVAL, "filter_probe must be in 1..min(n_centroids, 1024), got %u", filter_probe);
    if (filter_k == 0 || filter_k > 16384) return fail(DESSERT_EINVAL, "filter_k must be in 1..16384, got %u", filter_k);
    if ((uintptr_t)workspace_dev % 256 || (uintptr_t)q_vectors_dev % 16)
        return fail(DESSERT_EINVAL, "workspace_dev must be 256-byte and q_vectors_dev 16-byte aligned");
    std::vector<uint32_t> q_off(n_queries + 1, 0);
    uint32_t q_uniform = q_lengths_host[0], max_q = 0;
    for (uint32_t b = 0; b < n_queries; ++b) {
        if (q_lengths_host[b] == 0) return fail(DESSERT_EINVAL, "q_lengths_host[%u] = 0", b);
        uint64_t nxt = (uint64_t)q_off[b] + q_lengths_host[b];
        if (nxt > 0x7FFFFFFFull) return fail(DESSERT_EINVAL, "too many query vectors");
        q_off[b + 1] = (uint32_t)nxt;
        if (q_lengths_host[b] != q_uniform) q_uniform = 0;
        if (q_lengths_host[b] > max_q) max_q = q_lengths_host[b];
    }
    const uint64_t total_q = q_off[n_queries];
    if ((uint64_t)max_q * filter_probe > 0x7FFFFFFEull) return fail(DESSERT_EINVAL, "count range too large");
    FilterWorkspace w = carve_filter(ix, n_queries, total_q, max_q, filter_probe);
    if (workspace_bytes < w.total)
        return fail(DESSERT_EINVAL, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, w.total);
    DeviceGuard guard(ix->cfg.device);
    if (!guard.ok) return fail(DESSERT_EHIP, "hipSetDevice(%d) failed", ix->cfg.device);
    char* ws = (char*)workspace_dev;
    int32_t* dist = (int32_t*)(ws + w.dist);
    uint32_t* probe_ids = (uint32_t*)(ws + w.probe_ids);
    uint32_t* d_q_off = (uint32_t*)(ws + w.q_off);
    uint32_t* cursor = (uint32_t*)(ws + w.cursor);
    uint64_t* lists = (uint64_t*)(ws + w.lists);
    if (!q_uniform) {
        if (stream_capturing(ix))
            return fail(DESSERT_ESTATE, "graph capture needs query sets of equal length");
        dessert_status_t st = upload_small(ix, q_off.data(), ((size_t)n_queries + 1) * 4, d_q_off);
        if (st != DESSERT_OK) return st;
    }
    const FilterProbePlan pl = filter_probe_plan(total_q, ix->f_K, filter_probe);
    const FilterHistPlan hp = filter_hist_plan(n_queries, max_q * filter_probe, ix->n_docs, ix->f_sub);
    // A few query vectors (one query set, the unit of the paper's latency figures): the chain is bound by its launches, so
    // the probe GEMM also clears the counting kernel's list lengths: one launch fewer.
    const uint64_t zero_words = filter_count_zero_words(hp, n_queries);
    const bool gemm_clears = pl.ranges && total_q <= 512 && zero_words <= 4096;
    if (pl.ranges) {
        HIP_TRY(launch_filter_probe_lists((const int8_t*)q_vectors_dev, total_q, ix->cfg.d, ix->f_K, ix->f_cent,
                                          ix->f_table, filter_probe, pl, (int64_t*)dist, probe_ids, ix->stream,
                                          gemm_clears ? cursor : nullptr, gemm_clears ? (uint32_t)zero_words : 0u));
    } else {
        HIP_TRY(launch_filter_distances((const int8_t*)q_vectors_dev, total_q, ix->cfg.d, ix->f_K, ix->f_cent,
                                        ix->f_table, dist, ix->stream));
        HIP_TRY(launch_filter_probe(dist, total_q, ix->f_K, filter_probe, probe_ids, ix->stream));
    }
    HIP_TRY(launch_filter_count(probe_ids, total_q, filter_probe, max_q * filter_probe, d_q_off, q_uniform, n_queries,
                                ix->f_sub_off, ix->f_sub, ix->f_bucket_docs, ix->n_docs, lists, w.list_stride, cursor,
                                ix->stream, gemm_clears));
    HIP_TRY(launch_topk_lists(lists, w.list_stride, cursor, n_queries, filter_k, max_q * filter_probe,
                              ix->n_docs ? ix->n_docs - 1 : 0, (ix->n_docs && total_q) ? &hp : nullptr, out_ids_dev,
                              out_counts_dev, ordered, ix->stream,
                              (!ordered && n_queries <= FILTER_FEW_LISTS) ? (uint32_t*)(ws + w.emit_plan) : nullptr));
    return DESSERT_OK;
}

// Workspace of dessert_filter_search: the filter's, the search's, and the candidate lists between them.
struct ChainWorkspace {
    size_t filter, filter_bytes, ids, counts, search, search_bytes, total;
};
ChainWorkspace carve_chain(const dessert_index* ix, uint32_t B, uint64_t total_q, uint32_t max_q, uint32_t probe,
                           uint32_t filter_k, uint32_t k) {
    ChainWorkspace w{};
    size_t p = 0;
    w.filter_bytes = carve_filter(ix, B, total_q, max_q, probe).total;
    w.filter = p;  p += align_up(w.filter_bytes, 256);
    w.ids = p;     p += align_up((size_t)B * filter_k * 4, 256);
    w.counts = p;  p += align_up((size_t)B * filter_k * 4, 256);
    const uint64_t scored = (uint64_t)B * filter_k;
    w.search_bytes = carve(ix, B, total_q, scored, filter_k, k, true).total;
    w.search = p;  p += align_up(w.search_bytes, 256);
    w.total = p;
    return w;
}
}  // namespace

dessert_status_t dessert_filter_query(const dessert_index_t* ix, const void* q_vectors_dev,
                                      const uint32_t* q_lengths_host, uint32_t n_queries, uint32_t filter_probe,
                                      uint32_t filter_k, void* workspace_dev, size_t workspace_bytes,
                                      uint32_t* out_ids_dev, int32_t* out_counts_dev) {
    return filter_query_impl(ix, q_vectors_dev, q_lengths_host, n_queries, filter_probe, filter_k, workspace_dev,
                             workspace_bytes, out_ids_dev, out_counts_dev, true);
}

size_t dessert_filter_search_workspace_bytes(const dessert_index_t* ix, uint32_t n_queries, uint64_t total_q_vectors,
                                             uint32_t max_q_len, uint32_t filter_probe, uint32_t filter_k, uint32_t k) {
    if (!ix || !ix->f_built || !ix->built) return 0;
    return carve_chain(ix, n_queries, total_q_vectors, max_q_len, filter_probe, filter_k, k).total;
}

dessert_status_t dessert_filter_search(const dessert_index_t* ix, const void* q_vectors_dev, const uint32_t* q_lengths_host,
                                       uint32_t n_queries, uint32_t filter_probe, uint32_t filter_k, uint32_t k,
                                       void* workspace_dev, size_t workspace_bytes, uint32_t* out_ids_dev,
                                       int32_t* out_scores_dev) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    if (!ix->f_built) return fail(DESSERT_ESTATE, "dessert_filter_build has not been called");
    if (k == 0 || k > 16384) return fail(DESSERT_EINVAL, "k must be in 1..16384, got %u", k);
    if (filter_k == 0 || filter_k > 16384) return fail(DESSERT_EINVAL, "filter_k must be in 1..16384, got %u", filter_k);
    if (filter_probe == 0 || filter_probe > ix->f_K || filter_probe > 1024)
        return fail(DESSERT_EINVAL, "filter_probe must be in 1..min(n_centroids, 1024), got %u", filter_probe);
    if (n_queries == 0) return DESSERT_OK;
    if (!q_lengths_host || !workspace_dev || !out_ids_dev || !out_scores_dev) return fail(DESSERT_EINVAL, "NULL argument");
    if ((uintptr_t)workspace_dev % 256) return fail(DESSERT_EINVAL, "workspace_dev must be 256-byte aligned");
    uint64_t total_q = 0;
    uint32_t max_q = 0;
    for (uint32_t b = 0; b < n_queries && b < 65536; ++b) {
        total_q += q_lengths_host[b];
        if (q_lengths_host[b] > max_q) max_q = q_lengths_host[b];
    }
    const ChainWorkspace w = carve_chain(ix, n_queries, total_q, max_q, filter_probe, filter_k, k);
    if (workspace_bytes < w.total)
        return fail(DESSERT_EINVAL, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, w.total);
    char* ws = (char*)workspace_dev;
    uint32_t* cand = (uint32_t*)(ws + w.ids);
    // the candidates go straight into the scoring, which does not care about their order: the filter skips its sort
    dessert_status_t st = filter_query_impl(ix, q_vectors_dev, q_lengths_host, n_queries, filter_probe, filter_k, ws + w.filter,
                                            w.filter_bytes, cand, (int32_t*)(ws + w.counts), false);
    if (st != DESSERT_OK) return st;
    // lists of equal length filter_k (unused slots hold 0xFFFFFFFF, which the scoring marks -1 and the top-k skips)
    Batch bt;
    st = check_batch(ix, q_vectors_dev, q_lengths_host, n_queries, nullptr, nullptr, &bt);
    if (st != DESSERT_OK) return st;
    bt.max_scored = bt.cand_uniform = filter_k;
    bt.total_scored = (uint64_t)n_queries * filter_k;
    return search_impl(const_cast<dessert_index*>(ix), bt, q_vectors_dev, n_queries, cand, nullptr, k, ws + w.search,
                       w.search_bytes, nullptr, out_ids_dev, out_scores_dev);
}

dessert_status_t dessert_enable_timing(dessert_index_t* ix, int enable) {
    if (!ix) return fail(DESSERT_EINVAL, "index is NULL");
    DeviceGuard guard(ix->cfg.device);
    if (enable && !ix->slots[0].ev[0])
        for (auto& slot : ix->slots)
            for (auto& ev : slot.ev) HIP_TRY(hipEventCreate(&ev));
    ix->timing = enable != 0;
    ix->timing_period = enable > 1 ? (uint32_t)enable : 1;
    ix->timing_seen = 0;
    ix->timed_calls = 0;
    for (auto& slot : ix->slots) slot.any = false;
    return DESSERT_OK;
}

dessert_status_t dessert_get_timing(dessert_index_t* ix, uint32_t calls_back, float ms[4]) {
    if (!ix || !ms) return fail(DESSERT_EINVAL, "NULL argument");
    ms[0] = ms[1] = ms[2] = ms[3] = 0.f;
    if (calls_back >= dessert_index::kTimingSlots || calls_back >= ix->timed_calls)
        return fail(DESSERT_ESTATE, "no timed call recorded %u calls back", calls_back);
    const dessert_index::TimingSlot& ts = ix->slots[(ix->timed_calls - 1 - calls_back) % dessert_index::kTimingSlots];
    if (!ts.any) return fail(DESSERT_ESTATE, "no timed call recorded %u calls back", calls_back);
    DeviceGuard guard(ix->cfg.device);
    HIP_TRY(hipEventSynchronize(ts.ev[4]));
    if (ts.hash) HIP_TRY(hipEventElapsedTime(&ms[0], ts.ev[0], ts.ev[1]));
    if (ts.score) HIP_TRY(hipEventElapsedTime(&ms[1], ts.ev[1], ts.ev[2]));
    if (ts.topk) HIP_TRY(hipEventElapsedTime(&ms[2], ts.ev[2], ts.ev[3]));
    HIP_TRY(hipEventElapsedTime(&ms[3], ts.ev[0], ts.ev[4]));
    return DESSERT_OK;
}

}  // extern "C"
