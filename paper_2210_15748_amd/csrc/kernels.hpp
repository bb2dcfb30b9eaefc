// Internal launch interface between the C ABI (api.hip) and the gfx950 kernels.
// Nothing here is exported; every function enqueues work on `stream` and
// returns the launch status without synchronising.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cand_order.hpp"

namespace dessert {

// ---- hashing (Sec. 3 SRP family, Sec. 5 concatenation trick) ----------------
// Fill R [P][d] with the seed-derived Rademacher matrix.
hipError_t launch_rademacher(uint64_t seed, uint32_t P, uint32_t d, int8_t* R, hipStream_t stream);

// Bytes of the MFMA-ordered copy of an int8 projection matrix, 0 if (d, L, C) has no MFMA kernel.
size_t mfma_proj_bytes(uint32_t d, uint32_t L, uint32_t C);
hipError_t launch_repack_proj_i8(const int8_t* R, uint32_t d, uint32_t L, uint32_t C, void* Rp, hipStream_t stream);
bool hash_mfma_supported(uint32_t d, uint32_t L, uint32_t C);
// fused: nullptr, or a candidate grouping (cand_order_plan with max_ranges = hash_mfma_fused_ranges) that extra
// workgroups of the same launch carry out beside the hashing (a search hashes few vectors: both are short, latency-bound
// jobs, and one launch instead of two saves a kernel boundary on the stream).
uint32_t hash_mfma_fused_ranges(uint32_t d, uint32_t L, uint32_t C);
hipError_t launch_hash_mfma_i8(const int8_t* X, uint64_t n, uint32_t d, uint32_t L, uint32_t C, const void* Rp,
                               uint8_t* codes, const CandOrderArgs* fused, hipStream_t stream);

// fp16 vectors x fp32 Gaussian projections on fp16 MFMA (projection matrix split hi + lo).
size_t mfma_f16_proj_bytes(uint32_t d, uint32_t L);
hipError_t launch_repack_proj_f16(const float* R, uint32_t d, uint32_t L, uint32_t C, void* Rp, hipStream_t stream);
bool hash_mfma_f16_supported(uint32_t d, uint32_t L, uint32_t C);
hipError_t launch_hash_mfma_f16(const void* X, uint64_t n, uint32_t d, uint32_t L, uint32_t C, const void* Rp,
                                uint8_t* codes, hipStream_t stream);

// One thread per (vector, table); any d, L, C <= 16.  dtype/proj_kind as in dessert.h.  Codes are one byte
// per table for C <= 8, else two.
hipError_t launch_hash_scalar(const void* X, uint32_t dtype, uint64_t n, uint32_t d, const void* R, uint32_t proj_kind,
                              uint32_t L, uint32_t C, uint8_t* codes, hipStream_t stream);

// ---- measurement aid: one pass of a plain streaming read over [buf, buf+bytes) ------------
hipError_t launch_read_probe(const void* buf, size_t bytes, hipStream_t stream);
// one pass that reads 4 * out_bytes from `in` and writes out_bytes to `out` (index building's traffic without its arithmetic)
hipError_t launch_mix_probe(const void* in, void* out, size_t out_bytes, hipStream_t stream);

// ---- scoring (Alg. 2: collision counts, sigma = max, A = sum) ---------------
struct ScoreArgs {
    const uint8_t* codes;       // [V][L] codes of code_bytes bytes each
    uint32_t code_bytes;        // 1 (C <= 8) or 2
    const uint64_t* offsets;    // [n_docs+1]
    uint64_t n_docs;
    uint32_t L, C;
    const uint8_t* qcodes;      // [total_q][L], same code width
    const uint32_t* q_off;      // dev [B+1]; unused when q_uniform != 0
    uint32_t q_uniform;         // != 0: every query set has this many vectors (q_off[b] = b * q_uniform)
    uint32_t n_queries;
    uint32_t max_q_len;
    const uint32_t* cand_ids;   // dev or nullptr
    const uint64_t* cand_off;   // dev [B+1] (candidate mode); unused when cand_uniform != 0
    uint64_t cand_uniform;      // != 0: every candidate list has this many ids
    const uint32_t* order;      // dev [total_cand] or nullptr: per list, its slots grouped by document id range
                                // (launch_cand_order); the mask-table kernel then takes a list's slots in that order
    uint64_t max_scored;        // largest number of documents scored by one query set
    uint64_t total_scored;      // all output slots (candidate mode: sum of the list lengths)
    uint64_t n_vectors;         // vectors in the index (launch heuristics only)
    int32_t* scores;            // out: candidate mode [total_cand], else [B][n_docs]
    const uint32_t* remap;      // dev [L+1] fixed-point phi per collision count (Eq. 1, Sec. 4.1 examples), or nullptr: raw counts
    uint32_t sigma_mean;        // != 0: sigma = rounded mean of remap[count] over the document's vectors (else the max)
    uint32_t phi_identity;      // != 0: remap[count] = 65536 / L * count exactly (phi = identity and L a power of two); the
                                // mask-table kernel then forms the mean from sums of counts
    const uint32_t* q_weights;  // dev [total_q] Q16 weights of the outer sum (Sec. 4.2), or nullptr
};
// first query vector / first candidate slot of query set b (b may be n_queries: one past the end)
__device__ inline uint32_t q_begin(const ScoreArgs& a, uint32_t b) { return a.q_uniform ? b * a.q_uniform : a.q_off[b]; }
__device__ inline uint64_t cand_begin(const ScoreArgs& a, uint32_t b) {
    return a.cand_uniform ? (uint64_t)b * a.cand_uniform : a.cand_off[b];
}
// desc (optional, desc_len bytes): receives the name of the kernel instantiation that was launched, spelled as a
// profiler prints it ("" when nothing was launched).
hipError_t launch_score_bytecmp(const ScoreArgs& a, hipStream_t stream, char* desc = nullptr, size_t desc_len = 0);
// Candidate lists gathered from all over the code array: order[list start + p] = the slots of a list grouped by
// range of document id (a counting sort over the leading id bits; the order inside a range is unspecified).
// Workgroups that take the same run of positions of different lists then read neighbouring parts of the code array
// at about the same time.  Worth it from score_order_min() candidates per list on.
uint64_t score_order_min();
// Fills *out for lists of at most max_scored ids (ranges a power of two <= max_ranges); false: not applicable.
bool cand_order_plan(const uint32_t* cand_ids, const uint64_t* cand_off, uint64_t cand_uniform, uint32_t n_queries,
                     uint64_t max_scored, uint64_t n_docs, uint32_t max_ranges, uint32_t* order, CandOrderArgs* out);
hipError_t launch_cand_order(const CandOrderArgs& a, hipStream_t stream);  // a.ranges <= 4096
// Write the n <= SCORE_TABLE_MAX words of a host table to dst (device) in stream order: the values travel as the launch's argument.
constexpr uint32_t SCORE_TABLE_MAX = 192;   // L + 1 entries with L <= 128
hipError_t launch_write_table(const uint32_t* table_host, uint32_t n, uint32_t* dst, hipStream_t stream);
// Debug aid: *first_bad = the lowest slot whose id is neither below n_docs nor the empty-slot value 0xFFFFFFFF,
// all ones if every id is fine (two launches: reset, then a scan of the n ids).
hipError_t launch_check_cand_ids(const uint32_t* cand_ids, uint64_t n, uint64_t n_docs, unsigned long long* first_bad,
                                 hipStream_t stream);
bool score_masklut_supported(uint32_t L, uint32_t C);
// longest document (in vectors) for which the mask-table kernel can form sigma = mean (32-bit numerators)
constexpr uint64_t MASKLUT_MEAN_MAX_LEN = 65535;
hipError_t launch_score_masklut(const ScoreArgs& a, hipStream_t stream, char* desc = nullptr, size_t desc_len = 0);

// ---- candidate filter (Sec. 5 "Filtering") ---------------------------------------------
bool filter_supported(uint32_t d);
uint32_t filter_tiles(uint32_t K);
size_t filter_centroid_bytes(uint32_t K, uint32_t d);   // MFMA-ordered centroids
size_t filter_table_bytes(uint32_t K);                  // per-row key constants
hipError_t launch_filter_prep(const int8_t* Cn, uint32_t K, uint32_t d, void* Cp, void* T2, hipStream_t stream);
hipError_t launch_filter_assign(const int8_t* X, uint64_t n, uint32_t d, uint32_t K, const void* Cp, const void* T2,
                                uint32_t* assign, hipStream_t stream);
hipError_t launch_filter_distances(const int8_t* X, uint64_t n, uint32_t d, uint32_t K, const void* Cp, const void* T2,
                                   int32_t* out /*[n][filter_tiles(K)*32]*/, hipStream_t stream);
// Update step of Lloyd's k-means: per-cluster coordinate sums and counts of the assigned vectors, then the rounded means
// written over Cn [K][d] (clusters without vectors keep their centroid).  sums [K][d] i32, counts [K] u32 are scratch.
hipError_t launch_kmeans_update(const int8_t* X, uint64_t n, uint32_t d, const uint32_t* assign, uint32_t K,
                                int32_t* sums, uint32_t* counts, int8_t* Cn, hipStream_t stream);
// Probe selection inside the GEMM for probe <= FILTER_LIST_MAX (ranges = 0: not applicable, use the
// distance matrix + launch_filter_probe instead).
constexpr uint32_t FILTER_LIST_MAX = 8;
struct FilterProbePlan {
    uint32_t ranges, tiles_per_range, width;
    uint32_t nt;        // 32-vector column tiles per wave (2 when there are enough query vectors to fill the chip so)
    size_t list_bytes;  // int64 lists[n][ranges][2][width]
};
FilterProbePlan filter_probe_plan(uint64_t n, uint32_t K, uint32_t probe);
// zero / zero_words: words the launch also clears (nullptr / 0: none), for the kernel that follows it.
hipError_t launch_filter_probe_lists(const int8_t* X, uint64_t n, uint32_t d, uint32_t K, const void* Cp, const void* T2,
                                     uint32_t probe, const FilterProbePlan& plan, int64_t* lists, uint32_t* probe_ids,
                                     hipStream_t stream, uint32_t* zero = nullptr, uint32_t zero_words = 0);
// A bucket is stored as S sub-buckets by document range (sub-bucket s of centroid c holds the bucket's documents
// with id >> sub_shift == s), so that a query-side workgroup that counts one range of documents reads only that
// part of every bucket it probes.  sub_off [K*S+1] are the sub-bucket starts in bucket_docs; bucket_off[c] = sub_off[c*S].
struct FilterSubPlan {
    uint32_t S;          // sub-buckets per bucket
    uint32_t sub_shift;  // log2 of the documents per sub-bucket range
};
FilterSubPlan filter_sub_plan(uint64_t n_docs, uint32_t K);
hipError_t launch_filter_buckets(const uint32_t* assign, const uint64_t* doc_off, uint64_t n_docs, uint32_t K,
                                 FilterSubPlan sp, uint32_t* cursor /*[K*S] scratch*/, uint32_t* sub_off /*[K*S+1]*/,
                                 uint32_t* bucket_off /*[K+1]*/, uint32_t* bucket_docs, hipStream_t stream);
hipError_t launch_filter_probe(const int32_t* dist, uint64_t total_q, uint32_t K, uint32_t probe, uint32_t* probe_ids,
                               hipStream_t stream);
// Layout of the counting kernel's small outputs, one u32 array ("cursor"): the B list lengths, then what lets the
// selection that follows skip passes over the lists (launch_topk_lists takes the same plan):
//   rows: per (query set, slab of documents) the histogram of the slab's keys by score field [B][slabs][bins] and the
//         slab's run within the list [B][slabs][2] (plain stores by the workgroup that owns the slab); or
//   one histogram per query set [B][bins], added up with atomics (more than 128 bins or very many slabs); or nothing
//   (score field wider than a digit of the selection).
struct FilterHistPlan {
    uint32_t bins;    // 0: no histogram
    uint32_t slabs;   // document slabs of the counting kernel (its grid.x)
    uint32_t slab_docs, counter_bytes;
    bool rows;
    size_t hist_off, seg_off, words;  // in u32 words from the start of the array
};
FilterHistPlan filter_hist_plan(uint32_t n_queries, uint32_t max_pairs, uint64_t n_docs, FilterSubPlan sp);
// Per query set: one key (count, id) per document that at least one probed bucket holds, lists[b][0..cursor[b]).
// max_pairs bounds (vectors of a query set) * probe, i.e. the largest possible count.  cursor: filter_hist_plan().words
// u32 words (see above).
// The kernel needs the first filter_count_zero_words() words of cursor cleared: zeroed = true says an earlier launch
// has done that.
uint64_t filter_count_zero_words(const FilterHistPlan& hp, uint32_t n_queries);
hipError_t launch_filter_count(const uint32_t* probe_ids, uint64_t total_q, uint32_t probe, uint32_t max_pairs,
                               const uint32_t* q_off, uint32_t q_uniform, uint32_t n_queries, const uint32_t* sub_off,
                               FilterSubPlan sp, const uint32_t* bucket_docs, uint64_t n_docs, uint64_t* lists,
                               uint64_t list_stride, uint32_t* cursor /*out*/, hipStream_t stream, bool zeroed = false);

// ---- top-k (Alg. 2 last line, k best instead of argmax) ---------------------
struct TopkArgs {
    const int32_t* scores;      // as written by the scoring kernels
    const uint32_t* cand_ids;   // dev or nullptr
    const uint64_t* cand_off;   // dev [B+1] or nullptr
    uint64_t cand_uniform;      // != 0: every candidate list has this many ids (cand_off unused)
    uint64_t n_docs;
    uint32_t n_queries;
    uint64_t max_scored;
    uint32_t k;
    uint32_t max_score;         // largest possible score (longest query set * L)
    uint64_t* partial;          // workspace for the two-level path: [B][slices][k] keys
    uint32_t* out_ids;          // [B][k]
    int32_t* out_scores;        // [B][k]
};
uint32_t topk_slices(uint64_t max_scored, uint32_t n_queries);
hipError_t launch_topk(const TopkArgs& a, hipStream_t stream);
// k best of stored key lists: lists[b][0..counts[b]) (counts on the device), keys as built by make_key with
// id_bits = bits of max_id; one workgroup per list.  When the score and id fields fit 32 bits together the lists hold
// u32 keys (list b starts list_stride u32 entries after list b-1); launch_filter_count writes them the same way.
// lists must be 16-byte aligned and list_stride a multiple of 4 (the lists are read 16 bytes at a time).
// hp: nullptr, or the plan by which launch_filter_count laid out its histograms behind the counts (counts = the
// start of that array): the selection then skips its first pass over a list and, with rows, decides the id digits
// inside one slab's run.  ordered = false: the k best of a list are written in no particular order (their set is
// the same; saves the sort when only the set matters).
// emit_plan (unordered results only): nullptr, or TOPK_LISTS_EMIT_WORDS u32 words of scratch per list; the selection
// then runs as two launches, the second of which copies the selected keys with many workgroups per list (for a handful
// of long lists, where one workgroup per list would leave the chip idle during that pass).
constexpr uint32_t TOPK_LISTS_EMIT_WORDS = 8;
hipError_t launch_topk_lists(const uint64_t* lists, uint64_t list_stride, const uint32_t* counts, uint32_t n_queries,
                             uint32_t k, uint32_t max_score, uint64_t max_id, const FilterHistPlan* hp, uint32_t* out_ids,
                             int32_t* out_scores, bool ordered, hipStream_t stream, uint32_t* emit_plan = nullptr);

}  // namespace dessert
