/*
 * CPU oracle for hashed set-to-set scoring (DESSERT, arxiv 2210.15748).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition that the
 * GPU library is compared against.  It shares no code, header, table or
 * constant with the HIP sources and must never be called from the product
 * path.  Every function follows one passage of the paper, cited above it, in
 * scalar loops with no blocking, fusion or reordering.  The only parallelism
 * is an optional OpenMP loop over documents (or vectors), which does not
 * change any result because each iteration writes its own outputs.
 *
 * Integer arithmetic is exact (int32/int64).  The floating-point hash path
 * accumulates in double.
 *
 * Readings of the paper taken here (the paper is silent on each):
 *   - LSH family: signed random projections, one sign bit per projection
 *     (Sec. 3 lists SRP for cosine; Sec. 5 "concatenation trick" joins C
 *     hashes per table; a hash range of 128 with C = 7 in Sec. 5 / App. B
 *     means one bit per hash).
 *   - bit c of table t comes from projection row t*C + c and lands in bit c
 *     of the table's code.
 *   - sign(0): a projection that is exactly zero gives bit 1 (p >= 0).
 *   - sigma = max, A = sum (Sec. 2, ColBERT's sum of max similarities); in
 *     oracle_scores the division by L in Alg. 2 and the remap of Eq. 1 are left
 *     out, so the score is an integer in [0, |Q|*L]; oracle_scores_eq1 applies
 *     both.
 *   - an empty document scores 0 (Alg. 2 starts every count at 0).
 *   - top-k order: score descending, ties by ascending document id.
 *
 * Parity pins: see tests/test_oracle_pins.py (brute-force sum-of-max on tiny
 * inputs, the SRP collision-probability closed form, the binomial model of
 * the counts, invariants, the literal bucket form of Alg. 1 + Alg. 2, a
 * hand-computed example, numpy lexsort for top-k).  What stays unpinned:
 * recall / latency on the paper's real datasets (not available).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- projection matrix from a seed ------------------------------------
 * Counter-based Rademacher rule shared by definition (not by code) with the
 * library: entry (row, col) of the [P][d] matrix is +1 when the top bit of
 * mix64(seed + GOLDEN * (row*d + col + 1)) is set, else -1, where mix64 is
 * the finalizer of the SplitMix64 generator (Steele, Lea, Flood 2014).
 */
static uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

void oracle_rademacher(uint64_t seed, uint32_t P, uint32_t d, int8_t *R)
{
    for (uint32_t row = 0; row < P; ++row)
        for (uint32_t col = 0; col < d; ++col) {
            uint64_t ctr = (uint64_t)row * d + col + 1;
            uint64_t z = mix64(seed + 0x9E3779B97F4A7C15ULL * ctr);
            R[(size_t)row * d + col] = (z >> 63) ? 1 : -1;
        }
}

/* ---- hashing: Sec. 3 (SRP family), Sec. 5 concatenation trick, Alg. 1 line
 * "h = f_t(x_j)" and Alg. 2 line "h_{t,q} = f_t(q)".
 * X [n][d] int8, R [L*C][d] int8, codes [n][L] u8.
 * proj (optional, may be NULL) receives the raw projections [n][L*C] int32.
 */
void oracle_hash_i8(const int8_t *X, uint64_t n, uint32_t d, const int8_t *R,
                    uint32_t L, uint32_t C, uint8_t *codes, int32_t *proj)
{
    const uint32_t P = L * C;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < (int64_t)n; ++v) {
        const int8_t *x = X + (size_t)v * d;
        for (uint32_t t = 0; t < L; ++t) {
            uint32_t code = 0;
            for (uint32_t c = 0; c < C; ++c) {
                const int8_t *r = R + (size_t)(t * C + c) * d;
                int32_t p = 0;
                for (uint32_t i = 0; i < d; ++i)
                    p += (int32_t)r[i] * (int32_t)x[i];
                if (proj)
                    proj[(size_t)v * P + t * C + c] = p;
                if (p >= 0)
                    code |= 1u << c;
            }
            codes[(size_t)v * L + t] = (uint8_t)code;
        }
    }
}

/* Same, for real-valued inputs (the values of the fp16 vectors and of the
 * fp32 Gaussian matrix, both widened exactly to double by the caller's
 * float arrays).  proj (optional) receives the double projections.
 */
void oracle_hash_fp(const float *X, uint64_t n, uint32_t d, const float *R,
                    uint32_t L, uint32_t C, uint8_t *codes, double *proj)
{
    const uint32_t P = L * C;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < (int64_t)n; ++v) {
        const float *x = X + (size_t)v * d;
        for (uint32_t t = 0; t < L; ++t) {
            uint32_t code = 0;
            for (uint32_t c = 0; c < C; ++c) {
                const float *r = R + (size_t)(t * C + c) * d;
                double p = 0.0;
                for (uint32_t i = 0; i < d; ++i)
                    p += (double)r[i] * (double)x[i];
                if (proj)
                    proj[(size_t)v * P + t * C + c] = p;
                if (p >= 0.0)
                    code |= 1u << c;
            }
            codes[(size_t)v * L + t] = (uint8_t)code;
        }
    }
}

/* ---- scoring: Alg. 2, the loop over documents i, query vectors q, tables t
 * with sigma = max over the document's vectors and A = sum over q.
 * doc_codes [V][L], offsets [N+1] (document i owns rows offsets[i] ..
 * offsets[i+1]-1), q_codes [mq][L].  doc_ids [n_scored] selects which
 * documents to score (NULL: documents 0 .. n_scored-1).  scores [n_scored].
 */
void oracle_scores(const uint8_t *doc_codes, const int64_t *offsets, uint32_t L,
                   const uint8_t *q_codes, uint32_t mq,
                   const int64_t *doc_ids, uint64_t n_scored, int32_t *scores)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t s = 0; s < (int64_t)n_scored; ++s) {
        int64_t i = doc_ids ? doc_ids[s] : s;
        int64_t lo = offsets[i], hi = offsets[i + 1];
        int32_t score = 0;
        for (uint32_t q = 0; q < mq; ++q) {
            const uint8_t *hq = q_codes + (size_t)q * L;
            int32_t agg = 0;                       /* max over an empty set = 0 */
            for (int64_t j = lo; j < hi; ++j) {
                const uint8_t *hx = doc_codes + (size_t)j * L;
                int32_t cnt = 0;
                for (uint32_t t = 0; t < L; ++t)
                    cnt += (hq[t] == hx[t]);
                if (cnt > agg)
                    agg = cnt;
            }
            score += agg;
        }
        scores[s] = score;
    }
}

/* ---- scoring with the similarity remap of Sec. 5 ("concatenation trick", Eq. 1):
 * Alg. 2 as the paper's implementation runs it: count / L  ->  Eq. 1  ->  sigma = max  ->  A.
 * Eq. 1: sim = exp(ln(p_hat) / C) with p_hat = count / L; a count of 0 gives similarity 0
 * (the limit of Eq. 1).  The L+1 possible values are tabulated once, as the paper says its
 * implementation does.  Reading taken here (the paper does not fix a number format): each
 * per-query-vector maximum enters the sum as the fixed-point integer round(65536 * sim)
 * (llround: half away from zero), so the result does not depend on summation order;
 * score / (65536 * mq) is the paper's average of max similarities.  sim_table (optional,
 * [L+1] doubles) receives the table.
 */
void oracle_scores_eq1(const uint8_t *doc_codes, const int64_t *offsets, uint32_t L, uint32_t C,
                       const uint8_t *q_codes, uint32_t mq,
                       const int64_t *doc_ids, uint64_t n_scored, int32_t *scores, double *sim_table)
{
    double *sim = (double *)malloc((L + 1) * sizeof(double));
    for (uint32_t c = 0; c <= L; ++c) {
        double p_hat = (double)c / (double)L;                       /* Alg. 2: s_hat / L */
        sim[c] = (c == 0) ? 0.0 : exp(log(p_hat) / (double)C);      /* Eq. 1 */
        if (sim_table)
            sim_table[c] = sim[c];
    }
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t s = 0; s < (int64_t)n_scored; ++s) {
        int64_t i = doc_ids ? doc_ids[s] : s;
        int64_t lo = offsets[i], hi = offsets[i + 1];
        int64_t score = 0;
        for (uint32_t q = 0; q < mq; ++q) {
            const uint8_t *hq = q_codes + (size_t)q * L;
            double agg = 0.0;                                       /* sigma = max, empty set -> 0 */
            for (int64_t j = lo; j < hi; ++j) {
                const uint8_t *hx = doc_codes + (size_t)j * L;
                int32_t cnt = 0;
                for (uint32_t t = 0; t < L; ++t)
                    cnt += (hq[t] == hx[t]);
                if (sim[cnt] > agg)
                    agg = sim[cnt];
            }
            score += llround(65536.0 * agg);                        /* A = sum, in Q16 */
        }
        scores[s] = (int32_t)score;
    }
    free(sim);
}

/* ---- wide codes: more than 8 hashes per table (Sec. 6.1: the synthetic experiment sets
 * C = log2(m) + 1, up to 11 at m = 1024).  The same definitions as above with the table's
 * code kept in 16 bits (C <= 16): bit c of table t still comes from projection row t*C + c.
 */
void oracle_hash_i8_wide(const int8_t *X, uint64_t n, uint32_t d, const int8_t *R,
                         uint32_t L, uint32_t C, uint16_t *codes)
{
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < (int64_t)n; ++v) {
        const int8_t *x = X + (size_t)v * d;
        for (uint32_t t = 0; t < L; ++t) {
            uint32_t code = 0;
            for (uint32_t c = 0; c < C; ++c) {
                const int8_t *r = R + (size_t)(t * C + c) * d;
                int32_t p = 0;
                for (uint32_t i = 0; i < d; ++i)
                    p += (int32_t)r[i] * (int32_t)x[i];
                if (p >= 0)
                    code |= 1u << c;
            }
            codes[(size_t)v * L + t] = (uint16_t)code;
        }
    }
}

void oracle_hash_fp_wide(const float *X, uint64_t n, uint32_t d, const float *R,
                         uint32_t L, uint32_t C, uint16_t *codes, double *proj)
{
    const uint32_t P = L * C;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < (int64_t)n; ++v) {
        const float *x = X + (size_t)v * d;
        for (uint32_t t = 0; t < L; ++t) {
            uint32_t code = 0;
            for (uint32_t c = 0; c < C; ++c) {
                const float *r = R + (size_t)(t * C + c) * d;
                double p = 0.0;
                for (uint32_t i = 0; i < d; ++i)
                    p += (double)r[i] * (double)x[i];
                if (proj)
                    proj[(size_t)v * P + t * C + c] = p;
                if (p >= 0.0)
                    code |= 1u << c;
            }
            codes[(size_t)v * L + t] = (uint16_t)code;
        }
    }
}

/* Alg. 2 with sigma = max, A = sum on 16-bit codes; eq1_C = 0: raw counts, else the
 * remap of Eq. 1 with C = eq1_C in the same Q16 form as oracle_scores_eq1.
 */
void oracle_scores_wide(const uint16_t *doc_codes, const int64_t *offsets, uint32_t L, uint32_t eq1_C,
                        const uint16_t *q_codes, uint32_t mq,
                        const int64_t *doc_ids, uint64_t n_scored, int32_t *scores)
{
    double *sim = (double *)malloc((L + 1) * sizeof(double));
    for (uint32_t c = 0; c <= L; ++c)
        sim[c] = (c == 0 || eq1_C == 0) ? 0.0 : exp(log((double)c / (double)L) / (double)eq1_C);   /* Eq. 1 */
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t s = 0; s < (int64_t)n_scored; ++s) {
        int64_t i = doc_ids ? doc_ids[s] : s;
        int64_t lo = offsets[i], hi = offsets[i + 1];
        int64_t score = 0;
        for (uint32_t q = 0; q < mq; ++q) {
            const uint16_t *hq = q_codes + (size_t)q * L;
            int32_t agg = 0;                        /* max over an empty set = 0 */
            for (int64_t j = lo; j < hi; ++j) {
                const uint16_t *hx = doc_codes + (size_t)j * L;
                int32_t cnt = 0;
                for (uint32_t t = 0; t < L; ++t)
                    cnt += (hq[t] == hx[t]);
                if (cnt > agg)
                    agg = cnt;                      /* Eq. 1 is increasing: max of sims = sim of max */
            }
            score += eq1_C ? llround(65536.0 * sim[agg]) : agg;
        }
        scores[s] = (int32_t)score;
    }
    free(sim);
}

/* ---- other inner aggregations and a weighted outer aggregation (Sec. 4.1, the lemma on
 * sigma(x) = (1/m) sum_i phi(x_i); Sec. 4.2, F(Q,S) = (1/m_q) sum_j w_j sigma(s_hat(q_j, S))).
 * Alg. 2 in the paper's order: s_hat = count / L  ->  phi  ->  sigma over the document's vectors
 * ->  weighted sum over the query vectors.
 *   phi: 0 identity phi(x) = x;  1 phi(x) = e^x - 1;  2 debiased sigmoid 1/(1+e^-x) - 1/2
 *        (the three examples the paper gives for that lemma);  3 the similarity remap of Eq. 1
 *        with C = eq1_C, phi(x) = x^(1/C) (Sec. 5; phi(0) = 0);
 *   sigma: 0 max over the document's vectors, 1 mean (1/m) sum.
 * Number format (reading taken here; the paper fixes none): phi(s_hat) enters as the integer
 * round(65536 * phi) (llround); the mean is the integer (sum + floor(m/2)) / m (round half up; an
 * empty document gives 0); a weight is an integer w in [0, 65536] standing for w / 65536 and a
 * query vector contributes (w * sigma + 32768) >> 16, which is sigma itself for w = 65536 and when
 * weights is NULL.  The division by m_q of Sec. 4.2 is left out (same ranking).
 * code_bytes = 1 or 2 selects the code width.
 */
void oracle_scores_general(const void *doc_codes, const int64_t *offsets, uint32_t L, uint32_t code_bytes,
                           uint32_t phi, uint32_t eq1_C, uint32_t sigma, const void *q_codes, uint32_t mq,
                           const uint32_t *weights, const int64_t *doc_ids, uint64_t n_scored, int32_t *scores,
                           double *phi_table)
{
    int64_t *T = (int64_t *)malloc((L + 1) * sizeof(int64_t));
    for (uint32_t c = 0; c <= L; ++c) {
        double s_hat = (double)c / (double)L;                       /* Alg. 2: s_hat / L */
        double y = phi == 0 ? s_hat
                 : phi == 1 ? exp(s_hat) - 1.0
                 : phi == 2 ? 1.0 / (1.0 + exp(-s_hat)) - 0.5
                 : (c == 0 ? 0.0 : exp(log(s_hat) / (double)eq1_C));    /* Eq. 1 */
        if (phi_table)
            phi_table[c] = y;
        T[c] = llround(65536.0 * y);
    }
    const uint8_t *d8 = (const uint8_t *)doc_codes, *q8 = (const uint8_t *)q_codes;
    const uint16_t *d16 = (const uint16_t *)doc_codes, *q16 = (const uint16_t *)q_codes;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t s = 0; s < (int64_t)n_scored; ++s) {
        int64_t i = doc_ids ? doc_ids[s] : s;
        int64_t lo = offsets[i], hi = offsets[i + 1], m = hi - lo;
        int64_t score = 0;
        for (uint32_t q = 0; q < mq; ++q) {
            int64_t best = 0, sum = 0;
            for (int64_t j = lo; j < hi; ++j) {
                int32_t cnt = 0;
                for (uint32_t t = 0; t < L; ++t)
                    cnt += code_bytes == 1 ? (q8[(size_t)q * L + t] == d8[(size_t)j * L + t])
                                           : (q16[(size_t)q * L + t] == d16[(size_t)j * L + t]);
                int64_t y = T[cnt];                                  /* phi(s_hat) in Q16 */
                if (y > best)
                    best = y;
                sum += y;
            }
            int64_t sg = sigma == 0 ? best : (m ? (sum + m / 2) / m : 0);
            score += weights ? (((int64_t)weights[q] * sg + 32768) >> 16) : sg;
        }
        scores[s] = (int32_t)score;
    }
    free(T);
}

/* ---- top-k: Alg. 2 last line (argmax), widened to the k best.
 * Order: score descending, then document id ascending.  ids may be NULL
 * (then the id of entry s is s).  Missing slots (n < k) get id 0xFFFFFFFF,
 * score -1.  Plain selection: k passes, each picking the best remaining.
 */
void oracle_topk(const int32_t *scores, const int64_t *ids, uint64_t n, uint32_t k,
                 uint32_t *out_ids, int32_t *out_scores)
{
    uint8_t *taken = (uint8_t *)calloc(n ? n : 1, 1);
    for (uint32_t r = 0; r < k; ++r) {
        int64_t best = -1;
        for (uint64_t s = 0; s < n; ++s) {
            if (taken[s])
                continue;
            if (best < 0) {
                best = (int64_t)s;
                continue;
            }
            int64_t id_s = ids ? ids[s] : (int64_t)s;
            int64_t id_b = ids ? ids[best] : best;
            if (scores[s] > scores[best] || (scores[s] == scores[best] && id_s < id_b))
                best = (int64_t)s;
        }
        if (best < 0) {
            out_ids[r] = 0xFFFFFFFFu;
            out_scores[r] = -1;
        } else {
            taken[best] = 1;
            out_ids[r] = (uint32_t)(ids ? ids[best] : best);
            out_scores[r] = scores[best];
        }
    }
    free(taken);
}

/* ---- candidate filter: Sec. 5 "Filtering".
 * The paper clusters a sample of the item vectors with k-means and keeps an inverted index
 * from centroid ids to document ids; a document is added to the bucket of the closest centroid
 * of each of its vectors.  At query time the buckets of the filter_probe closest centroids of
 * every query vector are aggregated into a count per document id, and only the filter_k
 * documents with the highest count go on to be scored.
 * Readings taken here (the paper does not say): "closest" is the squared Euclidean distance
 * (the k-means objective), ties go to the lower centroid id; a bucket is a set (a document
 * appears once however many of its vectors chose the centroid); a document's count is the number
 * of (query vector, probed centroid) pairs whose bucket holds it; the filter_k best are taken by
 * (count descending, document id ascending) among documents with count >= 1.  The centroids
 * themselves are an input: k-means training is not part of this oracle.
 */

/* closest centroid of every vector: assign[v] = argmin_k sum_i (x_i - c_{k,i})^2 */
void oracle_assign_centroids(const int8_t *X, uint64_t n, uint32_t d, const int8_t *Cn, uint32_t K,
                             int32_t *assign)
{
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < (int64_t)n; ++v) {
        const int8_t *x = X + (size_t)v * d;
        int64_t best = -1;
        int32_t best_k = -1;
        for (uint32_t k = 0; k < K; ++k) {
            const int8_t *c = Cn + (size_t)k * d;
            int64_t dist = 0;
            for (uint32_t i = 0; i < d; ++i) {
                int64_t diff = (int64_t)x[i] - (int64_t)c[i];
                dist += diff * diff;
            }
            if (best_k < 0 || dist < best) {
                best = dist;
                best_k = (int32_t)k;
            }
        }
        assign[v] = best_k;
    }
}

/* the filter_probe closest centroids of one vector, closest first (ties: lower id first) */
static void closest_centroids(const int8_t *x, uint32_t d, const int8_t *Cn, uint32_t K, uint32_t probe,
                              int32_t *out)
{
    uint8_t *taken = (uint8_t *)calloc(K ? K : 1, 1);
    for (uint32_t r = 0; r < probe; ++r) {
        int64_t best = -1;
        int32_t best_k = -1;
        for (uint32_t k = 0; k < K; ++k) {
            if (taken[k])
                continue;
            const int8_t *c = Cn + (size_t)k * d;
            int64_t dist = 0;
            for (uint32_t i = 0; i < d; ++i) {
                int64_t diff = (int64_t)x[i] - (int64_t)c[i];
                dist += diff * diff;
            }
            if (best_k < 0 || dist < best) {
                best = dist;
                best_k = (int32_t)k;
            }
        }
        out[r] = best_k;
        if (best_k >= 0)
            taken[best_k] = 1;
    }
    free(taken);
}

/* inverted index from the assignments: bucket k = sorted set of documents with a vector assigned
 * to centroid k.  Call with bucket_docs == NULL to get only bucket_offsets [K+1] (sizes), then
 * again with room for bucket_offsets[K] ids. */
void oracle_inverted_index(const int32_t *assign, const int64_t *offsets, uint64_t n_docs, uint32_t K,
                           int64_t *bucket_offsets, uint32_t *bucket_docs)
{
    int64_t *size = (int64_t *)calloc((size_t)K + 1, sizeof(int64_t));
    uint8_t *seen = (uint8_t *)calloc(K ? K : 1, 1);
    for (int pass = 0; pass < 2; ++pass) {
        if (pass == 1) {
            int64_t run = 0;
            for (uint32_t k = 0; k < K; ++k) {
                bucket_offsets[k] = run;
                run += size[k];
                size[k] = 0;
            }
            bucket_offsets[K] = run;
            if (!bucket_docs)
                break;
        }
        for (uint64_t i = 0; i < n_docs; ++i) {           /* documents in id order: buckets come out sorted */
            for (int64_t j = offsets[i]; j < offsets[i + 1]; ++j) {
                int32_t k = assign[j];
                if (seen[k])
                    continue;
                seen[k] = 1;
                if (pass == 1)
                    bucket_docs[bucket_offsets[k] + size[k]] = (uint32_t)i;
                size[k] += 1;
            }
            for (int64_t j = offsets[i]; j < offsets[i + 1]; ++j)
                seen[assign[j]] = 0;
        }
    }
    free(size);
    free(seen);
}

/* one query set through the filter: counts per document, then the filter_k best.
 * out_ids / out_counts [filter_k]; unused slots get id 0xFFFFFFFF, count -1 (the padding of oracle_topk). */
void oracle_filter_query(const int8_t *Q, uint32_t mq, uint32_t d, const int8_t *Cn, uint32_t K,
                         const int64_t *bucket_offsets, const uint32_t *bucket_docs, uint64_t n_docs,
                         uint32_t probe, uint32_t filter_k, uint32_t *out_ids, int32_t *out_counts)
{
    int32_t *count = (int32_t *)calloc(n_docs ? n_docs : 1, sizeof(int32_t));
    int32_t *near = (int32_t *)malloc((probe ? probe : 1) * sizeof(int32_t));
    for (uint32_t q = 0; q < mq; ++q) {
        closest_centroids(Q + (size_t)q * d, d, Cn, K, probe, near);
        for (uint32_t r = 0; r < probe; ++r) {
            if (near[r] < 0)
                continue;
            for (int64_t e = bucket_offsets[near[r]]; e < bucket_offsets[near[r] + 1]; ++e)
                count[bucket_docs[e]] += 1;
        }
    }
    for (uint32_t r = 0; r < filter_k; ++r) {             /* plain selection, best remaining first */
        int64_t best = -1;
        for (uint64_t i = 0; i < n_docs; ++i)
            if (count[i] > 0 && (best < 0 || count[i] > count[best]))
                best = (int64_t)i;                          /* strict '>' keeps the lower id on ties */
        if (best < 0) {
            out_ids[r] = 0xFFFFFFFFu;
            out_counts[r] = -1;
        } else {
            out_ids[r] = (uint32_t)best;
            out_counts[r] = count[best];
            count[best] = -count[best];                     /* taken */
        }
    }
    free(count);
    free(near);
}

/* ---- k-means for the filter's centroids (Sec. 5 "Filtering": k-means clustering on a sample of the
 * vectors at the start of indexing).  The paper names the method only; taken here: Lloyd's iteration with
 * the squared Euclidean distance, starting from the centroids the caller passes, a fixed number of
 * iterations, everything in integers: each iteration assigns every sample vector to its closest centroid
 * (ties to the lower id, as oracle_assign_centroids) and replaces every centroid that received vectors by
 * the coordinate-wise mean rounded to the nearest integer (half rounds up: floor((2 sum + n) / (2 n)));
 * a centroid that received none stays.  Cn [K][d] is updated in place; inertia (optional, [iters]) receives
 * the sum of squared distances of each iteration's assignment step.
 */
static int64_t floor_div(int64_t a, int64_t b)   /* b > 0 */
{
    int64_t q = a / b;
    return (a % b != 0 && a < 0) ? q - 1 : q;
}

void oracle_kmeans(const int8_t *X, uint64_t n, uint32_t d, int8_t *Cn, uint32_t K, uint32_t iters,
                   int64_t *inertia)
{
    int32_t *assign = (int32_t *)malloc((n ? n : 1) * sizeof(int32_t));
    int64_t *sum = (int64_t *)malloc((size_t)K * d * sizeof(int64_t));
    int64_t *cnt = (int64_t *)malloc((size_t)K * sizeof(int64_t));
    for (uint32_t it = 0; it < iters; ++it) {
        oracle_assign_centroids(X, n, d, Cn, K, assign);
        memset(sum, 0, (size_t)K * d * sizeof(int64_t));
        memset(cnt, 0, (size_t)K * sizeof(int64_t));
        int64_t total = 0;
        for (uint64_t v = 0; v < n; ++v) {
            const int8_t *x = X + (size_t)v * d, *c = Cn + (size_t)assign[v] * d;
            cnt[assign[v]] += 1;
            for (uint32_t i = 0; i < d; ++i) {
                sum[(size_t)assign[v] * d + i] += x[i];
                total += ((int64_t)x[i] - c[i]) * ((int64_t)x[i] - c[i]);
            }
        }
        if (inertia)
            inertia[it] = total;
        for (uint32_t k = 0; k < K; ++k)
            if (cnt[k])
                for (uint32_t i = 0; i < d; ++i)
                    Cn[(size_t)k * d + i] = (int8_t)floor_div(2 * sum[(size_t)k * d + i] + cnt[k], 2 * cnt[k]);
    }
    free(assign);
    free(sum);
    free(cnt);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
