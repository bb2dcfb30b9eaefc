/* Runs every routine of the CPU oracle on small random inputs, edge cases included (no vectors, empty
 * documents, k larger than the list, one centroid), inside a binary built with
 * -fsanitize=address,undefined: an out-of-bounds access, a leak of the routines' own scratch memory
 * or undefined integer behaviour ends the run with a report.  It also checks the invariants that need no
 * second implementation (score bounds, a document that contains the query scores |Q|*L, top-k order).
 * Test infrastructure: compiled and run by tests/test_oracle_sanitized.py. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void oracle_rademacher(uint64_t seed, uint32_t P, uint32_t d, int8_t *R);
void oracle_hash_i8(const int8_t *X, uint64_t n, uint32_t d, const int8_t *R, uint32_t L, uint32_t C, uint8_t *codes,
                    int32_t *proj);
void oracle_hash_fp(const float *X, uint64_t n, uint32_t d, const float *R, uint32_t L, uint32_t C, uint8_t *codes,
                    double *proj);
void oracle_scores(const uint8_t *doc_codes, const int64_t *offsets, uint32_t L, const uint8_t *q_codes, uint32_t mq,
                   const int64_t *doc_ids, uint64_t n_scored, int32_t *scores);
void oracle_scores_eq1(const uint8_t *doc_codes, const int64_t *offsets, uint32_t L, uint32_t C, const uint8_t *q_codes,
                       uint32_t mq, const int64_t *doc_ids, uint64_t n_scored, int32_t *scores, double *sim_table);
void oracle_hash_i8_wide(const int8_t *X, uint64_t n, uint32_t d, const int8_t *R, uint32_t L, uint32_t C,
                         uint16_t *codes);
void oracle_hash_fp_wide(const float *X, uint64_t n, uint32_t d, const float *R, uint32_t L, uint32_t C,
                         uint16_t *codes, double *proj);
void oracle_scores_wide(const uint16_t *doc_codes, const int64_t *offsets, uint32_t L, uint32_t eq1_C,
                        const uint16_t *q_codes, uint32_t mq, const int64_t *doc_ids, uint64_t n_scored,
                        int32_t *scores);
void oracle_scores_general(const void *doc_codes, const int64_t *offsets, uint32_t L, uint32_t code_bytes, uint32_t phi,
                           uint32_t eq1_C, uint32_t sigma, const void *q_codes, uint32_t mq, const uint32_t *weights,
                           const int64_t *doc_ids, uint64_t n_scored, int32_t *scores, double *phi_table);
void oracle_topk(const int32_t *scores, const int64_t *ids, uint64_t n, uint32_t k, uint32_t *out_ids,
                 int32_t *out_scores);
void oracle_assign_centroids(const int8_t *X, uint64_t n, uint32_t d, const int8_t *Cn, uint32_t K, int32_t *assign);
void oracle_inverted_index(const int32_t *assign, const int64_t *offsets, uint64_t n_docs, uint32_t K,
                           int64_t *bucket_offsets, uint32_t *bucket_docs);
void oracle_filter_query(const int8_t *Q, uint32_t mq, uint32_t d, const int8_t *Cn, uint32_t K,
                         const int64_t *bucket_offsets, const uint32_t *bucket_docs, uint64_t n_docs, uint32_t probe,
                         uint32_t filter_k, uint32_t *out_ids, int32_t *out_counts);
void oracle_kmeans(const int8_t *X, uint64_t n, uint32_t d, int8_t *Cn, uint32_t K, uint32_t iters, int64_t *inertia);
int oracle_num_threads(void);

static uint64_t rng_state = 0x243F6A8885A308D3ULL;
static uint32_t rnd(void)
{
    rng_state = rng_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (uint32_t)(rng_state >> 33);
}
static int8_t rnd_i8(void) { return (int8_t)((int)(rnd() % 255) - 127); }

#define CHECK(cond)                                                               \
    do {                                                                          \
        if (!(cond)) {                                                            \
            fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond);    \
            exit(1);                                                              \
        }                                                                         \
    } while (0)

/* exact-size heap blocks so that the sanitizer sees every overrun; malloc(0) is avoided */
static void *block(size_t bytes) { return calloc(bytes ? bytes : 1, 1); }

static void one_case(uint32_t d, uint32_t L, uint32_t C, uint32_t n_docs, uint32_t max_len, uint32_t mq, uint32_t k)
{
    const uint32_t P = L * C;
    int64_t *off = block((n_docs + 1) * sizeof(int64_t));
    for (uint32_t i = 0; i < n_docs; ++i) off[i + 1] = off[i] + (max_len ? rnd() % (max_len + 1) : 0);
    const uint64_t V = (uint64_t)off[n_docs];
    int8_t *X = block(V * d), *Q = block((size_t)mq * d), *R = block((size_t)P * d);
    for (uint64_t i = 0; i < V * d; ++i) X[i] = rnd_i8();
    for (uint64_t i = 0; i < (uint64_t)mq * d; ++i) Q[i] = rnd_i8();
    oracle_rademacher(7 + d + L, P, d, R);
    for (uint64_t i = 0; i < (uint64_t)P * d; ++i) CHECK(R[i] == 1 || R[i] == -1);
    /* the last document, if it has vectors, gets the query's vectors: it must reach the maximum score */
    uint32_t full_doc = n_docs;
    if (n_docs && (uint64_t)(off[n_docs] - off[n_docs - 1]) >= mq && mq) {
        full_doc = n_docs - 1;
        memcpy(X + (size_t)off[full_doc] * d, Q, (size_t)mq * d);
    }

    if (C <= 8) {
        uint8_t *dc = block(V * L), *qc = block((size_t)mq * L);
        int32_t *proj = block(V * P * sizeof(int32_t));
        oracle_hash_i8(X, V, d, R, L, C, dc, proj);
        oracle_hash_i8(Q, mq, d, R, L, C, qc, NULL);
        for (uint64_t i = 0; i < V * L; ++i) CHECK(dc[i] < (1u << C));
        int32_t *sc = block(n_docs * sizeof(int32_t)), *sc2 = block(n_docs * sizeof(int32_t));
        oracle_scores(dc, off, L, qc, mq, NULL, n_docs, sc);
        for (uint32_t i = 0; i < n_docs; ++i) CHECK(sc[i] >= 0 && sc[i] <= (int32_t)(mq * L));
        if (full_doc < n_docs) CHECK(sc[full_doc] == (int32_t)(mq * L));
        double *sim = block((L + 1) * sizeof(double));
        oracle_scores_eq1(dc, off, L, C, qc, mq, NULL, n_docs, sc2, sim);
        CHECK(sim[0] == 0.0 && sim[L] == 1.0);
        if (full_doc < n_docs) CHECK(sc2[full_doc] == (int32_t)(mq * 65536));
        /* a candidate list with repeats, scored through every aggregation */
        const uint32_t n_c = n_docs ? 2 * n_docs + 3 : 0;
        int64_t *cand = block(n_c * sizeof(int64_t));
        for (uint32_t i = 0; i < n_c; ++i) cand[i] = rnd() % n_docs;
        int32_t *sc3 = block(n_c * sizeof(int32_t));
        uint32_t *w = block(mq * sizeof(uint32_t));
        for (uint32_t q = 0; q < mq; ++q) w[q] = rnd() % 65537;
        double *tab = block((L + 1) * sizeof(double));
        for (uint32_t phi = 0; phi < 4; ++phi)
            for (uint32_t sigma = 0; sigma < 2; ++sigma) {
                oracle_scores_general(dc, off, L, 1, phi, C, sigma, qc, mq, (phi & 1) ? w : NULL, cand, n_c, sc3, tab);
                for (uint32_t i = 0; i < n_c; ++i) CHECK(sc3[i] >= 0);
            }
        oracle_scores(dc, off, L, qc, mq, cand, n_c, sc3);
        for (uint32_t i = 0; i < n_c; ++i) CHECK(sc3[i] == sc[cand[i]]);
        /* top-k: descending scores, ties by ascending id, padding when k exceeds the list */
        uint32_t *ids = block(k * sizeof(uint32_t));
        int32_t *ts = block(k * sizeof(int32_t));
        oracle_topk(sc, NULL, n_docs, k, ids, ts);
        for (uint32_t r = 0; r < k; ++r) {
            if (r >= n_docs) { CHECK(ids[r] == 0xFFFFFFFFu && ts[r] == -1); continue; }
            CHECK(ts[r] == sc[ids[r]]);
            if (r) CHECK(ts[r - 1] > ts[r] || (ts[r - 1] == ts[r] && ids[r - 1] < ids[r]));
        }
        free(dc); free(qc); free(proj); free(sc); free(sc2); free(sim); free(cand); free(sc3); free(w); free(tab);
        free(ids); free(ts);
        /* fp path on the same numbers */
        float *Xf = block(V * d * sizeof(float)), *Rf = block((size_t)P * d * sizeof(float));
        for (uint64_t i = 0; i < V * d; ++i) Xf[i] = (float)X[i] / 127.0f;
        for (uint64_t i = 0; i < (uint64_t)P * d; ++i) Rf[i] = (float)((int)(rnd() % 2001) - 1000) / 500.0f;
        uint8_t *fc = block(V * L);
        double *fp = block(V * P * sizeof(double));
        oracle_hash_fp(Xf, V, d, Rf, L, C, fc, fp);
        for (uint64_t i = 0; i < V * L; ++i) CHECK(fc[i] < (1u << C));
        free(Xf); free(Rf); free(fc); free(fp);
    } else {
        uint16_t *dc = block(V * L * 2), *qc = block((size_t)mq * L * 2);
        oracle_hash_i8_wide(X, V, d, R, L, C, dc);
        oracle_hash_i8_wide(Q, mq, d, R, L, C, qc);
        for (uint64_t i = 0; i < V * L; ++i) CHECK(dc[i] < (1u << C));
        int32_t *sc = block(n_docs * sizeof(int32_t));
        oracle_scores_wide(dc, off, L, 0, qc, mq, NULL, n_docs, sc);
        for (uint32_t i = 0; i < n_docs; ++i) CHECK(sc[i] >= 0 && sc[i] <= (int32_t)(mq * L));
        if (full_doc < n_docs) CHECK(sc[full_doc] == (int32_t)(mq * L));
        oracle_scores_wide(dc, off, L, C, qc, mq, NULL, n_docs, sc);
        double *tab = block((L + 1) * sizeof(double));
        oracle_scores_general(dc, off, L, 2, 1, C, 1, qc, mq, NULL, NULL, n_docs, sc, tab);
        float *Xf = block(V * d * sizeof(float)), *Rf = block((size_t)P * d * sizeof(float));
        for (uint64_t i = 0; i < V * d; ++i) Xf[i] = (float)X[i];
        for (uint64_t i = 0; i < (uint64_t)P * d; ++i) Rf[i] = (float)R[i];
        uint16_t *fc = block(V * L * 2);
        oracle_hash_fp_wide(Xf, V, d, Rf, L, C, fc, NULL);
        for (uint64_t i = 0; i < V * L; ++i) CHECK(fc[i] == dc[i]);  /* same numbers in float: same codes */
        free(dc); free(qc); free(sc); free(tab); free(Xf); free(Rf); free(fc);
    }

    /* candidate filter and k-means */
    const uint32_t K = 1 + rnd() % 9;
    int8_t *Cn = block((size_t)K * d);
    for (uint64_t i = 0; i < (uint64_t)K * d; ++i) Cn[i] = rnd_i8();
    int32_t *assign = block(V * sizeof(int32_t));
    oracle_assign_centroids(X, V, d, Cn, K, assign);
    for (uint64_t v = 0; v < V; ++v) CHECK(assign[v] >= 0 && assign[v] < (int32_t)K);
    int64_t *boff = block((K + 1) * sizeof(int64_t));
    uint32_t *bdocs = block(V * sizeof(uint32_t));
    oracle_inverted_index(assign, off, n_docs, K, boff, bdocs);
    CHECK(boff[0] == 0 && boff[K] <= (int64_t)V);
    for (int64_t e = 0; e < boff[K]; ++e) CHECK(bdocs[e] < n_docs);
    const uint32_t probe = 1 + rnd() % K, fk = 1 + rnd() % (n_docs + 4);
    uint32_t *fid = block(fk * sizeof(uint32_t));
    int32_t *fcn = block(fk * sizeof(int32_t));
    oracle_filter_query(Q, mq, d, Cn, K, boff, bdocs, n_docs, probe, fk, fid, fcn);
    for (uint32_t r = 0; r < fk; ++r) {
        CHECK((fid[r] == 0xFFFFFFFFu) == (fcn[r] == -1));
        if (fcn[r] > 0) CHECK(fcn[r] <= (int32_t)(mq * probe) && fid[r] < n_docs);
        if (r && fcn[r] != -1) CHECK(fcn[r - 1] > fcn[r] || (fcn[r - 1] == fcn[r] && fid[r - 1] < fid[r]));
    }
    int64_t inertia[4] = {0, 0, 0, 0};
    oracle_kmeans(X, V, d, Cn, K, 3, inertia);
    if (V) CHECK(inertia[0] >= inertia[1] && inertia[1] >= inertia[2]);  /* Lloyd steps with exact means would never go up; rounded means may by rounding only */
    free(Cn); free(assign); free(boff); free(bdocs); free(fid); free(fcn);
    free(off); free(X); free(Q); free(R);
}

int main(void)
{
    CHECK(oracle_num_threads() >= 1);
    /* d, L, C, documents, longest document, query vectors, k */
    one_case(8, 4, 3, 0, 0, 1, 3);       /* no documents at all */
    one_case(8, 4, 3, 5, 0, 2, 7);       /* only empty documents */
    one_case(16, 8, 7, 1, 9, 4, 1);
    one_case(33, 5, 8, 40, 12, 9, 64);   /* odd d and L, k above the number of documents */
    one_case(64, 32, 7, 60, 40, 32, 10);
    one_case(24, 16, 1, 30, 5, 40, 5);   /* one-bit codes, a query longer than 32 vectors */
    one_case(16, 8, 11, 25, 20, 6, 4);   /* 16-bit codes */
    one_case(10, 3, 16, 12, 7, 3, 20);
    for (int i = 0; i < 12; ++i)
        one_case(4 + rnd() % 60, 1 + rnd() % 40, 1 + rnd() % 8, rnd() % 50, rnd() % 30, 1 + rnd() % 50, 1 + rnd() % 70);
    puts("oracle sanitizer run: ok");
    return 0;
}
