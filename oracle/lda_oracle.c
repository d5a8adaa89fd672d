/*
 * CPU oracle for one iteration of collapsed Gibbs sampling for LDA.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the GPU library must compute.  It shares no code with that library; only
 * tests, the smoke check and the benchmark's CPU-baseline leg may call it.
 *
 * What it follows (paper sections / equations):
 *   - Eq. 1 (Section 2.1): p(k) ~ (theta_dk + alpha)(phi_kv + beta) / (sum_v phi_kv + beta V).
 *   - Eq. 6-8 (Section 6.1): p = p1 + p2, p1 = theta_dk p*(k), p2 = alpha p*(k),
 *     p*(k) = (phi_kv + beta)/(n_k + beta V); S = sum p1, Q = sum p2.
 *   - Section 6.1.1 / Algorithm 2: one uniform picks the bucket (p1 if it falls
 *     below S/(S+Q), else p2) and the topic inside it is the smallest k whose
 *     prefix sum exceeds the draw.
 *   - Section 2.1: a full pass over all tokens is an iteration; theta and phi
 *     are rebuilt after the pass.
 *
 * Readings where the paper is silent (each listed in the design notes):
 *   - counts are frozen for the whole iteration and the token's own assignment
 *     is removed from theta, phi and n_k before its conditional is formed;
 *   - p*(k) is the fp64 quotient rounded once to fp32; every product and sum is
 *     fp64, taken in ascending k;
 *   - one 53-bit uniform u per (seed, iteration, token) from Philox4x32-10;
 *     x = u (S+Q); x < S selects the p1 bucket at position x, otherwise the p2
 *     bucket at position x - S; if rounding leaves no prefix above the draw the
 *     last candidate is taken;
 *   - initial topics: iteration 0 of the same generator, z = floor(u K);
 *   - log-likelihood: the joint collapsed log p(w, z) (Dirichlet-multinomial
 *     closed form with lgamma).
 *
 * All arrays are in the caller's document-major token order.
 * Parity pins: tests/test_oracle_*.py (closed-form chi-square, exact rational
 * CDF boundaries, special cases, count invariants, chain-rule likelihood,
 * Philox known answers).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ Philox */

/* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random
 * numbers: as easy as 1, 2, 3", SC'11), written from the paper's round
 * definition: two 32x32->64 multiplies, the high halves xor-ed with the other
 * counter words and the round key; the key advances by the Weyl constants. */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* u in [0,1) with 53 random bits; counter = (token lo, token hi, iteration, 0),
 * key = (seed lo, seed hi). */
double oracle_uniform(uint64_t seed, uint32_t iter, uint64_t token) {
    uint32_t ctr[4] = {(uint32_t)token, (uint32_t)(token >> 32), iter, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t r[4];
    oracle_philox4x32_10(ctr, key, r);
    uint64_t bits = (((uint64_t)r[0] << 32) | (uint64_t)r[1]) >> 11;
    return (double)bits * (1.0 / 9007199254740992.0);
}

void oracle_uniforms(uint64_t seed, uint32_t iter, uint64_t token0, int64_t n, double* u) {
    for (int64_t i = 0; i < n; ++i) u[i] = oracle_uniform(seed, iter, token0 + (uint64_t)i);
}

/* Random initial topics (Section 2.1): every token starts with a uniformly drawn topic. */
void oracle_init_topics(int64_t T, int32_t K, uint64_t seed, uint16_t* z) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        int32_t k = (int32_t)(oracle_uniform(seed, 0u, (uint64_t)t) * (double)K);
        if (k > K - 1) k = K - 1;
        z[t] = (uint16_t)k;
    }
}

/* ------------------------------------------------------------------ counts */

/* phi as a word-major matrix n_wk[v*K + k] and its column sums n_k[k]. */
void oracle_count_word_topic(int64_t T, const int32_t* word_ids, const uint16_t* z,
                             int32_t V, int32_t K, int32_t* n_wk, int32_t* n_k) {
    memset(n_wk, 0, sizeof(int32_t) * (size_t)V * (size_t)K);
    memset(n_k, 0, sizeof(int32_t) * (size_t)K);
    for (int64_t t = 0; t < T; ++t) {
        n_wk[(size_t)word_ids[t] * (size_t)K + z[t]] += 1;
        n_k[z[t]] += 1;
    }
}

/* One dense row of theta: n_d[k] = number of tokens of the document with topic k. */
static void count_doc_row(const uint16_t* z, int64_t begin, int64_t end, int32_t K, int32_t* n_d) {
    memset(n_d, 0, sizeof(int32_t) * (size_t)K);
    for (int64_t t = begin; t < end; ++t) n_d[z[t]] += 1;
}

/* theta in CSR form: per document the topics with a non-zero count, ascending,
 * and their counts.  row_ptr has D+1 entries.  Returns the number of entries. */
int64_t oracle_doc_topic_csr(int64_t D, const int64_t* doc_ptr, const uint16_t* z, int32_t K,
                             int64_t* row_ptr, uint16_t* topics, int32_t* counts) {
    int32_t* n_d = (int32_t*)malloc(sizeof(int32_t) * (size_t)K);
    int64_t nnz = 0;
    row_ptr[0] = 0;
    for (int64_t d = 0; d < D; ++d) {
        count_doc_row(z, doc_ptr[d], doc_ptr[d + 1], K, n_d);
        for (int32_t k = 0; k < K; ++k)
            if (n_d[k] > 0) {
                if (topics) topics[nnz] = (uint16_t)k;
                if (counts) counts[nnz] = n_d[k];
                ++nnz;
            }
        row_ptr[d + 1] = nnz;
    }
    free(n_d);
    return nnz;
}

/* ------------------------------------------------------------- one token */

/*
 * Resample one token.  n_d, n_w, n_k are the frozen dense count rows of the
 * token's document, of its word, and the topic totals, all INCLUDING the token
 * itself; o is its current topic; u its uniform.  work holds 2K doubles.
 * Optionally reports S and Q.
 */
int32_t oracle_resample_token(int32_t K, int32_t V, double alpha, double beta,
                              const int32_t* n_d, const int32_t* n_w, const int32_t* n_k,
                              int32_t o, double u, double* work, double* S_out, double* Q_out) {
    double* p1 = work;
    double* p2 = work + K;
    const double beta_V = beta * (double)V;
    double S = 0.0, Q = 0.0;
    for (int32_t k = 0; k < K; ++k) {
        const int32_t own = (k == o) ? 1 : 0;
        const int32_t th = n_d[k] - own;
        const int32_t ph = n_w[k] - own;
        const int32_t nk = n_k[k] - own;
        const float pstar = (float)(((double)ph + beta) / ((double)nk + beta_V));   /* Eq. 8 */
        p1[k] = (double)th * (double)pstar;                                           /* Eq. 6 */
        p2[k] = alpha * (double)pstar;
        S += p1[k];                                                                   /* Eq. 7 */
        Q += p2[k];
    }
    if (S_out) *S_out = S;
    if (Q_out) *Q_out = Q;
    const double x = u * (S + Q);
    if (x < S) {
        double prefix = 0.0;
        int32_t last = -1;
        for (int32_t k = 0; k < K; ++k) {
            if (p1[k] > 0.0) last = k;
            prefix += p1[k];
            if (prefix > x) return k;
        }
        return last;              /* rounding left no prefix above x */
    } else {
        const double y = x - S;
        double prefix = 0.0;
        for (int32_t k = 0; k < K; ++k) {
            prefix += p2[k];
            if (prefix > y) return k;
        }
        return K - 1;
    }
}

/* ---------------------------------------------------------- one iteration */

/*
 * One full pass: every token is resampled from the counts of z as they stand
 * at the start of the pass.  n_wk / n_k must be the counts of z (see
 * oracle_count_word_topic).  iter >= 1 keys the uniforms.  Tokens are
 * independent, so documents are spread over threads.
 */
void oracle_iteration(int64_t D, const int64_t* doc_ptr, const int32_t* word_ids, const uint16_t* z,
                      int32_t V, int32_t K, double alpha, double beta, uint64_t seed, uint32_t iter,
                      const int32_t* n_wk, const int32_t* n_k, uint16_t* z_new, int nthreads) {
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
#pragma omp parallel
    {
        int32_t* n_d = (int32_t*)malloc(sizeof(int32_t) * (size_t)K);
        double* work = (double*)malloc(sizeof(double) * 2 * (size_t)K);
#pragma omp for schedule(dynamic, 64)
        for (int64_t d = 0; d < D; ++d) {
            count_doc_row(z, doc_ptr[d], doc_ptr[d + 1], K, n_d);
            for (int64_t t = doc_ptr[d]; t < doc_ptr[d + 1]; ++t) {
                const double u = oracle_uniform(seed, iter, (uint64_t)t);
                z_new[t] = (uint16_t)oracle_resample_token(
                    K, V, alpha, beta, n_d, n_wk + (size_t)word_ids[t] * (size_t)K, n_k,
                    (int32_t)z[t], u, work, 0, 0);
            }
        }
        free(n_d);
        free(work);
    }
}

/*
 * The same draw for a chosen list of tokens only (token index, document-major,
 * with the document of each given): lets a test check single outputs of a
 * corpus too large to pass over on the CPU.  Listed tokens are independent, so
 * they are spread over threads (each with its own dense row and work space).
 */
void oracle_resample_listed(int64_t n_listed, const int64_t* token, const int64_t* doc,
                            const int64_t* doc_ptr, const int32_t* word_ids, const uint16_t* z,
                            int32_t V, int32_t K, double alpha, double beta, uint64_t seed,
                            uint32_t iter, const int32_t* n_wk, const int32_t* n_k,
                            uint16_t* z_new) {
#pragma omp parallel
    {
        int32_t* row = (int32_t*)malloc(sizeof(int32_t) * (size_t)K);
        double* scratch = (double*)malloc(sizeof(double) * 2 * (size_t)K);
#pragma omp for schedule(dynamic, 256)
        for (int64_t i = 0; i < n_listed; ++i) {
            const int64_t t = token[i], d = doc[i];
            count_doc_row(z, doc_ptr[d], doc_ptr[d + 1], K, row);
            const double u = oracle_uniform(seed, iter, (uint64_t)t);
            const int32_t* n_w = n_wk + (size_t)word_ids[t] * (size_t)K;
            z_new[i] = (uint16_t)oracle_resample_token(K, V, alpha, beta, row, n_w, n_k,
                                                       (int32_t)z[t], u, scratch, 0, 0);
        }
        free(row);
        free(scratch);
    }
}

/* -------------------------------------------------------- log-likelihood */

/*
 * Joint collapsed log-likelihood log p(w, z | alpha, beta):
 *   sum_k [ lgG(V beta) - lgG(n_k + V beta) + sum_v (lgG(n_wk + beta) - lgG(beta)) ]
 * + sum_d [ lgG(K alpha) - lgG(N_d + K alpha) + sum_k (lgG(n_dk + alpha) - lgG(alpha)) ].
 * Zero counts contribute nothing to the inner sums.
 */
double oracle_loglik(int64_t D, const int64_t* doc_ptr, const uint16_t* z, int32_t V, int32_t K,
                     double alpha, double beta, const int32_t* n_wk, const int32_t* n_k) {
    const double v_beta = (double)V * beta, k_alpha = (double)K * alpha;
    const double lg_beta = lgamma(beta), lg_alpha = lgamma(alpha);
    double word_side = 0.0, doc_side = 0.0;
    for (int32_t k = 0; k < K; ++k) word_side += lgamma(v_beta) - lgamma((double)n_k[k] + v_beta);
    for (size_t i = 0; i < (size_t)V * (size_t)K; ++i)
        if (n_wk[i] > 0) word_side += lgamma((double)n_wk[i] + beta) - lg_beta;
    int32_t* n_d = (int32_t*)malloc(sizeof(int32_t) * (size_t)K);
    for (int64_t d = 0; d < D; ++d) {
        const int64_t len = doc_ptr[d + 1] - doc_ptr[d];
        count_doc_row(z, doc_ptr[d], doc_ptr[d + 1], K, n_d);
        doc_side += lgamma(k_alpha) - lgamma((double)len + k_alpha);
        for (int32_t k = 0; k < K; ++k)
            if (n_d[k] > 0) doc_side += lgamma((double)n_d[k] + alpha) - lg_alpha;
    }
    free(n_d);
    return word_side + doc_side;
}

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
