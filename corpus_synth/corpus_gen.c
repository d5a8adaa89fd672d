/*
 * Seeded synthetic LDA corpora.
 *
 * This module only makes INPUTS (documents, word ids, and the topics the
 * generative process used).  It holds none of the sampler's arithmetic and is
 * the one module that both the CPU oracle's tests and the GPU library's tests
 * may use.
 *
 * The corpus follows the LDA generative process in its collapsed (urn) form,
 * which has exactly the same distribution as drawing theta_d ~ Dir(alpha_gen)
 * and phi_k ~ Dir(beta_gen * V * m) first, but costs O(#tokens):
 *
 *   topic of the i-th token of a document (i = 0,1,..):
 *       with probability K*alpha_gen / (i + K*alpha_gen)  a uniform topic,
 *       otherwise the topic of a uniformly chosen earlier token of the document;
 *   word of the i-th token that carries topic k (tokens taken in corpus order):
 *       with probability beta_gen*V / (i + beta_gen*V)    a word drawn from the
 *       base measure m (Zipf over frequency ranks, m_r ~ (r+1)^-s),
 *       otherwise the word of a uniformly chosen earlier token of topic k.
 *
 * Word ids are a fixed random permutation of the frequency ranks.  Every random
 * stream is keyed by (seed, purpose, document-or-topic index), so the result
 * does not depend on the number of threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct { uint64_t s; } stream_t;

static inline uint64_t sm64_next(stream_t* g) {
    uint64_t z = (g->s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline stream_t stream_open(uint64_t seed, uint64_t purpose, uint64_t index) {
    stream_t g;
    g.s = seed;
    uint64_t a = sm64_next(&g);
    g.s = a ^ (purpose * 0xD6E8FEB86659FD93ull);
    uint64_t b = sm64_next(&g);
    g.s = b ^ (index * 0xA0761D6478BD642Full);
    (void)sm64_next(&g);
    return g;
}

static inline double stream_u01(stream_t* g) {           /* [0,1) */
    return (double)(sm64_next(g) >> 11) * (1.0 / 9007199254740992.0);
}

static inline uint64_t stream_below(stream_t* g, uint64_t n) {   /* [0,n), n >= 1 */
    /* 128-bit multiply keeps the bias below 2^-64 * n, irrelevant here */
    return (uint64_t)(((__uint128_t)sm64_next(g) * (__uint128_t)n) >> 64);
}

static double stream_normal(stream_t* g) {
    double u1 = 1.0 - stream_u01(g);                    /* (0,1] */
    double u2 = stream_u01(g);
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
}

static int64_t stream_poisson_small(stream_t* g, double lambda) {
    /* product-of-uniforms method; exp(-lambda) must stay a normal number */
    double limit = exp(-lambda), p = 1.0;
    int64_t n = -1;
    do { p *= stream_u01(g); ++n; } while (p > limit);
    return n;
}

static int64_t stream_poisson(stream_t* g, double lambda) {
    /* a Poisson variate of large mean is the sum of independent ones of small means */
    int64_t n = 0;
    while (lambda > 500.0) { n += stream_poisson_small(g, 500.0); lambda -= 500.0; }
    return n + stream_poisson_small(g, lambda);
}

/*
 * Document lengths -> doc_ptr[0..D] (doc_ptr[0] = 0).
 * law 0: Poisson(p1), law 1: lognormal with log-mean p1 and log-sd p2, rounded.
 * Every document has at least one token.  Returns the token count.
 */
int64_t corpus_doc_lengths(int64_t D, int law, double p1, double p2, uint64_t seed,
                           int64_t* doc_ptr) {
    doc_ptr[0] = 0;
#pragma omp parallel for schedule(static)
    for (int64_t d = 0; d < D; ++d) {
        stream_t g = stream_open(seed, 1, (uint64_t)d);
        int64_t n;
        if (law == 0) n = stream_poisson(&g, p1);
        else          n = (int64_t)llround(exp(p1 + p2 * stream_normal(&g)));
        if (n < 1) n = 1;
        doc_ptr[d + 1] = n;
    }
    for (int64_t d = 0; d < D; ++d) doc_ptr[d + 1] += doc_ptr[d];
    return doc_ptr[D];
}

/* Walker alias table for the Zipf base measure over ranks 0..V-1. */
typedef struct { double* prob; int32_t* alias; int32_t n; } alias_t;

static int alias_build(alias_t* a, int32_t V, double s) {
    a->n = V;
    a->prob = (double*)malloc(sizeof(double) * (size_t)V);
    a->alias = (int32_t*)malloc(sizeof(int32_t) * (size_t)V);
    double* w = (double*)malloc(sizeof(double) * (size_t)V);
    int32_t* small = (int32_t*)malloc(sizeof(int32_t) * (size_t)V);
    int32_t* large = (int32_t*)malloc(sizeof(int32_t) * (size_t)V);
    if (!a->prob || !a->alias || !w || !small || !large) return -1;
    double tot = 0.0;
    for (int32_t r = 0; r < V; ++r) { w[r] = pow((double)r + 1.0, -s); tot += w[r]; }
    int32_t ns = 0, nl = 0;
    for (int32_t r = 0; r < V; ++r) {
        w[r] = w[r] * (double)V / tot;
        if (w[r] < 1.0) small[ns++] = r; else large[nl++] = r;
    }
    while (ns > 0 && nl > 0) {
        int32_t sidx = small[--ns], lidx = large[--nl];
        a->prob[sidx] = w[sidx];
        a->alias[sidx] = lidx;
        w[lidx] = (w[lidx] + w[sidx]) - 1.0;
        if (w[lidx] < 1.0) small[ns++] = lidx; else large[nl++] = lidx;
    }
    while (nl > 0) { int32_t i = large[--nl]; a->prob[i] = 1.0; a->alias[i] = i; }
    while (ns > 0) { int32_t i = small[--ns]; a->prob[i] = 1.0; a->alias[i] = i; }
    free(w); free(small); free(large);
    return 0;
}

static inline int32_t alias_draw(const alias_t* a, stream_t* g) {
    int32_t i = (int32_t)stream_below(g, (uint64_t)a->n);
    return (stream_u01(g) < a->prob[i]) ? i : a->alias[i];
}

/*
 * Fill word_ids[T] (int32, document-major) and z_true[T] (uint16, the topic the
 * process used for each token) for the documents laid out by doc_ptr.
 * Returns 0, or -1 on allocation failure / bad arguments.
 */
int corpus_fill(int64_t D, const int64_t* doc_ptr, int32_t V, int32_t K,
                double alpha_gen, double beta_gen, double zipf_s, uint64_t seed,
                int32_t* word_ids, uint16_t* z_true, int nthreads) {
    if (D < 0 || V < 1 || K < 1 || K > 65535) return -1;
    const int64_t T = doc_ptr[D];
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif

    /* 1. topics, document by document */
    const double ka = (double)K * alpha_gen;
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t d = 0; d < D; ++d) {
        stream_t g = stream_open(seed, 2, (uint64_t)d);
        const int64_t b = doc_ptr[d], n = doc_ptr[d + 1] - b;
        for (int64_t i = 0; i < n; ++i) {
            if (stream_u01(&g) * ((double)i + ka) < ka)
                z_true[b + i] = (uint16_t)stream_below(&g, (uint64_t)K);
            else
                z_true[b + i] = z_true[b + (int64_t)stream_below(&g, (uint64_t)i)];
        }
    }

    /* 2. tokens of each topic, in corpus order */
    int64_t* start = (int64_t*)calloc((size_t)K + 1, sizeof(int64_t));
    int32_t* rank_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    int64_t* member = (int64_t*)malloc(sizeof(int64_t) * (size_t)(T > 0 ? T : 1));
    int32_t* perm = (int32_t*)malloc(sizeof(int32_t) * (size_t)V);
    alias_t base;
    if (!start || !rank_of || !member || !perm || alias_build(&base, V, zipf_s) != 0) return -1;
    for (int64_t t = 0; t < T; ++t) start[z_true[t] + 1]++;
    for (int32_t k = 0; k < K; ++k) start[k + 1] += start[k];
    {
        int64_t* cur = (int64_t*)malloc(sizeof(int64_t) * (size_t)K);
        if (!cur) return -1;
        memcpy(cur, start, sizeof(int64_t) * (size_t)K);
        for (int64_t t = 0; t < T; ++t) member[cur[z_true[t]]++] = t;
        free(cur);
    }

    /* 3. words, topic by topic (frequency ranks first) */
    const double bv = beta_gen * (double)V;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t k = 0; k < K; ++k) {
        stream_t g = stream_open(seed, 3, (uint64_t)k);
        int32_t* mine = rank_of + start[k];
        const int64_t n = start[k + 1] - start[k];
        for (int64_t i = 0; i < n; ++i) {
            if (stream_u01(&g) * ((double)i + bv) < bv) mine[i] = alias_draw(&base, &g);
            else mine[i] = mine[stream_below(&g, (uint64_t)i)];
        }
    }

    /* 4. rank -> word id through a fixed random permutation */
    {
        stream_t g = stream_open(seed, 4, 0);
        for (int32_t r = 0; r < V; ++r) perm[r] = r;
        for (int32_t r = V - 1; r > 0; --r) {
            int32_t j = (int32_t)stream_below(&g, (uint64_t)r + 1);
            int32_t tmp = perm[r]; perm[r] = perm[j]; perm[j] = tmp;
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < T; ++i) word_ids[member[i]] = perm[rank_of[i]];

    free(start); free(rank_of); free(member); free(perm);
    free(base.prob); free(base.alias);
    return 0;
}

int corpus_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
