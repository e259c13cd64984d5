/*
 * Seeded synthetic LDA corpus generator (test / benchmark input only).
 *
 * Draws a corpus from the LDA generative process: planted topics over a
 * Zipf-ordered vocabulary, per-document topic mixtures, document lengths from a
 * Poisson or a lognormal law.  It stands in for the corpora of Table 3 (NYTimes,
 * PubMed, ClueWeb12 subset), which are not available; only their shape
 * (D, V, T, T/D) is reproduced.
 *
 * This file holds none of the sampler's arithmetic: it only produces
 * (doc_ptr, word_ids, true_topic).  Both the CPU oracle and the GPU path consume
 * its output; neither shares code with it.
 *
 * Every random stream is a function of (seed, stream kind, index) only, so the
 * output does not depend on the number of threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct { uint64_t s[4]; } rng_t;

static inline uint64_t splitmix64(uint64_t *x) {
    uint64_t z = (*x += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static inline uint64_t rotl64(uint64_t x, int k) { return (x << k) | (x >> (64 - k)); }

static void rng_seed(rng_t *r, uint64_t seed, uint64_t kind, uint64_t index) {
    uint64_t x = seed * 0xD1342543DE82EF95ull + kind * 0x2545F4914F6CDD1Dull + index;
    x ^= index << 32;
    for (int i = 0; i < 4; i++) r->s[i] = splitmix64(&x);
}
/* xoshiro256** step */
static inline uint64_t rng_next(rng_t *r) {
    uint64_t *s = r->s;
    uint64_t result = rotl64(s[1] * 5, 7) * 9;
    uint64_t t = s[1] << 17;
    s[2] ^= s[0]; s[3] ^= s[1]; s[1] ^= s[2]; s[0] ^= s[3];
    s[2] ^= t; s[3] = rotl64(s[3], 45);
    return result;
}
/* uniform in (0,1) */
static inline double rng_u(rng_t *r) { return ((double)(rng_next(r) >> 11) + 0.5) * (1.0 / 9007199254740992.0); }
static double rng_normal(rng_t *r) {
    double u1 = rng_u(r), u2 = rng_u(r);
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586 * u2);
}
/* log of a Gamma(a,1) variate; works for very small a without underflow */
static double rng_log_gamma(rng_t *r, double a) {
    double boost = 0.0;
    if (a < 1.0) { boost = log(rng_u(r)) / a; a += 1.0; }
    double d = a - 1.0 / 3.0, c = 1.0 / sqrt(9.0 * d);
    for (;;) {
        double x = rng_normal(r), v = 1.0 + c * x;
        if (v <= 0.0) continue;
        v = v * v * v;
        double u = rng_u(r);
        if (log(u) < 0.5 * x * x + d - d * v + d * log(v)) return log(d * v) + boost;
    }
}
static int64_t rng_poisson(rng_t *r, double lam) {
    /* sum of exponentials for small lambda, normal approximation rounded for large */
    if (lam < 30.0) {
        double L = exp(-lam), p = 1.0; int64_t k = 0;
        do { k++; p *= rng_u(r); } while (p > L);
        return k - 1;
    }
    /* PTRS would be exact; a split into chunks of <30 keeps it exact and simple */
    int64_t total = 0; double rest = lam;
    while (rest > 0.0) { double part = rest < 25.0 ? rest : 25.0; total += rng_poisson(r, part); rest -= part; }
    return total;
}

/* first index i in [0,n) with cdf[i] >= x (cdf non-decreasing, cdf[n-1] is the total) */
static inline int32_t cdf_find(const double *cdf, int32_t n, double x) {
    int32_t lo = 0, hi = n - 1;
    while (lo < hi) { int32_t mid = (lo + hi) >> 1; if (cdf[mid] >= x) hi = mid; else lo = mid + 1; }
    return lo;
}

/*
 * length_kind: 0 = Poisson(length_mean) (sum left as drawn),
 *              1 = lognormal with mean length_mean and log-sigma length_sigma,
 *                  rescaled so that the lengths sum to T_target exactly.
 * Step 1: lda_corpus_lengths fills doc_ptr[D+1] and returns T.
 * Step 2: lda_corpus_fill writes word_ids[T] (and true_topic[T] if not NULL).
 */
int64_t lda_corpus_lengths(uint64_t seed, int64_t D, int length_kind, double length_mean,
                           double length_sigma, int64_t T_target, int64_t *doc_ptr) {
    if (D < 0 || !doc_ptr) return -1;
    doc_ptr[0] = 0;
    if (length_kind == 0) {
        for (int64_t d = 0; d < D; d++) {
            rng_t r; rng_seed(&r, seed, 1, (uint64_t)d);
            int64_t len = rng_poisson(&r, length_mean);
            doc_ptr[d + 1] = doc_ptr[d] + len;
        }
        return doc_ptr[D];
    }
    double *raw = (double *)malloc(sizeof(double) * (size_t)(D > 0 ? D : 1));
    if (!raw) return -2;
    double mu = log(length_mean) - 0.5 * length_sigma * length_sigma, sum = 0.0;
    for (int64_t d = 0; d < D; d++) {
        rng_t r; rng_seed(&r, seed, 1, (uint64_t)d);
        raw[d] = exp(mu + length_sigma * rng_normal(&r));
        sum += raw[d];
    }
    double scale = (T_target > 0 && sum > 0) ? (double)T_target / sum : 1.0;
    int64_t total = 0;
    for (int64_t d = 0; d < D; d++) {
        int64_t len = (int64_t)llround(raw[d] * scale);
        if (len < 1) len = 1;
        doc_ptr[d + 1] = len; total += len;
    }
    free(raw);
    if (T_target > 0 && D > 0) {
        /* spread the rounding remainder one token at a time over the documents in order */
        int64_t diff = T_target - total, d = 0, guard = 0;
        while (diff != 0 && guard < 64 * D) {
            if (diff > 0) { doc_ptr[d + 1]++; diff--; }
            else if (doc_ptr[d + 1] > 1) { doc_ptr[d + 1]--; diff++; }
            d = (d + 1) % D; guard++;
        }
    }
    for (int64_t d = 0; d < D; d++) doc_ptr[d + 1] += doc_ptr[d];
    return doc_ptr[D];
}

int lda_corpus_fill(uint64_t seed, int64_t D, int32_t V, int32_t K_true, double zipf_s,
                    double topic_conc, double doc_conc, const int64_t *doc_ptr,
                    int32_t *word_ids, int32_t *true_topic, int nthreads) {
    if (D < 0 || V < 1 || K_true < 1 || !doc_ptr || !word_ids) return -1;
    if (nthreads < 1) nthreads = 1;
    /* mean word frequencies m_v ~ (v+1)^-s */
    double *logm = (double *)malloc(sizeof(double) * (size_t)V);
    double *tw = (double *)malloc(sizeof(double) * (size_t)V * (size_t)K_true); /* per-topic word cdf */
    if (!logm || !tw) { free(logm); free(tw); return -2; }
    double H = 0.0;
    for (int32_t v = 0; v < V; v++) H += pow((double)v + 1.0, -zipf_s);
    for (int32_t v = 0; v < V; v++) logm[v] = -zipf_s * log((double)v + 1.0) - log(H);

    /* topic k ~ Dirichlet(topic_conc * V * m): gammas in log space, then normalise */
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int32_t k = 0; k < K_true; k++) {
        rng_t r; rng_seed(&r, seed, 2, (uint64_t)k);
        double *row = tw + (size_t)k * (size_t)V;
        double mx = -INFINITY;
        for (int32_t v = 0; v < V; v++) {
            double a = topic_conc * (double)V * exp(logm[v]);
            row[v] = rng_log_gamma(&r, a);
            if (row[v] > mx) mx = row[v];
        }
        double run = 0.0;
        for (int32_t v = 0; v < V; v++) { run += exp(row[v] - mx); row[v] = run; }
    }

    /* LDA_CORPUS_PROGRESS=n: report on stderr every time another n documents are done (long generations) */
    const char *prog_env = getenv("LDA_CORPUS_PROGRESS");
    const int64_t prog_every = prog_env ? atoll(prog_env) : 0;
    int64_t docs_done = 0;
#pragma omp parallel num_threads(nthreads)
    {
        double *theta = (double *)malloc(sizeof(double) * (size_t)K_true);
#pragma omp for schedule(dynamic, 64)
        for (int64_t d = 0; d < D; d++) {
            if (prog_every > 0) {
                int64_t n;
#pragma omp atomic capture
                n = ++docs_done;
                if (n % prog_every == 0) { fprintf(stderr, "[corpusgen] %lld of %lld documents\n", (long long)n, (long long)D); fflush(stderr); }
            }
            int64_t b = doc_ptr[d], e = doc_ptr[d + 1];
            if (e <= b) continue;
            rng_t r; rng_seed(&r, seed, 3, (uint64_t)d);
            double mx = -INFINITY;
            for (int32_t k = 0; k < K_true; k++) { theta[k] = rng_log_gamma(&r, doc_conc); if (theta[k] > mx) mx = theta[k]; }
            double run = 0.0;
            for (int32_t k = 0; k < K_true; k++) { run += exp(theta[k] - mx); theta[k] = run; }
            for (int64_t t = b; t < e; t++) {
                int32_t k = cdf_find(theta, K_true, rng_u(&r) * run);
                const double *row = tw + (size_t)k * (size_t)V;
                int32_t w = cdf_find(row, V, rng_u(&r) * row[V - 1]);
                word_ids[t] = w;
                if (true_topic) true_topic[t] = k;
            }
        }
        free(theta);
    }
    free(logm); free(tw);
    return 0;
}
