/*
 * CPU ORACLE for the sparsity-aware LDA sampler (ESCA E-step + M-step).
 *
 * TEST INFRASTRUCTURE ONLY.  A plain, slow, single-pass implementation written
 * from the paper's definitions, used to check the GPU library and to report a
 * CPU baseline.  It shares no code with the GPU path and must never be called
 * by it.  Only tests, the smoke check and the benchmark's cpu_baseline leg may
 * load this file.
 *
 * What follows the paper, and where:
 *   - E-step distribution p(k) ~ (A_dk + alpha) * Bhat_vk            (Sec. 2.2, Eq. 1)
 *   - Bhat_vk = (B_vk + beta) / (sum_v B_vk + V beta)                (Sec. 2.2, Eq. 2)
 *   - inverse-CDF draw: first k with u <= c_k                        (Sec. 2.3, steps 1-3)
 *   - sparsity-aware split: branch 1 w.p. S/(S+Q_v),
 *       S = sum_k A_dk Bhat_vk,  Q_v = alpha sum_k Bhat_vk           (Sec. 2.3; Alg. 2)
 *   - BSP iteration: all tokens sample from counts frozen at the
 *     previous M-step; then CountByDZ, CountByVZ, Preprocess,
 *     BuildTree                                                      (Alg. 1; Sec. 2.4)
 *   - W-ary tree: bottom level = prefix sums, node i of an upper
 *     level = node (i+1)W-1 of the level below (0-based), child
 *     window of node i is [iW, iW+W-1]                               (Sec. 3.2.4; Fig. 4)
 *
 * Readings of points the paper leaves open (all listed in the design notes):
 *   - no "minus current token" correction (Eq. 1 has none);
 *   - rows of A are kept in ascending topic order (the segmented count sorts by k);
 *   - random numbers: Philox4x32-10, key = seed, counter = (token index lo, hi,
 *     iteration, 0); word 0 -> coin, word 1 -> position; u = top 24 bits * 2^-24;
 *   - initial assignment (iteration 0): z = floor(word0 * K / 2^32);
 *   - Bhat is stored in binary32, each operation of Eq. 2 rounded once;
 *   - S and the sparse-branch prefix sums are accumulated in binary64 (products of a
 *     count and a binary32 Bhat are exact in binary64);
 *   - the per-word prefix table is stored in binary32 like the paper's tree levels:
 *     c32[k] = round32(sum_{j<=k} Bhat_j accumulated in binary64); the dense-branch
 *     decision "first k with c32[k] >= x" is taken in binary32 with
 *     x = round32(u1 * c32[K-1]);
 *   - if rounding leaves no index satisfying the test, the last one is returned.
 *
 * Pins (see tests/, all run without a GPU): Philox known-answer vectors, the
 * worked inverse-CDF example of Fig. 2, count invariants and brute-force
 * histograms, column sums of Bhat, K=1 closed forms, tree query == linear scan
 * for several W, the split sampler's induced measure and chi-square against the
 * dense Eq. 1, planted-topic recovery, dense evaluation of the log-likelihood;
 * holdout log-likelihood: K=1 closed form, the no-observation closed form, dense
 * evaluation from the returned assignments, improvement under fold-in; alias tables:
 * two hand-worked tables, the mass every table must encode, the measure a grid of
 * draws induces, chi-square of the alias E-step against the dense Eq. 1.
 * The realised sample path z itself has no printed reference in the paper:
 * "parity unpinned" beyond the distributional and invariant pins above.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ Philox4x32-10 */
/* Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3" (SC'11). */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; round++) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static void token_random(uint64_t seed, uint64_t t, uint32_t iter, uint32_t out[4]) {
    uint32_t ctr[4] = { (uint32_t)t, (uint32_t)(t >> 32), iter, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    orc_philox4x32_10(ctr, key, out);
}
static double unit24(uint32_t r) { return (double)(r >> 8) * (1.0 / 16777216.0); }

/* the two uniforms of token t at iteration iter (exported for tests) */
void orc_token_uniforms(uint64_t seed, uint64_t t, uint32_t iter, double *u0, double *u1) {
    uint32_t r[4]; token_random(seed, t, iter, r);
    *u0 = unit24(r[0]); *u1 = unit24(r[1]);
}

/* iteration 0: uniform topic per token */
void orc_init_z(int64_t T, int32_t K, uint64_t seed, int32_t *z) {
    for (int64_t t = 0; t < T; t++) {
        uint32_t r[4]; token_random(seed, (uint64_t)t, 0u, r);
        z[t] = (int32_t)(((uint64_t)r[0] * (uint64_t)(uint32_t)K) >> 32);
    }
}

/* ------------------------------------------------------------------ M-step */
/* CountByDZ (Alg. 1; Sec. 3.3): A as CSR with ascending topics, rebuilt per document by
 * sorting the document's assignments and counting runs.  cd_topic/cd_count hold T entries. */
static int cmp_i32(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}
int orc_count_by_dz(int64_t D, const int64_t *doc_ptr, const int32_t *z, int32_t K,
                    int64_t *cd_ptr, int32_t *cd_topic, int32_t *cd_count) {
    int64_t maxlen = 1;
    for (int64_t d = 0; d < D; d++) if (doc_ptr[d + 1] - doc_ptr[d] > maxlen) maxlen = doc_ptr[d + 1] - doc_ptr[d];
    int32_t *keys = (int32_t *)malloc(sizeof(int32_t) * (size_t)maxlen);
    if (!keys) return -2;
    int64_t n = 0;
    cd_ptr[0] = 0;
    for (int64_t d = 0; d < D; d++) {
        int64_t len = doc_ptr[d + 1] - doc_ptr[d];
        for (int64_t i = 0; i < len; i++) {
            keys[i] = z[doc_ptr[d] + i];
            if (keys[i] < 0 || keys[i] >= K) { free(keys); return -1; }
        }
        qsort(keys, (size_t)len, sizeof(int32_t), cmp_i32);
        for (int64_t i = 0; i < len; i++) {
            if (i == 0 || keys[i] != keys[i - 1]) { cd_topic[n] = keys[i]; cd_count[n] = 1; n++; }
            else cd_count[n - 1]++;
        }
        cd_ptr[d + 1] = n;
    }
    free(keys);
    return 0;
}

/* CountByVZ (Alg. 1): B dense V x K (row = word), and the topic totals C_k = sum_v B_vk. */
void orc_count_by_vz(int64_t T, const int32_t *word_ids, const int32_t *z, int32_t V, int32_t K,
                     int32_t *cwk, int64_t *ck) {
    memset(cwk, 0, sizeof(int32_t) * (size_t)V * (size_t)K);
    memset(ck, 0, sizeof(int64_t) * (size_t)K);
    for (int64_t t = 0; t < T; t++) cwk[(size_t)word_ids[t] * (size_t)K + (size_t)z[t]]++;
    for (int32_t v = 0; v < V; v++)
        for (int32_t k = 0; k < K; k++) ck[k] += cwk[(size_t)v * (size_t)K + (size_t)k];
}

/* Preprocess (Eq. 2) in binary32, one rounding per operation:
 * Bhat_vk = (float(B_vk) + beta) / (float(C_k) + float(V)*beta). */
int orc_preprocess(const int32_t *cwk, const int64_t *ck, int32_t V, int32_t K, float beta, float *phi) {
    float *denom = (float *)malloc(sizeof(float) * (size_t)K);
    if (!denom) return -2;
    volatile float vbeta = (float)V * beta;
    for (int32_t k = 0; k < K; k++) { volatile float dk = (float)ck[k] + vbeta; denom[k] = dk; }
    for (int32_t v = 0; v < V; v++)
        for (int32_t k = 0; k < K; k++) {
            volatile float num = (float)cwk[(size_t)v * (size_t)K + (size_t)k] + beta;
            phi[(size_t)v * (size_t)K + (size_t)k] = num / denom[k];
        }
    free(denom);
    return 0;
}

/* BuildTree, bottom level (Alg. 1; Sec. 3.2.4): prefix sums of Bhat_v, binary64 accumulation,
 * stored binary32.  sum64[v] is the binary64 total (used for Q_v = alpha * sum). */
void orc_build_prefix(const float *phi, int32_t V, int32_t K, float *c32, double *sum64) {
    for (int32_t v = 0; v < V; v++) {
        double run = 0.0;
        for (int32_t k = 0; k < K; k++) {
            run += (double)phi[(size_t)v * (size_t)K + (size_t)k];
            c32[(size_t)v * (size_t)K + (size_t)k] = (float)run;
        }
        sum64[v] = run;
    }
}

/* ------------------------------------------------------------------ W-ary tree (Sec. 3.2.4, Fig. 4) */
/*
 * Generic W-ary tree over a non-decreasing bottom array of n values.
 * levels[0] is the bottom; level l+1 has ceil(n_l / W) nodes, node i = level l node
 * min((i+1)W-1, n_l-1).  Building stops at the first level with at most W nodes.
 * Storage: tree[] receives all levels back to back, level_off[l] / level_len[l] index it.
 * Returns the number of levels, or -1 if the caller's capacity is too small.
 */
int orc_wary_build(const float *bottom, int32_t n, int32_t W, float *tree, int64_t tree_cap,
                   int64_t *level_off, int32_t *level_len, int max_levels) {
    if (n < 1 || W < 2 || max_levels < 1 || n > tree_cap) return -1;
    memcpy(tree, bottom, sizeof(float) * (size_t)n);
    int levels = 1; int64_t off = 0; int32_t len = n;
    level_off[0] = 0; level_len[0] = n;
    while (len > W) {
        int32_t up = (len + W - 1) / W;
        if (levels >= max_levels || off + len + up > tree_cap) return -1;
        for (int32_t i = 0; i < up; i++) {
            int64_t j = (int64_t)(i + 1) * W - 1; if (j > len - 1) j = len - 1;
            tree[off + len + i] = tree[off + j];
        }
        off += len; len = up;
        level_off[levels] = off; level_len[levels] = len; levels++;
    }
    return levels;
}

/* position of x: first bottom index whose value is >= x, found by descending from the top level */
int32_t orc_wary_query(const float *tree, const int64_t *level_off, const int32_t *level_len, int levels,
                       int32_t W, float x) {
    int32_t pos = 0;
    for (int l = levels - 1; l >= 0; l--) {
        int32_t lo = pos * W, hi = lo + W;  /* child window of node pos; the top level is one window */
        if (l == levels - 1) { lo = 0; hi = level_len[l]; }
        if (hi > level_len[l]) hi = level_len[l];
        int32_t found = hi - 1;
        for (int32_t i = lo; i < hi; i++)
            if (tree[level_off[l] + i] >= x) { found = i; break; }
        pos = found;
    }
    return pos;
}

/* first index with c[i] >= x by binary search (Sec. 2.3, step 3); last index if none */
static int32_t position_in_prefix32(const float *c, int32_t n, float x) {
    int32_t lo = 0, hi = n - 1;
    while (lo < hi) { int32_t mid = lo + ((hi - lo) >> 1); if (c[mid] >= x) hi = mid; else lo = mid + 1; }
    return lo;
}
int32_t orc_position_in_prefix32(const float *c, int32_t n, float x) { return position_in_prefix32(c, n, x); }

/* ------------------------------------------------------------------ Sample (Alg. 2) */
typedef struct {
    double S;        /* sum_k A_dk Bhat_vk */
    double Q;        /* alpha * sum_k Bhat_vk */
    double p_sparse; /* S / (S + Q) */
    int32_t branch;  /* 1 = sparse (problem 1), 2 = dense (problem 2) */
    int32_t pad;
    double margin;   /* distance, in units of the uniform draws, from the nearest decision boundary */
} orc_detail;

int32_t orc_sample(int32_t nnz, const int32_t *topic, const int32_t *count, const float *phi_w,
                   const float *c32_w, int32_t K, double Q, double u0, double u1, orc_detail *det) {
    double S = 0.0;
    for (int32_t j = 0; j < nnz; j++) S += (double)count[j] * (double)phi_w[topic[j]];
    double thr = S / (S + Q);
    int32_t result; double margin = fabs(u0 - thr); int branch;
    if (u0 < thr) {
        branch = 1;
        double x = u1 * S, run = 0.0, prev = 0.0; int32_t j = 0;
        for (; j < nnz; j++) {
            prev = run; run += (double)count[j] * (double)phi_w[topic[j]];
            if (run >= x) break;
        }
        if (j >= nnz) { j = nnz - 1; }
        result = topic[j];
        double m = fmin(fabs(x - prev), fabs(run - x)) / S;
        if (m < margin) margin = m;
    } else {
        branch = 2;
        float total = c32_w[K - 1];
        volatile float x = (float)u1 * total;
        int32_t k = position_in_prefix32(c32_w, K, x);
        result = k;
        double lo = (k > 0) ? (double)c32_w[k - 1] : 0.0, hi = (double)c32_w[k];
        double m = fmin(fabs((double)x - lo), fabs(hi - (double)x)) / (double)total;
        if (k == 0) m = fabs(hi - (double)x) / (double)total;
        if (m < margin) margin = m;
    }
    if (det) { det->S = S; det->Q = Q; det->p_sparse = thr; det->branch = branch; det->pad = 0; det->margin = margin; }
    return result;
}

/* E-step over all tokens (Alg. 1, E step).  Reads frozen A (CSR), Bhat, prefix table; writes z_new.
 * Optional per-token outputs (may be NULL): S, p_sparse, branch, margin. */
void orc_estep(int64_t D, const int64_t *doc_ptr, const int32_t *word_ids, int32_t K, float alpha,
               const int64_t *cd_ptr, const int32_t *cd_topic, const int32_t *cd_count,
               const float *phi, const float *c32, const double *sum64,
               uint64_t seed, uint32_t iter, int32_t *z_new,
               double *out_S, double *out_p, int8_t *out_branch, double *out_margin, int nthreads) {
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 16) num_threads(nthreads)
    for (int64_t d = 0; d < D; d++) {
        int64_t a = cd_ptr[d]; int32_t nnz = (int32_t)(cd_ptr[d + 1] - a);
        for (int64_t t = doc_ptr[d]; t < doc_ptr[d + 1]; t++) {
            int32_t w = word_ids[t];
            double u0, u1; orc_token_uniforms(seed, (uint64_t)t, iter, &u0, &u1);
            double Q = (double)alpha * sum64[w];
            orc_detail det;
            z_new[t] = orc_sample(nnz, cd_topic + a, cd_count + a, phi + (size_t)w * (size_t)K,
                                  c32 + (size_t)w * (size_t)K, K, Q, u0, u1, &det);
            if (out_S) out_S[t] = det.S;
            if (out_p) out_p[t] = det.p_sparse;
            if (out_branch) out_branch[t] = (int8_t)det.branch;
            if (out_margin) out_margin[t] = det.margin;
        }
    }
}

/* ------------------------------------------------------------------ alias table (the other per-word structure)
 * Sec. 3.2.3 weighs the alias table (Walker's method: O(1) per draw, O(K) sequential construction) against the
 * W-ary tree for the dense term alpha * Bhat_v.  The paper does not say how its table was built; the reading
 * taken here is the sweep construction, which is deterministic given the weights:
 *   q_k = K p_k / sum_j p_j;  items with q_k <= 1 are light, the others heavy; both kinds are visited in index
 *   order.  j = current heavy item, r = what is left of its weight (q_j at first).
 *     while r > 1 and a light item i remains:  bucket i keeps i with probability q_i, else yields j;
 *                                              r -= 1 - q_i;  next light
 *     when r <= 1 and another heavy j' exists: bucket j keeps j with probability r, else yields j';
 *                                              r = q_j' - (1 - r);  j = j'
 *   the last heavy item's bucket is full (r = 1 up to rounding); a light item that finds every heavy one used up
 *   (rounding only) is paired with the last heavy item.
 * Every bucket then holds mass 1/K: bucket k yields k with probability prob[k] and alias[k] otherwise, so that
 * P(k) = (prob[k] + sum over buckets b with alias[b] = k of (1 - prob[b])) / K = p_k / sum p.
 * Arithmetic in binary64; prob is stored rounded to binary32. */
void orc_alias_build(const float *p, int32_t K, float *prob, int32_t *alias) {
    double total = 0.0;
    for (int32_t k = 0; k < K; k++) total += (double)p[k];
    const double scale = (double)K / total;
    int32_t i = 0, j = 0, last_heavy = -1;           /* next light, current heavy */
    while (j < K && !((double)p[j] * scale > 1.0)) j++;
    double r = j < K ? (double)p[j] * scale : 0.0;
    for (;;) {
        while (i < K && (double)p[i] * scale > 1.0) i++;              /* next light item */
        if (j >= K) break;                                            /* no heavy item (left) */
        if (r > 1.0 && i < K) {
            const double q = (double)p[i] * scale;
            prob[i] = (float)q; alias[i] = j;
            r -= 1.0 - q;
            i++;
        } else {
            int32_t jn = j + 1;
            while (jn < K && !((double)p[jn] * scale > 1.0)) jn++;    /* next heavy item */
            last_heavy = j;
            if (jn >= K || !(r <= 1.0)) { prob[j] = 1.0f; alias[j] = j; j = jn; if (jn >= K) break; r = (double)p[jn] * scale; continue; }
            prob[j] = (float)(r < 0.0 ? 0.0 : r); alias[j] = jn;
            r = (double)p[jn] * scale - (1.0 - r);
            j = jn;
        }
    }
    for (; i < K; i++) {                                              /* light items left over */
        if ((double)p[i] * scale > 1.0) continue;
        const double q = (double)p[i] * scale;
        prob[i] = last_heavy >= 0 ? (float)q : 1.0f; alias[i] = last_heavy >= 0 ? last_heavy : i;
    }
}

/* Walker's draw with the 24 random bits behind u (u = bits * 2^-24): bucket b = floor(u K), taken in integers;
 * the bucket's own item if the fraction of u K lies below prob[b], its alias otherwise.  *margin (may be NULL):
 * distance of u from the boundary prob[b] inside the bucket, in units of u. */
int32_t orc_alias_draw(const float *prob, const int32_t *alias, int32_t K, uint32_t bits24, double *margin) {
    const uint64_t prod = (uint64_t)bits24 * (uint64_t)K;
    const int32_t b = (int32_t)(prod >> 24);
    const float frac = (float)(prod & 0xffffffu) * (1.0f / 16777216.0f);
    if (margin) *margin = fabs((double)frac - (double)prob[b]) / (double)K;
    return frac < prob[b] ? b : alias[b];
}

/* Alg. 2 with the dense term drawn from alias tables (prob, alias: [V][K]); otherwise as orc_estep. */
void orc_estep_alias(int64_t D, const int64_t *doc_ptr, const int32_t *word_ids, int32_t K, float alpha,
                     const int64_t *cd_ptr, const int32_t *cd_topic, const int32_t *cd_count,
                     const float *phi, const double *sum64, const float *prob, const int32_t *alias,
                     uint64_t seed, uint32_t iter, int32_t *z_new, int8_t *out_branch, double *out_margin, int nthreads) {
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 16) num_threads(nthreads)
    for (int64_t d = 0; d < D; d++) {
        const int64_t a = cd_ptr[d]; const int32_t nnz = (int32_t)(cd_ptr[d + 1] - a);
        const int32_t *topic = cd_topic + a, *count = cd_count + a;
        for (int64_t t = doc_ptr[d]; t < doc_ptr[d + 1]; t++) {
            const int32_t w = word_ids[t];
            const float *phi_w = phi + (size_t)w * (size_t)K;
            double u0, u1; orc_token_uniforms(seed, (uint64_t)t, iter, &u0, &u1);
            const double Q = (double)alpha * sum64[w];
            double S = 0.0;
            for (int32_t j = 0; j < nnz; j++) S += (double)count[j] * (double)phi_w[topic[j]];
            const double thr = S / (S + Q);
            double margin = fabs(u0 - thr); int32_t result; int branch;
            if (u0 < thr) {                                           /* problem 1, as in orc_sample */
                branch = 1;
                double x = u1 * S, run = 0.0, prev = 0.0; int32_t j = 0;
                for (; j < nnz; j++) { prev = run; run += (double)count[j] * (double)phi_w[topic[j]]; if (run >= x) break; }
                if (j >= nnz) j = nnz - 1;
                result = topic[j];
                const double m = fmin(fabs(x - prev), fabs(run - x)) / S;
                if (m < margin) margin = m;
            } else {                                                  /* problem 2 from the word's alias table */
                branch = 2;
                double m;
                result = orc_alias_draw(prob + (size_t)w * (size_t)K, alias + (size_t)w * (size_t)K, K,
                                        (uint32_t)(u1 * 16777216.0), &m);
                if (m < margin) margin = m;
            }
            z_new[t] = result;
            if (out_branch) out_branch[t] = (int8_t)branch;
            if (out_margin) out_margin[t] = margin;
        }
    }
}

/* per-token training log-likelihood on the current counts:
 *   (1/T) sum_t [ ln(S_t + Q_w) - ln(L_d + K alpha) ]  =  (1/T) sum_t ln sum_k theta_dk Bhat_wk,
 *   theta_dk = (A_dk + alpha) / (L_d + K alpha).  (The paper names the metric, Sec. 4, but prints no formula.) */
double orc_loglik(int64_t D, const int64_t *doc_ptr, const int32_t *word_ids, int32_t K, float alpha,
                  const int64_t *cd_ptr, const int32_t *cd_topic, const int32_t *cd_count,
                  const float *phi, const double *sum64) {
    double total = 0.0; int64_t T = doc_ptr[D];
    for (int64_t d = 0; d < D; d++) {
        int64_t a = cd_ptr[d]; int32_t nnz = (int32_t)(cd_ptr[d + 1] - a);
        double Ld = (double)(doc_ptr[d + 1] - doc_ptr[d]);
        double lognorm = log(Ld + (double)K * (double)alpha);
        for (int64_t t = doc_ptr[d]; t < doc_ptr[d + 1]; t++) {
            const float *phi_w = phi + (size_t)word_ids[t] * (size_t)K;
            double S = 0.0;
            for (int32_t j = 0; j < nnz; j++) S += (double)cd_count[a + j] * (double)phi_w[cd_topic[a + j]];
            total += log(S + (double)alpha * sum64[word_ids[t]]) - lognorm;
        }
    }
    return T > 0 ? total / (double)T : 0.0;
}

/* ------------------------------------------------------------------ whole-model handle (Alg. 1) */
typedef struct {
    int64_t D, T; int32_t V, K; float alpha, beta; uint64_t seed; uint32_t iter;
    const int64_t *doc_ptr; const int32_t *word_ids; /* borrowed from the caller */
    int32_t *z, *z_new;
    int64_t *cd_ptr; int32_t *cd_topic, *cd_count;
    int32_t *cwk; int64_t *ck;
    float *phi, *c32; double *sum64;
} orc_model;

static int model_mstep(orc_model *m) {
    int rc = orc_count_by_dz(m->D, m->doc_ptr, m->z, m->K, m->cd_ptr, m->cd_topic, m->cd_count);
    if (rc) return rc;
    orc_count_by_vz(m->T, m->word_ids, m->z, m->V, m->K, m->cwk, m->ck);
    rc = orc_preprocess(m->cwk, m->ck, m->V, m->K, m->beta, m->phi);
    if (rc) return rc;
    orc_build_prefix(m->phi, m->V, m->K, m->c32, m->sum64);
    return 0;
}

void orc_model_free(orc_model *m) {
    if (!m) return;
    free(m->z); free(m->z_new); free(m->cd_ptr); free(m->cd_topic); free(m->cd_count);
    free(m->cwk); free(m->ck); free(m->phi); free(m->c32); free(m->sum64); free(m);
}

/* doc_ptr / word_ids must outlive the model. */
orc_model *orc_model_create(const int64_t *doc_ptr, const int32_t *word_ids, int64_t D, int32_t V, int32_t K,
                            float alpha, float beta, uint64_t seed) {
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    if (!m) return NULL;
    int64_t T = doc_ptr[D]; size_t vk = (size_t)V * (size_t)K, tt = (size_t)(T > 0 ? T : 1);
    m->D = D; m->T = T; m->V = V; m->K = K; m->alpha = alpha; m->beta = beta; m->seed = seed; m->iter = 0;
    m->doc_ptr = doc_ptr; m->word_ids = word_ids;
    m->z = (int32_t *)malloc(sizeof(int32_t) * tt); m->z_new = (int32_t *)malloc(sizeof(int32_t) * tt);
    m->cd_ptr = (int64_t *)malloc(sizeof(int64_t) * (size_t)(D + 1));
    m->cd_topic = (int32_t *)malloc(sizeof(int32_t) * tt); m->cd_count = (int32_t *)malloc(sizeof(int32_t) * tt);
    m->cwk = (int32_t *)malloc(sizeof(int32_t) * vk); m->ck = (int64_t *)malloc(sizeof(int64_t) * (size_t)K);
    m->phi = (float *)malloc(sizeof(float) * vk); m->c32 = (float *)malloc(sizeof(float) * vk);
    m->sum64 = (double *)malloc(sizeof(double) * (size_t)V);
    if (!m->z || !m->z_new || !m->cd_ptr || !m->cd_topic || !m->cd_count || !m->cwk || !m->ck || !m->phi ||
        !m->c32 || !m->sum64) { orc_model_free(m); return NULL; }
    orc_init_z(T, K, seed, m->z);
    if (model_mstep(m)) { orc_model_free(m); return NULL; }
    return m;
}

/* replace the assignments (T values) and redo the M-step; the iteration counter is set by the caller */
int orc_model_set_z(orc_model *m, const int32_t *z, uint32_t iter) {
    for (int64_t t = 0; t < m->T; t++) if (z[t] < 0 || z[t] >= m->K) return -1;
    memcpy(m->z, z, sizeof(int32_t) * (size_t)m->T);
    m->iter = iter;
    return model_mstep(m);
}

/* n iterations of Alg. 1: E-step for every token on frozen counts, then the M-step */
int orc_model_iterate(orc_model *m, int32_t n, int nthreads) {
    for (int32_t i = 0; i < n; i++) {
        m->iter++;
        orc_estep(m->D, m->doc_ptr, m->word_ids, m->K, m->alpha, m->cd_ptr, m->cd_topic, m->cd_count,
                  m->phi, m->c32, m->sum64, m->seed, m->iter, m->z_new, NULL, NULL, NULL, NULL, nthreads);
        int32_t *tmp = m->z; m->z = m->z_new; m->z_new = tmp;
        int rc = model_mstep(m); if (rc) return rc;
    }
    return 0;
}

/* E-step only, from the model's current state, for iteration m->iter + 1; does not change the model */
void orc_model_estep_detail(orc_model *m, int32_t *z_out, double *out_S, double *out_p, int8_t *out_branch,
                            double *out_margin, int nthreads) {
    orc_estep(m->D, m->doc_ptr, m->word_ids, m->K, m->alpha, m->cd_ptr, m->cd_topic, m->cd_count,
              m->phi, m->c32, m->sum64, m->seed, m->iter + 1, z_out, out_S, out_p, out_branch, out_margin, nthreads);
}

/* Alg. 2 for a list of tokens (canonical indices), from the model's current state, for iteration m->iter + 1 */
void orc_model_sample_tokens(orc_model *m, const int64_t *tok, int64_t n, int32_t *z_out, double *out_S,
                             double *out_p, int8_t *out_branch, double *out_margin) {
    for (int64_t i = 0; i < n; i++) {
        int64_t t = tok[i];
        /* document of token t: last d with doc_ptr[d] <= t */
        int64_t lo = 0, hi = m->D - 1;
        while (lo < hi) { int64_t mid = lo + (hi - lo + 1) / 2; if (m->doc_ptr[mid] <= t) lo = mid; else hi = mid - 1; }
        int64_t d = lo, a = m->cd_ptr[d]; int32_t nnz = (int32_t)(m->cd_ptr[d + 1] - a);
        int32_t w = m->word_ids[t];
        double u0, u1; orc_token_uniforms(m->seed, (uint64_t)t, m->iter + 1, &u0, &u1);
        orc_detail det;
        z_out[i] = orc_sample(nnz, m->cd_topic + a, m->cd_count + a, m->phi + (size_t)w * (size_t)m->K,
                              m->c32 + (size_t)w * (size_t)m->K, m->K, (double)m->alpha * m->sum64[w], u0, u1, &det);
        if (out_S) out_S[i] = det.S;
        if (out_p) out_p[i] = det.p_sparse;
        if (out_branch) out_branch[i] = (int8_t)det.branch;
        if (out_margin) out_margin[i] = det.margin;
    }
}

double orc_model_loglik(orc_model *m) {
    return orc_loglik(m->D, m->doc_ptr, m->word_ids, m->K, m->alpha, m->cd_ptr, m->cd_topic, m->cd_count,
                      m->phi, m->sum64);
}

/* ------------------------------------------------------------------ holdout log-likelihood
 * The quality metric Sec. 4 names: log-likelihood per token of held-out documents, "partially-observed
 * document" approach.  The paper prints no formula; the reading taken is document completion: every held-out
 * document is split into an observed part and a scored part (the caller's mask).  The model's Bhat, prefix
 * table and row sums stay frozen.  Fold-in: the observed tokens get assignments by the same ESCA iteration as
 * training (Alg. 1 restricted to these documents and to A): iteration 0 assigns z = floor(word0 K / 2^32) with
 * the Philox counter = position of the token among the observed tokens, or the caller supplies z_init;
 * iterations 1..n_fold run Alg. 2 for every observed token against A' = counts of the document's observed
 * assignments (frozen during the iteration), then rebuild A'.  Score:
 *     (1/T_s) sum over scored tokens t of [ ln(S_t + Q_w) - ln(L'_d + K alpha) ],
 * S_t = sum_k A'_dk Bhat_wk, L'_d = observed tokens of the document: the predictive probability
 * sum_k theta_dk Bhat_wk with theta_dk = (A'_dk + alpha) / (L'_d + K alpha).
 * z_out (may be NULL) receives the final assignments of the observed tokens, in corpus order.
 * Returns 0, or -1 on a bad argument / allocation failure. */
int orc_holdout_loglik(const orc_model *m, int64_t D, const int64_t *doc_ptr, const int32_t *word_ids,
                       const uint8_t *observed, int32_t n_fold, uint64_t seed, const int32_t *z_init,
                       int nthreads, double *out_ll, int64_t *out_scored, int32_t *z_out) {
    int64_t T = doc_ptr[D], To = 0;
    for (int64_t t = 0; t < T; t++) { if (word_ids[t] < 0 || word_ids[t] >= m->V) return -1; To += observed[t] ? 1 : 0; }
    size_t no = (size_t)(To > 0 ? To : 1);
    int64_t *optr = (int64_t *)malloc(sizeof(int64_t) * (size_t)(D + 1));
    int32_t *ow = (int32_t *)malloc(sizeof(int32_t) * no), *z = (int32_t *)malloc(sizeof(int32_t) * no);
    int32_t *zn = (int32_t *)malloc(sizeof(int32_t) * no);
    int64_t *cd_ptr = (int64_t *)malloc(sizeof(int64_t) * (size_t)(D + 1));
    int32_t *cd_topic = (int32_t *)malloc(sizeof(int32_t) * no), *cd_count = (int32_t *)malloc(sizeof(int32_t) * no);
    int rc = -1;
    if (!optr || !ow || !z || !zn || !cd_ptr || !cd_topic || !cd_count) goto done;
    /* the observed part as a corpus of its own */
    optr[0] = 0;
    for (int64_t d = 0, k = 0; d < D; d++) {
        for (int64_t t = doc_ptr[d]; t < doc_ptr[d + 1]; t++) if (observed[t]) ow[k++] = word_ids[t];
        optr[d + 1] = k;
    }
    if (z_init) {
        for (int64_t t = 0; t < To; t++) { if (z_init[t] < 0 || z_init[t] >= m->K) goto done; z[t] = z_init[t]; }
    } else {
        orc_init_z(To, m->K, seed, z);
    }
    for (int32_t it = 1; it <= n_fold; it++) {
        if (orc_count_by_dz(D, optr, z, m->K, cd_ptr, cd_topic, cd_count)) goto done;
        orc_estep(D, optr, ow, m->K, m->alpha, cd_ptr, cd_topic, cd_count, m->phi, m->c32, m->sum64, seed,
                  (uint32_t)it, zn, NULL, NULL, NULL, NULL, nthreads);
        int32_t *tmp = z; z = zn; zn = tmp;
    }
    if (orc_count_by_dz(D, optr, z, m->K, cd_ptr, cd_topic, cd_count)) goto done;
    {
        double total = 0.0; int64_t scored = 0;
        for (int64_t d = 0; d < D; d++) {
            int64_t a = cd_ptr[d]; int32_t nnz = (int32_t)(cd_ptr[d + 1] - a);
            double lognorm = log((double)(optr[d + 1] - optr[d]) + (double)m->K * (double)m->alpha);
            for (int64_t t = doc_ptr[d]; t < doc_ptr[d + 1]; t++) {
                if (observed[t]) continue;
                const float *phi_w = m->phi + (size_t)word_ids[t] * (size_t)m->K;
                double S = 0.0;
                for (int32_t j = 0; j < nnz; j++) S += (double)cd_count[a + j] * (double)phi_w[cd_topic[a + j]];
                total += log(S + (double)m->alpha * m->sum64[word_ids[t]]) - lognorm;
                scored++;
            }
        }
        *out_ll = scored > 0 ? total / (double)scored : 0.0;
        *out_scored = scored;
    }
    if (z_out) memcpy(z_out, z, sizeof(int32_t) * (size_t)To);
    rc = 0;
done:
    free(optr); free(ow); free(z); free(zn); free(cd_ptr); free(cd_topic); free(cd_count);
    return rc;
}

/* accessors (pointers into the model; valid until the next mutating call) */
int32_t *orc_model_z(orc_model *m) { return m->z; }
int64_t *orc_model_cd_ptr(orc_model *m) { return m->cd_ptr; }
int32_t *orc_model_cd_topic(orc_model *m) { return m->cd_topic; }
int32_t *orc_model_cd_count(orc_model *m) { return m->cd_count; }
int32_t *orc_model_cwk(orc_model *m) { return m->cwk; }
int64_t *orc_model_ck(orc_model *m) { return m->ck; }
float *orc_model_phi(orc_model *m) { return m->phi; }
float *orc_model_c32(orc_model *m) { return m->c32; }
double *orc_model_sum64(orc_model *m) { return m->sum64; }
uint32_t orc_model_iter(orc_model *m) { return m->iter; }
