/*
 * saber.h - C ABI of the MI355X (gfx950) sparsity-aware LDA sampler.
 *
 * The library runs the ESCA iteration of the paper (Alg. 1): an E-step in which
 * every token draws a topic from p(k) ~ (A_dk + alpha) * Bhat_vk (Eq. 1) through
 * the sparsity-aware split of Alg. 2, then an M-step that rebuilds the sparse
 * document-topic counts A (CountByDZ), the dense word-topic counts B (CountByVZ),
 * Bhat by Eq. 2 (Preprocess) and the per-word prefix-sum trees (BuildTree).
 * All of it executes in hand-written HIP kernels; there is no CPU fallback.
 *
 * Conventions
 *   - Every pointer argument is a HOST pointer unless its comment says "device".
 *   - The caller owns all input and output buffers.  saber_init copies what it
 *     needs; inputs may be freed when it returns.
 *   - Indices are 0-based.  Tokens are identified by their position t in the
 *     caller's doc-major word_ids array ("canonical token index").
 *   - Every function returns SABER_OK (0) or a negative saber_status and never
 *     throws; saber_last_error() gives a message for the calling thread's last
 *     failure.  A context is not thread-safe: one thread at a time per context.
 *   - Random numbers: Philox4x32-10, key = seed, counter = (t lo, t hi, iteration, 0);
 *     word 0 decides the branch, word 1 the position; u = (word >> 8) * 2^-24.
 *     Results therefore do not depend on the internal token order, tile sizes or
 *     chunk count.
 *   - Limits: 1 <= K <= 262144 (three searched tree levels of width 64), D < 2^31, T < 2^40 (the corpus is cut
 *     into document chunks of fewer than 2^30 tokens when it is larger), and the longest document must be
 *     shorter than 2^(32 - ceil(log2 K)).  Device memory: about 16 bytes per token plus 8*K bytes per frequent
 *     word and 8 bytes per non-zero count of the others when everything is resident; about 6 bytes per token
 *     and 4 bytes per token of pinned host memory with host streaming (saber_options.stream_workers).
 */
#ifndef SABER_H
#define SABER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct saber_ctx saber_ctx; /* opaque, owned by the library */

typedef enum saber_status {
    SABER_OK = 0,
    SABER_EINVAL = -1,  /* null pointer, bad size, malformed CSR, word id or topic out of range */
    SABER_ENOMEM = -2,  /* host or device allocation failed */
    SABER_EDEVICE = -3, /* no usable GPU, or a HIP call failed */
    SABER_ESTATE = -4,  /* call not valid in the context's current state */
    SABER_ERANGE = -5   /* a size exceeds a documented limit */
} saber_status;

/* Tunables; none of them changes any result.  Zero / negative means "library default". */
typedef struct saber_options {
    int32_t n_chunks;       /* document chunks the corpus is cut into (Sec. 3.1.2); 0 (default): chunks of about
                               80 M tokens (T / 80 M rounded to the nearest whole number, at least 1), so that the rows of A
                               a chunk's sampling pass re-reads stay in the 256 MB Infinity Cache; always at least one
                               chunk per 2^30 tokens */
    int32_t block_threads;  /* threads per workgroup of the sampling kernel (multiple of 64 up to 1024);
                               default: the size that lets a CU hold the most wavefronts given the LDS the Bhat row takes */
    int32_t tile_tokens;    /* most tokens of one word handled by one workgroup; default 0: a 2560th of a chunk's tokens,
                               not below 8,192 and not above 32,768 */
    int32_t stage_phi;      /* 1: keep the word's Bhat row in LDS when it fits (up to 150 KB: K <= 37,800), 0: always
                               gather from global; default 1 */
    int32_t profile;        /* 1: time every kernel group with HIP events (see saber_get_stats); default 0 */
    int32_t long_doc_tokens;/* documents longer than this use a 256-thread workgroup in CountByDZ; default 512 */
    int32_t dz_lds_entries; /* LDS capacity (entries) of one CountByDZ workgroup before it falls back to
                               accumulating in the global row; default 2048 (a larger buffer halves the
                               workgroups a CU can hold) */
    int32_t stage_min_tokens;   /* tiles with at least this many tokens are launched with block_threads threads, smaller
                                   ones with light_block_threads; default 1 (one class) */
    int32_t light_block_threads;/* workgroup size for the smaller tiles; default: as block_threads */
    int32_t light_word_tokens;  /* words with fewer tokens than this keep their row of B sparse (rebuilt by a segmented
                                   count, like a row of A) and their Bhat row is formed in LDS from a base vector and
                                   the non-zeros; default K/2; negative: every word keeps a dense row */
    int32_t stream_workers;     /* 1..8: host streaming (Sec. 3.1.2) with this many workers: the chunks' token lists stay
                                   in pinned host memory (4 bytes per token) and each chunk is copied into one of this
                                   many device buffers for its pass, so that with two or more the copy of one chunk
                                   overlaps the sampling of another (three hide it reliably).  The chunk's rows of A
                                   are rebuilt right after its sampling, while its new assignments are in the
                                   buffer; resident are the rows of A and 2 bytes per token (the word-major
                                   assignments), which is what lets a corpus several times the device memory run.
                                   0 (default): everything stays in device memory if the estimate of what that takes
                                   fits what is free, else host streaming with three workers (saber_stats says which;
                                   SABER_ENOMEM if that does not fit either).  -1: never stream.  Results are the
                                   same.  With profile=1 and streaming, ms_sample covers the whole chunk loop (copies
                                   waited for, sampling, CountByDZ) and ms_count_dz is zero. */
    int32_t ablation;           /* measurement aid, default 0: bit 0 samples the tokens in document order instead of
                                   word order (the layout before Sec. 3.1.3: the row of A is fetched once per document,
                                   Bhat is gathered from global memory; every word then keeps a dense row and
                                   stream_workers must be 0); bit 1 rebuilds A by a radix sort of all (document, topic)
                                   pairs instead of the segmented count of Sec. 3.3.  Results are the same.
                                   Bit 2 draws the dense term from per-word alias tables instead of the prefix-sum tree
                                   (the alternative Sec. 3.2.3 weighs): every word keeps a dense row, the tables (8 K
                                   bytes per word) are rebuilt after every M-step, K <= 13,500, not with bit 0.  This
                                   variant maps the uniform draw to another topic than the tree does: its assignments
                                   differ from the default path's and follow the same distribution. */
    int32_t device_mem_limit_mb;/* device memory the automatic choice above may plan with, in MB; 0 (default): what
                                   hipMemGetInfo reports as free */
    int32_t quarter_row_entries;/* rows of A of at most this many entries (default and at most 64) are sampled four at a time,
                                   one (word, document) run per 16 lanes of a wavefront; negative: none */
    int32_t half_row_entries;   /* longer rows of at most this many entries (default and at most 128) two at a time, one per 32
                                   lanes; negative: none.  Rows beyond both get all 64 lanes, in blocks of 256 entries */
    int32_t reserved[1];
} saber_options;

/* Sums over the iterations run since the last saber_reset_stats.  The ms_* fields need profile=1. */
typedef struct saber_stats {
    int64_t iterations;       /* iterations counted */
    double ms_sample;         /* E-step sampling kernel (all chunks) */
    double ms_count_dz;       /* CountByDZ */
    double ms_ck;             /* topic totals C_k */
    double ms_phi;            /* Preprocess + BuildTree */
    double ms_total;          /* whole iterations, first kernel to last */
    int64_t sample_launches;  /* sampling-kernel launches timed */
    int64_t sum_tokens;       /* tokens sampled */
    int64_t sum_tokens_dense; /* of those, tokens that took the dense branch (problem 2) */
    int64_t sum_row_entries;  /* sum over sampled tokens of K_d: entries of A_d each token's product loop read */
    /* state after the last M-step: */
    int64_t nnz_cd;           /* non-zeros of A */
    int64_t next_row_entries; /* sum_d K_d * L_d: what the next E-step will read */
    /* layout constants: */
    int64_t tokens;           /* T */
    int64_t words_present;    /* (word, chunk) pairs with at least one token */
    int64_t tiles;            /* workgroups of one E-step */
    int64_t sum_row_fetch;    /* like sum_row_entries, counting a row once per run of consecutive tokens of one
                                 (word, document) pair: the entries the sampler has to fetch */
    int64_t next_row_fetch;   /* sum_d K_d * U_d, U_d = distinct words of document d */
    /* words whose row of B is kept sparse (light words): */
    int64_t light_words_present; /* (light word, chunk) pairs with at least one token (layout constant) */
    int64_t light_tokens;        /* tokens of light words (layout constant) */
    int64_t sum_light_entries;   /* non-zeros of the sparse rows the counted E-steps staged, once per word */
    int64_t next_light_entries;  /* non-zeros of the sparse rows after the last M-step */
    int64_t stream_workers;      /* device buffers of host streaming in use; 0: everything is resident */
    int64_t chunks;              /* document chunks the corpus is cut into (Sec. 3.1.2; layout constant) */
} saber_stats;

/*
 * Where device memory and the compute stream come from (Sec. 2.1's problem statement leaves both to the host
 * program; a caller that runs PyTorch hands over its caching allocator and its current stream).
 *   alloc(bytes)   returns DEVICE memory of at least `bytes` bytes, 256-byte aligned, on the current device, or NULL
 *   dealloc(ptr)   takes back what alloc returned
 *   hip_stream     a hipStream_t on which every kernel and every ordered copy of the library then runs; NULL: each
 *                  context creates (and destroys) a stream of its own
 * alloc and dealloc are given together; both NULL restores hipMalloc / hipFree.  The setting is process-wide and
 * applies to contexts created afterwards (and to saber_bandwidth_probe); a context keeps the hooks it was created
 * with until saber_free, so they must stay callable until then, and the stream must outlive the context.  With a
 * caller's stream the library still synchronises that stream before it returns from a call that promises completed
 * work.  Pinned host memory of host streaming is always the library's own.  Errors: EINVAL (only one of alloc/dealloc).
 */
int saber_set_hooks(void *(*alloc)(size_t bytes), void (*dealloc)(void *ptr), void *hip_stream);

/* Fill *opt with the defaults. */
void saber_options_default(saber_options *opt);

/*
 * Create a sampler for one corpus (problem statement of Sec. 2.1).
 *   doc_ptr  [D+1]  doc_ptr[0]=0, non-decreasing, doc_ptr[D]=T; empty documents are legal
 *   word_ids [T]    doc-major token list, each in [0,V)
 *   K, alpha, beta  number of topics and the two Dirichlet parameters (alpha>0, beta>0)
 * On return the state is "iteration 0": z_t = floor(PhiloxWord0(t, 0) * K / 2^32), and A, B, Bhat and
 * the trees are built from it, so saber_counts / saber_loglik are valid immediately.
 * opt may be NULL.  Errors: EINVAL, ERANGE, ENOMEM, EDEVICE.  *out is NULL on failure.
 */
int saber_init_ex(saber_ctx **out, const int64_t *doc_ptr, const int32_t *word_ids, int64_t D, int32_t V,
                  int32_t K, float alpha, float beta, uint64_t seed, const saber_options *opt);
int saber_init(saber_ctx **out, const int64_t *doc_ptr, const int32_t *word_ids, int64_t D, int32_t V,
               int32_t K, float alpha, float beta, uint64_t seed);

/* Run n iterations of Alg. 1 (E-step for every token on the frozen counts, then the M-step).
 * Synchronous: all work has finished when it returns.  n = 0 is a no-op.  Errors: EINVAL (n<0), EDEVICE. */
int saber_iterate(saber_ctx *ctx, int32_t n);

/* Number of non-zeros of the document-topic count matrix A of Sec. 2.1 (A_dk = tokens of document d assigned
 * to topic k), i.e. the size of cd_topic / cd_count for saber_counts.  Errors: EINVAL, ENOMEM, EDEVICE. */
int saber_counts_nnz(saber_ctx *ctx, int64_t *nnz_cd);

/*
 * Copy out the count matrices of Sec. 2.1 as the last completed M-step of Alg. 1 (CountByDZ, CountByVZ) left them:
 * A (D x K, sparse: A_dk = tokens of document d with topic k) and B (V x K, dense: B_vk = tokens of word v with
 * topic k).
 *   cd_row_ptr [D+1], cd_topic [nnz], cd_count [nnz]: A in CSR, topics ascending within a row (the order the
 *                                                     segmented count of Sec. 3.3 produces; the sparse draw of
 *                                                     Alg. 2 depends on it)
 *   cwk [V*K] row-major by word (B);  ck [K] topic totals sum_v B_vk (the denominators of Eq. 2 without V beta)
 * Any of the five may be NULL to skip it (cd_topic and cd_count need cd_row_ptr).  All are host buffers owned by
 * the caller.  Errors: EINVAL, ENOMEM, EDEVICE.
 */
int saber_counts(saber_ctx *ctx, int64_t *cd_row_ptr, int32_t *cd_topic, int32_t *cd_count, int32_t *cwk,
                 int64_t *ck);

/*
 * Per-token training log-likelihood on the counts of the last M-step:
 *   (1/T) sum_t [ ln(S_t + Q_w) - ln(L_d + K alpha) ]  =  (1/T) sum_t ln sum_k theta_dk Bhat_wk
 * (the paper names per-token log-likelihood as its quality metric in Sec. 4 and gives no formula;
 * this is the predictive likelihood of the training tokens, a by-product of the sampler's normaliser).
 * Both sums are reduced on the device in binary64 and in a fixed order (the result is the same in every run); one
 * double comes back.  per_token_ll is a host pointer.  T = 0 gives 0.  Errors: EINVAL, EDEVICE.
 */
int saber_loglik(saber_ctx *ctx, double *per_token_ll);

/*
 * saber_loglik for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same kernels and the same order of additions, hence the same number, but the
 * work space of the reduction (per-workgroup partial sums) is a static device array of the library instead of memory
 * of the context, and the call itself allocates nothing on host or device.
 *   d_result  DEVICE pointer to one double, owned by the caller; written on the context's stream, which the call
 *             waits for before it returns
 * Limit: at most 2^20 sampling workgroups per document chunk (8 MB of static work space per GPU, held until the
 * process ends); more is refused with ERANGE.  All calls on one GPU share that array: it keeps the last call's
 * contents (nothing in it has to start at zero), and calls that overlap in time on one GPU race.
 * Errors: EINVAL, ERANGE, ESTATE (the context's device has no work space), EDEVICE.
 */
int saber_loglik_static(saber_ctx *ctx, double *d_result);

/*
 * Holdout log-likelihood per token of held-out documents, "partially-observed document" approach (the quality
 * metric of Sec. 4; the paper prints no formula, the reading taken is document completion).  The model of ctx
 * (Bhat, trees) stays frozen and ctx is not changed.
 *   doc_ptr [D+1], word_ids [T]  the held-out documents, as for saber_init (same V)
 *   observed [T]                 non-zero: the token is folded in; zero: the token is scored
 *   n_foldin                     iterations of Alg. 1 restricted to these documents and to A: the observed
 *                                tokens sample from p(k) ~ (A'_dk + alpha) Bhat_vk, A' = counts of the document's
 *                                observed assignments, frozen during an iteration and rebuilt after it
 *   seed                         Philox key of the fold-in; the counter of a token is its position among the
 *                                observed tokens; iteration 0 assigns z = floor(word0 K / 2^32)
 *   z_init                       NULL, or the assignments of the observed tokens (corpus order) to start from
 *                                instead of iteration 0
 *   z_out                        NULL, or receives the final assignments of the observed tokens
 *   loglik, n_scored             (1/T_s) sum over scored tokens of [ ln(S_t + Q_w) - ln(L'_d + K alpha) ] with
 *                                S_t = sum_k A'_dk Bhat_wk and L'_d = observed tokens of the document; T_s
 * All pointers are host pointers owned by the caller.  Documents longer than the count bits of the model's
 * packing allow are refused (ERANGE).  Allocates and frees device memory for the held-out documents.
 */
int saber_holdout_loglik(saber_ctx *ctx, const int64_t *doc_ptr, const int32_t *word_ids, const uint8_t *observed,
                         int64_t D, int32_t n_foldin, uint64_t seed, const int32_t *z_init, int32_t *z_out,
                         double *loglik, int64_t *n_scored);

void saber_free(saber_ctx *ctx);

/* Message of the calling thread's last failed call (static storage, never NULL). */
const char *saber_last_error(void);

/* ---- state exchange (checkpointing, and the hooks the parity tests need) ---- */

/* The state of Alg. 1 between iterations is the topic assignment k of every token of the list L (Sec. 2.1: tokens
 * are triplets (d, v, k)); everything else (A, B, Bhat, the trees) is rebuilt from it by the M-step.
 * saber_get_z: current assignments, z[T] (host) in canonical token order.  Errors: EINVAL, ENOMEM, EDEVICE. */
int saber_get_z(saber_ctx *ctx, int32_t *z);
/* Replace the assignments (z[T], host, each in [0,K)), set the iteration counter to iter and redo the M-step of
 * Alg. 1 (CountByDZ, CountByVZ, Preprocess, BuildTree) on them.  The next E-step then uses Philox counter word
 * 2 = iter + 1.  Errors: EINVAL (a topic out of range), ENOMEM, EDEVICE. */
int saber_set_z(saber_ctx *ctx, const int32_t *z, uint32_t iter);
/* Number of iterations of Alg. 1's outer loop completed so far (0 after init, or the value given to
 * saber_set_z); it is the third word of the Philox counter of the last E-step. */
int saber_get_iteration(saber_ctx *ctx, uint32_t *iter);

/*
 * Normalisers of Alg. 2 for m tokens (canonical indices tok[m], each in [0,T)) on the current counts:
 *   S = sum_k A_dk Bhat_vk,  Q = alpha sum_k Bhat_vk,  p_sparse = S / (S + Q).  Outputs may be NULL.
 */
int saber_token_probs(saber_ctx *ctx, const int64_t *tok, int64_t m, float *S, float *Q, float *p_sparse);

/* Rows of Bhat (Eq. 2) and of the per-word inclusive prefix table (bottom tree level) for m words:
 * phi[m*K], prefix[m*K]; either may be NULL.  The prefix rows are not kept in memory; they are rebuilt here with
 * the arithmetic of the sampler's dense branch. */
int saber_get_phi(saber_ctx *ctx, const int32_t *words, int32_t m, float *phi, float *prefix);

/* ---- measurement ---- */
int saber_get_stats(saber_ctx *ctx, saber_stats *out);
int saber_reset_stats(saber_ctx *ctx);
/* HIP stream the library launches on (a hipStream_t), for callers that want to order work against it. */
int saber_get_stream(saber_ctx *ctx, void **hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SABER_H */
