// Host side of the C ABI declared in include/saber.h: validation, the device data layout, and the
// per-iteration launch sequence of Alg. 1.  Every step of the path runs in the kernels of
// saber_kernels.hpp; nothing here computes counts or samples on the CPU.
#include "saber_kernels.hpp"
#include "saber_ablation.hpp"
#include "../../include/saber.h"
#include "../../include/saber_measure.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include <rocprim/rocprim.hpp>

using namespace saber;

// ------------------------------------------------------------------------------------------------
// errors
// ------------------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";
static int fail(int code, const char *fmt, ...) {
    va_list ap; va_start(ap, fmt); vsnprintf(g_err, sizeof(g_err), fmt, ap); va_end(ap);
    return code;
}
#define HIP_TRY(expr)                                                                                     \
    do {                                                                                                  \
        hipError_t e_ = (expr);                                                                           \
        if (e_ != hipSuccess)                                                                             \
            return fail(e_ == hipErrorOutOfMemory ? SABER_ENOMEM : SABER_EDEVICE, "%s failed: %s (%s:%d)", \
                        #expr, hipGetErrorString(e_), __FILE__, __LINE__);                                \
    } while (0)
#define SABER_TRY(expr) do { int rc_ = (expr); if (rc_ != SABER_OK) return rc_; } while (0)

extern "C" const char *saber_last_error(void) { return g_err; }

// ------------------------------------------------------------------------------------------------
// device memory
// ------------------------------------------------------------------------------------------------
// Work space of the log-likelihood reduction: the per-tile sums of one chunk, then kLlTail doubles - the workgroup sums
// of one reduction pass, the running total over chunks, the normaliser and the result.
constexpr size_t kLlTail = (size_t)kReduceBlocks + 3;
struct LlScratch { double *tile_part, *block_part, *acc, *norm, *result; };
static LlScratch ll_scratch(double *base, size_t max_tiles) {
    LlScratch w;
    w.tile_part = base; w.block_part = base + max_tiles; w.acc = w.block_part + kReduceBlocks; w.norm = w.acc + 1; w.result = w.norm + 1;
    return w;
}

// Where device memory and the compute stream come from (saber_set_hooks).  A context keeps the hooks it was created
// with, so its memory goes back through the deallocator that matches its allocator.
struct Hooks {
    void *(*alloc)(size_t) = nullptr;
    void (*dealloc)(void *) = nullptr;
    hipStream_t stream = nullptr;
    bool have_stream = false;
};
static Hooks g_hooks;

static int hook_alloc(const Hooks &h, void **p, size_t bytes) {
    *p = nullptr;
    bytes = std::max<size_t>(bytes, 1);
    if (h.alloc) {
        *p = h.alloc(bytes);
        if (!*p) return fail(SABER_ENOMEM, "the caller's allocator returned no memory for %zu bytes", bytes);
        if (reinterpret_cast<uintptr_t>(*p) & 255u) {
            void *q = *p; *p = nullptr;
            if (h.dealloc) h.dealloc(q);
            return fail(SABER_EINVAL, "the caller's allocator returned memory that is not 256-byte aligned");
        }
        return SABER_OK;
    }
    HIP_TRY(hipMalloc(p, bytes));
    return SABER_OK;
}
static void hook_free(const Hooks &h, void *p) {
    if (!p) return;
    if (h.alloc) { if (h.dealloc) h.dealloc(p); }
    else (void)hipFree(p);
}
template <typename T>
static int dev_alloc(const Hooks &h, T **p, size_t n) { return hook_alloc(h, (void **)p, std::max<size_t>(n, 1) * sizeof(T)); }
static void dev_free(const Hooks &h, void *p) { hook_free(h, p); }

// ------------------------------------------------------------------------------------------------
// context
// ------------------------------------------------------------------------------------------------
struct Chunk {
    int64_t d0 = 0, d1 = 0;   // document range
    int64_t t0 = 0, ntok = 0; // canonical token range [t0, t0+ntok)
    int64_t tile0 = 0, ntiles = 0, words_present = 0;
    // tiles of the chunk: [0, n_dense) belong to words with dense B rows, sorted by size, the first n_heavy of
    // them forming the class of large tiles; [n_dense, ntiles) belong to light words (sparse B rows)
    int64_t n_heavy = 0, n_dense = 0;
    // the chunk's documents inside the (ascending) lists of short and of long documents
    int64_t short0 = 0, nshort = 0, long0 = 0, nlong = 0;
    // the rows of A of the chunk's documents: first row and extent, in units of 32 entries (128 bytes)
    int64_t row_unit0 = 0, row_units = 0;
};

constexpr int kMaxSlots = 8;

constexpr int kMaxTimedIters = 32;
constexpr int kCtr = 8;   // device counters per timed iteration
enum { EV_BEGIN = 0, EV_SAMPLE, EV_DZ, EV_CK, EV_PHI, EV_PER_ITER };

struct saber_ctx {
    Hooks hooks;                      // allocator and stream in force when the context was created
    bool own_stream = false;
    int device = 0;                   // the HIP device the context lives on
    int64_t D = 0, T = 0;
    int32_t V = 0, K = 0, Kpad = 0, n3 = 0, n3pad = 0, nwords = 0;
    float alpha = 0, beta = 0, vbeta = 0;
    uint64_t seed = 0;
    uint32_t iter = 0, topic_bits = 0, topic_mask = 0;
    bool z16 = false, staged = false, b16 = false;
    saber_options opt{};
    int32_t tile_tokens_asked = 0;    // the caller's tile_tokens (0: automatic), before the default was filled in
    int64_t max_doc_len = 0;
    hipStream_t stream = nullptr;
    // device arrays
    void *z = nullptr;                // [T] uint16 or int32, canonical (document) order
    int32_t *tok_doc = nullptr;       // [T] word-major inside every chunk
    uint32_t *tok_t = nullptr;        // [T]
    Tile *tiles = nullptr;
    uint2 *docrec = nullptr;          // [D]
    uint32_t *cd_ent = nullptr;       // [cd_cap]
    int64_t cd_cap = 0;
    int64_t *doc_ptr = nullptr;       // [D+1]
    int32_t *short_docs = nullptr, *long_docs = nullptr;
    int64_t n_short = 0, n_long = 0;
    // words: V_dense keep dense rows of B and Bhat (row V_dense is an all-zero row that yields the base vector);
    // V_light keep B sparse, like the rows of A
    int32_t V_dense = 0, V_light = 0;
    int32_t *row_word = nullptr;      // [V_dense+1] word of each dense row (the zero row maps to word index V)
    int32_t *light_words = nullptr;   // [V_light] word of each light row
    int32_t *light_short = nullptr, *light_long = nullptr;   // light rows by token count, for the count launches
    int64_t n_light_short = 0, n_light_long = 0;
    int64_t *light_tok_ptr = nullptr; // [V_light+1] positions of the light words' tokens in z_wm
    uint2 *wrec = nullptr;            // [V_light] {row start / 32, non-zeros}
    uint32_t *lw_ent = nullptr;       // packed rows of B of the light words
    float *lw_phi = nullptr;          // Bhat of each such entry
    void *z_wm = nullptr;             // [T] word-major assignments: the light words' tokens first, then the dense rows' ones
    int64_t T_light = 0, lw_cap = 0;
    VzItem *vz_items = nullptr;       // slabs of the dense-row words' segments of z_wm
    int64_t n_vz_items = 0;
    std::vector<int32_t> h_word_row;  // host: word -> dense row (>= 0) or -(light row) - 1
    // A context built on a trained model (held-out documents): it borrows the model's word classes, Bhat, tree
    // levels and sparse rows, owns only its own tokens, z and rows of A, and never rebuilds B.
    const saber_ctx *parent = nullptr;
    bool no_state = false;            // no assignments of its own (tokens that are only scored)
    int32_t *cwk = nullptr;           // [V_dense+1][Kpad]
    unsigned long long *ck = nullptr; // [K] topic totals
    float *denom = nullptr;           // [K] denominators of Eq. 2
    float *phi = nullptr, *l3 = nullptr, *sumphi = nullptr;
    double *l3_64 = nullptr;          // [V][n3]
    uint32_t *doc_words = nullptr;    // [D] distinct words of the document
    unsigned long long *dense_slots = nullptr; // [kMaxTimedIters][kDenseSlots] dense-branch tokens, spread over slots
    unsigned long long *counters = nullptr; // [kMaxTimedIters][kCtr]: dense-branch tokens, nnz(A), sum K_d L_d, sum K_d U_d,
                                            // non-zeros of the sparse rows of B
    // log-likelihood reduction: [max tiles per chunk] per-tile sums, then kLlTail doubles (LlScratch below)
    double *ll_partial = nullptr;
    std::vector<Chunk> chunks;
    int64_t total_tiles = 0, max_chunk_tiles = 0;
    // measurement
    hipEvent_t ev[kMaxTimedIters * EV_PER_ITER] = {};
    bool have_events = false;
    saber_stats stats{};
    std::vector<int64_t> doc_len;     // host copy of the document lengths (statistics only)
    // Host streaming (Sec. 3.1.2), n_slots > 0: tok_t lives in pinned host memory; a chunk's part of it is copied
    // into one of n_slots device buffers for the chunk's pass (4 bytes per token and iteration over the host link).
    // The rest is derived or kept on the device: the chunk's tok_doc follows from one look-up per token in
    // doc_blocks (16 bytes per 64 canonical tokens: where documents start); its assignments in document order exist only in the
    // buffer, between the sampling kernel that writes them and the CountByDZ that turns them into rows of A, and
    // are re-created from the word-major copy when asked for; z_wm (2 bytes per token) and the rows of A are
    // resident.  Copies run on a stream of their own and are ordered against the compute stream with two events
    // per buffer.
    int n_slots = 0, next_slot = 0;
    int64_t slot_tokens = 0;
    uint32_t *h_tok_t = nullptr;
    uint4 *doc_blocks = nullptr;      // [ceil(T/64)] see expand_tok_doc_kernel
    int32_t *ne_doc = nullptr;        // [non-empty documents] their numbers; null when no document is empty
    int32_t *slot_tok_doc[kMaxSlots] = {}; uint32_t *slot_tok_t[kMaxSlots] = {}; void *slot_z[kMaxSlots] = {};
    hipStream_t s_in = nullptr;
    hipEvent_t ev_loaded[kMaxSlots] = {}, ev_done[kMaxSlots] = {};
    bool slot_used[kMaxSlots] = {};
    // ablation variants (saber_options.ablation): document-order sampling needs the words in canonical order and
    // the word -> row map; the sort-based rebuild of A needs key buffers and the sort's work space
    int32_t *word_ids_d = nullptr, *word_row_d = nullptr;
    uint64_t *sort_keys = nullptr, *sort_keys_out = nullptr;
    uint32_t *sort_rank = nullptr;
    void *sort_tmp = nullptr;
    size_t sort_tmp_bytes = 0;
    unsigned sort_end_bit = 0;
    uint2 *alias_table = nullptr;     // [V_dense][K] {prob bits, alias} when the dense term is drawn from alias tables
};

static inline int grid_for(int64_t n, int block, int cap = 65535 * 16) {
    int64_t g = (n + block - 1) / block;
    return (int)std::max<int64_t>(1, std::min<int64_t>(g, cap));
}

extern "C" int saber_set_hooks(void *(*alloc)(size_t), void (*dealloc)(void *), void *hip_stream) {
    if ((alloc == nullptr) != (dealloc == nullptr))
        return fail(SABER_EINVAL, "saber_set_hooks: alloc and dealloc must be given together");
    g_hooks.alloc = alloc; g_hooks.dealloc = dealloc;
    g_hooks.stream = reinterpret_cast<hipStream_t>(hip_stream); g_hooks.have_stream = hip_stream != nullptr;
    return SABER_OK;
}

extern "C" void saber_options_default(saber_options *opt) {
    if (!opt) return;
    memset(opt, 0, sizeof(*opt));
    opt->n_chunks = 0; opt->block_threads = 0; opt->tile_tokens = 0; opt->stage_phi = 1; opt->profile = 0;
    opt->quarter_row_entries = 64; opt->half_row_entries = 128;
    opt->long_doc_tokens = 512; opt->dz_lds_entries = 2048; opt->stage_min_tokens = 0; opt->light_block_threads = 0; opt->light_word_tokens = 0;
}

extern "C" void saber_free(saber_ctx *c) {
    if (!c) return;
    if (c->stream) (void)hipStreamSynchronize(c->stream);
    auto release = [c](void *p) { dev_free(c->hooks, p); };
    release(c->z); release(c->tok_doc); release(c->tok_t); release(c->tiles); release(c->docrec);
    release(c->cd_ent); release(c->doc_ptr); release(c->short_docs); release(c->long_docs);
    release(c->doc_words); release(c->counters); release(c->dense_slots); release(c->ll_partial); release(c->z_wm);
    if (!c->parent) {   // the model's arrays belong to the model
        release(c->cwk); release(c->ck); release(c->denom); release(c->phi); release(c->l3_64); release(c->l3);
        release(c->sumphi); release(c->row_word); release(c->light_words); release(c->light_short);
        release(c->light_long); release(c->light_tok_ptr); release(c->wrec); release(c->lw_ent); release(c->lw_phi);
        release(c->vz_items);
    }
    if (c->have_events) for (auto &e : c->ev) if (e) (void)hipEventDestroy(e);
    if (c->s_in) { (void)hipStreamSynchronize(c->s_in); (void)hipStreamDestroy(c->s_in); }
    for (int s = 0; s < kMaxSlots; s++) {
        release(c->slot_tok_doc[s]); release(c->slot_tok_t[s]); release(c->slot_z[s]);
        if (c->ev_loaded[s]) (void)hipEventDestroy(c->ev_loaded[s]);
        if (c->ev_done[s]) (void)hipEventDestroy(c->ev_done[s]);
    }
    release(c->doc_blocks); release(c->ne_doc);
    release(c->word_ids_d); release(c->word_row_d); release(c->sort_keys); release(c->sort_keys_out);
    release(c->sort_rank); release(c->sort_tmp); release(c->alias_table);
    if (c->h_tok_t) (void)hipHostFree(c->h_tok_t);
    if (c->stream && c->own_stream) (void)hipStreamDestroy(c->stream);
    delete c;
}

// ------------------------------------------------------------------------------------------------
// launch helpers
// ------------------------------------------------------------------------------------------------
// The assignments of a chunk in canonical order: the resident array, which holds all tokens (`first` = 0: its first
// element is token 0), or the streaming buffer that holds the chunk (`first` = the chunk's first token).
struct ZView { void *z; int64_t first; };
static ZView z_view(const saber_ctx *c, const Chunk &ch, int slot) {
    return slot < 0 ? ZView{c->z, 0} : ZView{c->slot_z[slot], ch.t0};
}

// The rows of A the sampling kernel reads for the documents of chunk `ch` of context `theta`: all of them sit behind
// one buffer descriptor and are addressed by 32-bit byte offsets (build() keeps every chunk's rows below 4 GB).
static void set_rows(EStepParams &p, const saber_ctx *theta, const Chunk &ch) {
    p.docrec = theta->docrec;
    p.cd_rows = theta->cd_ent + (size_t)ch.row_unit0 * 32u;
    p.row_unit0 = (uint32_t)ch.row_unit0;
    p.rows_bytes = (uint32_t)((uint64_t)ch.row_units * 128u);
    p.quarter_row_bytes = 4u * (uint32_t)theta->opt.quarter_row_entries; p.half_row_bytes = 4u * (uint32_t)theta->opt.half_row_entries;
}

static EStepParams make_params(saber_ctx *c, const Chunk &ch, int slot = -1) {
    EStepParams p{};
    p.tiles = c->tiles + ch.tile0;
    if (slot < 0) { p.tok_doc = c->tok_doc + ch.t0; p.tok_t = c->tok_t + ch.t0; }
    else { p.tok_doc = c->slot_tok_doc[slot]; p.tok_t = c->slot_tok_t[slot]; }
    set_rows(p, c, ch);
    p.phi = c->phi; p.l3 = c->l3; p.l3_64 = c->l3_64; p.sumphi = c->sumphi;
    const ZView zv = z_view(c, ch, slot);
    p.z = zv.z; p.z_rel = ch.t0 - zv.first;
    p.base = c->phi + (size_t)c->V_dense * (size_t)c->Kpad;
    p.wrec = c->wrec; p.lw_ent = c->lw_ent; p.lw_phi = c->lw_phi; p.z_wm = c->z_wm;
    p.alias_table = c->alias_table;
    p.t_base = ch.t0; p.K = c->K; p.Kpad = c->Kpad; p.n3 = c->n3; p.n3pad = c->n3pad;
    p.topic_bits = c->topic_bits; p.topic_mask = c->topic_mask; p.alpha = c->alpha;
    p.seed_lo = (uint32_t)c->seed; p.seed_hi = (uint32_t)(c->seed >> 32); p.iter = c->iter;
    return p;
}

// LDS of a staged sampling workgroup's row: the Bhat row (K rounded to 4 floats) and the tree level (n3 rounded to 4)
static size_t estep_row_bytes(const saber_ctx *c) {
    return ((size_t)((c->K + 3) & ~3) + (size_t)((c->n3 + 3) & ~3)) * sizeof(float);
}
// dynamic LDS of a sampling workgroup: the row when staged, 16 bytes of control words, and in log-likelihood mode
// one double per wavefront
static size_t estep_lds_bytes(const saber_ctx *c, int mode) {
    return (c->staged ? estep_row_bytes(c) : 0) + 16 + (mode == MODE_LOGLIK ? 16 * sizeof(double) : 0);
}

// a workgroup may use more than the default 64 KB of LDS (up to the CU's 160 KB) once the kernel has been told so
template <typename Kern>
static void launch_with_lds(Kern kern, dim3 grid, dim3 block, size_t lds, hipStream_t stream, const EStepParams &p) {
    if (lds > 64 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kern, grid, block, lds, stream, p);
}

template <int MODE, bool STAGED, typename ZT>
static void launch_estep_b16(saber_ctx *c, dim3 grid, dim3 block, size_t lds, const EStepParams &p, bool light) {
    if (light) {   // light words exist only in the staged, 16-bit-z configuration
        if (c->b16) launch_with_lds(estep_kernel<MODE, true, uint16_t, true, true>, grid, block, lds, c->stream, p);
        else launch_with_lds(estep_kernel<MODE, true, uint16_t, false, true>, grid, block, lds, c->stream, p);
        return;
    }
    if (c->b16) launch_with_lds(estep_kernel<MODE, STAGED, ZT, true, false>, grid, block, lds, c->stream, p);
    else launch_with_lds(estep_kernel<MODE, STAGED, ZT, false, false>, grid, block, lds, c->stream, p);
}

// The staged 16/16 sampler addresses its Bhat row from LDS address 0: its kernels must have no static LDS in
// front of the dynamic part.
template <typename F>
static int static_lds_is_zero(F kernel) {
    hipFuncAttributes a;
    HIP_TRY(hipFuncGetAttributes(&a, reinterpret_cast<const void *>(kernel)));
    if (a.sharedSizeBytes != 0) return fail(SABER_EDEVICE, "sampling kernel built with %zu bytes of static LDS", (size_t)a.sharedSizeBytes);
    return SABER_OK;
}
static int check_estep_lds_layout() {
    SABER_TRY(static_lds_is_zero(estep_kernel<MODE_SAMPLE, true, uint16_t, true, false>));
    SABER_TRY(static_lds_is_zero(estep_kernel<MODE_SAMPLE, true, uint16_t, true, true>));
    SABER_TRY(static_lds_is_zero(estep_kernel<MODE_PROBS, true, uint16_t, true, false>));
    SABER_TRY(static_lds_is_zero(estep_kernel<MODE_PROBS, true, uint16_t, true, true>));
    SABER_TRY(static_lds_is_zero(estep_kernel<MODE_LOGLIK, true, uint16_t, true, false>));
    SABER_TRY(static_lds_is_zero(estep_kernel<MODE_LOGLIK, true, uint16_t, true, true>));
    SABER_TRY(static_lds_is_zero(estep_kernel<MODE_SAMPLE, true, int32_t, true, false>));
    SABER_TRY(static_lds_is_zero(estep_kernel<MODE_PROBS, true, int32_t, true, false>));
    SABER_TRY(static_lds_is_zero(estep_kernel<MODE_LOGLIK, true, int32_t, true, false>));
    return SABER_OK;
}

// One E-step launch per tile class.  Dense-row tiles with at least stage_min_tokens tokens run with block_threads
// threads, smaller ones with light_block_threads (so that a word with few tokens does not hold a large workgroup
// whose wavefronts have nothing to do); tiles of light words run the variant that builds the Bhat row from the
// base vector and the word's non-zeros.  All stage the row in LDS when it fits.
template <int MODE>
static int launch_estep(saber_ctx *c, const Chunk &ch, EStepParams &p0) {
    struct Class { int64_t first, count; int block; bool light; };
    const Class classes[3] = {
        {0, ch.n_heavy, c->opt.block_threads, false},
        {ch.n_heavy, ch.n_dense - ch.n_heavy, c->opt.light_block_threads, false},
        {ch.n_dense, ch.ntiles - ch.n_dense, c->opt.light_block_threads, true},
    };
    for (const Class &cl : classes) {
        if (cl.count == 0) continue;
        EStepParams p = p0;
        p.tiles = p0.tiles + cl.first;
        if (p0.out_ll) p.out_ll = p0.out_ll + cl.first;
        const dim3 grid((unsigned)cl.count), block((unsigned)cl.block);
        const size_t lds = estep_lds_bytes(c, MODE);
        if (c->staged) {
            if (c->z16) launch_estep_b16<MODE, true, uint16_t>(c, grid, block, lds, p, cl.light);
            else launch_estep_b16<MODE, true, int32_t>(c, grid, block, lds, p, false);
        } else {
            if (c->z16) launch_estep_b16<MODE, false, uint16_t>(c, grid, block, lds, p, false);
            else launch_estep_b16<MODE, false, int32_t>(c, grid, block, lds, p, false);
        }
        HIP_TRY(hipGetLastError());
    }
    return SABER_OK;
}

// Segmented count of one grouping of the assignments: documents over z (CountByDZ -> rows of A) or light words
// over z_wm (CountByVZ -> sparse rows of B).  Two launches: short segments with one wavefront each, long ones
// with 256 threads.
static int launch_segmented_count(saber_ctx *c, const int32_t *short_list, int64_t n_short, const int32_t *long_list,
                                  int64_t n_long, const int64_t *seg_ptr, const void *z, int64_t z_first, uint2 *rec,
                                  uint32_t *ent) {
    for (int pass = 0; pass < 2; pass++) {
        const int64_t n = pass == 0 ? n_short : n_long;
        const int32_t *list = pass == 0 ? short_list : long_list;
        const int block = pass == 0 ? 64 : 256;
        if (n == 0) continue;
        // LDS: bitmap + rank prefix (2 * nwords) + the row under construction; a short segment's row has at
        // most long_doc_tokens entries, so its workgroup asks for no more than that
        const int budget = std::max(0, (int)((63 * 1024 - 8 * (int64_t)c->nwords) / 4));
        const int want = pass == 0 ? std::min(c->opt.long_doc_tokens, c->K) : c->opt.dz_lds_entries;
        const int entries = std::min(want, budget);
        const size_t lds = ((size_t)2 * c->nwords + (size_t)entries) * sizeof(uint32_t);
        if (lds > 63 * 1024) {   // K > 2^17: the two bitmap arrays alone pass 64 KB; gfx950 has 160 KB per workgroup
            const void *fn = c->z16 ? (const void *)count_dz_kernel<uint16_t> : (const void *)count_dz_kernel<int32_t>;
            HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        }
        const dim3 grid((unsigned)n), blk((unsigned)block);
        if (c->z16)
            hipLaunchKernelGGL((count_dz_kernel<uint16_t>), grid, blk, lds, c->stream, list, seg_ptr,
                               (const uint16_t *)z, z_first, rec, ent, c->K, c->topic_bits, c->nwords, entries);
        else
            hipLaunchKernelGGL((count_dz_kernel<int32_t>), grid, blk, lds, c->stream, list, seg_ptr,
                               (const int32_t *)z, z_first, rec, ent, c->K, c->topic_bits, c->nwords, entries);
        HIP_TRY(hipGetLastError());
    }
    return SABER_OK;
}

// Ablation: A rebuilt by sorting the (document, topic) pairs of all tokens
static int launch_sort_rebuild(saber_ctx *c) {
    if (c->T == 0 || c->D == 0) return SABER_OK;
    const dim3 grid((unsigned)((c->D + 3) / 4)), block(256);
    if (c->z16)
        hipLaunchKernelGGL((sort_keys_kernel<uint16_t>), grid, block, 0, c->stream, c->doc_ptr, (const uint16_t *)c->z, c->D,
                           c->topic_bits, c->sort_keys);
    else
        hipLaunchKernelGGL((sort_keys_kernel<int32_t>), grid, block, 0, c->stream, c->doc_ptr, (const int32_t *)c->z, c->D,
                           c->topic_bits, c->sort_keys);
    HIP_TRY(hipGetLastError());
    size_t bytes = c->sort_tmp_bytes;
    HIP_TRY(rocprim::radix_sort_keys(c->sort_tmp, bytes, c->sort_keys, c->sort_keys_out, (size_t)c->T, 0u, c->sort_end_bit,
                                     c->stream));
    hipLaunchKernelGGL(sort_mark_kernel, grid, block, 0, c->stream, c->doc_ptr, c->sort_keys_out, c->D, c->topic_mask,
                       c->docrec, c->cd_ent, c->sort_rank);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(sort_count_kernel, grid, block, 0, c->stream, c->doc_ptr, c->sort_rank, c->D, c->docrec, c->cd_ent,
                       c->topic_bits);
    HIP_TRY(hipGetLastError());
    return SABER_OK;
}

static int launch_count_dz(saber_ctx *c) {
    if (c->opt.ablation & 2) return launch_sort_rebuild(c);
    return launch_segmented_count(c, c->short_docs, c->n_short, c->long_docs, c->n_long, c->doc_ptr, c->z, 0, c->docrec,
                                  c->cd_ent);
}

// CountByDZ for the documents of one chunk whose assignments sit in a buffer
static int launch_count_dz_chunk(saber_ctx *c, const Chunk &ch, int slot) {
    const ZView zv = z_view(c, ch, slot);
    return launch_segmented_count(c, c->short_docs + ch.short0, ch.nshort, c->long_docs + ch.long0, ch.nlong, c->doc_ptr,
                                  zv.z, zv.first, c->docrec, c->cd_ent);
}

// ---- host streaming ----
// Takes the next buffer (round robin) for chunk `ch`: once the kernels of the buffer's previous user have run, the
// chunk's tok_t is copied in and tok_doc derived from it (both on the copy stream), and the compute stream is made to
// wait for that.
static int stream_acquire(saber_ctx *c, const Chunk &ch, int *slot) {
    const int s = c->next_slot;
    c->next_slot = (c->next_slot + 1) % c->n_slots;
    if (ch.ntok > c->slot_tokens) return fail(SABER_ESTATE, "chunk of %lld tokens exceeds the streaming buffers", (long long)ch.ntok);
    if (c->slot_used[s]) HIP_TRY(hipStreamWaitEvent(c->s_in, c->ev_done[s], 0));
    *slot = s;
    if (ch.ntok == 0) return SABER_OK;
    HIP_TRY(hipMemcpyAsync(c->slot_tok_t[s], c->h_tok_t + ch.t0, (size_t)ch.ntok * sizeof(uint32_t), hipMemcpyHostToDevice, c->s_in));
    // on the copy stream as well: the look-ups of this kernel wait for memory most of the time and run beside the
    // sampling of the chunk before (1.7 ms per 123 M tokens of short documents when it ran in line with it)
    hipLaunchKernelGGL(expand_tok_doc_kernel, dim3(grid_for(ch.ntok, 256)), dim3(256), 0, c->s_in, c->slot_tok_t[s],
                       ch.ntok, ch.t0, c->doc_blocks, c->ne_doc, c->slot_tok_doc[s]);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(c->ev_loaded[s], c->s_in));
    HIP_TRY(hipStreamWaitEvent(c->stream, c->ev_loaded[s], 0));
    return SABER_OK;
}
// After the chunk's kernels have been queued: the buffer may be overwritten once they have run.
static int stream_release(saber_ctx *c, int s) {
    HIP_TRY(hipEventRecord(c->ev_done[s], c->stream));
    c->slot_used[s] = true;
    return SABER_OK;
}
static int sync_all(saber_ctx *c) {
    HIP_TRY(hipStreamSynchronize(c->stream));
    if (c->n_slots) HIP_TRY(hipStreamSynchronize(c->s_in));
    return SABER_OK;
}

// CountByVZ + Preprocess + BuildTree for the light words (sparse rows of B); needs the base vector, i.e. runs
// after launch_phi
static int launch_light_words(saber_ctx *c) {
    if (c->V_light == 0) return SABER_OK;
    SABER_TRY(launch_segmented_count(c, c->light_short, c->n_light_short, c->light_long, c->n_light_long,
                                     c->light_tok_ptr, c->z_wm, 0, c->wrec, c->lw_ent));
    const size_t lds = (size_t)c->n3 * (sizeof(double) + sizeof(int));
    hipLaunchKernelGGL(light_tree_kernel, dim3((unsigned)c->V_light), dim3(64), lds, c->stream, c->light_words, c->wrec,
                       c->lw_ent, c->lw_phi, c->denom, c->phi + (size_t)c->V_dense * (size_t)c->Kpad,
                       c->l3_64 + (size_t)c->V * (size_t)c->n3, c->l3, c->l3_64, c->sumphi, c->n3, c->n3pad,
                       c->topic_bits, c->beta);
    HIP_TRY(hipGetLastError());
    return SABER_OK;
}

// nnz(A), sum_d K_d L_d, sum_d K_d U_d and the non-zeros of the sparse rows of B (what the next E-step will
// read) into four device counters
static int launch_row_stats(saber_ctx *c, unsigned long long *out2) {
    if (c->D == 0) return SABER_OK;
    hipLaunchKernelGGL(row_stats_kernel, dim3(grid_for(c->D, 256, 1024)), dim3(256), 0, c->stream, c->docrec,
                       c->doc_ptr, c->doc_words, c->D, out2);
    HIP_TRY(hipGetLastError());
    if (c->V_light) {
        hipLaunchKernelGGL(light_stats_kernel, dim3(grid_for(c->V_light, 256, 256)), dim3(256), 0, c->stream, c->wrec,
                           c->V_light, out2 + 3);
        HIP_TRY(hipGetLastError());
    }
    return SABER_OK;
}

static int launch_topic_totals(saber_ctx *c) {
    hipLaunchKernelGGL(fill_u32_kernel, dim3(grid_for(2 * (int64_t)c->K, 256)), dim3(256), 0, c->stream, (uint32_t *)c->ck, 0u, (size_t)c->K * 2);
    HIP_TRY(hipGetLastError());
    if (c->T == 0) return SABER_OK;
    const int use_lds = (size_t)c->K * 4 <= 60 * 1024;
    // every workgroup ends with up to K atomics into the K totals: few, large workgroups (about 500 of them, each
    // over at least 65,536 and at most 2^20 assignments) keep those from dominating
    const int64_t per_block = std::min<int64_t>(1 << 20, std::max<int64_t>(65536, ((c->T / 512 + 4095) / 4096) * 4096));
    const int64_t nblocks = (c->T + per_block - 1) / per_block;
    const size_t lds = use_lds ? (size_t)c->K * 4 : 0;
    // a histogram of all assignments: their order does not matter, and with host streaming the word-major copy is
    // the one that is resident
    const void *zsrc = c->n_slots ? c->z_wm : c->z;
    if (c->z16)
        hipLaunchKernelGGL((topic_totals_kernel<uint16_t>), dim3((unsigned)nblocks), dim3(1024), lds, c->stream,
                           (const uint16_t *)zsrc, c->T, per_block, c->ck, c->K, use_lds);
    else
        hipLaunchKernelGGL((topic_totals_kernel<int32_t>), dim3((unsigned)nblocks), dim3(1024), lds, c->stream,
                           (const int32_t *)zsrc, c->T, per_block, c->ck, c->K, use_lds);
    HIP_TRY(hipGetLastError());
    return SABER_OK;
}

// LDS of one workgroup of the alias-table build: K + 1 prefix sums (binary64) and K item numbers
static size_t alias_lds_bytes(int K) { return ((size_t)K + 1) * sizeof(double) + (size_t)K * sizeof(uint32_t); }

static int launch_phi(saber_ctx *c) {
    hipLaunchKernelGGL(denominators_kernel, dim3(grid_for(c->K, 256)), dim3(256), 0, c->stream, c->ck, c->denom, c->K, c->vbeta);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(phi_tree_kernel, dim3((unsigned)(c->V_dense + 1)), dim3(256), 0, c->stream, c->cwk, c->denom, c->phi,
                       c->l3, c->l3_64, c->sumphi, c->row_word, c->K, c->Kpad, c->n3, c->n3pad, c->beta, 1);
    HIP_TRY(hipGetLastError());
    if (c->alias_table && c->V_dense > 0) {   // measurement variant: an alias table per word on top of the tree level
        const size_t lds = alias_lds_bytes(c->K);
        if (lds > 64 * 1024)
            HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(alias_sweep_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(alias_sweep_kernel, dim3((unsigned)c->V_dense), dim3(kAliasThreads), lds, c->stream, c->phi, c->K, c->Kpad, c->alias_table);
        HIP_TRY(hipGetLastError());
    }
    return SABER_OK;
}

// Word-major copy of z (after init / set_z; an E-step writes it itself).
static int launch_fill_zwm_chunk(saber_ctx *c, const Chunk &ch, int slot) {
    if (ch.ntiles == 0) return SABER_OK;
    const uint32_t *tok_t = slot < 0 ? c->tok_t + ch.t0 : c->slot_tok_t[slot];
    const ZView zv = z_view(c, ch, slot);
    if (c->z16)
        hipLaunchKernelGGL((fill_zwm_kernel<uint16_t>), dim3((unsigned)ch.ntiles), dim3(256), 0, c->stream,
                           c->tiles + ch.tile0, tok_t, (const uint16_t *)zv.z, ch.t0 - zv.first, (uint16_t *)c->z_wm);
    else
        hipLaunchKernelGGL((fill_zwm_kernel<int32_t>), dim3((unsigned)ch.ntiles), dim3(256), 0, c->stream,
                           c->tiles + ch.tile0, tok_t, (const int32_t *)zv.z, ch.t0 - zv.first, (int32_t *)c->z_wm);
    HIP_TRY(hipGetLastError());
    return SABER_OK;
}
static int launch_fill_zwm(saber_ctx *c) {
    for (const Chunk &ch : c->chunks) SABER_TRY(launch_fill_zwm_chunk(c, ch, -1));
    return SABER_OK;
}

// Ablation: the E-step over the tokens in document order, then the word-major copy from z
static int launch_estep_docmajor(saber_ctx *c, unsigned long long *n_dense) {
    if (c->T == 0 || c->D == 0) return SABER_OK;
    DocMajorParams p{};
    p.doc_ptr = c->doc_ptr; p.word_ids = c->word_ids_d; p.word_row = c->word_row_d;
    p.docrec = c->docrec; p.cd_ent = c->cd_ent;
    p.phi = c->phi; p.l3 = c->l3; p.sumphi = c->sumphi; p.l3_64 = c->l3_64;
    p.z = c->z; p.n_dense = n_dense; p.D = c->D;
    p.K = c->K; p.Kpad = c->Kpad; p.n3 = c->n3; p.n3pad = c->n3pad;
    p.topic_bits = c->topic_bits; p.topic_mask = c->topic_mask; p.alpha = c->alpha;
    p.seed_lo = (uint32_t)c->seed; p.seed_hi = (uint32_t)(c->seed >> 32); p.iter = c->iter;
    const dim3 grid((unsigned)((c->D + 3) / 4)), block(256);
    if (c->z16) hipLaunchKernelGGL((estep_docmajor_kernel<uint16_t>), grid, block, 0, c->stream, p);
    else hipLaunchKernelGGL((estep_docmajor_kernel<int32_t>), grid, block, 0, c->stream, p);
    HIP_TRY(hipGetLastError());
    return launch_fill_zwm(c);
}

// CountByVZ for the dense rows of B out of the word-major assignments; the rows must be all zero on entry
// (the Bhat kernel leaves them so).
static int launch_count_vz(saber_ctx *c) {
    if (c->n_vz_items == 0) return SABER_OK;
    const int use_lds = (size_t)c->K * 4 <= 60 * 1024;
    const size_t lds = use_lds ? (size_t)c->K * 4 : 0;
    const dim3 grid((unsigned)c->n_vz_items), block(use_lds ? 1024u : 256u);
    if (c->z16)
        hipLaunchKernelGGL((count_vz_kernel<uint16_t>), grid, block, lds, c->stream, c->vz_items, (const uint16_t *)c->z_wm,
                           c->cwk, c->K, c->Kpad, use_lds);
    else
        hipLaunchKernelGGL((count_vz_kernel<int32_t>), grid, block, lds, c->stream, c->vz_items, (const int32_t *)c->z_wm,
                           c->cwk, c->K, c->Kpad, use_lds);
    HIP_TRY(hipGetLastError());
    return SABER_OK;
}

// iteration 0: the Philox draw of Alg. 1's initialisation for the canonical tokens [t0, t1), stored from z[z_rel] on
static int launch_init_z(saber_ctx *c, void *z, int64_t z_rel, int64_t t0, int64_t t1) {
    if (t1 <= t0) return SABER_OK;
    if (c->z16)
        hipLaunchKernelGGL((init_z_kernel<uint16_t>), dim3(grid_for(t1 - t0, 256, 8192)), dim3(256), 0, c->stream,
                           (uint16_t *)z, z_rel, t0, t1, (uint32_t)c->K, (uint32_t)c->seed, (uint32_t)(c->seed >> 32));
    else
        hipLaunchKernelGGL((init_z_kernel<int32_t>), dim3(grid_for(t1 - t0, 256, 8192)), dim3(256), 0, c->stream,
                           (int32_t *)z, z_rel, t0, t1, (uint32_t)c->K, (uint32_t)c->seed, (uint32_t)(c->seed >> 32));
    HIP_TRY(hipGetLastError());
    return SABER_OK;
}

// The M-step after the assignments changed outside an E-step: all four rebuilds of Alg. 1.
// With host streaming the assignments are not on the device: they come chunk by chunk from user_z, or when that
// is null from the Philox draw of iteration 0.
static int full_mstep(saber_ctx *c, const int32_t *user_z = nullptr) {
    if (c->n_slots) {   // chunk by chunk: rows of A and the word-major copy
        std::vector<uint16_t> stage;
        for (const Chunk &ch : c->chunks) {
            int s;
            SABER_TRY(stream_acquire(c, ch, &s));
            if (user_z && ch.ntok) {
                HIP_TRY(hipStreamSynchronize(c->stream));   // the buffer's earlier kernels are done: plain copy
                const void *src = user_z + ch.t0;
                if (c->z16) {
                    stage.resize((size_t)ch.ntok);
                    for (int64_t i = 0; i < ch.ntok; i++) stage[(size_t)i] = (uint16_t)user_z[ch.t0 + i];
                    src = stage.data();
                }
                HIP_TRY(hipMemcpy(c->slot_z[s], src, (size_t)ch.ntok * (c->z16 ? 2 : 4), hipMemcpyHostToDevice));
            } else {
                SABER_TRY(launch_init_z(c, c->slot_z[s], 0, ch.t0, ch.t0 + ch.ntok));
            }
            SABER_TRY(launch_count_dz_chunk(c, ch, s));
            SABER_TRY(launch_fill_zwm_chunk(c, ch, s));
            SABER_TRY(stream_release(c, s));
        }
    } else {
        SABER_TRY(launch_count_dz(c));
    }
    if (c->parent) {   // held-out documents: A only, the model stays frozen
        HIP_TRY(hipStreamSynchronize(c->stream));
        return SABER_OK;
    }
    if (!c->n_slots) SABER_TRY(launch_fill_zwm(c));
    SABER_TRY(launch_count_vz(c));
    SABER_TRY(launch_topic_totals(c));
    SABER_TRY(launch_phi(c));
    SABER_TRY(launch_light_words(c));
    SABER_TRY(sync_all(c));
    return SABER_OK;
}

// Workload numbers of the E-step that will read the current A: nnz(A) and sum_d K_d * L_d.
static int refresh_workload_stats(saber_ctx *c) {
    hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, c->stream, (uint32_t *)c->counters, 0u, (size_t)kCtr * 2);
    HIP_TRY(hipGetLastError());
    SABER_TRY(launch_row_stats(c, c->counters + 1));
    HIP_TRY(hipStreamSynchronize(c->stream));
    unsigned long long h[kCtr];
    HIP_TRY(hipMemcpy(h, c->counters, sizeof(h), hipMemcpyDeviceToHost));
    c->stats.nnz_cd = (int64_t)h[1]; c->stats.next_row_entries = (int64_t)h[2]; c->stats.next_row_fetch = (int64_t)h[3];
    c->stats.next_light_entries = (int64_t)h[4];
    return SABER_OK;
}

// ------------------------------------------------------------------------------------------------
// saber_init
// ------------------------------------------------------------------------------------------------
static int build(saber_ctx *c, const int64_t *doc_ptr, const int32_t *word_ids) {
    const int64_t D = c->D, T = c->T; const int32_t V = c->V, K = c->K;
    if (c->hooks.have_stream) { c->stream = c->hooks.stream; c->own_stream = false; }
    else { HIP_TRY(hipStreamCreate(&c->stream)); c->own_stream = true; }
    if (c->opt.profile) {
        for (auto &e : c->ev) HIP_TRY(hipEventCreate(&e));
        c->have_events = true;
    }
    // ---- chunks: contiguous document ranges of about equal token count (Sec. 3.1.2) ----
    // A chunk also ends before its rows of A (128-byte aligned slots of capacity min(L_d, K)) would pass 4 GB: the
    // sampling kernel addresses them by 32-bit byte offsets.  That only happens with far fewer chunks than the default.
    const int nch = std::max(1, c->opt.n_chunks);
    const int64_t unit_limit = (int64_t)0xfff00000ll / 128;
    c->chunks.clear();
    {
        int64_t d = 0;
        for (int i = 0; i < nch || d < D; i++) {
            Chunk ch; ch.d0 = d; ch.t0 = doc_ptr[d];
            const int64_t target = i < nch - 1 ? (T * (int64_t)(i + 1)) / nch : T;
            int64_t units = 0;
            while (d < D && doc_ptr[d + 1] <= target) {
                const int64_t u = (std::min<int64_t>(doc_ptr[d + 1] - doc_ptr[d], K) + 31) / 32;
                if (units + u > unit_limit) break;
                units += u; d++;
            }
            ch.d1 = d; ch.ntok = doc_ptr[d] - ch.t0;
            if (ch.ntok >= (1ll << 31)) return fail(SABER_ERANGE, "saber_init: a document chunk holds %lld tokens (limit 2^31)", (long long)ch.ntok);
            if (ch.d1 > ch.d0) c->chunks.push_back(ch);
        }
    }
    // ---- words: dense rows of B for the frequent ones, sparse rows for the rest ----
    // A word with n tokens has at most n non-zero counts; below light_word_tokens tokens its sparse row
    // (8 bytes per non-zero, rebuilt by a segmented count like a row of A) is cheaper than 12*K bytes of dense B / Bhat
    // traffic per iteration.  Needs the LDS-staged sampler and 16-bit assignments.
    std::vector<int64_t> n_v((size_t)V, 0);
    for (int64_t t = 0; t < T; t++) n_v[(size_t)word_ids[t]]++;
    const bool light_ok = c->staged && c->z16 && c->opt.light_word_tokens > 0;
    const saber_ctx *par = c->parent;   // then the model's word classes are taken over
    // a packed entry of a sparse row has at least 16 count bits when the assignments are 16-bit
    c->opt.light_word_tokens = std::min(c->opt.light_word_tokens, 65536);
    c->h_word_row.assign((size_t)V, 0);
    std::vector<int32_t> h_row_word, h_light_words, h_light_short, h_light_long;
    std::vector<int64_t> h_light_tok_ptr(1, 0);
    std::vector<uint2> h_wrec;
    {
        int64_t lunits = 0;
        for (int32_t v = 0; v < V; v++) {
            if (par ? par->h_word_row[(size_t)v] < 0 : (light_ok && n_v[(size_t)v] < c->opt.light_word_tokens)) {
                const int32_t li = (int32_t)h_light_words.size();
                c->h_word_row[(size_t)v] = -li - 1;
                h_light_words.push_back(v);
                h_light_tok_ptr.push_back(h_light_tok_ptr.back() + n_v[(size_t)v]);
                if (lunits > 0xffffffffll) return fail(SABER_ERANGE, "sparse rows of B exceed 2^32 * 128 bytes");
                h_wrec.push_back(make_uint2((uint32_t)lunits, 0u));
                lunits += (std::min<int64_t>(n_v[(size_t)v], K) + 31) / 32;
                (n_v[(size_t)v] > c->opt.long_doc_tokens ? h_light_long : h_light_short).push_back(li);
            } else {
                c->h_word_row[(size_t)v] = (int32_t)h_row_word.size();
                h_row_word.push_back(v);
            }
        }
        c->V_dense = (int32_t)h_row_word.size(); c->V_light = (int32_t)h_light_words.size();
        h_row_word.push_back(V);   // the all-zero row: its Bhat is the base vector, its tree level the base running sums
        c->T_light = h_light_tok_ptr.back(); c->lw_cap = lunits * 32;
        c->n_light_short = (int64_t)h_light_short.size(); c->n_light_long = (int64_t)h_light_long.size();
    }
    // ---- resident or streamed?  stream_workers = 0 keeps everything on the device when it fits and falls back to
    // host streaming with three buffers when it does not ----
    if (!par && c->opt.stream_workers == 0 && c->opt.ablation == 0 && T > 0) {
        const size_t zs = c->z16 ? 2 : 4;
        size_t row_units = 0, slot_tokens = 0, tiles_bound = (size_t)(T / std::max(1, c->opt.tile_tokens));
        for (int64_t d = 0; d < D; d++) row_units += (size_t)((std::min<int64_t>(doc_ptr[d + 1] - doc_ptr[d], K) + 31) / 32);
        for (const Chunk &ch : c->chunks) {
            slot_tokens = std::max(slot_tokens, (size_t)ch.ntok);
            tiles_bound += (size_t)std::min<int64_t>(V, ch.ntok);
        }
        const size_t common = row_units * 128 + (size_t)D * 32 + tiles_bound * sizeof(Tile) +
                              ((size_t)c->V_dense + 1) * (size_t)c->Kpad * 8 +
                              ((size_t)V + 1) * ((size_t)c->n3pad * 4 + (size_t)c->n3 * 8 + 4) + (size_t)c->lw_cap * 8 +
                              (size_t)T * zs + ((size_t)32 << 20);
        const size_t resident = common + (size_t)T * (8 + zs);
        const size_t streamed = common + 3 * slot_tokens * (8 + zs) + (size_t)T / 4 + (size_t)D * 4;
        size_t limit = (size_t)std::max(0, c->opt.device_mem_limit_mb) << 20;
        if (limit == 0) {
            size_t free_b = 0, total_b = 0;
            HIP_TRY(hipMemGetInfo(&free_b, &total_b));
            limit = free_b;
        }
        if (resident > limit - limit / 16) {
            if (streamed > limit - limit / 16)
                return fail(SABER_ENOMEM, "saber_init: the corpus needs about %.1f GB of device memory (%.1f GB with the token "
                            "lists streamed from the host) and %.1f GB are available; more chunks shrink the streaming buffers",
                            resident / 1e9, streamed / 1e9, limit / 1e9);
            c->n_slots = 3;
        }
    }
    c->stats.stream_workers = c->n_slots;

    // ---- word-major token arrays and tiles per chunk (host counting sort; layout only) ----
    // position of every word's segment in the word-major order (light words first, then dense rows) and the
    // slabs CountByVZ cuts the dense rows' segments into
    std::vector<int64_t> wm_ptr((size_t)V, 0), wm_seen((size_t)V, 0);   // wm_seen: tokens placed so far (chunk by chunk)
    std::vector<VzItem> h_vz_items;
    {
        for (int32_t li = 0; li < c->V_light; li++) wm_ptr[(size_t)h_light_words[(size_t)li]] = h_light_tok_ptr[(size_t)li];
        int64_t pos = c->T_light;
        const int64_t slab = 131072;
        for (int32_t r = 0; r < c->V_dense; r++) {
            const int32_t v = h_row_word[(size_t)r];
            wm_ptr[(size_t)v] = pos;
            for (int64_t s = 0; s < n_v[(size_t)v]; s += slab)
                h_vz_items.push_back(VzItem{r, (int32_t)std::min<int64_t>(slab, n_v[(size_t)v] - s), pos + s});
            pos += n_v[(size_t)v];
        }
        c->n_vz_items = (int64_t)h_vz_items.size();
    }
    // the word-major token arrays: ordinary host memory on the way to the device, or with host streaming the
    // pinned arrays that stay
    std::vector<int32_t> v_tok_doc; std::vector<uint32_t> v_tok_t;
    int32_t *h_tok_doc; uint32_t *h_tok_t;
    if (c->n_slots) {
        const size_t n = (size_t)std::max<int64_t>(T, 1);
        HIP_TRY(hipHostMalloc((void **)&c->h_tok_t, n * sizeof(uint32_t), hipHostMallocDefault));
        h_tok_doc = nullptr; h_tok_t = c->h_tok_t;   // tok_doc is derived on the device
    } else {
        v_tok_doc.resize((size_t)std::max<int64_t>(T, 1)); v_tok_t.resize((size_t)std::max<int64_t>(T, 1));
        h_tok_doc = v_tok_doc.data(); h_tok_t = v_tok_t.data();
    }
    std::vector<Tile> h_tiles;
    std::vector<int64_t> wcount((size_t)V + 1);
    const int tile_tokens = c->opt.tile_tokens;
    for (Chunk &ch : c->chunks) {
        std::fill(wcount.begin(), wcount.end(), 0);
        for (int64_t t = ch.t0; t < ch.t0 + ch.ntok; t++) wcount[(size_t)word_ids[t] + 1]++;
        for (int32_t v = 0; v < V; v++) wcount[(size_t)v + 1] += wcount[(size_t)v];
        const size_t first_tile = h_tiles.size();
        for (int32_t v = 0; v < V; v++) {
            const int64_t b = wcount[(size_t)v], e = wcount[(size_t)v + 1];
            const int32_t row = c->h_word_row[(size_t)v];
            if (e > b) { ch.words_present++; if (row < 0) c->stats.light_words_present++; }
            for (int64_t s = b; s < e; s += tile_tokens) {
                const int32_t cnt = (int32_t)std::min<int64_t>(tile_tokens, e - s);
                h_tiles.push_back(Tile{v, (int32_t)s, cnt, row >= 0 ? row : -row - 1, wm_ptr[(size_t)v] + wm_seen[(size_t)v], 0});
                wm_seen[(size_t)v] += cnt;
            }
        }
        for (int64_t d = ch.d0; d < ch.d1; d++)
            for (int64_t t = doc_ptr[d]; t < doc_ptr[d + 1]; t++) {
                const int64_t pos = ch.t0 + wcount[(size_t)word_ids[t]]++;
                if (h_tok_doc) h_tok_doc[(size_t)pos] = (int32_t)d;
                h_tok_t[(size_t)pos] = (uint32_t)(t - ch.t0);
            }
        // tiles of dense-row words first, then those of light words; inside each group heavy tiles first so the
        // tail of a launch is made of small ones (Sec. 3.4)
        const std::vector<int32_t> &wr = c->h_word_row;
        std::stable_sort(h_tiles.begin() + (ptrdiff_t)first_tile, h_tiles.end(), [&wr](const Tile &a, const Tile &b) {
            const bool la = wr[(size_t)a.word] < 0, lb = wr[(size_t)b.word] < 0;
            return la != lb ? lb : a.count > b.count;
        });
        ch.tile0 = (int64_t)first_tile; ch.ntiles = (int64_t)(h_tiles.size() - first_tile);
        for (size_t i = first_tile; i < h_tiles.size(); i++) {
            if (wr[(size_t)h_tiles[i].word] < 0) continue;
            ch.n_dense++;
            if (h_tiles[i].count >= c->opt.stage_min_tokens) ch.n_heavy++;
        }
        c->max_chunk_tiles = std::max(c->max_chunk_tiles, ch.ntiles);
    }
    c->total_tiles = (int64_t)h_tiles.size();
    // ---- rows of A: fixed, 128-byte aligned slots of capacity min(L_d, K) (Sec. 3.4 aligns rows likewise) ----
    std::vector<uint2> h_rec((size_t)std::max<int64_t>(D, 1));
    std::vector<int32_t> h_short, h_long;
    std::vector<uint32_t> h_doc_words((size_t)std::max<int64_t>(D, 1));
    {   // distinct words per document (layout statistic for the bandwidth model)
        std::vector<int64_t> last_doc((size_t)V, -1);
        for (int64_t d = 0; d < D; d++) {
            uint32_t u = 0;
            for (int64_t t = doc_ptr[d]; t < doc_ptr[d + 1]; t++)
                if (last_doc[(size_t)word_ids[t]] != d) { last_doc[(size_t)word_ids[t]] = d; u++; }
            h_doc_words[(size_t)d] = u;
        }
    }
    c->doc_len.resize((size_t)D);
    int64_t units = 0;
    for (int64_t d = 0; d < D; d++) {
        const int64_t len = doc_ptr[d + 1] - doc_ptr[d];
        c->doc_len[(size_t)d] = len;
        if (units > 0xffffffffll) return fail(SABER_ERANGE, "rows of A exceed 2^32 * 128 bytes");
        h_rec[(size_t)d] = make_uint2((uint32_t)units, 0u);
        units += (std::min<int64_t>(len, K) + 31) / 32;
        (len > c->opt.long_doc_tokens ? h_long : h_short).push_back((int32_t)d);
    }
    c->cd_cap = units * 32;
    c->n_short = (int64_t)h_short.size(); c->n_long = (int64_t)h_long.size();
    for (Chunk &ch : c->chunks) {   // both lists ascend by document: a chunk's documents are a contiguous part of each
        ch.row_unit0 = (int64_t)h_rec[(size_t)ch.d0].x;
        ch.row_units = (ch.d1 < D ? (int64_t)h_rec[(size_t)ch.d1].x : units) - ch.row_unit0;
        ch.short0 = std::lower_bound(h_short.begin(), h_short.end(), (int32_t)ch.d0) - h_short.begin();
        ch.nshort = (std::lower_bound(h_short.begin(), h_short.end(), (int32_t)std::min<int64_t>(ch.d1, 0x7fffffff)) - h_short.begin()) - ch.short0;
        ch.long0 = std::lower_bound(h_long.begin(), h_long.end(), (int32_t)ch.d0) - h_long.begin();
        ch.nlong = (std::lower_bound(h_long.begin(), h_long.end(), (int32_t)std::min<int64_t>(ch.d1, 0x7fffffff)) - h_long.begin()) - ch.long0;
        c->slot_tokens = std::max(c->slot_tokens, ch.ntok);
    }

    // ---- device memory ----
    const size_t vk = ((size_t)c->V_dense + 1) * (size_t)c->Kpad;
    if (c->n_slots) {
        HIP_TRY(hipStreamCreateWithFlags(&c->s_in, hipStreamNonBlocking));
        for (int s = 0; s < c->n_slots; s++) {
            SABER_TRY(dev_alloc(c->hooks, &c->slot_tok_doc[s], (size_t)c->slot_tokens)); SABER_TRY(dev_alloc(c->hooks, &c->slot_tok_t[s], (size_t)c->slot_tokens));
            if (c->z16) SABER_TRY(dev_alloc(c->hooks, (uint16_t **)&c->slot_z[s], (size_t)c->slot_tokens));
            else SABER_TRY(dev_alloc(c->hooks, (int32_t **)&c->slot_z[s], (size_t)c->slot_tokens));
            HIP_TRY(hipEventCreateWithFlags(&c->ev_loaded[s], hipEventDisableTiming));
            HIP_TRY(hipEventCreateWithFlags(&c->ev_done[s], hipEventDisableTiming));
        }
        std::vector<uint4> blocks((size_t)((T + 63) / 64) + 1, make_uint4(0u, 0u, 0u, 0u));
        std::vector<int32_t> ne;
        for (int64_t d = 0; d < D; d++) {
            const int64_t t = doc_ptr[d], end = doc_ptr[d + 1];
            if (end <= t) continue;
            const uint32_t r = (uint32_t)ne.size();
            ne.push_back((int32_t)d);
            const int j = (int)(t & 63);
            if (j) { uint4 &q = blocks[(size_t)(t >> 6)]; if (j < 32) q.y |= 1u << j; else q.z |= 1u << (j - 32); }
            for (int64_t b = (t + 63) >> 6; b <= (end - 1) >> 6; b++) blocks[(size_t)b].x = r;   // blocks that begin inside d
        }
        SABER_TRY(dev_alloc(c->hooks, &c->doc_blocks, blocks.size()));
        HIP_TRY(hipMemcpy(c->doc_blocks, blocks.data(), sizeof(uint4) * blocks.size(), hipMemcpyHostToDevice));
        if ((int64_t)ne.size() != D) {   // some document is empty: ordinals are not document numbers
            SABER_TRY(dev_alloc(c->hooks, &c->ne_doc, ne.size()));
            if (!ne.empty()) HIP_TRY(hipMemcpy(c->ne_doc, ne.data(), sizeof(int32_t) * ne.size(), hipMemcpyHostToDevice));
        }
    } else {
        if (c->z16) SABER_TRY(dev_alloc(c->hooks, (uint16_t **)&c->z, (size_t)T)); else SABER_TRY(dev_alloc(c->hooks, (int32_t **)&c->z, (size_t)T));
        SABER_TRY(dev_alloc(c->hooks, &c->tok_doc, (size_t)T)); SABER_TRY(dev_alloc(c->hooks, &c->tok_t, (size_t)T));
    }
    SABER_TRY(dev_alloc(c->hooks, &c->tiles, h_tiles.size())); SABER_TRY(dev_alloc(c->hooks, &c->docrec, (size_t)D));
    SABER_TRY(dev_alloc(c->hooks, &c->cd_ent, (size_t)c->cd_cap)); SABER_TRY(dev_alloc(c->hooks, &c->doc_ptr, (size_t)D + 1));
    SABER_TRY(dev_alloc(c->hooks, &c->short_docs, h_short.size())); SABER_TRY(dev_alloc(c->hooks, &c->long_docs, h_long.size()));
    if (par) {
        // borrowed from the model: everything the sampler reads about words
        c->phi = par->phi; c->l3 = par->l3; c->l3_64 = par->l3_64; c->sumphi = par->sumphi;
        c->wrec = par->wrec; c->lw_ent = par->lw_ent; c->lw_phi = par->lw_phi;
    } else {
    SABER_TRY(dev_alloc(c->hooks, &c->cwk, vk)); SABER_TRY(dev_alloc(c->hooks, &c->ck, (size_t)K)); SABER_TRY(dev_alloc(c->hooks, &c->denom, (size_t)K));
    SABER_TRY(dev_alloc(c->hooks, &c->phi, vk)); SABER_TRY(dev_alloc(c->hooks, &c->l3_64, ((size_t)V + 1) * (size_t)c->n3));
    SABER_TRY(dev_alloc(c->hooks, &c->row_word, h_row_word.size())); SABER_TRY(dev_alloc(c->hooks, &c->light_words, h_light_words.size()));
    SABER_TRY(dev_alloc(c->hooks, &c->light_short, h_light_short.size())); SABER_TRY(dev_alloc(c->hooks, &c->light_long, h_light_long.size()));
    SABER_TRY(dev_alloc(c->hooks, &c->light_tok_ptr, h_light_tok_ptr.size())); SABER_TRY(dev_alloc(c->hooks, &c->wrec, h_wrec.size()));
    SABER_TRY(dev_alloc(c->hooks, &c->lw_ent, (size_t)c->lw_cap)); SABER_TRY(dev_alloc(c->hooks, &c->lw_phi, (size_t)c->lw_cap));
    }
    if (c->z16) SABER_TRY(dev_alloc(c->hooks, (uint16_t **)&c->z_wm, (size_t)T)); else SABER_TRY(dev_alloc(c->hooks, (int32_t **)&c->z_wm, (size_t)T));
    if (!par) {
    SABER_TRY(dev_alloc(c->hooks, &c->vz_items, h_vz_items.size()));
    if (!h_vz_items.empty())
        HIP_TRY(hipMemcpy(c->vz_items, h_vz_items.data(), sizeof(VzItem) * h_vz_items.size(), hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(c->row_word, h_row_word.data(), sizeof(int32_t) * h_row_word.size(), hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(c->light_tok_ptr, h_light_tok_ptr.data(), sizeof(int64_t) * h_light_tok_ptr.size(), hipMemcpyHostToDevice));
    }
    if (c->V_light && !par) {
        HIP_TRY(hipMemcpy(c->light_words, h_light_words.data(), sizeof(int32_t) * h_light_words.size(), hipMemcpyHostToDevice));
        HIP_TRY(hipMemcpy(c->wrec, h_wrec.data(), sizeof(uint2) * h_wrec.size(), hipMemcpyHostToDevice));
        if (!h_light_short.empty()) HIP_TRY(hipMemcpy(c->light_short, h_light_short.data(), sizeof(int32_t) * h_light_short.size(), hipMemcpyHostToDevice));
        if (!h_light_long.empty()) HIP_TRY(hipMemcpy(c->light_long, h_light_long.data(), sizeof(int32_t) * h_light_long.size(), hipMemcpyHostToDevice));
    }
    SABER_TRY(dev_alloc(c->hooks, &c->doc_words, (size_t)D));
    if (c->opt.ablation & 1) {
        SABER_TRY(dev_alloc(c->hooks, &c->word_ids_d, (size_t)T)); SABER_TRY(dev_alloc(c->hooks, &c->word_row_d, (size_t)V));
        if (T) HIP_TRY(hipMemcpy(c->word_ids_d, word_ids, sizeof(int32_t) * (size_t)T, hipMemcpyHostToDevice));
        HIP_TRY(hipMemcpy(c->word_row_d, c->h_word_row.data(), sizeof(int32_t) * (size_t)V, hipMemcpyHostToDevice));
    }
    if (c->opt.ablation & 4)
        SABER_TRY(dev_alloc(c->hooks, &c->alias_table, (size_t)std::max(c->V_dense, 1) * (size_t)K));
    if (c->opt.ablation & 2) {
        unsigned dbits = 1; while (dbits < 32 && (1ll << dbits) < std::max<int64_t>(D, 1)) dbits++;
        c->sort_end_bit = c->topic_bits + dbits;
        SABER_TRY(dev_alloc(c->hooks, &c->sort_keys, (size_t)T)); SABER_TRY(dev_alloc(c->hooks, &c->sort_keys_out, (size_t)T));
        SABER_TRY(dev_alloc(c->hooks, &c->sort_rank, (size_t)T));
        size_t bytes = 0;
        HIP_TRY(rocprim::radix_sort_keys(nullptr, bytes, c->sort_keys, c->sort_keys_out, (size_t)std::max<int64_t>(T, 1), 0u,
                                         c->sort_end_bit, c->stream));
        c->sort_tmp_bytes = std::max<size_t>(bytes, 1);
        SABER_TRY(hook_alloc(c->hooks, &c->sort_tmp, c->sort_tmp_bytes));
    }
    if (!par) { SABER_TRY(dev_alloc(c->hooks, &c->l3, ((size_t)V + 1) * (size_t)c->n3pad)); SABER_TRY(dev_alloc(c->hooks, &c->sumphi, (size_t)V + 1)); }
    SABER_TRY(dev_alloc(c->hooks, &c->counters, (size_t)kMaxTimedIters * kCtr));
    SABER_TRY(dev_alloc(c->hooks, &c->dense_slots, (size_t)kMaxTimedIters * kDenseSlots));
    SABER_TRY(dev_alloc(c->hooks, &c->ll_partial, (size_t)std::max<int64_t>(c->max_chunk_tiles, 1) + kLlTail));
    if (T && !c->n_slots) {
        HIP_TRY(hipMemcpy(c->tok_doc, h_tok_doc, sizeof(int32_t) * (size_t)T, hipMemcpyHostToDevice));
        HIP_TRY(hipMemcpy(c->tok_t, h_tok_t, sizeof(uint32_t) * (size_t)T, hipMemcpyHostToDevice));
    }
    if (!h_tiles.empty()) HIP_TRY(hipMemcpy(c->tiles, h_tiles.data(), sizeof(Tile) * h_tiles.size(), hipMemcpyHostToDevice));
    if (D) HIP_TRY(hipMemcpy(c->docrec, h_rec.data(), sizeof(uint2) * (size_t)D, hipMemcpyHostToDevice));
    if (D) HIP_TRY(hipMemcpy(c->doc_words, h_doc_words.data(), sizeof(uint32_t) * (size_t)D, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(c->doc_ptr, doc_ptr, sizeof(int64_t) * ((size_t)D + 1), hipMemcpyHostToDevice));
    if (!h_short.empty()) HIP_TRY(hipMemcpy(c->short_docs, h_short.data(), sizeof(int32_t) * h_short.size(), hipMemcpyHostToDevice));
    if (!h_long.empty()) HIP_TRY(hipMemcpy(c->long_docs, h_long.data(), sizeof(int32_t) * h_long.size(), hipMemcpyHostToDevice));
    if (!par) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(grid_for((int64_t)vk, 256, 8192)), dim3(256), 0, c->stream, (uint32_t *)c->cwk, 0u, vk);
        HIP_TRY(hipGetLastError());
    }
    c->stats.tokens = T; c->stats.tiles = c->total_tiles; c->stats.chunks = (int64_t)c->chunks.size();
    if (c->no_state) { HIP_TRY(hipStreamSynchronize(c->stream)); return SABER_OK; }

    // ---- iteration 0: Philox assignment, then the M-step ----
    if (!c->n_slots) SABER_TRY(launch_init_z(c, c->z, 0, 0, T));   // with host streaming: chunk by chunk, in full_mstep
    SABER_TRY(full_mstep(c));
    if (par) return SABER_OK;
    SABER_TRY(refresh_workload_stats(c));
    c->stats.words_present = 0;
    for (const Chunk &ch : c->chunks) c->stats.words_present += ch.words_present;
    c->stats.light_tokens = c->T_light;
    return SABER_OK;
}

static int static_scratch_init(int device);

// saber_init_ex, or with `parent` a context for held-out documents that borrows the parent's model
static int create_ctx(saber_ctx **out, const int64_t *doc_ptr, const int32_t *word_ids, int64_t D, int32_t V,
                      int32_t K, float alpha, float beta, uint64_t seed, const saber_options *opt_in,
                      const saber_ctx *parent, bool no_state) {
    if (out) *out = nullptr;
    if (!out || !doc_ptr) return fail(SABER_EINVAL, "saber_init: null argument");
    if (D < 0 || V < 1 || K < 1) return fail(SABER_EINVAL, "saber_init: need D >= 0, V >= 1, K >= 1");
    if (!(alpha > 0.f) || !(beta > 0.f) || !std::isfinite(alpha) || !std::isfinite(beta))
        return fail(SABER_EINVAL, "saber_init: alpha and beta must be positive and finite");
    if (K > 262144) return fail(SABER_ERANGE, "saber_init: K = %d exceeds 262144 (three tree levels of width 64)", K);
    if (D > 0x7fffffffll) return fail(SABER_ERANGE, "saber_init: D exceeds 2^31 - 1");
    if (doc_ptr[0] != 0) return fail(SABER_EINVAL, "saber_init: doc_ptr[0] must be 0");
    int64_t maxlen = 0;
    for (int64_t d = 0; d < D; d++) {
        if (doc_ptr[d + 1] < doc_ptr[d]) return fail(SABER_EINVAL, "saber_init: doc_ptr decreases at document %lld", (long long)d);
        maxlen = std::max(maxlen, doc_ptr[d + 1] - doc_ptr[d]);
    }
    const int64_t T = doc_ptr[D];
    if (T >= (1ll << 40)) return fail(SABER_ERANGE, "saber_init: T = %lld tokens exceeds 2^40", (long long)T);
    if (T > 0 && !word_ids) return fail(SABER_EINVAL, "saber_init: word_ids is null");
    for (int64_t t = 0; t < T; t++)
        if (word_ids[t] < 0 || word_ids[t] >= V)
            return fail(SABER_EINVAL, "saber_init: word id %d at token %lld is outside [0,%d)", word_ids[t], (long long)t, V);
    uint32_t bits = 1; while ((1u << bits) < (uint32_t)K) bits++;
    bool b16 = K <= 65536 && maxlen < 65536;   // the common case: topic and count both fit 16 bits
    if (b16) bits = 16;
    if (parent) { b16 = parent->b16; bits = parent->topic_bits; }   // the model's sparse rows of B fix the packing
    if (maxlen >= (1ll << (32 - bits)))
        return fail(SABER_ERANGE, "saber_init: longest document (%lld tokens) does not fit the %u count bits left by K = %d",
                    (long long)maxlen, 32 - bits, K);

    saber_options opt; saber_options_default(&opt);
    if (opt_in) {
        if (opt_in->n_chunks > 0) opt.n_chunks = opt_in->n_chunks;
        if (opt_in->block_threads > 0) opt.block_threads = opt_in->block_threads;
        if (opt_in->tile_tokens > 0) opt.tile_tokens = opt_in->tile_tokens;
        if (opt_in->long_doc_tokens > 0) opt.long_doc_tokens = opt_in->long_doc_tokens;
        if (opt_in->dz_lds_entries > 0) opt.dz_lds_entries = opt_in->dz_lds_entries;
        if (opt_in->stage_min_tokens > 0) opt.stage_min_tokens = opt_in->stage_min_tokens;
        if (opt_in->light_block_threads > 0) opt.light_block_threads = opt_in->light_block_threads;
        opt.light_word_tokens = opt_in->light_word_tokens;
        opt.stream_workers = opt_in->stream_workers;
        opt.ablation = opt_in->ablation;
        opt.device_mem_limit_mb = opt_in->device_mem_limit_mb;
        if (opt_in->quarter_row_entries != 0) opt.quarter_row_entries = std::max(0, opt_in->quarter_row_entries);
        if (opt_in->half_row_entries != 0) opt.half_row_entries = std::max(0, opt_in->half_row_entries);
        opt.stage_phi = opt_in->stage_phi; opt.profile = opt_in->profile;
        if (opt_in->stage_phi < 0) opt.stage_phi = 1;
    }
    if (opt.block_threads <= 0) opt.block_threads = 256;   // replaced below, once the LDS footprint is known
    if (opt.block_threads % 64 || opt.block_threads < 64 || opt.block_threads > 1024)
        return fail(SABER_EINVAL, "saber_init: block_threads must be a multiple of 64 in [64,1024]");
    if (opt.light_block_threads > 0 && (opt.light_block_threads % 64 || opt.light_block_threads > 1024))
        return fail(SABER_EINVAL, "saber_init: light_block_threads must be a multiple of 64 in [64,1024]");
    if (opt.stage_min_tokens <= 0) opt.stage_min_tokens = 1;
    if (opt.stream_workers < -1 || opt.stream_workers > kMaxSlots)
        return fail(SABER_EINVAL, "saber_init: stream_workers must be in [-1,%d]", kMaxSlots);
    if (parent) { opt.stream_workers = 0; opt.ablation = 0; }   // held-out documents are few: always resident, regular kernels
    if (opt.ablation < 0 || opt.ablation > 7 || (opt.ablation & 5) == 5)
        return fail(SABER_EINVAL, "saber_init: ablation must be in [0,7], and document order (bit 0) excludes alias tables (bit 2)");
    if (opt.ablation && opt.stream_workers) return fail(SABER_EINVAL, "saber_init: the ablation variants need stream_workers = 0");
    if (opt.ablation & 5) opt.light_word_tokens = -1;   // document order gathers Bhat from dense rows; alias tables are built from them
    if ((opt.ablation & 4) && alias_lds_bytes(K) > 159 * 1024)
        return fail(SABER_ERANGE, "saber_init: the alias-table variant needs 12 K bytes of LDS per workgroup, K = %d is beyond 13,500", K);
    if (opt.light_word_tokens == 0) opt.light_word_tokens = std::max(1, K / 2);   // < 0 keeps every word dense
    // automatic: chunks of about 80 M tokens (T / 80 M, rounded to the nearest whole number).  The sampling pass of a
    // chunk reads every row of A of the chunk once per word of the document; at 0.4 to 0.7 non-zeros per token these rows
    // (4 bytes per entry) then fit the 256 MB Infinity Cache, and a corpus of several hundred million tokens samples
    // 20 % faster than in one chunk.  (Every chunk stages every word's Bhat row again: a 100 M-token corpus is fastest
    // in one chunk, and below 60 M tokens per chunk a large one slows down again.)
    if (opt.n_chunks <= 0) opt.n_chunks = (int32_t)std::max<int64_t>(1, (T + (40ll << 20)) / (80ll << 20));
    if (opt.n_chunks > 65536) return fail(SABER_EINVAL, "saber_init: n_chunks too large");
    if (opt.quarter_row_entries > 64 || opt.half_row_entries > 128)
        return fail(SABER_EINVAL, "saber_init: quarter_row_entries must not exceed 64 and half_row_entries 128");
    if (opt.dz_lds_entries > 12288) return fail(SABER_EINVAL, "saber_init: dz_lds_entries must not exceed 12288");
    // token positions inside a chunk are 32-bit: keep every chunk below 2^30 tokens (documents are far shorter)
    opt.n_chunks = (int32_t)std::max<int64_t>(opt.n_chunks, (T >> 30) + 1);
    if ((int64_t)opt.n_chunks > std::max<int64_t>(D, 1)) opt.n_chunks = (int32_t)std::max<int64_t>(D, 1);
    // automatic tile size: a heavy word's Bhat row is staged once per tile, so larger tiles stage less; but a tile is
    // the work of one workgroup, and with about a thousand workgroups in flight a tile of chunk / 2560 tokens takes 40 %
    // of the chunk's pass (heavy tiles are launched first; at chunk / 1500 the pass waits for them: + 5 to 20 %).
    // Between 8,192 and 32,768 tokens.
    const int32_t tile_tokens_asked = opt.tile_tokens;
    if (opt.tile_tokens <= 0) {
        const int64_t per_chunk = T / std::max(1, opt.n_chunks);
        opt.tile_tokens = (int32_t)std::min<int64_t>(32768, std::max<int64_t>(8192, (per_chunk / 2560) & ~255ll));
    }

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(SABER_EDEVICE, "saber_init: no HIP device available");

    saber_ctx *c = new (std::nothrow) saber_ctx();
    if (!c) return fail(SABER_ENOMEM, "saber_init: out of host memory");
    c->hooks = parent ? parent->hooks : g_hooks;
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return fail(SABER_EDEVICE, "saber_init: hipGetDevice failed"); }
    { const int rc0 = static_scratch_init(c->device); if (rc0 != SABER_OK) { delete c; return rc0; } }
    c->D = D; c->T = T; c->V = V; c->K = K; c->alpha = alpha; c->beta = beta; c->seed = seed; c->opt = opt; c->tile_tokens_asked = tile_tokens_asked;
    c->parent = parent; c->no_state = no_state;
    c->n_slots = std::max(0, opt.stream_workers);
    c->Kpad = (K + 63) / 64 * 64;
    c->n3 = c->Kpad / 64;
    c->n3pad = (c->n3 + 63) / 64 * 64;
    c->b16 = b16;
    c->nwords = (K + 31) / 32;
    c->topic_bits = bits; c->topic_mask = (1u << bits) - 1u;
    c->z16 = K <= 65536;
    // the word's Bhat row is staged in LDS when it fits a workgroup's share: up to 150 KB of the CU's 160 KB
    int lds_per_cu = 0;
    if (hipDeviceGetAttribute(&lds_per_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, 0) != hipSuccess || lds_per_cu <= 0)
        lds_per_cu = 64 * 1024;
    const size_t stage_limit = std::min<size_t>(150 * 1024, (size_t)lds_per_cu > 10 * 1024 ? (size_t)lds_per_cu - 10 * 1024 : 0);
    c->staged = opt.stage_phi && estep_row_bytes(c) <= std::max<size_t>(stage_limit, 54 * 1024);
    if (opt_in == nullptr || opt_in->block_threads <= 0) {
        // automatic workgroup size: the one that lets a CU hold the most wavefronts given the LDS footprint
        // (LDS is handed out in 512-byte pieces; a CU holds at most 32 wavefronts); ties go to the smaller size
        int lds_cu = 0;
        if (hipDeviceGetAttribute(&lds_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, 0) != hipSuccess || lds_cu <= 0)
            lds_cu = 64 * 1024;
        const size_t need = c->staged ? ((estep_lds_bytes(c, MODE_SAMPLE) + 144 + 511) / 512) * 512 : 512;
        int best = 256, best_waves = 0;
        for (int block : {256, 512, 1024}) {
            const int by_lds = (int)std::min<size_t>(64, (size_t)lds_cu / need), by_waves = 32 / (block / 64);
            const int waves = std::min(by_lds, by_waves) * (block / 64);
            if (waves > best_waves) { best_waves = waves; best = block; }
        }
        c->opt.block_threads = best;
    }
    if (c->opt.light_block_threads <= 0) c->opt.light_block_threads = c->opt.block_threads;
    c->vbeta = (float)V * beta;
    c->max_doc_len = maxlen;
    int rc;
    if ((rc = check_estep_lds_layout()) != SABER_OK) { delete c; return rc; }
    try { rc = build(c, doc_ptr, word_ids); }
    catch (const std::bad_alloc &) { rc = fail(SABER_ENOMEM, "saber_init: out of host memory"); }
    if (rc != SABER_OK) { saber_free(c); return rc; }
    *out = c;
    return SABER_OK;
}

extern "C" int saber_init_ex(saber_ctx **out, const int64_t *doc_ptr, const int32_t *word_ids, int64_t D, int32_t V,
                             int32_t K, float alpha, float beta, uint64_t seed, const saber_options *opt_in) {
    return create_ctx(out, doc_ptr, word_ids, D, V, K, alpha, beta, seed, opt_in, nullptr, false);
}

extern "C" int saber_init(saber_ctx **out, const int64_t *doc_ptr, const int32_t *word_ids, int64_t D, int32_t V,
                          int32_t K, float alpha, float beta, uint64_t seed) {
    return saber_init_ex(out, doc_ptr, word_ids, D, V, K, alpha, beta, seed, nullptr);
}

// ------------------------------------------------------------------------------------------------
// saber_iterate
// ------------------------------------------------------------------------------------------------
extern "C" int saber_iterate(saber_ctx *c, int32_t n) {
    if (!c) return fail(SABER_EINVAL, "saber_iterate: null context");
    if (n < 0) return fail(SABER_EINVAL, "saber_iterate: n must be >= 0");
    const bool prof = c->opt.profile != 0;
    int32_t done = 0;
    while (done < n) {
        const int batch = std::min<int32_t>(n - done, kMaxTimedIters);
        // per-iteration device counters: {dense-branch tokens, nnz(A), sum_d K_d L_d}
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, c->stream, (uint32_t *)c->counters, 0u,
                           (size_t)kMaxTimedIters * kCtr * 2);
        HIP_TRY(hipGetLastError());
        hipLaunchKernelGGL(fill_u32_kernel, dim3(grid_for((int64_t)batch * kDenseSlots * 2, 256)), dim3(256), 0, c->stream,
                           (uint32_t *)c->dense_slots, 0u, (size_t)batch * kDenseSlots * 2);
        HIP_TRY(hipGetLastError());
        for (int b = 0; b < batch; b++) {
            hipEvent_t *ev = c->ev + (size_t)b * EV_PER_ITER;
            c->iter++;
            if (prof) HIP_TRY(hipEventRecord(ev[EV_BEGIN], c->stream));
            // E-step: z <- Sample(A_d, Bhat_v, Q_v, T_v) for every token, written in document order and in word order
            if (c->opt.ablation & 1) SABER_TRY(launch_estep_docmajor(c, c->dense_slots + (size_t)kDenseSlots * b));
            else for (const Chunk &ch : c->chunks) {
                int s = -1;
                if (c->n_slots) SABER_TRY(stream_acquire(c, ch, &s));
                EStepParams p = make_params(c, ch, s);
                p.n_dense = c->dense_slots + (size_t)kDenseSlots * b;
                SABER_TRY(launch_estep<MODE_SAMPLE>(c, ch, p));
                if (c->n_slots) {
                    // the chunk's rows of A are rebuilt while its new assignments are in the buffer (the sampling
                    // of later chunks reads other documents' rows only); after that only z_wm keeps them
                    SABER_TRY(launch_count_dz_chunk(c, ch, s));
                    SABER_TRY(stream_release(c, s));
                }
            }
            if (prof) HIP_TRY(hipEventRecord(ev[EV_SAMPLE], c->stream));
            // M-step
            if (!c->n_slots) SABER_TRY(launch_count_dz(c));
            if (prof) HIP_TRY(hipEventRecord(ev[EV_DZ], c->stream));
            SABER_TRY(launch_topic_totals(c));
            if (prof) HIP_TRY(hipEventRecord(ev[EV_CK], c->stream));
            SABER_TRY(launch_count_vz(c));
            SABER_TRY(launch_phi(c));
            SABER_TRY(launch_light_words(c));
            if (prof) HIP_TRY(hipEventRecord(ev[EV_PHI], c->stream));
            hipLaunchKernelGGL(sum_slots_kernel, dim3(1), dim3(256), 0, c->stream, c->dense_slots + (size_t)kDenseSlots * b,
                               kDenseSlots, c->counters + kCtr * b);
            HIP_TRY(hipGetLastError());
            SABER_TRY(launch_row_stats(c, c->counters + kCtr * b + 1));
        }
        SABER_TRY(sync_all(c));
        unsigned long long h[kMaxTimedIters * kCtr];
        HIP_TRY(hipMemcpy(h, c->counters, sizeof(h), hipMemcpyDeviceToHost));
        for (int b = 0; b < batch; b++) {
            // the E-step of this iteration read the rows counted at the end of the previous one
            c->stats.sum_tokens += c->T;
            c->stats.sum_tokens_dense += (int64_t)h[kCtr * b];
            c->stats.sum_row_entries += c->stats.next_row_entries;
            c->stats.sum_row_fetch += c->stats.next_row_fetch;
            c->stats.sum_light_entries += c->stats.next_light_entries;
            c->stats.nnz_cd = (int64_t)h[kCtr * b + 1];
            c->stats.next_row_entries = (int64_t)h[kCtr * b + 2];
            c->stats.next_row_fetch = (int64_t)h[kCtr * b + 3];
            c->stats.next_light_entries = (int64_t)h[kCtr * b + 4];
            if (prof) {
                hipEvent_t *ev = c->ev + (size_t)b * EV_PER_ITER;
                float ms[4], tot;
                for (int s = 0; s < 4; s++) HIP_TRY(hipEventElapsedTime(&ms[s], ev[s], ev[s + 1]));
                HIP_TRY(hipEventElapsedTime(&tot, ev[EV_BEGIN], ev[EV_PHI]));
                c->stats.ms_sample += ms[0]; c->stats.ms_count_dz += ms[1]; c->stats.ms_ck += ms[2];
                c->stats.ms_phi += ms[3]; c->stats.ms_total += tot;
                c->stats.sample_launches += (int64_t)c->chunks.size();
            }
            c->stats.iterations++;
        }
        done += batch;
    }
    return SABER_OK;
}

// ------------------------------------------------------------------------------------------------
// outputs
// ------------------------------------------------------------------------------------------------
extern "C" int saber_counts_nnz(saber_ctx *c, int64_t *nnz) {
    if (!c || !nnz) return fail(SABER_EINVAL, "saber_counts_nnz: null argument");
    try {
        std::vector<uint2> rec((size_t)c->D);
        if (c->D) HIP_TRY(hipMemcpy(rec.data(), c->docrec, sizeof(uint2) * (size_t)c->D, hipMemcpyDeviceToHost));
        int64_t s = 0; for (auto &r : rec) s += r.y;
        *nnz = s;
    } catch (const std::bad_alloc &) { return fail(SABER_ENOMEM, "saber_counts_nnz: out of host memory"); }
    return SABER_OK;
}

extern "C" int saber_counts(saber_ctx *c, int64_t *cd_row_ptr, int32_t *cd_topic, int32_t *cd_count, int32_t *cwk,
                            int64_t *ck) {
    if (!c) return fail(SABER_EINVAL, "saber_counts: null context");
    if ((cd_topic || cd_count) && !cd_row_ptr) return fail(SABER_EINVAL, "saber_counts: cd_topic/cd_count need cd_row_ptr");
    try {
        if (cd_row_ptr) {
            std::vector<uint2> rec((size_t)c->D);
            if (c->D) HIP_TRY(hipMemcpy(rec.data(), c->docrec, sizeof(uint2) * (size_t)c->D, hipMemcpyDeviceToHost));
            cd_row_ptr[0] = 0;
            for (int64_t d = 0; d < c->D; d++) cd_row_ptr[d + 1] = cd_row_ptr[d] + rec[(size_t)d].y;
            if (cd_topic || cd_count) {
                // unpack the device rows slab by slab (format conversion only)
                const int64_t slab_docs = 65536;
                std::vector<uint32_t> buf;
                for (int64_t d0 = 0; d0 < c->D; d0 += slab_docs) {
                    const int64_t d1 = std::min(c->D, d0 + slab_docs);
                    const int64_t e0 = (int64_t)rec[(size_t)d0].x * 32;
                    const int64_t e1 = d1 < c->D ? (int64_t)rec[(size_t)d1].x * 32 : c->cd_cap;
                    buf.resize((size_t)std::max<int64_t>(e1 - e0, 1));
                    if (e1 > e0) HIP_TRY(hipMemcpy(buf.data(), c->cd_ent + e0, sizeof(uint32_t) * (size_t)(e1 - e0), hipMemcpyDeviceToHost));
                    for (int64_t d = d0; d < d1; d++) {
                        const uint32_t *row = buf.data() + ((int64_t)rec[(size_t)d].x * 32 - e0);
                        int64_t o = cd_row_ptr[d];
                        for (uint32_t j = 0; j < rec[(size_t)d].y; j++, o++) {
                            if (cd_topic) cd_topic[o] = (int32_t)(row[j] & c->topic_mask);
                            if (cd_count) cd_count[o] = (int32_t)(row[j] >> c->topic_bits);
                        }
                    }
                }
            }
        }
        if (cwk) {
            // dense rows: B is consumed (and cleared) by the Bhat kernel; rebuild it from z for export
            SABER_TRY(launch_count_vz(c));
            HIP_TRY(hipStreamSynchronize(c->stream));
            const int64_t slab = 2048;   // rows per host staging buffer
            std::vector<int32_t> buf((size_t)slab * (size_t)c->Kpad);
            std::vector<int32_t> row_word((size_t)c->V_dense + 1);
            HIP_TRY(hipMemcpy(row_word.data(), c->row_word, sizeof(int32_t) * row_word.size(), hipMemcpyDeviceToHost));
            for (int64_t r0 = 0; r0 < c->V_dense; r0 += slab) {
                const int64_t r1 = std::min<int64_t>(c->V_dense, r0 + slab);
                HIP_TRY(hipMemcpy(buf.data(), c->cwk + (size_t)r0 * (size_t)c->Kpad,
                                  sizeof(int32_t) * (size_t)(r1 - r0) * (size_t)c->Kpad, hipMemcpyDeviceToHost));
                for (int64_t r = r0; r < r1; r++)
                    memcpy(cwk + (size_t)row_word[(size_t)r] * (size_t)c->K, buf.data() + (size_t)(r - r0) * (size_t)c->Kpad,
                           sizeof(int32_t) * (size_t)c->K);
            }
            const size_t vk = (size_t)c->V_dense * (size_t)c->Kpad;
            hipLaunchKernelGGL(fill_u32_kernel, dim3(grid_for((int64_t)vk, 256, 8192)), dim3(256), 0, c->stream,
                               (uint32_t *)c->cwk, 0u, vk);
            HIP_TRY(hipGetLastError());
            HIP_TRY(hipStreamSynchronize(c->stream));
            // light words: unpack the sparse rows (format conversion only)
            if (c->V_light) {
                std::vector<uint2> wrec((size_t)c->V_light);
                std::vector<int32_t> lwords((size_t)c->V_light);
                HIP_TRY(hipMemcpy(wrec.data(), c->wrec, sizeof(uint2) * wrec.size(), hipMemcpyDeviceToHost));
                HIP_TRY(hipMemcpy(lwords.data(), c->light_words, sizeof(int32_t) * lwords.size(), hipMemcpyDeviceToHost));
                std::vector<uint32_t> ent((size_t)std::max<int64_t>(c->lw_cap, 1));
                if (c->lw_cap) HIP_TRY(hipMemcpy(ent.data(), c->lw_ent, sizeof(uint32_t) * (size_t)c->lw_cap, hipMemcpyDeviceToHost));
                for (int32_t li = 0; li < c->V_light; li++) {
                    int32_t *row = cwk + (size_t)lwords[(size_t)li] * (size_t)c->K;
                    memset(row, 0, sizeof(int32_t) * (size_t)c->K);
                    const uint32_t *e = ent.data() + (size_t)wrec[(size_t)li].x * 32u;
                    for (uint32_t j = 0; j < wrec[(size_t)li].y; j++) row[e[j] & c->topic_mask] = (int32_t)(e[j] >> c->topic_bits);
                }
            }
        }
        if (ck) {
            std::vector<unsigned long long> h((size_t)c->K);
            HIP_TRY(hipMemcpy(h.data(), c->ck, sizeof(unsigned long long) * (size_t)c->K, hipMemcpyDeviceToHost));
            for (int32_t k = 0; k < c->K; k++) ck[k] = (int64_t)h[(size_t)k];
        }
    } catch (const std::bad_alloc &) { return fail(SABER_ENOMEM, "saber_counts: out of host memory"); }
    return SABER_OK;
}

// *result (device memory) = [ sum over the tokens of c of ln(S_t + Q_w)  -  sum_d w_d ln(len_d + K alpha) ] / T on the device, all
// sums in binary64 and in a fixed order.  `theta` holds the rows of A that S is formed with (c itself for the training
// log-likelihood; the observed part of the documents for the holdout score, whose document lengths then also give
// len_d while w_d counts the scored tokens).  Everything is queued on c's stream; nothing is waited for.
static int launch_loglik(saber_ctx *c, const saber_ctx *theta, const LlScratch &ws, double *result) {
    bool first = true;
    for (const Chunk &ch : c->chunks) {
        if (ch.ntiles == 0) continue;
        int s = -1;
        if (c->n_slots) SABER_TRY(stream_acquire(c, ch, &s));
        EStepParams p = make_params(c, ch, s);
        // theta's documents are c's documents (same D, same chunks: the held-out contexts have one chunk each)
        set_rows(p, theta, theta->chunks[(size_t)(&ch - c->chunks.data())]);
        p.out_ll = ws.tile_part;
        SABER_TRY(launch_estep<MODE_LOGLIK>(c, ch, p));
        if (c->n_slots) SABER_TRY(stream_release(c, s));
        hipLaunchKernelGGL(reduce_partials_kernel, dim3(kReduceBlocks), dim3(kReduceThreads), 0, c->stream, ws.tile_part,
                           ch.ntiles, ws.block_part);
        HIP_TRY(hipGetLastError());
        hipLaunchKernelGGL(reduce_final_kernel, dim3(1), dim3(kReduceThreads), 0, c->stream, ws.block_part, ws.acc, first ? 0 : 1);
        HIP_TRY(hipGetLastError());
        first = false;
    }
    hipLaunchKernelGGL(doc_norm_kernel, dim3(kReduceBlocks), dim3(kReduceThreads), 0, c->stream, c->doc_ptr, theta->doc_ptr,
                       c->D, (double)c->K * (double)c->alpha, ws.block_part);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(reduce_final_kernel, dim3(1), dim3(kReduceThreads), 0, c->stream, ws.block_part, ws.norm, 0);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(loglik_finish_kernel, dim3(1), dim3(64), 0, c->stream, ws.acc, ws.norm, (double)c->T, result);
    HIP_TRY(hipGetLastError());
    return SABER_OK;
}

extern "C" int saber_loglik(saber_ctx *c, double *out) {
    if (!c || !out) return fail(SABER_EINVAL, "saber_loglik: null argument");
    if (c->T == 0) { *out = 0.0; return SABER_OK; }
    const LlScratch ws = ll_scratch(c->ll_partial, (size_t)std::max<int64_t>(c->max_chunk_tiles, 1));
    SABER_TRY(launch_loglik(c, c, ws, ws.result));
    SABER_TRY(sync_all(c));
    HIP_TRY(hipMemcpy(out, ws.result, sizeof(double), hipMemcpyDeviceToHost));
    return SABER_OK;
}

// ---- the same reduction for callers that must not allocate ----
// The work space is a file-scope device array instead of the context's allocation.  Every device has its own copy of
// the array at its own address, looked up once per device (saber_init does it, with that device current); host code
// uses that address only, never the array's name.
constexpr size_t kStaticLlTiles = (size_t)1 << 20;   // per-tile sums of one chunk: 8 MB
constexpr int kMaxDevices = 64;
static __device__ __align__(256) double g_ll_static[kStaticLlTiles + kLlTail];
static double *g_ll_static_ptr[kMaxDevices] = {};

static int static_scratch_init(int device) {
    if (device < 0 || device >= kMaxDevices) return fail(SABER_ERANGE, "device %d is beyond the %d devices the library keeps work space for", device, kMaxDevices);
    if (g_ll_static_ptr[device]) return SABER_OK;
    double *ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(g_ll_static)));
    if (!ptr) return fail(SABER_EDEVICE, "hipGetSymbolAddress returned no address for the static work space");
    g_ll_static_ptr[device] = ptr;
    return SABER_OK;
}

extern "C" int saber_loglik_static(saber_ctx *c, double *d_result) {
    if (!c || !d_result) return fail(SABER_EINVAL, "saber_loglik_static: null argument");
    if ((size_t)c->max_chunk_tiles > kStaticLlTiles)
        return fail(SABER_ERANGE, "saber_loglik_static: a chunk of %lld sampling workgroups exceeds the static work space of %zu "
                    "(use saber_loglik, or more chunks)", (long long)c->max_chunk_tiles, kStaticLlTiles);
    double *base = (c->device >= 0 && c->device < kMaxDevices) ? g_ll_static_ptr[c->device] : nullptr;
    if (!base) return fail(SABER_ESTATE, "saber_loglik_static: no static work space on device %d", c->device);
    if (c->T == 0) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, c->stream, reinterpret_cast<uint32_t *>(d_result), 0u, (size_t)2);
        HIP_TRY(hipGetLastError());
    } else {
        SABER_TRY(launch_loglik(c, c, ll_scratch(base, kStaticLlTiles), d_result));
    }
    return sync_all(c);
}

// ------------------------------------------------------------------------------------------------
// holdout log-likelihood (document completion on held-out documents, model frozen)
// ------------------------------------------------------------------------------------------------
// n E-steps + CountByDZ on a context that borrows a model: Alg. 1 restricted to A
static int foldin_iterate(saber_ctx *c, int32_t n) {
    for (int32_t i = 0; i < n; i++) {
        c->iter++;
        hipLaunchKernelGGL(fill_u32_kernel, dim3(grid_for((int64_t)kDenseSlots * 2, 256)), dim3(256), 0, c->stream,
                           (uint32_t *)c->dense_slots, 0u, (size_t)kDenseSlots * 2);
        HIP_TRY(hipGetLastError());
        for (const Chunk &ch : c->chunks) {
            EStepParams p = make_params(c, ch);
            p.n_dense = c->dense_slots;
            SABER_TRY(launch_estep<MODE_SAMPLE>(c, ch, p));
        }
        SABER_TRY(launch_count_dz(c));
    }
    HIP_TRY(hipStreamSynchronize(c->stream));
    return SABER_OK;
}

extern "C" int saber_holdout_loglik(saber_ctx *m, const int64_t *doc_ptr, const int32_t *word_ids,
                                    const uint8_t *observed, int64_t D, int32_t n_foldin, uint64_t seed,
                                    const int32_t *z_init, int32_t *z_out, double *loglik, int64_t *n_scored) {
    if (!m || !doc_ptr || !loglik || !n_scored || D < 0 || n_foldin < 0)
        return fail(SABER_EINVAL, "saber_holdout_loglik: bad argument");
    if (m->parent) return fail(SABER_EINVAL, "saber_holdout_loglik: the model must be a context made by saber_init");
    if (doc_ptr[0] != 0) return fail(SABER_EINVAL, "saber_holdout_loglik: doc_ptr[0] must be 0");
    for (int64_t d = 0; d < D; d++)
        if (doc_ptr[d + 1] < doc_ptr[d]) return fail(SABER_EINVAL, "saber_holdout_loglik: doc_ptr decreases at document %lld", (long long)d);
    const int64_t T = doc_ptr[D];
    if (T > 0 && (!word_ids || !observed)) return fail(SABER_EINVAL, "saber_holdout_loglik: null token arrays");
    saber_ctx *obs = nullptr, *scr = nullptr;
    int rc = SABER_OK;
    try {
        // the observed part and the scored part as two corpora over the same documents
        std::vector<int64_t> optr((size_t)D + 1, 0), sptr((size_t)D + 1, 0);
        std::vector<int32_t> ow, sw;
        ow.reserve((size_t)T / 2 + 1); sw.reserve((size_t)T / 2 + 1);
        for (int64_t d = 0; d < D; d++) {
            for (int64_t t = doc_ptr[d]; t < doc_ptr[d + 1]; t++) (observed[t] ? ow : sw).push_back(word_ids[t]);
            optr[(size_t)d + 1] = (int64_t)ow.size(); sptr[(size_t)d + 1] = (int64_t)sw.size();
        }
        saber_options opt = m->opt;
        opt.profile = 0; opt.n_chunks = 1; opt.tile_tokens = m->tile_tokens_asked;   // (0: sized for these documents)
        rc = create_ctx(&obs, optr.data(), ow.data(), D, m->V, m->K, m->alpha, m->beta, seed, &opt, m, false);
        if (rc == SABER_OK && z_init) rc = saber_set_z(obs, z_init, 0);
        if (rc == SABER_OK) rc = foldin_iterate(obs, n_foldin);
        if (rc == SABER_OK && z_out) rc = saber_get_z(obs, z_out);
        if (rc == SABER_OK) rc = create_ctx(&scr, sptr.data(), sw.data(), D, m->V, m->K, m->alpha, m->beta, seed, &opt, m, true);
        double ll = 0.0;
        if (rc == SABER_OK && scr->T > 0) {
            // theta comes from the observed part: its rows of A, and its document lengths in the normaliser
            const LlScratch ws = ll_scratch(scr->ll_partial, (size_t)std::max<int64_t>(scr->max_chunk_tiles, 1));
            rc = launch_loglik(scr, obs, ws, ws.result);
            if (rc == SABER_OK) {
                hipError_t e = hipStreamSynchronize(scr->stream);
                if (e == hipSuccess) e = hipMemcpy(&ll, ws.result, sizeof(double), hipMemcpyDeviceToHost);
                if (e != hipSuccess) rc = fail(SABER_EDEVICE, "saber_holdout_loglik: %s", hipGetErrorString(e));
            }
        }
        if (rc == SABER_OK) {
            *n_scored = scr->T;
            *loglik = ll;
        }
    } catch (const std::bad_alloc &) { rc = fail(SABER_ENOMEM, "saber_holdout_loglik: out of host memory"); }
    saber_free(scr); saber_free(obs);
    return rc;
}

extern "C" int saber_get_z(saber_ctx *c, int32_t *z) {
    if (!c || !z) return fail(SABER_EINVAL, "saber_get_z: null argument");
    if (c->T == 0) return SABER_OK;
    if (c->n_slots) {   // document order is re-created chunk by chunk from the word-major copy
        try {
            std::vector<uint16_t> stage;
            for (const Chunk &ch : c->chunks) {
                if (ch.ntok == 0) continue;
                int s;
                SABER_TRY(stream_acquire(c, ch, &s));
                if (c->z16)
                    hipLaunchKernelGGL((scatter_zwm_kernel<uint16_t>), dim3((unsigned)ch.ntiles), dim3(256), 0, c->stream,
                                       c->tiles + ch.tile0, c->slot_tok_t[s], (const uint16_t *)c->z_wm, (uint16_t *)c->slot_z[s]);
                else
                    hipLaunchKernelGGL((scatter_zwm_kernel<int32_t>), dim3((unsigned)ch.ntiles), dim3(256), 0, c->stream,
                                       c->tiles + ch.tile0, c->slot_tok_t[s], (const int32_t *)c->z_wm, (int32_t *)c->slot_z[s]);
                HIP_TRY(hipGetLastError());
                SABER_TRY(stream_release(c, s));
                HIP_TRY(hipStreamSynchronize(c->stream));
                if (c->z16) {
                    stage.resize((size_t)ch.ntok);
                    HIP_TRY(hipMemcpy(stage.data(), c->slot_z[s], (size_t)ch.ntok * 2, hipMemcpyDeviceToHost));
                    for (int64_t i = 0; i < ch.ntok; i++) z[ch.t0 + i] = (int32_t)stage[(size_t)i];
                } else {
                    HIP_TRY(hipMemcpy(z + ch.t0, c->slot_z[s], (size_t)ch.ntok * 4, hipMemcpyDeviceToHost));
                }
            }
        } catch (const std::bad_alloc &) { return fail(SABER_ENOMEM, "saber_get_z: out of host memory"); }
        return SABER_OK;
    }
    if (!c->z16) { HIP_TRY(hipMemcpy(z, c->z, sizeof(int32_t) * (size_t)c->T, hipMemcpyDeviceToHost)); return SABER_OK; }
    int32_t *tmp = nullptr;
    SABER_TRY(dev_alloc(c->hooks, &tmp, (size_t)c->T));
    hipLaunchKernelGGL((z_to_i32_kernel<uint16_t>), dim3(grid_for(c->T, 256, 8192)), dim3(256), 0, c->stream,
                       (const uint16_t *)c->z, tmp, c->T);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e == hipSuccess) e = hipMemcpy(z, tmp, sizeof(int32_t) * (size_t)c->T, hipMemcpyDeviceToHost);
    dev_free(c->hooks, tmp);
    if (e != hipSuccess) return fail(SABER_EDEVICE, "saber_get_z: %s", hipGetErrorString(e));
    return SABER_OK;
}

extern "C" int saber_set_z(saber_ctx *c, const int32_t *z, uint32_t iter) {
    if (!c || (!z && c->T)) return fail(SABER_EINVAL, "saber_set_z: null argument");
    for (int64_t t = 0; t < c->T; t++)
        if (z[t] < 0 || z[t] >= c->K) return fail(SABER_EINVAL, "saber_set_z: topic %d at token %lld is outside [0,%d)", z[t], (long long)t, c->K);
    if (c->T && !c->n_slots) {
        int32_t *tmp = nullptr;
        SABER_TRY(dev_alloc(c->hooks, &tmp, (size_t)c->T));
        hipError_t e = hipMemcpy(tmp, z, sizeof(int32_t) * (size_t)c->T, hipMemcpyHostToDevice);
        if (e == hipSuccess) {
            if (c->z16)
                hipLaunchKernelGGL((z_from_i32_kernel<uint16_t>), dim3(grid_for(c->T, 256, 8192)), dim3(256), 0, c->stream, (uint16_t *)c->z, tmp, c->T);
            else
                hipLaunchKernelGGL((z_from_i32_kernel<int32_t>), dim3(grid_for(c->T, 256, 8192)), dim3(256), 0, c->stream, (int32_t *)c->z, tmp, c->T);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
        dev_free(c->hooks, tmp);
        if (e != hipSuccess) return fail(SABER_EDEVICE, "saber_set_z: %s", hipGetErrorString(e));
    }
    c->iter = iter;
    try { SABER_TRY(full_mstep(c, c->n_slots ? z : nullptr)); }
    catch (const std::bad_alloc &) { return fail(SABER_ENOMEM, "saber_set_z: out of host memory"); }
    SABER_TRY(refresh_workload_stats(c));
    return SABER_OK;
}

extern "C" int saber_get_iteration(saber_ctx *c, uint32_t *iter) {
    if (!c || !iter) return fail(SABER_EINVAL, "saber_get_iteration: null argument");
    *iter = c->iter;
    return SABER_OK;
}

extern "C" int saber_token_probs(saber_ctx *c, const int64_t *tok, int64_t m, float *S, float *Q, float *p_sparse) {
    if (!c || (m > 0 && !tok) || m < 0) return fail(SABER_EINVAL, "saber_token_probs: bad argument");
    for (int64_t i = 0; i < m; i++)
        if (tok[i] < 0 || tok[i] >= c->T) return fail(SABER_EINVAL, "saber_token_probs: token index %lld is outside [0,%lld)", (long long)tok[i], (long long)c->T);
    if (m == 0) return SABER_OK;
    // S and Q of every token of a chunk (inspection mode of the sampling kernel), then the requested tokens of that
    // chunk are picked out and S / (S + Q) is formed, all on the device; the work space is sized for one chunk
    int64_t max_tok = 1;
    for (const Chunk &ch : c->chunks) max_tok = std::max(max_tok, ch.ntok);
    float *dS = nullptr, *dQ = nullptr, *g3 = nullptr; int64_t *dtok = nullptr;
    int rc = SABER_OK;
    auto cleanup = [&]() { dev_free(c->hooks, dS); dev_free(c->hooks, dQ); dev_free(c->hooks, g3); dev_free(c->hooks, dtok); };
    if ((rc = dev_alloc(c->hooks, &dS, (size_t)max_tok)) || (rc = dev_alloc(c->hooks, &dQ, (size_t)max_tok)) ||
        (rc = dev_alloc(c->hooks, &g3, 3 * (size_t)m)) || (rc = dev_alloc(c->hooks, &dtok, (size_t)m))) { cleanup(); return rc; }
    hipError_t e = hipMemcpy(dtok, tok, sizeof(int64_t) * (size_t)m, hipMemcpyHostToDevice);
    for (const Chunk &ch : c->chunks) {
        if (e != hipSuccess) break;
        if (ch.ntiles == 0) continue;
        int s = -1;
        if (c->n_slots && (rc = stream_acquire(c, ch, &s))) { cleanup(); return rc; }
        EStepParams p = make_params(c, ch, s);
        p.out_S = dS; p.out_Q = dQ;
        if ((rc = launch_estep<MODE_PROBS>(c, ch, p))) { cleanup(); return rc; }
        if (c->n_slots && (rc = stream_release(c, s))) { cleanup(); return rc; }
        hipLaunchKernelGGL(gather_probs_kernel, dim3(grid_for(m, 256)), dim3(256), 0, c->stream, dS, dQ, dtok, m, ch.t0, ch.ntok,
                           g3, g3 + m, g3 + 2 * m);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e == hipSuccess && S) e = hipMemcpy(S, g3, sizeof(float) * (size_t)m, hipMemcpyDeviceToHost);
    if (e == hipSuccess && Q) e = hipMemcpy(Q, g3 + m, sizeof(float) * (size_t)m, hipMemcpyDeviceToHost);
    if (e == hipSuccess && p_sparse) e = hipMemcpy(p_sparse, g3 + 2 * m, sizeof(float) * (size_t)m, hipMemcpyDeviceToHost);
    cleanup();
    if (e != hipSuccess) return fail(SABER_EDEVICE, "saber_token_probs: %s", hipGetErrorString(e));
    return SABER_OK;
}

extern "C" int saber_get_phi(saber_ctx *c, const int32_t *words, int32_t m, float *phi, float *prefix) {
    if (!c || (m > 0 && !words) || m < 0) return fail(SABER_EINVAL, "saber_get_phi: bad argument");
    for (int32_t i = 0; i < m; i++)
        if (words[i] < 0 || words[i] >= c->V) return fail(SABER_EINVAL, "saber_get_phi: word %d is outside [0,%d)", words[i], c->V);
    if (m == 0) return SABER_OK;
    // assemble the requested Bhat rows on the device: dense rows are copied, light rows are the base vector
    // overwritten at the word's non-zeros; the prefix rows are then rebuilt the way the dense branch does
    float *drows = nullptr, *dout = nullptr; int32_t *dw = nullptr, *dlight = nullptr;
    auto cleanup = [&]() { dev_free(c->hooks, drows); dev_free(c->hooks, dout); dev_free(c->hooks, dw); dev_free(c->hooks, dlight); };
    int rc;
    if ((rc = dev_alloc(c->hooks, &drows, (size_t)m * (size_t)c->K)) || (rc = dev_alloc(c->hooks, &dout, (size_t)m * (size_t)c->K)) ||
        (rc = dev_alloc(c->hooks, &dw, (size_t)m)) || (rc = dev_alloc(c->hooks, &dlight, (size_t)m))) { cleanup(); return rc; }
    hipError_t e = hipMemcpy(dw, words, sizeof(int32_t) * (size_t)m, hipMemcpyHostToDevice);
    for (int32_t i = 0; i < m && e == hipSuccess; i++) {
        const int32_t row = c->h_word_row[(size_t)words[i]];
        if (row >= 0) {
            e = hipMemcpyAsync(drows + (size_t)i * (size_t)c->K, c->phi + (size_t)row * (size_t)c->Kpad,
                               sizeof(float) * (size_t)c->K, hipMemcpyDeviceToDevice, c->stream);
        } else {
            const int32_t li = -row - 1;
            e = hipMemcpyAsync(dlight, &li, sizeof(int32_t), hipMemcpyHostToDevice, c->stream);
            if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
            if (e == hipSuccess) {
                hipLaunchKernelGGL(light_rows_export_kernel, dim3(1), dim3(256), 0, c->stream, dlight, 1, c->wrec, c->lw_ent,
                                   c->lw_phi, c->phi + (size_t)c->V_dense * (size_t)c->Kpad, c->K, c->topic_bits,
                                   drows + (size_t)i * (size_t)c->K, (int32_t *)nullptr);
                e = hipGetLastError();
            }
            if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
        }
    }
    if (e == hipSuccess && prefix) {
        const int64_t items = (int64_t)m * ((c->K + 63) / 64);
        hipLaunchKernelGGL(prefix_export_kernel, dim3((unsigned)items), dim3(64), 0, c->stream, drows, c->l3_64, dw, m,
                           c->K, c->n3, dout);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e == hipSuccess && phi) e = hipMemcpy(phi, drows, sizeof(float) * (size_t)m * (size_t)c->K, hipMemcpyDeviceToHost);
    if (e == hipSuccess && prefix) e = hipMemcpy(prefix, dout, sizeof(float) * (size_t)m * (size_t)c->K, hipMemcpyDeviceToHost);
    cleanup();
    if (e != hipSuccess) return fail(SABER_EDEVICE, "saber_get_phi: %s", hipGetErrorString(e));
    return SABER_OK;
}

// ------------------------------------------------------------------------------------------------
// alias-table construction (measurement aid)
// ------------------------------------------------------------------------------------------------
extern "C" int saber_alias_build_probe(saber_ctx *c, const int32_t *words, int32_t m, float *prob, int32_t *alias,
                                       double *ms_build, int32_t *rows_built) {
    if (!c || m < 0 || (m > 0 && (!words || !prob || !alias)) || !ms_build)
        return fail(SABER_EINVAL, "saber_alias_build_probe: bad argument");
    if (c->parent) return fail(SABER_EINVAL, "saber_alias_build_probe: needs a context made by saber_init");
    std::vector<int32_t> rows((size_t)std::max(m, 1));
    for (int32_t i = 0; i < m; i++) {
        if (words[i] < 0 || words[i] >= c->V) return fail(SABER_EINVAL, "saber_alias_build_probe: word %d is outside [0,%d)", words[i], c->V);
        rows[(size_t)i] = c->h_word_row[(size_t)words[i]];
        if (rows[(size_t)i] < 0) return fail(SABER_EINVAL, "saber_alias_build_probe: word %d keeps a sparse row (no dense Bhat row to build from)", words[i]);
    }
    const int nrows = c->V_dense, K = c->K;
    if (rows_built) *rows_built = nrows;
    *ms_build = 0.0;
    if (nrows == 0) return m ? fail(SABER_EINVAL, "saber_alias_build_probe: no dense rows") : (int)SABER_OK;
    const size_t cells = (size_t)nrows * (size_t)K;
    if (cells * 20 > ((size_t)64 << 30)) return fail(SABER_ERANGE, "saber_alias_build_probe: tables of %zu bytes exceed 64 GB", cells * 20);
    double *scaled = nullptr; int32_t *stack = nullptr, *d_alias = nullptr, *d_rows = nullptr, *o_alias = nullptr;
    float *d_prob = nullptr, *o_prob = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    auto cleanup = [&]() {
        dev_free(c->hooks, scaled); dev_free(c->hooks, stack); dev_free(c->hooks, d_alias); dev_free(c->hooks, d_rows); dev_free(c->hooks, o_alias); dev_free(c->hooks, d_prob); dev_free(c->hooks, o_prob);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    };
    int rc;
    if ((rc = dev_alloc(c->hooks, &scaled, cells)) || (rc = dev_alloc(c->hooks, &stack, cells)) || (rc = dev_alloc(c->hooks, &d_alias, cells)) ||
        (rc = dev_alloc(c->hooks, &d_prob, cells)) || (rc = dev_alloc(c->hooks, &d_rows, (size_t)std::max(m, 1))) ||
        (rc = dev_alloc(c->hooks, &o_prob, (size_t)std::max(m, 1) * (size_t)K)) || (rc = dev_alloc(c->hooks, &o_alias, (size_t)std::max(m, 1) * (size_t)K))) {
        cleanup(); return rc;
    }
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e == hipSuccess) e = hipEventRecord(e0, c->stream);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(alias_build_kernel, dim3((unsigned)((nrows + 255) / 256)), dim3(256), 0, c->stream, c->phi, nrows, K,
                           c->Kpad, scaled, stack, d_prob, d_alias);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(e1, c->stream);
    if (e == hipSuccess && m) e = hipMemcpyAsync(d_rows, rows.data(), sizeof(int32_t) * (size_t)m, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess && m) {
        hipLaunchKernelGGL(alias_export_kernel, dim3(grid_for((int64_t)m * K, 256, 4096)), dim3(256), 0, c->stream, d_rows, m,
                           nrows, K, d_prob, d_alias, o_prob, o_alias);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess && m) e = hipMemcpy(prob, o_prob, sizeof(float) * (size_t)m * (size_t)K, hipMemcpyDeviceToHost);
    if (e == hipSuccess && m) e = hipMemcpy(alias, o_alias, sizeof(int32_t) * (size_t)m * (size_t)K, hipMemcpyDeviceToHost);
    cleanup();
    if (e != hipSuccess) return fail(SABER_EDEVICE, "saber_alias_build_probe: %s", hipGetErrorString(e));
    *ms_build = (double)ms;
    return SABER_OK;
}

extern "C" int saber_get_alias(saber_ctx *c, const int32_t *words, int32_t m, float *prob, int32_t *alias) {
    if (!c || m < 0 || (m > 0 && (!words || !prob || !alias))) return fail(SABER_EINVAL, "saber_get_alias: bad argument");
    if (!c->alias_table) return fail(SABER_ESTATE, "saber_get_alias: the context keeps no alias tables (saber_options.ablation bit 2)");
    try {
        std::vector<uint2> rowbuf((size_t)c->K);
        for (int32_t i = 0; i < m; i++) {
            if (words[i] < 0 || words[i] >= c->V) return fail(SABER_EINVAL, "saber_get_alias: word %d is outside [0,%d)", words[i], c->V);
            const int32_t row = c->h_word_row[(size_t)words[i]];
            if (row < 0) return fail(SABER_ESTATE, "saber_get_alias: word %d keeps a sparse row", words[i]);
            HIP_TRY(hipMemcpy(rowbuf.data(), c->alias_table + (size_t)row * (size_t)c->K, sizeof(uint2) * (size_t)c->K, hipMemcpyDeviceToHost));
            for (int32_t k = 0; k < c->K; k++) {   // format conversion only
                memcpy(&prob[(size_t)i * (size_t)c->K + (size_t)k], &rowbuf[(size_t)k].x, sizeof(float));
                alias[(size_t)i * (size_t)c->K + (size_t)k] = (int32_t)rowbuf[(size_t)k].y;
            }
        }
    } catch (const std::bad_alloc &) { return fail(SABER_ENOMEM, "saber_get_alias: out of host memory"); }
    return SABER_OK;
}

extern "C" int saber_get_stats(saber_ctx *c, saber_stats *out) {
    if (!c || !out) return fail(SABER_EINVAL, "saber_get_stats: null argument");
    *out = c->stats;
    return SABER_OK;
}

extern "C" int saber_reset_stats(saber_ctx *c) {
    if (!c) return fail(SABER_EINVAL, "saber_reset_stats: null context");
    c->stats.iterations = 0; c->stats.ms_sample = c->stats.ms_count_dz = c->stats.ms_ck = c->stats.ms_phi = c->stats.ms_total = 0.0;
    c->stats.sample_launches = 0; c->stats.sum_tokens = c->stats.sum_tokens_dense = c->stats.sum_row_entries = c->stats.sum_row_fetch = c->stats.sum_light_entries = 0;
    return SABER_OK;
}

extern "C" int saber_get_stream(saber_ctx *c, void **s) {
    if (!c || !s) return fail(SABER_EINVAL, "saber_get_stream: null argument");
    *s = (void *)c->stream;
    return SABER_OK;
}

// ------------------------------------------------------------------------------------------------
// bandwidth probe (measurement aid; independent of any context)
// ------------------------------------------------------------------------------------------------
extern "C" int saber_bandwidth_probe(int64_t bytes, int32_t reps, double *gb_per_s) {
    if (bytes < 16 || reps < 1 || !gb_per_s) return fail(SABER_EINVAL, "saber_bandwidth_probe: bad argument");
    const size_t n16 = (size_t)bytes / 16;
    uint4 *src = nullptr, *dst = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = SABER_OK;
    auto cleanup = [&]() { dev_free(g_hooks, src); dev_free(g_hooks, dst); if (e0) (void)hipEventDestroy(e0); if (e1) (void)hipEventDestroy(e1); };
    if ((rc = dev_alloc(g_hooks, &src, n16)) || (rc = dev_alloc(g_hooks, &dst, n16))) { cleanup(); return rc; }
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(8192), dim3(256), 0, 0, (uint32_t *)src, 1u, n16 * 4);
        hipLaunchKernelGGL(copy_probe_kernel, dim3(8192), dim3(256), 0, 0, src, dst, n16);   // warm-up
        e = hipEventRecord(e0, 0);
        for (int r = 0; r < reps; r++) hipLaunchKernelGGL(copy_probe_kernel, dim3(8192), dim3(256), 0, 0, src, dst, n16);
        if (e == hipSuccess) e = hipEventRecord(e1, 0);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipGetLastError();
    }
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    cleanup();
    if (e != hipSuccess) return fail(SABER_EDEVICE, "saber_bandwidth_probe: %s", hipGetErrorString(e));
    *gb_per_s = 2.0 * (double)(n16 * 16) * reps / ((double)ms * 1e-3) / 1e9;   // read + write
    return SABER_OK;
}
