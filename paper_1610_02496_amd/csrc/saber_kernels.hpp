// Device code of the sparsity-aware LDA sampler for gfx950 (wave64).
// Included once by saber.hip.  Citations refer to the SaberLDA paper.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace saber {

constexpr int kWave = 64;

// ---------------------------------------------------------------------------------------------
// Wavefront primitives (the wave64 counterparts of warp_sum / warp_prefix_sum / warp_vote /
// warp_copy in Sec. 3.2.3): DPP row shifts + row broadcasts for scans, a 64-bit ballot + count
// trailing zeros for the vote, readlane for the copy.
// ---------------------------------------------------------------------------------------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f32(float v) {
    // lanes without a valid source (or masked rows) receive 0, the identity of the sums below
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64(double v) {
    long long b = __double_as_longlong(v);
    int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffll), CTRL, ROW_MASK, 0xf, false);
    int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, ROW_MASK, 0xf, false);
    return __longlong_as_double(((long long)hi << 32) | (long long)(uint32_t)lo);
}

// inclusive scan over the 64 lanes: 4 shifts inside each row of 16, then two row broadcasts
#define SABER_SCAN_BODY(T, DPP)                                                            \
    v += DPP<0x111, 0xf>(v); /* row_shr:1 */                                               \
    v += DPP<0x112, 0xf>(v); /* row_shr:2 */                                               \
    v += DPP<0x114, 0xf>(v); /* row_shr:4 */                                               \
    v += DPP<0x118, 0xf>(v); /* row_shr:8 */                                               \
    v += DPP<0x142, 0xa>(v); /* row_bcast:15 into rows 1 and 3 */                          \
    v += DPP<0x143, 0xc>(v); /* row_bcast:31 into rows 2 and 3 */                          \
    return v;
__device__ __forceinline__ float wave_incl_scan(float v) { SABER_SCAN_BODY(float, dpp_f32) }
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) { SABER_SCAN_BODY(uint32_t, dpp_u32) }
__device__ __forceinline__ double wave_incl_scan(double v) { SABER_SCAN_BODY(double, dpp_f64) }
#undef SABER_SCAN_BODY

// binary32 scan used in the sampler's inner loop: the two row-broadcast steps as single fused DPP adds (rows
// outside the row mask keep their value, which is exactly what the scan wants; the compiler fuses a masked DPP
// move into an integer add but not into a float add, hence the two lines of assembly).  s_nop 1 covers the two
// wait states a DPP read needs after the VALU write of its source.  The compiler's hazard recogniser does not see
// inside the assembly, so the one other hazard of a DPP instruction is the caller's to exclude: no VALU write of
// EXEC (v_cmpx, v_readlane into EXEC) within five instructions before the call.  Every call site sits in
// wave-uniform control flow, where EXEC is only ever written by scalar instructions (on gfx9 the compiler forms
// no v_cmpx), which need no wait.
__device__ __forceinline__ float wave_incl_scan_fast(float v) {
    v += dpp_f32<0x111, 0xf>(v);
    v += dpp_f32<0x112, 0xf>(v);
    v += dpp_f32<0x114, 0xf>(v);
    v += dpp_f32<0x118, 0xf>(v);
    asm volatile("s_nop 1\n\tv_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf" : "+v"(v));
    asm volatile("s_nop 1\n\tv_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf" : "+v"(v));
    return v;
}

// write a wave-uniform value into one lane of a register
__device__ unsigned int llvm_amdgcn_writelane_u32(unsigned int value, unsigned int lane, unsigned int old)
    __asm("llvm.amdgcn.writelane.i32");

__device__ __forceinline__ float readlane_f32(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ uint32_t readlane_u32(uint32_t v, int lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}
__device__ __forceinline__ double readlane_f64(double v, int lane) {
    long long b = __double_as_longlong(v);
    int lo = __builtin_amdgcn_readlane((int)(b & 0xffffffffll), lane);
    int hi = __builtin_amdgcn_readlane((int)(b >> 32), lane);
    return __longlong_as_double(((long long)hi << 32) | (long long)(uint32_t)lo);
}
__device__ __forceinline__ float wave_sum(float v) { return readlane_f32(wave_incl_scan(v), 63); }
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) { return readlane_u32(wave_incl_scan(v), 63); }

// inclusive running maximum over the 64 lanes
__device__ __forceinline__ int wave_incl_scan_max(int v) {
    const int lo = -2147483647 - 1;
    v = max(v, __builtin_amdgcn_update_dpp(lo, v, 0x111, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(lo, v, 0x112, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(lo, v, 0x114, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(lo, v, 0x118, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(lo, v, 0x142, 0xa, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(lo, v, 0x143, 0xc, 0xf, false));
    return v;
}

// index of the first lane whose predicate holds, or -1
__device__ __forceinline__ int wave_vote_first(bool pred) {
    unsigned long long m = __builtin_amdgcn_ballot_w64(pred);
    return m ? (int)__builtin_ctzll(m) : -1;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11), written for the device; the CPU checker has its own.
// counter = (token lo, token hi, iteration, 0), key = (seed lo, seed hi).
// ---------------------------------------------------------------------------------------------
struct Rand2 { uint32_t r0, r1; };
__device__ __forceinline__ Rand2 philox_token(uint32_t seed_lo, uint32_t seed_hi, uint64_t t, uint32_t iter) {
    uint32_t c0 = (uint32_t)t, c1 = (uint32_t)(t >> 32), c2 = iter, c3 = 0u;
    uint32_t k0 = seed_lo, k1 = seed_hi;
#pragma unroll
    for (int r = 0; r < 10; r++) {
        const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
        uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return Rand2{c0, c1};
}
__device__ __forceinline__ float unit24(uint32_t r) { return (float)(r >> 8) * (1.0f / 16777216.0f); }

// ---------------------------------------------------------------------------------------------
// Small utility kernels
// ---------------------------------------------------------------------------------------------
__global__ void fill_u32_kernel(uint32_t *p, uint32_t value, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = value;
}

// z[z_rel + i] belongs to the canonical token t0 + i
template <typename ZT>
__global__ void init_z_kernel(ZT *z, int64_t z_rel, int64_t t0, int64_t t1, uint32_t K, uint32_t seed_lo, uint32_t seed_hi) {
    int64_t t = t0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (int64_t)gridDim.x * blockDim.x;
    for (; t < t1; t += stride) {
        Rand2 r = philox_token(seed_lo, seed_hi, (uint64_t)t, 0u);
        z[z_rel + (t - t0)] = (ZT)__umulhi(r.r0, K);   // floor(word0 * K / 2^32)
    }
}

template <typename ZT>
__global__ void z_from_i32_kernel(ZT *z, const int32_t *src, int64_t T) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (int64_t)gridDim.x * blockDim.x;
    for (; t < T; t += stride) z[t] = (ZT)src[t];
}
template <typename ZT>
__global__ void z_to_i32_kernel(const ZT *z, int32_t *dst, int64_t T) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (int64_t)gridDim.x * blockDim.x;
    for (; t < T; t += stride) dst[t] = (int32_t)z[t];
}

// Normalisers of Alg. 2 for the requested tokens that lie in the chunk [t0, t0 + n): S and Q as the sampling
// kernel's inspection mode left them (indexed by the token's position in the chunk) and the probability of the
// sparse branch, S / (S + Q).
__global__ void gather_probs_kernel(const float *S, const float *Q, const int64_t *idx, int64_t m, int64_t t0, int64_t n,
                                    float *out_S, float *out_Q, float *out_p) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= m) return;
    const int64_t r = idx[i] - t0;
    if (r < 0 || r >= n) return;
    const float s = S[r], q = Q[r];
    out_S[i] = s; out_Q[i] = q; out_p[i] = s / (s + q);
}

// ---------------------------------------------------------------------------------------------
// Work description of the E-step: one tile = up to tile_tokens tokens of one word inside one chunk.
// Tokens of a chunk are stored word-major (partition-by-document, order-by-word, Sec. 3.1.4).
// ---------------------------------------------------------------------------------------------
// row: the word's row in the dense B / Bhat arrays, or its index among the light words (see below)
// wm_begin: position of the tile's first token in the corpus-wide word-major order
struct Tile { int32_t word; int32_t begin; int32_t count; int32_t row; int64_t wm_begin; int64_t pad; };

struct EStepParams {
    const Tile *tiles;
    const int32_t *tok_doc;     // [chunk tokens] document of the token (global document id)
    const uint32_t *tok_t;      // [chunk tokens] canonical token index relative to t_base
    const uint2 *docrec;        // [D] {row start in units of 32 entries, K_d}
    const uint32_t *cd_rows;    // packed rows of A (topic | count << topic_bits, ascending topic) from the first row of
                                // the chunk's documents on: the row of document d starts (docrec[d].x - row_unit0) * 32
                                // entries into it
    uint32_t row_unit0;         // row start of the chunk's first document
    uint32_t rows_bytes;        // bytes from cd_rows to the end of the chunk's last row (below 2^32)
    uint32_t quarter_row_bytes; // rows up to this padded length (at most 256 bytes) are sampled four at a time, one per 16 lanes
    uint32_t half_row_bytes;    // longer rows up to this length (at most 512 bytes) two at a time, one per 32 lanes
    const float *phi;           // [dense rows][Kpad]  Bhat
    const float *l3;            // [V][n3pad] binary32 prefix sum of the Bhat row at the end of every 64-topic block,
                                //            padded with the row total (tree level above the bottom)
    const double *l3_64;        // [V][n3]    the same running sums before rounding (base of each bottom block)
    const float *sumphi;        // [V]        prefix sum at topic K-1 = l3[n3-1]
    void *z;                    // assignments in canonical order (uint16 or int32): the chunk's token t_base + i is
                                // element z_rel + i (the resident array holds all tokens, a streaming buffer one chunk)
    // light words (few tokens): B is kept sparse, Bhat = base + the word's non-zeros
    const float *base;          // [Kpad] Bhat of a zero count, beta / denom_k (pad columns 0)
    const uint2 *wrec;          // [light words] {row start in units of 32 entries, non-zeros}
    const uint32_t *lw_ent;     // packed (topic, count) rows of B for the light words, ascending topic
    const float *lw_phi;        // Bhat value of every such entry
    void *z_wm;                 // [T] new assignments in word-major order (light words first): input of CountByVZ
    const uint2 *alias_table;   // null, or [dense rows][K] {prob bits, alias}: the dense term is then drawn from these
                                // alias tables instead of the prefix-sum tree (measurement variant, Sec. 3.2.3)
    float *out_S;               // probs mode: S per token of the chunk, indexed by the token's position in the chunk
    float *out_Q;               // probs mode: Q likewise
    double *out_ll;             // loglik mode: one partial sum per tile
    unsigned long long *n_dense;// sample mode: kDenseSlots dense-branch token counters (workgroup b adds to slot b mod
                                // kDenseSlots: one hot address would serialise the atomics of the whole launch)
    int64_t t_base;             // canonical index of the chunk's first token
    int64_t z_rel;              // position of that token in z
    int32_t K, Kpad, n3, n3pad;
    uint32_t topic_bits, topic_mask;
    float alpha;
    uint32_t seed_lo, seed_hi, iter;
};

enum { MODE_SAMPLE = 0, MODE_PROBS = 1, MODE_LOGLIK = 2 };
constexpr int kDenseSlots = 1024;

// Sums and scans inside one DPP row (16 lanes): the dense branch serves four tokens at a time, one per row.
__device__ __forceinline__ uint32_t row16_allsum(uint32_t v) {
    v += dpp_u32<0x128, 0xf>(v);   // row_ror:8
    v += dpp_u32<0x124, 0xf>(v);   // row_ror:4
    v += dpp_u32<0x122, 0xf>(v);   // row_ror:2
    v += dpp_u32<0x121, 0xf>(v);   // row_ror:1
    return v;
}
__device__ __forceinline__ double row16_incl_scan(double v) {
    v += dpp_f64<0x111, 0xf>(v);
    v += dpp_f64<0x112, 0xf>(v);
    v += dpp_f64<0x114, 0xf>(v);
    v += dpp_f64<0x118, 0xf>(v);
    return v;
}

__device__ __forceinline__ float row16_incl_scan(float v) {
    v += dpp_f32<0x111, 0xf>(v);
    v += dpp_f32<0x112, 0xf>(v);
    v += dpp_f32<0x114, 0xf>(v);
    v += dpp_f32<0x118, 0xf>(v);
    return v;
}

// Dense branch (problem 2, Sec. 2.3): position of x in the prefix sums of the word's Bhat row, four tokens per
// call: the 16 lanes of DPP row g serve the token whose x they hold (all lanes of a row hold the same x).
// The descent follows Sec. 3.2.4 with the stored level l3 (binary32 prefix sum at the end of every 64-topic
// block; every 16th, 256th, ... entry of it acts as the levels above).  Prefix sums are non-decreasing, so
// "first entry >= x" is the number of entries below x: every lane tests one entry and one row-wide sum gives
// the position.  The bottom level is not stored: the 64 prefix sums of the chosen block are rebuilt from the
// Bhat values as round32(base + running sum in binary64), base = unrounded running sum at the block's start -
// the numbers a stored table would hold, so the search is exact.
// Those 64 numbers are first formed in binary32 alone (base = the stored, rounded running sum before the block):
// 12 roundings of positive numbers put each within 7.5e-7 of the exact one, relatively.  If none of them lies within
// 1.5e-6 x of x, the count of entries below x is the same for both and the binary64 arithmetic (and the load of its
// base) is skipped; otherwise (a few calls in a hundred at K = 10,000) the exact numbers decide.
// Returns the topic in every lane of the row.
__device__ __forceinline__ uint32_t dense_query4(const float *phi_row, int phi_len, const float *l3,
                                                 const double *__restrict__ l3_64, int n3, int K, float x, int li) {
    // 16-ary descent over l3: lane li looks at the last entry of the li-th sub-range of the current window; the
    // number of sub-ranges lying wholly below x is the index of the one holding the position
    int stride = 1;
    while (stride * 16 < n3) stride *= 16;
    int blk = 0;
    for (; stride >= 1; stride >>= 4) {
        const float c = l3[min(blk + (li + 1) * stride - 1, n3 - 1)];
        blk += min((int)row16_allsum(c < x ? 1u : 0u), 15) * stride;
    }
    blk = min(blk, n3 - 1);                                 // rounding left no block: the last one
    const int k0 = blk * kWave + li * 4;
    float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k0 < phi_len) f = *reinterpret_cast<const float4 *>(phi_row + k0);   // columns K..phi_len-1 hold zeros
    const float t0 = f.x, t1 = t0 + f.y, t2 = t1 + f.z, t3 = t2 + f.w;
    const float a2 = (blk > 0 ? l3[blk - 1] : 0.f) + (row16_incl_scan(t3) - t3);
    const float c0 = a2 + t0, c1 = a2 + t1, c2 = a2 + t2, c3 = a2 + t3;
    uint32_t below = (c0 < x ? 1u : 0u) + (c1 < x ? 1u : 0u) + (c2 < x ? 1u : 0u) + (c3 < x ? 1u : 0u);
    const float nearest = fminf(fminf(fabsf(c0 - x), fabsf(c1 - x)), fminf(fabsf(c2 - x), fabsf(c3 - x)));
    if (__builtin_amdgcn_ballot_w64(nearest <= x * 1.5e-6f)) {   // wave-uniform: some entry is too close to x to call
        const double base = blk > 0 ? l3_64[blk - 1] : 0.0;
        const double s0 = (double)f.x, s1 = s0 + (double)f.y, s2 = s1 + (double)f.z, s3 = s2 + (double)f.w;
        const double b2 = base + (row16_incl_scan(s3) - s3);
        below = ((float)(b2 + s0) < x ? 1u : 0u) + ((float)(b2 + s1) < x ? 1u : 0u) +
                ((float)(b2 + s2) < x ? 1u : 0u) + ((float)(b2 + s3) < x ? 1u : 0u);
    }
    const int k = blk * kWave + min((int)row16_allsum(below), kWave - 1);
    return (uint32_t)min(k, K - 1);
}

// How many of the 16 lanes of this lane's DPP row satisfy pred (row_shift = 16 * row): one compare into a
// wave-wide mask, the row's 16 bits of it, a bit count.
__device__ __forceinline__ uint32_t row16_count(bool pred, uint32_t row_shift) {
    const unsigned long long m = __builtin_amdgcn_ballot_w64(pred);
    return (uint32_t)__builtin_popcount((uint32_t)(m >> row_shift) & 0xffffu);
}

// dense_query4 for a workgroup that holds the word's Bhat row and tree level in LDS, laid out as the sampling
// kernel stages them: the row from byte 0 to phi_bytes (K rounded to 4 floats), four control words of which the
// last is zero, then l3 from byte l3_addr = phi_bytes + 16.  Same numbers and same decisions as dense_query4; what
// differs is how they are fetched and counted.  Nothing is read conditionally: l3[-1] is the zero word before l3[0];
// a lane whose four columns lie past the row's end (last block only) reads the row's last four instead and is left
// out of the count afterwards (its sums would not be below x, and a prefix scan hands nothing of it to the lanes
// before it).  The descent's strides are powers of 16, applied as shifts (top_shift = 4 * number of levels above
// the lowest), and a row's count of entries below x comes from one wave-wide compare mask instead of four DPP additions.
__device__ __forceinline__ uint32_t dense_query4_staged(uint32_t phi_bytes, uint32_t l3_addr, const double *__restrict__ l3_64,
                                                        int n3, int top_shift, int K, float x, uint32_t li, uint32_t row_shift) {
    typedef __attribute__((address_space(3))) const float lds_cfloat;
    typedef float quad_t __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) const quad_t lds_cquad;
    uint32_t blk = 0;
    for (int sh = top_shift; sh >= 0; sh -= 4) {
        const uint32_t probe = min(blk + ((li + 1u) << sh), (uint32_t)n3);   // 1 + index of the entry this lane tests
        const float c = *reinterpret_cast<lds_cfloat *>(l3_addr - 4u + (probe << 2));
        blk += min(row16_count(c < x, row_shift), 15u) << sh;
    }
    blk = min(blk, (uint32_t)n3 - 1u);                      // rounding left no block: the last one
    const uint32_t col_bytes = (blk << 8) + (li << 4);
    const bool in_row = col_bytes < phi_bytes;
    const quad_t f = *reinterpret_cast<lds_cquad *>(min(col_bytes, phi_bytes - 16u));
    const float before = *reinterpret_cast<lds_cfloat *>(l3_addr - 4u + (blk << 2));
    const float t0 = f.x, t1 = t0 + f.y, t2 = t1 + f.z, t3 = t2 + f.w;
    const float a2 = before + (row16_incl_scan(t3) - t3);
    const float c0 = a2 + t0, c1 = a2 + t1, c2 = a2 + t2, c3 = a2 + t3;
    uint32_t below = (c0 < x ? 1u : 0u) + (c1 < x ? 1u : 0u) + (c2 < x ? 1u : 0u) + (c3 < x ? 1u : 0u);
    const float nearest = fminf(fminf(fabsf(c0 - x), fabsf(c1 - x)), fminf(fabsf(c2 - x), fabsf(c3 - x)));
    if (__builtin_amdgcn_ballot_w64(in_row && nearest <= x * 1.5e-6f)) {   // wave-uniform: some entry is too close to x to call
        const double base = blk > 0 ? l3_64[blk - 1] : 0.0;
        const double s0 = (double)f.x, s1 = s0 + (double)f.y, s2 = s1 + (double)f.z, s3 = s2 + (double)f.w;
        const double b2 = base + (row16_incl_scan(s3) - s3);
        below = ((float)(b2 + s0) < x ? 1u : 0u) + ((float)(b2 + s1) < x ? 1u : 0u) +
                ((float)(b2 + s2) < x ? 1u : 0u) + ((float)(b2 + s3) < x ? 1u : 0u);
    }
    const uint32_t k = (blk << 6) + min(row16_allsum(in_row ? below : 0u), (uint32_t)kWave - 1u);
    return min(k, (uint32_t)K - 1u);
}

// ---------------------------------------------------------------------------------------------
// E-step (Alg. 2).  One workgroup per tile; the word's Bhat row and the upper tree level are staged in
// LDS (STAGED) or read from global memory.  Each wavefront takes a batch of up to 64 tokens: the
// per-token scalars (document, row descriptor, Philox draws) are produced one token per lane.  Tokens are
// ordered by (word, document), so repeated occurrences of a word in a document are neighbours (a "run"): they
// share A_d (.) Bhat_v and S, and only the two draws differ.
//
// A row of A is consumed in pieces of 4 entries per lane (one 16-byte load per lane): the lane forms its four
// running partial products, a DPP scan over the lane sums yields both S and every prefix sum, and the draw is
// located with one ballot plus a four-way compare inside the winning lane.  How many lanes a run gets depends
// on the length of its row:
//   * rows of at most 64 entries: four runs at a time, one per DPP row of 16 lanes;
//   * rows of at most 128 entries: two runs at a time, one per half of the wavefront;
//   * longer rows: one run at a time over all 64 lanes, in blocks of 256 entries.
// A lane's 16 entries sit in the same order in all three layouts and a DPP scan never crosses the lanes of a
// group, so the sums come out bit-identical whichever layout a row gets.
// B16: entries are packed topic:16 | count:16 (compile-time shifts); otherwise topic_bits is a run-time value.
// ---------------------------------------------------------------------------------------------
struct RowBlock { float a0, a1, a2, a3, incl; };   // running sums inside the lane; inclusive scan of lane sums

// One 256-entry block of a row: lane l receives entries 4l..4l+3 through a buffer load whose descriptor ends
// at the row's padded length, so lanes past the end read zeros without any branch.  Rows are 128-byte
// aligned and padded to a multiple of 4 entries with (last topic, count 0).
__device__ __forceinline__ uint4 load_block(const uint32_t *row, int rel_kd, int lane) {
    const int bytes = rel_kd > 0 ? ((rel_kd + 3) & ~3) * 4 : 0;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)row, (short)0, bytes, 0x00020000);
    const auto v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane * 16, 0, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// The same for a row given by its address and padded length in bytes (wave-uniform values).
__device__ __forceinline__ uint4 load_block(const void *row, uint32_t row_bytes, int lane) {
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(row), (short)0, (int)row_bytes, 0x00020000);
    const auto v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane * 16, 0, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// The second 256-entry block of the same row (same descriptor, 1 KB further on).
__device__ __forceinline__ uint4 load_block2(const void *row, uint32_t row_bytes, int lane) {
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(row), (short)0, (int)row_bytes, 0x00020000);
    const auto v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane * 16, 16 * kWave, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// 16 bytes at a per-lane byte offset into the rows of a chunk; an offset of 0xffffffff (any offset past the
// descriptor's end) returns zeros and moves no data.
__device__ __forceinline__ uint4 load_rows_at(__amdgpu_buffer_rsrc_t rows, uint32_t byte_off) {
    const auto v = __builtin_amdgcn_raw_buffer_load_b128(rows, (int)byte_off, 0, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// clear bit `bit` of a wave-uniform mask (one scalar instruction)
__device__ __forceinline__ unsigned long long clear_bit(unsigned long long m, int bit) {
    asm("s_bitset0_b64 %0, %1" : "+s"(m) : "s"(bit));
    return m;
}

// lane permutations through the LDS crossbar (no LDS memory is touched); lane numbers are passed times 4
__device__ __forceinline__ uint32_t lane_pull(uint32_t v, uint32_t src_lane4) {
    return (uint32_t)__builtin_amdgcn_ds_bpermute((int)src_lane4, (int)v);      // every lane reads lane src
}
__device__ __forceinline__ float lane_pull(float v, uint32_t src_lane4) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute((int)src_lane4, __float_as_int(v)));
}
__device__ __forceinline__ uint32_t lane_push(uint32_t v, uint32_t dst_lane4) {
    return (uint32_t)__builtin_amdgcn_ds_permute((int)dst_lane4, (int)v);       // every lane writes lane dst; the
}                                                                               // highest writer wins, unwritten lanes get 0

// number of set bits of a wave-uniform mask at this lane or below it
__device__ __forceinline__ uint32_t bits_up_to_lane(unsigned long long m) {
    const unsigned long long h = m >> 1;
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(h >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)h, (uint32_t)(m & 1ull)));
}

// Inclusive scan over the lanes of each group of G lanes (G = 16: one DPP row; 32: half a wavefront; 64: all).
template <int G>
__device__ __forceinline__ float group_incl_scan(float v) {
    v += dpp_f32<0x111, 0xf>(v);
    v += dpp_f32<0x112, 0xf>(v);
    v += dpp_f32<0x114, 0xf>(v);
    v += dpp_f32<0x118, 0xf>(v);
    // see wave_incl_scan_fast for the two lines of assembly and their precondition
    if (G >= 32) asm volatile("s_nop 1\n\tv_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf" : "+v"(v));
    if (G >= 64) asm volatile("s_nop 1\n\tv_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf" : "+v"(v));
    return v;
}

// Bhat value of the entry's topic.  With 16/16 packing and the row in LDS the byte offset (topic * 4) is formed
// by one shift that reads the low half of the entry.
template <bool STAGED, bool B16>
__device__ __forceinline__ float phi_of(uint32_t e, uint32_t tmask, const float *lds_phi, const float *__restrict__ phi_row) {
    if (STAGED && B16) {
        uint32_t off;
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0"
            : "=v"(off) : "v"(2u), "v"(e));
        // the staged row starts at LDS address 0 (the kernel has no static LDS; the host checks that at start-up)
        typedef __attribute__((address_space(3))) const float lds_cfloat;
        return *reinterpret_cast<lds_cfloat *>(off);
    }
    return STAGED ? lds_phi[e & tmask] : phi_row[e & tmask];
}

// element-wise product A_d (.) Bhat_v of the lane's four entries as running sums, and their scan over the group
template <bool STAGED, bool B16, int G = kWave>
__device__ __forceinline__ void block_products(const uint4 e, uint32_t bits, uint32_t tmask,
                                               const float *lds_phi, const float *__restrict__ phi_row, RowBlock &b) {
    const float f0 = phi_of<STAGED, B16>(e.x, tmask, lds_phi, phi_row);
    const float f1 = phi_of<STAGED, B16>(e.y, tmask, lds_phi, phi_row);
    const float f2 = phi_of<STAGED, B16>(e.z, tmask, lds_phi, phi_row);
    const float f3 = phi_of<STAGED, B16>(e.w, tmask, lds_phi, phi_row);
    b.a0 = (float)(e.x >> bits) * f0;
    b.a1 = __builtin_fmaf((float)(e.y >> bits), f1, b.a0);
    b.a2 = __builtin_fmaf((float)(e.z >> bits), f2, b.a1);
    b.a3 = __builtin_fmaf((float)(e.w >> bits), f3, b.a2);
    b.incl = group_incl_scan<G>(b.a3);
}

// First entry of the block whose prefix sum (carry + sums inside the block) reaches x.  The lane is found
// with one ballot over the lanes' inclusive sums, the entry inside it with three compares.  If rounding
// leaves no entry, the choice falls on the block's last one (a row's padding repeats its last topic).
__device__ __forceinline__ uint32_t search_block(const uint4 e, const RowBlock &b, float carry, float x, int rel_kd,
                                                 uint32_t tmask) {
    const float base = carry + (b.incl - b.a3);
    const unsigned long long m3 = __builtin_amdgcn_ballot_w64(carry + b.incl >= x);
    const int nvalid = rel_kd < 4 * kWave ? rel_kd : 4 * kWave;
    const int L = m3 ? (int)__builtin_ctzll(m3) : ((nvalid - 1) >> 2);
    const uint32_t sel = (base + b.a0 >= x) ? e.x : (base + b.a1 >= x) ? e.y : (base + b.a2 >= x) ? e.z : e.w;
    return readlane_u32(sel, L) & tmask;
}

// New assignments are written twice: to z (canonical order) and to z_wm (word-major, coalesced), from which the
// M-step counts B; the sampler itself adds nothing to B.
// LIGHT: the tile's word keeps B sparse.  Its Bhat row is built in LDS from the base vector and the word's
// non-zeros.
template <int MODE, bool STAGED, typename ZT, bool B16, bool LIGHT>
__global__ void __launch_bounds__(1024, 8) estep_kernel(EStepParams p) {
    extern __shared__ float4 lds_f4[];
    // LDS, all of it dynamic so that the Bhat row starts at address 0 and a gather needs no base added:
    //   STAGED: [K rounded to 4] floats: the word's Bhat row
    //   [4] words: batch ticket, dense-branch tokens of the workgroup, 0, 0 (the last one doubles as the tree level's
    //           entry "before the first", which the dense branch reads for the first block)
    //   STAGED: [n3 rounded to 4] floats: the tree level above the bottom;  LOGLIK: [16] doubles, one per wavefront
    // The footprint is kept minimal because it decides how many wavefronts a CU can hold: at K = 10,000 it is
    // 40,656 bytes, which lets four 512-thread workgroups (32 wavefronts) share the 160 KB of a CU.
    const int K4 = STAGED ? (p.K + 3) & ~3 : 0;
    float *lds_phi = reinterpret_cast<float *>(lds_f4);
    int *ctrl = reinterpret_cast<int *>(lds_phi + K4);
    float *lds_l3 = lds_phi + K4 + 4;
    int &next_batch = ctrl[0];   // batches of a tile are handed out to wavefronts as they become free
    unsigned int &wg_dense = reinterpret_cast<unsigned int *>(ctrl)[1];   // dense-branch tokens of this workgroup
    double *ll_wave = reinterpret_cast<double *>(lds_l3 + (STAGED ? (p.n3 + 3) & ~3 : 0));
    const Tile tile = p.tiles[blockIdx.x];
    const int K = p.K;
    const float *__restrict__ phi_row = LIGHT ? p.base : p.phi + (size_t)tile.row * (size_t)p.Kpad;
    const float *__restrict__ l3_row = p.l3 + (size_t)tile.word * (size_t)p.n3pad;
    const double *__restrict__ l3_64_row = p.l3_64 + (size_t)tile.word * (size_t)p.n3;
    const int lane = lane_id(), nwaves = blockDim.x / kWave;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    // batch size: 64 tokens per wavefront, fewer when the tile is too small to keep every wavefront busy
    int bs = (tile.count + nwaves - 1) / nwaves;
    bs = __builtin_amdgcn_readfirstlane(bs > kWave ? kWave : bs);   // wave-uniform: keep it in a scalar register
    // The first batch of every wavefront is fixed (wavefront w takes batch w; the ticket counter starts behind these),
    // so its token records are requested here, before the word's row is staged, and the row records of their
    // documents before the workgroup waits at the barrier: for a small tile (one batch per wavefront) two of the three
    // dependent memory accesses in front of the first row then pass under the staging.
    int batch = wave * bs;
    int d = -1;
    uint32_t t = 0u;
    if (lane < min(bs, tile.count - batch)) {
        d = p.tok_doc[tile.begin + batch + lane];
        t = p.tok_t[tile.begin + batch + lane];
    }
    if (threadIdx.x == 0) { next_batch = nwaves; wg_dense = 0u; ctrl[2] = 0; ctrl[3] = 0; }
    if (STAGED) {
        // eight 16-byte loads per thread are requested before the first of them is written to LDS: one load, one
        // wait, one write at a time left a workgroup's start waiting for memory five times over at K = 10,000.
        // (No branch inside: past the end, the last piece is read and written once more.)
        typedef float quad_t __attribute__((ext_vector_type(4)));
        const quad_t *qsrc = reinterpret_cast<const quad_t *>(phi_row);
        quad_t *qdst = reinterpret_cast<quad_t *>(lds_phi);
        const int nq = K4 / 4, step = (int)blockDim.x;
        for (int i0 = threadIdx.x; i0 < nq; i0 += 8 * step) {
            const quad_t q0 = qsrc[min(i0, nq - 1)], q1 = qsrc[min(i0 + step, nq - 1)], q2 = qsrc[min(i0 + 2 * step, nq - 1)],
                         q3 = qsrc[min(i0 + 3 * step, nq - 1)], q4 = qsrc[min(i0 + 4 * step, nq - 1)],
                         q5 = qsrc[min(i0 + 5 * step, nq - 1)], q6 = qsrc[min(i0 + 6 * step, nq - 1)],
                         q7 = qsrc[min(i0 + 7 * step, nq - 1)];
            qdst[min(i0, nq - 1)] = q0; qdst[min(i0 + step, nq - 1)] = q1; qdst[min(i0 + 2 * step, nq - 1)] = q2;
            qdst[min(i0 + 3 * step, nq - 1)] = q3; qdst[min(i0 + 4 * step, nq - 1)] = q4; qdst[min(i0 + 5 * step, nq - 1)] = q5;
            qdst[min(i0 + 6 * step, nq - 1)] = q6; qdst[min(i0 + 7 * step, nq - 1)] = q7;
        }
        if (MODE == MODE_SAMPLE)
            for (int i = threadIdx.x; i < p.n3; i += blockDim.x) lds_l3[i] = l3_row[i];
    }
    uint2 rec = make_uint2(p.row_unit0, 0u);
    if (d >= 0) rec = p.docrec[d];
    __syncthreads();
    if (LIGHT) {
        // the staged row is the base vector so far; overwrite the topics this word has counts for
        const uint2 wr = p.wrec[tile.row];
        const uint32_t *__restrict__ ent = p.lw_ent + (size_t)wr.x * 32u;
        const float *__restrict__ val = p.lw_phi + (size_t)wr.x * 32u;
        const uint32_t tm = B16 ? 0xffffu : p.topic_mask;
        for (int j = threadIdx.x; j < (int)wr.y; j += blockDim.x) lds_phi[ent[j] & tm] = val[j];
        __syncthreads();
    }
    const float sum_w = p.sumphi[tile.word];
    const float Q = p.alpha * sum_w;
    int l3_top_shift = 0;                      // the dense branch's descent over l3 starts with stride 16^(l3_top_shift / 4)
    while ((16 << l3_top_shift) < p.n3) l3_top_shift += 4;
    const uint32_t bits = B16 ? 16u : p.topic_bits, tmask = B16 ? 0xffffu : p.topic_mask;
    // all rows of A of the chunk behind one buffer descriptor: a row is addressed by its 32-bit byte offset
    const __amdgpu_buffer_rsrc_t rows = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(p.cd_rows), (short)0,
                                                                          (int)p.rows_bytes, 0x00020000);
    double ll_acc = 0.0;

    // `batch`, and d, t, rec of its tokens, are in hand at the top of every turn: those of the first batch from above,
    // those of the later ones from the bottom of the turn before
    for (int round = 0;; round++) {
        if (batch >= tile.count) break;
        const int n = __builtin_amdgcn_readfirstlane(min(bs, tile.count - batch));   // wave-uniform by construction
        const bool act = lane < n;
        float u0 = 0.f, u1 = 0.f;
        if (MODE == MODE_SAMPLE) {
            Rand2 r = philox_token(p.seed_lo, p.seed_hi, (uint64_t)(p.t_base + (int64_t)t), p.iter);
            u0 = unit24(r.r0); u1 = unit24(r.r1);
        }
        uint32_t my_z = 0; float my_S = 0.f;
        unsigned long long dense_mask = 0ull;

        // Runs: bit i of `starts` marks a lane where the tokens of another document begin.
        const int d_prev = __builtin_amdgcn_update_dpp(-2, d, 0x138, 0xf, 0xf, false);   // wave_shr:1
        const bool first_of_run = act && d != d_prev;
        const unsigned long long starts = __builtin_amdgcn_ballot_w64(first_of_run) | 1ull;
        // the row of the lane's document: byte offset inside the chunk's rows and padded length in bytes
        const uint32_t row_off = (rec.x - p.row_unit0) << 7;
        const uint32_t row_bytes = ((rec.y + 3u) & ~3u) << 2;
        // position of the token inside its run
        const uint32_t jpos = (uint32_t)(lane - wave_incl_scan_max(first_of_run || lane == 0 ? lane : -1));
        // rows that fit a quarter or a half of the wavefront; runs are cut into pieces of at most G tokens there
        unsigned long long m16 = __builtin_amdgcn_ballot_w64(act && row_bytes <= p.quarter_row_bytes);
        unsigned long long m32 = __builtin_amdgcn_ballot_w64(act && row_bytes <= p.half_row_bytes) & ~m16;
        const unsigned long long cuts16 = __builtin_amdgcn_ballot_w64(act && (jpos & 15u) == 0u);   // where pieces begin
        const unsigned long long cuts32 = __builtin_amdgcn_ballot_w64(act && (jpos & 31u) == 0u);
        // a pass serves four (two) runs at the cost of about one: a class that would not fill most of one pass goes
        // with the next wider one
        if (__builtin_popcountll(m16 & cuts16) < 3) { if (p.half_row_bytes >= p.quarter_row_bytes) m32 |= m16; m16 = 0ull; }
        if (__builtin_popcountll(m32 & cuts32) < 2) m32 = 0ull;
        const unsigned long long cm16 = m16 & cuts16, cm32 = m32 & cuts32;
        unsigned long long wide_rest = starts & ~(m16 | m32);

        // ---- rows of at most 4 G entries: 64 / G runs at a time, one per group of G lanes ----
        // Token side: lane i holds token i of the batch.  Group side: the G lanes of group g hold the row of the
        // g-th run of the pass, 4 entries per lane.  Per class, the runs' row offsets and lengths are first packed
        // into the low lanes (slot r = r-th run of the class); a pass then pulls four (two) slots.
        auto run_class = [&](auto G_, const unsigned long long cm, const unsigned long long cuts, const bool in_class) {
            constexpr int G = decltype(G_)::value, NG = kWave / G, LG = G == 16 ? 4 : 5;
            const int nruns = (int)__builtin_popcountll(cm);   // wave-uniform
            if (nruns == 0) return;
            uint32_t zero = 0u;
            asm volatile("" : "+s"(zero));   // (keeps the compiler from running the set-up below ahead of this test)
            const int npass = (nruns + NG - 1) / NG;
            // (an opaque copy of the lane number: values derived from it are formed here, per class, instead of once
            // per kernel and then held in registers the kernel does not have to spare)
            uint32_t ln = (uint32_t)lane;
            asm volatile("" : "+v"(ln));
            const uint32_t gi = ln >> LG, li = ln & (uint32_t)(G - 1), li16 = li << 4;
            // Slot order: the pieces of one token first, the longer ones after them, each kind in batch order.  A pass
            // runs as many search steps as its longest piece has tokens, so like goes with like.  `rank` = 1 + slot of
            // the piece this lane belongs to.
            const unsigned long long sing = cm & ((cuts >> 1) | (1ull << (n - 1)));   // a piece that ends where the next begins
            const uint32_t nsing = (uint32_t)__builtin_popcountll(sing);
            const uint32_t rank = __builtin_amdgcn_inverse_ballot_w64(sing) ? bits_up_to_lane(sing)
                                                                            : nsing + bits_up_to_lane(cm & ~sing);
            // slots: a piece's first lane writes to slot rank - 1; all other lanes write to lane 63, which is a slot
            // only if every lane starts a piece
            const uint32_t dst4 = __builtin_amdgcn_inverse_ballot_w64(cm) ? (rank - 1u) << 2 : 252u + zero;
            const uint32_t slot_pk = lane_push(row_bytes | ((uint32_t)lane << 18), dst4);   // length | first token lane * 4 << 16
            const uint32_t slot_off = lane_push(row_off, dst4);
            const uint32_t my_piece = in_class ? rank - 1u : 0x80000000u;   // token side: piece of this token
            const uint32_t jg4 = (jpos & (uint32_t)(G - 1)) << 2;           // and its place in it, times 4
            constexpr unsigned long long ONES = G == 16 ? 0x0001000100010001ull : 0x0000000100000001ull;   // first lane of every group

            // request the rows of pass `ps` (past the last pass: nothing is moved)
            auto issue = [&](const int ps, uint4 &blk, uint32_t &pk) {
                uint32_t idx = (uint32_t)(ps * NG) + gi;
                idx = idx < (uint32_t)nruns ? idx : (uint32_t)(nruns - 1);   // spare groups repeat the last run
                pk = lane_pull(slot_pk, idx << 2);
                const uint32_t off = lane_pull(slot_off, idx << 2);
                const uint32_t lim = ps < npass ? pk & 0xffffu : 0u;
                blk = load_rows_at(rows, li16 < lim ? off + li16 : 0xffffffffu);
            };
            auto compute = [&](const int ps, const uint4 &cur, const uint32_t pk) {
                RowBlock b;
                block_products<STAGED, B16, G>(cur, bits, tmask, lds_phi, phi_row, b);
                // S of the group's run in all its lanes
                const float S = G == 16 ? dpp_f32<0x15f, 0xf>(b.incl)                    // row_newbcast:15
                                        : lane_pull(b.incl, (uint32_t)(lane | (G - 1)) << 2);
                // token side: is this token's piece part of the pass, and which lane will hold its result
                const uint32_t gt = my_piece - (uint32_t)(ps * NG);
                const bool in_pass = gt < (uint32_t)NG;
                const uint32_t src4 = (gt << (LG + 2)) + jg4;
                uint32_t zacc = 0u;
                if (MODE == MODE_SAMPLE) {
                    const float base = b.incl - b.a3;
                    const float p0 = base + b.a0, p1 = base + b.a1, p2 = base + b.a2;
                    // the last lane of every group's row: if rounding leaves no lane, the choice falls on it (its padding
                    // repeats the row's last topic)
                    const unsigned long long sent = __builtin_amdgcn_ballot_w64(li16 + 16u == (pk & 0xffffu));
                    const unsigned long long pass_mask = __builtin_amdgcn_ballot_w64(in_pass);
                    // Lane j of a group collects the result of the j-th token of the group's piece.  `todo` marks the
                    // token lanes at position j of the pass's pieces: when it is empty, no piece is that long.
                    unsigned long long todo = pass_mask & cuts, collect = ONES;
                    uint32_t ua = pk >> 16;                           // lane * 4 of the token that is served next
                    uint32_t da = (uint32_t)(lane & ~(G - 1)) << 2;   // lane * 4 of the group lane that collects its result
                    float x = lane_pull(u1, ua) * S;
                    while (todo) {
                        // problem 1 for one token per group: position of x in the prefix sums of P.  (Whether the
                        // token takes this branch is decided on the token side, once S has arrived there.)
                        ua += 4u;
                        const float x_next = lane_pull(u1, ua) * S;
                        const unsigned long long ge = __builtin_amdgcn_ballot_w64(b.incl >= x) | sent;
                        const unsigned long long win = ge & ~(ge - ONES);   // first such lane of every group
                        uint32_t sel = cur.w;
                        sel = p2 >= x ? cur.z : sel;
                        sel = p1 >= x ? cur.y : sel;
                        sel = p0 >= x ? cur.x : sel;
                        // the winning lane writes to the collecting lane, every other lane to the collecting lane's
                        // neighbour, whose own turn to collect is another one
                        const uint32_t got = lane_push(sel, da + (__builtin_amdgcn_inverse_ballot_w64(win) ? 0u : 4u));
                        zacc = __builtin_amdgcn_inverse_ballot_w64(collect) ? got : zacc;
                        da += 4u; collect <<= 1;
                        todo = (todo << 1) & pass_mask & ~cuts;
                        x = x_next;
                    }
                }
                const float St = lane_pull(S, src4);
                my_S = in_pass ? St : my_S;
                if (MODE == MODE_SAMPLE) {
                    const uint32_t zt = lane_pull(zacc, src4);
                    my_z = in_pass ? zt & tmask : my_z;
                }
            };
            uint4 blk_a, blk_b; uint32_t pk_a, pk_b;
            issue(0, blk_a, pk_a);
            for (int ps = 0;; ps += 2) {
                issue(ps + 1, blk_b, pk_b);
                compute(ps, blk_a, pk_a);
                if (ps + 1 >= npass) break;
                issue(ps + 2, blk_a, pk_a);
                compute(ps + 1, blk_b, pk_b);
                if (ps + 2 >= npass) break;
            }
        };
        // ---- longer rows: one run [s, s_end) at a time over the whole wavefront ----
        // `cur` and `cur2` hold the first two blocks of the run's row (fetched during the previous run) and cur_bytes the
        // row's padded length; the next run's row is fetched into `nxt`, `nxt2` before this run's arithmetic starts.
        const char *rows_base = reinterpret_cast<const char *>(p.cd_rows);
        auto fetch = [&](const int s, uint4 &blk, uint4 &blk2, uint32_t &bytes) {
            // Requested without any branch around the two loads: for s < 0 (no further run), and for the second
            // block of a short row, the descriptor's length makes every lane fall outside the row, which returns zeros
            // and moves no data.  A load inside a branch would make the compiler wait for ALL outstanding loads where
            // the branches meet, i.e. for the row just requested, before the current run's arithmetic.
            const int src = s < 0 ? 0 : s;
            bytes = s < 0 ? 0u : readlane_u32(row_bytes, src);
            const void *row = rows_base + readlane_u32(row_off, src);
            blk = load_block(row, bytes, lane);
            blk2 = load_block2(row, bytes, lane);
        };
        auto next_wide = [&]() {
            if (!wide_rest) return -1;
            const int s = (int)__builtin_ctzll(wide_rest);
            wide_rest = clear_bit(wide_rest, s);
            return s;
        };
        // the first of the long rows is requested now, so that it arrives while the short rows are worked on
        int s_a = next_wide(), s_b = -1;
        uint32_t bytes_a, bytes_b;
        uint4 blk_a, blk_a2, blk_b, blk_b2;
        fetch(s_a, blk_a, blk_a2, bytes_a);

        run_class(std::integral_constant<int, 16>{}, cm16, cuts16, __builtin_amdgcn_inverse_ballot_w64(m16));
        run_class(std::integral_constant<int, 32>{}, cm32, cuts32, __builtin_amdgcn_inverse_ballot_w64(m32));
        if (MODE == MODE_SAMPLE && (m16 | m32)) {
            // the coin of the tokens served above, all at once
            const unsigned long long sparse = __builtin_amdgcn_ballot_w64(u0 * (my_S + Q) < my_S);
            dense_mask = (m16 | m32) & ~sparse;
        }

        // ---- longer rows: one run [s, s_end) at a time over the whole wavefront (its first fetch went out above) ----
        auto do_run = [&](const int s, const uint4 &cur, const uint4 &cur2, const uint32_t cur_bytes, const int s_next, uint4 &nxt,
                          uint4 &nxt2, uint32_t &nxt_bytes) {
            fetch(s_next, nxt, nxt2, nxt_bytes);
            const unsigned long long later = starts & (~1ull << s);           // run starts after lane s
            const int s_end = later ? (int)__builtin_ctzll(later) : n;
            const unsigned long long in_run = (~0ull >> (kWave - s_end)) & (~0ull << s);   // 0 <= s < s_end <= 64
            // element-wise product A_d (.) Bhat_v, its prefix sums and its sum S (Alg. 2, product loop)
            RowBlock b0;
            block_products<STAGED, B16>(cur, bits, tmask, lds_phi, phi_row, b0);
            const float t0 = readlane_f32(b0.incl, 63);
            if (cur_bytes <= 16u * kWave) {
                // the whole row sits in this block (the common case): straight-line coin and search
                if (MODE == MODE_SAMPLE) {
                    unsigned long long sparse = __builtin_amdgcn_ballot_w64(u0 * (t0 + Q) < t0) & in_run;
                    dense_mask |= in_run & ~sparse;       // problem 2 is served after the runs, four tokens at a time
                    if (sparse) {
                        const float xs = u1 * t0;
                        const float base = b0.incl - b0.a3;
                        const float p0 = base + b0.a0, p1 = base + b0.a1, p2 = base + b0.a2;
                        // lanes past the row's end repeat its last inclusive sum: if rounding leaves no lane, the
                        // choice falls on the last one, whose padding repeats the row's last topic
                        const unsigned long long last_lane_bit = 1ull << ((cur_bytes >> 4) - 1u);
                        do {
                            // problem 1: position of x in the prefix sums of P
                            const int r = (int)__builtin_ctzll(sparse);
                            sparse = clear_bit(sparse, r);
                            const float x = readlane_f32(xs, r);
                            const int L = (int)__builtin_ctzll(__builtin_amdgcn_ballot_w64(b0.incl >= x) | last_lane_bit);
                            uint32_t sel = cur.w;
                            sel = p2 >= x ? cur.z : sel;
                            sel = p1 >= x ? cur.y : sel;
                            sel = p0 >= x ? cur.x : sel;
                            my_z = llvm_amdgcn_writelane_u32(readlane_u32(sel, L) & tmask, (unsigned)r, my_z);
                        } while (sparse);
                    }
                } else {
                    if (lane >= s && lane < s_end) my_S = t0;
                }
                return;
            }
            const int kd = (int)(cur_bytes >> 2);   // the row's length rounded up to 4 entries: the padding has count 0
            const uint32_t *row = reinterpret_cast<const uint32_t *>(rows_base + readlane_u32(row_off, s));
            const int nblk = (kd + 4 * kWave - 1) / (4 * kWave);
            const uint4 e1 = cur2;
            RowBlock b1;
            block_products<STAGED, B16>(e1, bits, tmask, lds_phi, phi_row, b1);
            const float t1 = readlane_f32(b1.incl, 63);
            float S = t0 + t1;
            for (int blk = 2; blk < nblk; blk++) {
                RowBlock bb;
                block_products<STAGED, B16>(load_block(row + blk * 4 * kWave, kd - blk * 4 * kWave, lane), bits, tmask,
                                            lds_phi, phi_row, bb);
                S = S + readlane_f32(bb.incl, 63);
            }
            if (MODE == MODE_SAMPLE) {
                // every lane evaluates the coin and the position for its own token; lanes of this run are used
                const unsigned long long sparse = __builtin_amdgcn_ballot_w64(u0 * (S + Q) < S);
                const float xs = u1 * S;
                dense_mask |= ~sparse & in_run;
                for (int r = s; r < s_end; r++) {
                    uint32_t topic;
                    if ((sparse >> r) & 1ull) {
                        const float x = readlane_f32(xs, r);
                        if (t0 >= x) topic = search_block(cur, b0, 0.f, x, kd, tmask);
                        else if (nblk == 2 || t0 + t1 >= x) topic = search_block(e1, b1, t0, x, kd - 4 * kWave, tmask);
                        else {
                            float carry = t0 + t1;
                            topic = 0u;
                            for (int blk = 2; blk < nblk; blk++) {
                                const int rel = kd - blk * 4 * kWave;
                                const uint4 e = load_block(row + blk * 4 * kWave, rel, lane);
                                RowBlock bb;
                                block_products<STAGED, B16>(e, bits, tmask, lds_phi, phi_row, bb);
                                const float tot = readlane_f32(bb.incl, 63);
                                if (blk == nblk - 1 || carry + tot >= x) { topic = search_block(e, bb, carry, x, rel, tmask); break; }
                                carry = carry + tot;
                            }
                        }
                        my_z = llvm_amdgcn_writelane_u32(topic, (unsigned)r, my_z);
                    }
                }
            } else {
                if (lane >= s && lane < s_end) my_S = S;
            }
        };

        if (s_a >= 0) {
            for (;;) {
                s_b = next_wide();
                do_run(s_a, blk_a, blk_a2, bytes_a, s_b, blk_b, blk_b2, bytes_b);
                if (s_b < 0) break;
                s_a = next_wide();
                do_run(s_b, blk_b, blk_b2, bytes_b, s_a, blk_a, blk_a2, bytes_a);
                if (s_a < 0) break;
            }
        }

        // The token's number is read again rather than carried through the batch in a register (the kernel is at its
        // register limit; the 4 bytes come from a cache line this wavefront loaded at the top of the batch).  Requested
        // here, it arrives while the dense branch below is served.
        uint32_t t_late = 0u;
        if (MODE != MODE_LOGLIK) {
            uint32_t pos_t = (uint32_t)(batch + lane);
            asm volatile("" : "+v"(pos_t));
            if (act) t_late = p.tok_t[tile.begin + (int)pos_t];
        }

        if (MODE == MODE_SAMPLE && dense_mask) {
            // problem 2 for the tokens whose coin chose it: DPP row g (16 lanes) serves the g-th of up to four tokens
            if (lane == 0) atomicAdd(&wg_dense, (unsigned int)__builtin_popcountll(dense_mask));   // statistic only
            if (!LIGHT && p.alias_table != nullptr) {
                // Walker's alias method for all these tokens at once: the bucket is floor(u1 K), taken in integers from
                // the 24 random bits behind u1; the bucket's own topic if the fraction of u1 K lies below its
                // probability, its alias otherwise
                const uint32_t bits24 = (uint32_t)(u1 * 16777216.0f);
                const uint32_t lo = bits24 * (uint32_t)K, hi = __umulhi(bits24, (uint32_t)K);
                const uint32_t bucket = (hi << 8) | (lo >> 24);
                const float frac = (float)(lo & 0xffffffu) * (1.0f / 16777216.0f);
                if (__builtin_amdgcn_inverse_ballot_w64(dense_mask)) {
                    const uint2 e = p.alias_table[(size_t)tile.row * (size_t)K + bucket];
                    my_z = frac < __uint_as_float(e.x) ? bucket : e.y;
                }
                dense_mask = 0ull;
            }
            const float xd = u1 * sum_w;
            uint32_t ln = (uint32_t)lane;
            asm volatile("" : "+v"(ln));               // (as above: lane-derived values formed where they are used)
            const uint32_t g = ln >> 4, li = ln & 15u;
            if (STAGED) {
                while (dense_mask) {
                    // the next four tokens (fewer at the end: the spare rows then repeat the first token's query, and
                    // arrive at the same answer)
                    const unsigned long long before = dense_mask;
                    uint32_t tl[4];
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        tl[q] = dense_mask ? (uint32_t)__builtin_ctzll(dense_mask) : tl[0];
                        if (dense_mask) dense_mask = clear_bit(dense_mask, (int)tl[q]);
                    }
                    // lane number * 4 of the row's token: the four of them packed into one scalar, a byte each
                    const uint32_t packed = (tl[0] | (tl[1] << 8) | (tl[2] << 16) | (tl[3] << 24)) << 2;
                    const uint32_t mine4 = __builtin_amdgcn_ubfe(packed, g << 3, 8u);
                    const float x = lane_pull(xd, mine4);
                    const uint32_t k = dense_query4_staged((uint32_t)K4 * 4u, (uint32_t)K4 * 4u + 16u, l3_64_row, p.n3, l3_top_shift, K,
                                                           x, li, ln & 48u);
                    // all 16 lanes of a row hold the row's answer and send it to the row's token
                    const uint32_t got = lane_push(k, mine4);
                    my_z = __builtin_amdgcn_inverse_ballot_w64(before ^ dense_mask) ? got : my_z;
                }
            }
            while (dense_mask) {
                int tl[4];
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    tl[q] = dense_mask ? (int)__builtin_ctzll(dense_mask) : -1;
                    if (dense_mask) dense_mask = clear_bit(dense_mask, tl[q]);
                }
                const int mine = g == 0 ? tl[0] : g == 1 ? tl[1] : g == 2 ? tl[2] : tl[3];
                const float x = __int_as_float(__builtin_amdgcn_ds_bpermute((mine < 0 ? lane : mine) << 2, __float_as_int(xd)));
                const uint32_t k = dense_query4(phi_row, p.Kpad, l3_row, l3_64_row, p.n3, K, x, (int)li);
#pragma unroll
                for (int q = 0; q < 4; q++)
                    if (tl[q] >= 0) my_z = llvm_amdgcn_writelane_u32(readlane_u32(k, 16 * q), (unsigned)tl[q], my_z);
            }
        }

        if (act) {
            if (MODE == MODE_SAMPLE) {
                reinterpret_cast<ZT *>(p.z)[p.z_rel + (int64_t)t_late] = (ZT)my_z;
                // the second copy, in word-major order, is what CountByVZ reads (coalesced here and there)
                uint32_t pos = (uint32_t)(batch + lane);   // of the token inside the tile
                asm volatile("" : "+v"(pos));
                reinterpret_cast<ZT *>(p.z_wm)[tile.wm_begin + (int64_t)pos] = (ZT)my_z;
            } else if (MODE == MODE_PROBS) {
                p.out_S[t_late] = my_S; p.out_Q[t_late] = Q;
            } else {
                ll_acc += log((double)(my_S + Q));
            }
        }
        // the next batch: taken from the ticket counter, as wavefronts become free.  (Asking for it and for its tokens'
        // records earlier, before the dense branch, changed nothing.)
        int ticket = 0;
        if (MODE == MODE_LOGLIK) ticket = (round + 1) * nwaves + wave;   // fixed assignment: the sums come out bit-identical every time
        else if (lane == 0) ticket = atomicAdd(&next_batch, 1);
        batch = __builtin_amdgcn_readfirstlane(ticket) * bs;   // wave-uniform: loop control stays scalar
        d = -1; t = 0u; rec = make_uint2(p.row_unit0, 0u);
        if (lane < min(bs, tile.count - batch)) {
            d = p.tok_doc[tile.begin + batch + lane];
            t = p.tok_t[tile.begin + batch + lane];
            rec = p.docrec[d];
        }
    }

    if (MODE == MODE_SAMPLE) {
        __syncthreads();
        if (threadIdx.x == 0 && wg_dense) atomicAdd(p.n_dense + (blockIdx.x & (kDenseSlots - 1)), (unsigned long long)wg_dense);
    }
    if (MODE == MODE_LOGLIK) {
        double tot = readlane_f64(wave_incl_scan(ll_acc), 63);
        if (lane == 0) ll_wave[wave] = tot;
        __syncthreads();
        if (threadIdx.x == 0) {
            double sum = 0.0;
            for (int w = 0; w < nwaves; w++) sum += ll_wave[w];
            p.out_ll[blockIdx.x] = sum;
        }
    }
}

// The bottom tree level (inclusive binary32 prefix sums of one Bhat row), rebuilt as the sampler's dense branch
// sees it; one wavefront per (row, 64-topic block).  rows[m][K] holds the Bhat rows of words[m].  Export / test aid.
__global__ void prefix_export_kernel(const float *rows, const double *l3_64, const int32_t *words, int m, int K, int n3,
                                     float *out) {
    const int nblk = (K + kWave - 1) / kWave;
    const int item = blockIdx.x, wi = item / nblk, blk = item % nblk, lane = lane_id();
    if (wi >= m) return;
    const size_t v = (size_t)words[wi];
    const int k = blk * kWave + lane;
    const double base = blk > 0 ? l3_64[v * (size_t)n3 + (size_t)(blk - 1)] : 0.0;
    const float f = k < K ? rows[(size_t)wi * (size_t)K + (size_t)k] : 0.f;
    const float c = (float)(base + wave_incl_scan((double)f));
    if (k < K) out[(size_t)wi * (size_t)K + (size_t)k] = c;
}

// ---------------------------------------------------------------------------------------------
// CountByVZ for the words with dense rows of B.  The assignments arrive word-major (z_wm), so a word's tokens are
// one contiguous segment; it is cut into slabs and each workgroup histograms one slab in LDS and adds the
// non-zero bins to the word's row: at most min(slab, K) global atomics per slab instead of one per token.
// Rows must be zero on entry (the Bhat kernel clears them after reading).  K too large for an LDS histogram:
// one global atomic per token.
// ---------------------------------------------------------------------------------------------
struct VzItem { int32_t row; int32_t count; int64_t begin; };   // slab: count tokens from z_wm[begin] on

// f(topic) for each of the n assignments at zs, the workgroup's threads sharing the work: 16-byte loads (8 or 4
// assignments per lane and load) over the aligned middle, single loads for the unaligned head and the tail.
// A one-assignment-per-load loop is bound by the latency of its dependent loads, not by bandwidth.
template <typename ZT, typename F>
__device__ __forceinline__ void block_for_each_z(const ZT *__restrict__ zs, int64_t n, F f) {
    constexpr int kPer = 16 / (int)sizeof(ZT);
    int64_t head = (int64_t)(((16u - (unsigned)(reinterpret_cast<uintptr_t>(zs) & 15u)) & 15u) / sizeof(ZT));
    if (head > n) head = n;
    for (int64_t i = threadIdx.x; i < head; i += blockDim.x) f((uint32_t)zs[i]);
    const int64_t nvec = (n - head) / kPer;
    const uint4 *__restrict__ v = reinterpret_cast<const uint4 *>(zs + head);
    // the next 16 bytes are requested before the current ones are handed to f: f's work (LDS atomics, as a rule)
    // does not depend on them, so their latency passes under it
    int64_t j = threadIdx.x;
    uint4 q = make_uint4(0u, 0u, 0u, 0u);
    if (j < nvec) q = v[j];
    while (j < nvec) {
        const int64_t jn = j + blockDim.x;
        uint4 qn = make_uint4(0u, 0u, 0u, 0u);
        if (jn < nvec) qn = v[jn];
        if (sizeof(ZT) == 2) {
            f(q.x & 0xffffu); f(q.x >> 16); f(q.y & 0xffffu); f(q.y >> 16);
            f(q.z & 0xffffu); f(q.z >> 16); f(q.w & 0xffffu); f(q.w >> 16);
        } else {
            f(q.x); f(q.y); f(q.z); f(q.w);
        }
        q = qn; j = jn;
    }
    for (int64_t i = head + nvec * kPer + threadIdx.x; i < n; i += blockDim.x) f((uint32_t)zs[i]);
}

template <typename ZT>
__global__ void __launch_bounds__(1024) count_vz_kernel(const VzItem *items, const ZT *z_wm, int32_t *cwk, int K,
                                                        int Kpad, int use_lds) {
    extern __shared__ uint32_t vz_hist[];
    const VzItem it = items[blockIdx.x];
    const ZT *__restrict__ zs = z_wm + it.begin;
    int32_t *row = cwk + (size_t)it.row * (size_t)Kpad;
    if (use_lds) {
        for (int k = threadIdx.x; k < K; k += blockDim.x) vz_hist[k] = 0u;
        __syncthreads();
        block_for_each_z(zs, (int64_t)it.count, [&](uint32_t k) { atomicAdd(&vz_hist[k], 1u); });
        __syncthreads();
        for (int k = threadIdx.x; k < K; k += blockDim.x) {
            const uint32_t h = vz_hist[k];
            if (h) atomicAdd(&row[k], (int)h);
        }
    } else {
        block_for_each_z(zs, (int64_t)it.count, [&](uint32_t k) { atomicAdd(&row[k], 1); });
    }
}

// Host streaming: a chunk's assignments in document order (relative to the chunk's first token) out of the
// word-major copy; the inverse of fill_zwm_kernel.
template <typename ZT>
__global__ void scatter_zwm_kernel(const Tile *tiles, const uint32_t *tok_t, const ZT *z_wm, ZT *z_chunk) {
    const Tile tile = tiles[blockIdx.x];
    for (int i = threadIdx.x; i < tile.count; i += blockDim.x)
        z_chunk[tok_t[tile.begin + i]] = z_wm[tile.wm_begin + i];
}

// Host streaming: the document of every token of a chunk, from the canonical token numbers, with one 16-byte
// look-up per token.  blocks[b] describes the canonical tokens 64 b .. 64 b + 63: .x = ordinal (among the non-empty
// documents) of the document that holds token 64 b, .y/.z = 64-bit mask whose bit j > 0 says that token 64 b + j is
// the first of its document.  The ordinal of token t's document is .x plus the mask bits up to t's own; ne_doc
// maps ordinals to document numbers when the corpus has empty documents (null: they are the same).
__global__ void expand_tok_doc_kernel(const uint32_t *__restrict__ tok_t, int64_t n, int64_t t0,
                                      const uint4 *__restrict__ blocks, const int32_t *__restrict__ ne_doc,
                                      int32_t *__restrict__ tok_doc) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int64_t t = t0 + (int64_t)tok_t[i];
        const uint4 q = blocks[t >> 6];
        const unsigned long long mask = (((unsigned long long)q.z << 32) | (unsigned long long)q.y) & (~0ull >> (63 - (int)(t & 63)));
        const int32_t ord = (int32_t)q.x + (int32_t)__popcll(mask);
        tok_doc[i] = ne_doc ? ne_doc[ord] : ord;
    }
}

// word-major copy of the assignments (after init / set_z; during iterations the E-step writes it)
template <typename ZT>
__global__ void fill_zwm_kernel(const Tile *tiles, const uint32_t *tok_t, const ZT *z, int64_t z_rel, ZT *z_wm) {
    const Tile tile = tiles[blockIdx.x];
    for (int i = threadIdx.x; i < tile.count; i += blockDim.x)
        z_wm[tile.wm_begin + i] = z[z_rel + (int64_t)tok_t[tile.begin + i]];
}

// ---------------------------------------------------------------------------------------------
// Block-wide exclusive scan of one uint32 per thread; returns the exclusive prefix, *total = block sum.
// scratch must hold blockDim.x/64 + 1 values.  Contains two __syncthreads() when the block has several wavefronts.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *scratch, uint32_t *total) {
    const int lane = lane_id(), wave = threadIdx.x / kWave, nwaves = (blockDim.x + kWave - 1) / kWave;
    const uint32_t incl = wave_incl_scan(v);
    if (blockDim.x <= kWave) {   // a single wavefront needs neither LDS nor barriers
        *total = readlane_u32(incl, kWave - 1);
        return incl - v;
    }
    if (lane == kWave - 1) scratch[wave] = incl;
    __syncthreads();
    uint32_t off = 0, tot = 0;
    for (int w = 0; w < nwaves; w++) { const uint32_t s = scratch[w]; if (w < wave) off += s; tot += s; }
    __syncthreads();
    *total = tot;
    return off + incl - v;
}

// ---------------------------------------------------------------------------------------------
// Segmented count of a short segment by one wavefront, in registers: the sort-and-count of Sec. 3.3 taken
// literally.  Lane i holds assignment i (lanes past the end an all-ones key); a bitonic network of 21
// compare-exchange steps sorts the 64 keys (partners at lane ^ m: DPP quad permutations and row mirrors for m = 1,
// 2, 3, 7, 15, the LDS crossbar for the others; the lower lane of a pair keeps the smaller key).  A lane whose key
// differs from its left neighbour's starts a topic: the number of such lanes before it is the topic's slot in the
// row, the distance to the next such lane (both read off the wave-wide mask of these lanes) its count, and the
// lane stores the entry.  Segments of 65 to 128 assignments hold two keys per lane and add one merge stage.  About
// 90 vector instructions per segment (200 with two keys per lane) where the bitmap version below spends 390: it
// clears, scans and enumerates K / 32 bitmap words whatever the segment's length.
// ---------------------------------------------------------------------------------------------
template <int XOR>
__device__ __forceinline__ uint32_t sort_exchange(uint32_t v, int lane) {
    uint32_t o;
    if (XOR == 1) o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true);            // quad_perm [1,0,3,2]
    else if (XOR == 2) o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, true);       // quad_perm [2,3,0,1]
    else if (XOR == 3) o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x1B, 0xf, 0xf, true);       // quad_perm [3,2,1,0]
    else if (XOR == 7) o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, true);      // row_half_mirror
    else if (XOR == 15) o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, true);     // row_mirror
    else if (XOR < 32) o = (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, (XOR << 10) | 0x1f);   // lane ^ XOR inside 32 lanes
    else o = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ XOR) << 2, (int)v);
    // lanes that are the upper one of their pair (the highest bit of XOR is set in the lane number)
    constexpr unsigned long long upper = XOR >= 32 ? 0xffffffff00000000ull : XOR >= 16 ? 0xffff0000ffff0000ull
                                       : XOR >= 8 ? 0xff00ff00ff00ff00ull : XOR >= 4 ? 0xf0f0f0f0f0f0f0f0ull
                                       : XOR >= 2 ? 0xccccccccccccccccull : 0xaaaaaaaaaaaaaaaaull;
    // the lower lane takes the partner's key if its own is larger, the upper lane if its own is not larger
    const unsigned long long take = __builtin_amdgcn_ballot_w64(v > o) ^ upper;
    return __builtin_amdgcn_inverse_ballot_w64(take) ? o : v;
}

// the 64 keys of one register, ascending over the lanes
__device__ __forceinline__ uint32_t sort64(uint32_t v, int lane) {
    v = sort_exchange<1>(v, lane);
    v = sort_exchange<3>(v, lane); v = sort_exchange<1>(v, lane);
    v = sort_exchange<7>(v, lane); v = sort_exchange<2>(v, lane); v = sort_exchange<1>(v, lane);
    v = sort_exchange<15>(v, lane); v = sort_exchange<4>(v, lane); v = sort_exchange<2>(v, lane); v = sort_exchange<1>(v, lane);
    v = sort_exchange<31>(v, lane); v = sort_exchange<8>(v, lane); v = sort_exchange<4>(v, lane); v = sort_exchange<2>(v, lane);
    v = sort_exchange<1>(v, lane);
    v = sort_exchange<63>(v, lane); v = sort_exchange<16>(v, lane); v = sort_exchange<8>(v, lane); v = sort_exchange<4>(v, lane);
    v = sort_exchange<2>(v, lane); v = sort_exchange<1>(v, lane);
    return v;
}
// two ascending registers of 64 keys -> one ascending sequence of 128 (v0's lanes, then v1's): the last stage of the network
__device__ __forceinline__ void merge128(uint32_t &v0, uint32_t &v1, int lane) {
    const uint32_t o1 = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ 63) << 2, (int)v1);   // key 127 - i for key i
    const uint32_t o0 = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ 63) << 2, (int)v0);
    v0 = min(v0, o1); v1 = max(v1, o0);
    v0 = sort_exchange<32>(v0, lane); v0 = sort_exchange<16>(v0, lane); v0 = sort_exchange<8>(v0, lane);
    v0 = sort_exchange<4>(v0, lane); v0 = sort_exchange<2>(v0, lane); v0 = sort_exchange<1>(v0, lane);
    v1 = sort_exchange<32>(v1, lane); v1 = sort_exchange<16>(v1, lane); v1 = sort_exchange<8>(v1, lane);
    v1 = sort_exchange<4>(v1, lane); v1 = sort_exchange<2>(v1, lane); v1 = sort_exchange<1>(v1, lane);
}

// R = 1: segments of at most 64 assignments; R = 2: of at most 128, two keys per lane (lane i holds keys i and 64 + i).
template <typename ZT, int R>
__device__ __forceinline__ void count_segment_wave(const ZT *__restrict__ zs, int len, uint2 *rec, uint32_t *__restrict__ row,
                                                   uint32_t topic_bits) {
    const int lane = lane_id();
    constexpr uint32_t kNone = 0xffffffffu;
    uint32_t v0 = lane < len ? (uint32_t)zs[lane] : kNone;
    uint32_t v1 = R > 1 && lane + kWave < len ? (uint32_t)zs[lane + kWave] : kNone;
    v0 = sort64(v0, lane);
    if (R > 1) { v1 = sort64(v1, lane); merge128(v0, v1, lane); }
    // the i-th smallest key now sits at position i (v0's lanes, then v1's); the all-ones keys follow the len real ones.
    // A key that differs from its left neighbour starts a topic: its slot in the row is the number of such keys
    // before it, its count the distance to the next one (or to the end of the segment).
    const uint32_t left0 = (uint32_t)__builtin_amdgcn_update_dpp((int)0xfffffffeu, (int)v0, 0x138, 0xf, 0xf, false);   // wave_shr:1
    const unsigned long long h0 = __builtin_amdgcn_ballot_w64(v0 != kNone && v0 != left0);
    unsigned long long h1 = 0ull;
    if (R > 1) {
        const uint32_t left1 = (uint32_t)__builtin_amdgcn_update_dpp((int)readlane_u32(v0, kWave - 1), (int)v1, 0x138, 0xf, 0xf, false);
        h1 = __builtin_amdgcn_ballot_w64(v1 != kNone && v1 != left1);
    }
    const int n0 = (int)__builtin_popcountll(h0), kd = n0 + (int)__builtin_popcountll(h1);
    const int after0 = h1 ? kWave + (int)__builtin_ctzll(h1) : len;        // first topic start behind v0's keys
    {
        const unsigned long long above = (h0 >> lane) >> 1;                // topic starts at the lanes above this one
        const int next = above ? lane + 1 + (int)__builtin_ctzll(above) : after0;
        const uint32_t slot = __builtin_amdgcn_mbcnt_hi((uint32_t)(h0 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)h0, 0u));
        if (__builtin_amdgcn_inverse_ballot_w64(h0)) row[slot] = v0 | ((uint32_t)(next - lane) << topic_bits);
    }
    if (R > 1 && h1) {
        const unsigned long long above = (h1 >> lane) >> 1;
        const int next = above ? lane + 1 + (int)__builtin_ctzll(above) : len - kWave;   // in v1's own numbering
        const uint32_t slot = (uint32_t)n0 + __builtin_amdgcn_mbcnt_hi((uint32_t)(h1 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)h1, 0u));
        if (__builtin_amdgcn_inverse_ballot_w64(h1)) row[slot] = v1 | ((uint32_t)(next - lane) << topic_bits);
    }
    // pad to the next multiple of 4 entries with (last topic, count 0), as the kernel below does
    const uint32_t last = R > 1 && len > kWave ? readlane_u32(v1, len - kWave - 1) : readlane_u32(v0, len - 1);
    if (lane < ((kd + 3) & ~3) - kd) row[kd + lane] = last;
    if (lane == 0) rec->y = (uint32_t)kd;
}

// ---------------------------------------------------------------------------------------------
// CountByDZ (Alg. 1; the "segmented count" of Sec. 3.3), one workgroup per document.
// The document's assignments are contiguous (z is kept in document order, so the "shuffle" of Sec. 3.3
// is the E-step's scattered store).  Instead of sorting, the workgroup marks the topics present in a
// K-bit LDS bitmap; popcount prefix sums over the bitmap give every present topic its rank, i.e. its
// slot in the ascending row; counts are accumulated per slot with LDS atomics.
// Rows whose K_d exceeds lds_entries are accumulated directly in the global row.
// ---------------------------------------------------------------------------------------------
// z[0] is the assignment at position z_first of the segment numbering (a streaming buffer holds one chunk only).
template <typename ZT>
__global__ void __launch_bounds__(1024) count_dz_kernel(const int32_t *doc_list, const int64_t *doc_ptr,
                                                        const ZT *z, int64_t z_first, uint2 *docrec, uint32_t *cd_ent, int K,
                                                        uint32_t topic_bits, int nwords, int lds_entries) {
    extern __shared__ uint32_t lds_u32[];
    __shared__ uint32_t scan_scratch[20];
    uint32_t *bitmap = lds_u32;            // [nwords]
    uint32_t *wpre = lds_u32 + nwords;     // [nwords] exclusive popcount prefix
    uint32_t *ent_lds = wpre + nwords;     // [lds_entries]
    const int d = doc_list[blockIdx.x];
    const int64_t begin = doc_ptr[d];
    const int len = (int)(doc_ptr[d + 1] - begin);
    if (len == 0) { if (threadIdx.x == 0) docrec[d].y = 0u; return; }
    const ZT *__restrict__ zd = z + (begin - z_first);
    if (blockDim.x == kWave && len <= 2 * kWave) {   // a short segment and a single wavefront: sorted in registers
        uint32_t *row = cd_ent + (size_t)docrec[d].x * 32u;
        if (len <= kWave) count_segment_wave<ZT, 1>(zd, len, docrec + d, row, topic_bits);
        else count_segment_wave<ZT, 2>(zd, len, docrec + d, row, topic_bits);
        return;
    }

    for (int w = threadIdx.x; w < nwords; w += blockDim.x) bitmap[w] = 0u;
    __syncthreads();
    block_for_each_z(zd, (int64_t)len, [&](uint32_t k) { atomicOr(&bitmap[k >> 5], 1u << (k & 31u)); });
    __syncthreads();
    // ranks: exclusive prefix of popcounts over the bitmap words.  Every thread takes a contiguous piece of the
    // bitmap (ascending topics), so one scan over the threads' totals serves all words
    const int wpt = (nwords + (int)blockDim.x - 1) / (int)blockDim.x;
    const int wb = min((int)threadIdx.x * wpt, nwords), we = min(wb + wpt, nwords);
    uint32_t mine = 0;
    for (int w = wb; w < we; w++) mine += (uint32_t)__popc(bitmap[w]);
    uint32_t total;
    const uint32_t first = block_excl_scan(mine, scan_scratch, &total);
    const int kd = (int)total;
    uint32_t *row = cd_ent + (size_t)docrec[d].x * 32u;
    const bool in_lds = kd <= lds_entries;
    uint32_t *ent = in_lds ? ent_lds : row;
    // slot r of the row starts as (topic, count 0): enumerate the set bits of the thread's words
    {
        uint32_t r = first;
        for (int w = wb; w < we; w++) {
            uint32_t m = bitmap[w];
            wpre[w] = r;
            while (m) { const int b = __ffs((int)m) - 1; m &= m - 1u; ent[r++] = (uint32_t)(w * 32 + b); }
        }
    }
    __syncthreads();
    block_for_each_z(zd, (int64_t)len, [&](uint32_t k) {
        const uint32_t wd = bitmap[k >> 5];
        const uint32_t r = wpre[k >> 5] + (uint32_t)__popc(wd & ((1u << (k & 31u)) - 1u));
        atomicAdd(&ent[r], 1u << topic_bits);
    });
    __syncthreads();
    if (in_lds)
        for (int r = threadIdx.x; r < kd; r += blockDim.x) row[r] = ent_lds[r];
    // pad to the next multiple of 4 entries with (last topic, count 0): the sampler reads rows in 16-byte pieces,
    // and a draw that rounding pushes past the end of the row then still lands on the last topic
    if (threadIdx.x < 4) {
        const int r = kd + (int)threadIdx.x;
        if (r < ((kd + 3) & ~3)) row[r] = ent[kd - 1] & ((1u << topic_bits) - 1u);
    }
    if (threadIdx.x == 0) docrec[d].y = (uint32_t)kd;
}

// ---------------------------------------------------------------------------------------------
// Topic totals C_k = sum_v B_vk, computed as the histogram of z (same numbers, 20x fewer bytes than
// column sums of B at K = 10^4).  LDS histogram when K fits, else global atomics.
// ---------------------------------------------------------------------------------------------
template <typename ZT>
__global__ void __launch_bounds__(1024) topic_totals_kernel(const ZT *z, int64_t T, int64_t per_block, unsigned long long *ck, int K,
                                                            int use_lds) {
    extern __shared__ uint32_t hist[];
    const int64_t b = (int64_t)blockIdx.x * per_block;
    int64_t e = b + per_block; if (e > T) e = T;
    if (use_lds) {
        for (int k = threadIdx.x; k < K; k += blockDim.x) hist[k] = 0u;
        __syncthreads();
        block_for_each_z(z + b, e - b, [&](uint32_t k) { atomicAdd(&hist[k], 1u); });
        __syncthreads();
        for (int k = threadIdx.x; k < K; k += blockDim.x) { const uint32_t h = hist[k]; if (h) atomicAdd(&ck[k], (unsigned long long)h); }
    } else {
        block_for_each_z(z + b, e - b, [&](uint32_t k) { atomicAdd(&ck[k], 1ull); });
    }
}

// ---------------------------------------------------------------------------------------------
// Preprocess + BuildTree (Alg. 1; Eq. 2; Sec. 3.2.4), one workgroup of 256 threads per word row.
//   Bhat_vk  = (float(B_vk) + beta) / denom_k,  denom_k = float(C_k) + float(V) * beta   -- single-rounded fp32 ops
//   l3_64[i] = running sum of Bhat_v through topic (i+1)*64 - 1, accumulated in binary64
//   l3[i]    = round32(l3_64[i])                                           -- tree level above the bottom, W = 64
// Pad columns k in [K, Kpad) get Bhat = 0, so the last block's running sum is the row total.
// The bottom level (one prefix sum per topic) is not stored; the sampler rebuilds the 64 entries it needs.
// The row of B is cleared after it has been read, ready for the next CountByVZ.
// ---------------------------------------------------------------------------------------------
// Denominators of Eq. 2, one per topic: float(C_k) + float(V) * beta (the conversion rounds to nearest even).
__global__ void denominators_kernel(const unsigned long long *ck, float *denom, int K, float vbeta) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k < K) denom[k] = (float)ck[k] + vbeta;
}

// row_word[r] is the word of dense row r (the tree levels are indexed by word); the last row is an all-zero
// row that yields the base vector (Bhat of a zero count) and its running sums for the light words.
__global__ void __launch_bounds__(256) phi_tree_kernel(int32_t *cwk, const float *denom, float *phi, float *l3,
                                                       double *l3_64, float *sumphi, const int32_t *row_word, int K,
                                                       int Kpad, int n3, int n3pad, float beta, int clear_cwk) {
    __shared__ double wave_tot[4];
    __shared__ float row_total;
    const int v = row_word[blockIdx.x];
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const size_t rbase = (size_t)blockIdx.x * (size_t)Kpad;
    double carry = 0.0;
    for (int base = 0; base < Kpad; base += 1024) {
        const int k0 = base + (int)threadIdx.x * 4;
        float f[4] = {0.f, 0.f, 0.f, 0.f};
        if (k0 < Kpad) {   // Kpad is a multiple of 64, so k0..k0+3 are all inside the padded row
            const int4 c = *reinterpret_cast<const int4 *>(cwk + rbase + k0);
            const int cc[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const int k = k0 + q;
                if (k < K) {
                    const float num = (float)cc[q] + beta;
                    f[q] = num / denom[k];
                }
            }
            *reinterpret_cast<float4 *>(phi + rbase + k0) = make_float4(f[0], f[1], f[2], f[3]);
            if (clear_cwk) *reinterpret_cast<int4 *>(cwk + rbase + k0) = make_int4(0, 0, 0, 0);
        }
        const double s3 = (((double)f[0] + (double)f[1]) + (double)f[2]) + (double)f[3];
        const double incl = wave_incl_scan(s3);
        if (lane == kWave - 1) wave_tot[wave] = incl;
        __syncthreads();
        double woff = 0.0, btot = 0.0;
#pragma unroll
        for (int w = 0; w < 4; w++) { const double tw = wave_tot[w]; if (w < wave) woff += tw; btot += tw; }
        if (k0 < Kpad && ((k0 + 3) & (kWave - 1)) == kWave - 1) {
            const double run = carry + woff + incl;       // running sum through topic k0+3, the end of a block
            const int i = (k0 + 3) / kWave;
            l3_64[(size_t)v * (size_t)n3 + (size_t)i] = run;
            l3[(size_t)v * (size_t)n3pad + (size_t)i] = (float)run;
            if (i == n3 - 1) row_total = (float)run;
        }
        carry += btot;
        __syncthreads();
    }
    const float total = row_total;   // written before the loop's last barrier
    for (int i = n3 + (int)threadIdx.x; i < n3pad; i += blockDim.x) l3[(size_t)v * (size_t)n3pad + i] = total;
    if (threadIdx.x == 0) sumphi[v] = total;
}

// ---------------------------------------------------------------------------------------------
// Preprocess + BuildTree for the light words (one wavefront per word).  Their Bhat row is the base vector
// except at the word's non-zeros, so only those are evaluated (Eq. 2, same three binary32 operations) and
// stored next to the entries.  The running sums at the block ends follow from the base vector's running sums
// plus the cumulative difference (Bhat - base) of the non-zeros up to each block, all in binary64: the same
// sum of the same binary32 numbers as for a dense row, associated differently.
// LDS: n3 doubles (cumulative difference at the last non-zero of each block) + n3 flags.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) light_tree_kernel(const int32_t *light_words, const uint2 *wrec,
                                                        const uint32_t *lw_ent, float *lw_phi, const float *denom,
                                                        const float *base, const double *basecum, float *l3,
                                                        double *l3_64, float *sumphi, int n3, int n3pad,
                                                        uint32_t topic_bits, float beta) {
    extern __shared__ double lds_dcum[];
    int *written = reinterpret_cast<int *>(lds_dcum + n3);
    const int v = light_words[blockIdx.x], lane = lane_id();
    const uint2 wr = wrec[blockIdx.x];
    const int nnz = (int)wr.y;
    const uint32_t *__restrict__ ent = lw_ent + (size_t)wr.x * 32u;
    float *__restrict__ val = lw_phi + (size_t)wr.x * 32u;
    const uint32_t tmask = (1u << topic_bits) - 1u;
    for (int i = lane; i < n3; i += kWave) written[i] = 0;
    __syncthreads();
    double carry = 0.0;
    for (int j0 = 0; j0 < nnz; j0 += kWave) {
        const int j = j0 + lane;
        const bool valid = j < nnz;
        const uint32_t e = valid ? ent[j] : 0u;
        const uint32_t k = e & tmask;
        double delta = 0.0;
        if (valid) {
            const float f = ((float)(e >> topic_bits) + beta) / denom[k];
            val[j] = f;
            delta = (double)f - (double)base[k];
        }
        const double incl = wave_incl_scan(delta) + carry;
        const int blk = (int)(k >> 6);
        const int next_blk = (j + 1 < nnz) ? (int)((ent[j + 1] & tmask) >> 6) : -1;
        if (valid && blk != next_blk) { lds_dcum[blk] = incl; written[blk] = 1; }
        carry = readlane_f64(incl, 63);
    }
    __syncthreads();
    int last = -1;   // last block at or before the current one that holds a non-zero
    float total = 0.f;
    for (int i0 = 0; i0 < n3; i0 += kWave) {
        const int i = i0 + lane;
        const int w = (i < n3 && written[i]) ? i : -1;
        const int idx = max(wave_incl_scan_max(w), last);
        if (i < n3) {
            const double run = basecum[i] + (idx >= 0 ? lds_dcum[idx] : 0.0);
            l3_64[(size_t)v * (size_t)n3 + (size_t)i] = run;
            l3[(size_t)v * (size_t)n3pad + (size_t)i] = (float)run;
            if (i == n3 - 1) total = (float)run;
        }
        last = __builtin_amdgcn_readlane(idx, 63);
    }
    total = readlane_f32(total, (n3 - 1) & (kWave - 1));
    for (int i = n3 + lane; i < n3pad; i += kWave) l3[(size_t)v * (size_t)n3pad + i] = total;
    if (lane == 0) sumphi[v] = total;
}

// Dense image of light words' rows for export: out[i][k] = base[k] (Bhat) or 0 (counts), then the non-zeros.
__global__ void light_rows_export_kernel(const int32_t *light_ids, int m, const uint2 *wrec, const uint32_t *lw_ent,
                                         const float *lw_phi, const float *base, int K, uint32_t topic_bits,
                                         float *out_phi, int32_t *out_cnt) {
    const int i = blockIdx.x;
    if (i >= m) return;
    const uint2 wr = wrec[light_ids[i]];
    const uint32_t tmask = (1u << topic_bits) - 1u;
    for (int k = threadIdx.x; k < K; k += blockDim.x) {
        if (out_phi) out_phi[(size_t)i * (size_t)K + k] = base[k];
        if (out_cnt) out_cnt[(size_t)i * (size_t)K + k] = 0;
    }
    __syncthreads();
    for (int j = threadIdx.x; j < (int)wr.y; j += blockDim.x) {
        const uint32_t e = lw_ent[(size_t)wr.x * 32u + j];
        if (out_phi) out_phi[(size_t)i * (size_t)K + (e & tmask)] = lw_phi[(size_t)wr.x * 32u + j];
        if (out_cnt) out_cnt[(size_t)i * (size_t)K + (e & tmask)] = (int32_t)(e >> topic_bits);
    }
}

// Statistics for the bandwidth model (exact in binary64 below 2^53): nnz(A), sum_d K_d * L_d (row entries
// touched if every token read its row) and sum_d K_d * U_d, U_d = distinct words of document d inside its
// chunk (row entries the sampler has to fetch: consecutive tokens of one (word, document) pair share the row).
__global__ void row_stats_kernel(const uint2 *docrec, const int64_t *doc_ptr, const uint32_t *doc_words, int64_t D,
                                 unsigned long long *out3) {
    double nnz = 0.0, reads = 0.0, fetch = 0.0;
    for (int64_t d = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; d < D; d += (int64_t)gridDim.x * blockDim.x) {
        const double kd = (double)docrec[d].y;
        nnz += kd; reads += kd * (double)(doc_ptr[d + 1] - doc_ptr[d]); fetch += kd * (double)doc_words[d];
    }
    nnz = readlane_f64(wave_incl_scan(nnz), 63); reads = readlane_f64(wave_incl_scan(reads), 63);
    fetch = readlane_f64(wave_incl_scan(fetch), 63);
    __shared__ double part[3][16];
    const int wave = threadIdx.x / kWave, nwaves = blockDim.x / kWave;
    if (lane_id() == 0) { part[0][wave] = nnz; part[1][wave] = reads; part[2][wave] = fetch; }
    __syncthreads();
    if (threadIdx.x < 3) {
        double sum = 0.0;
        for (int w = 0; w < nwaves; w++) sum += part[threadIdx.x][w];
        atomicAdd(&out3[threadIdx.x], (unsigned long long)sum);
    }
}

// Sum of the dense-branch counter slots, added to *out.
__global__ void sum_slots_kernel(const unsigned long long *slots, int n, unsigned long long *out) {
    unsigned long long v = 0;
    for (int i = threadIdx.x; i < n; i += blockDim.x) v += slots[i];
    __shared__ unsigned long long tot;
    if (threadIdx.x == 0) tot = 0ull;
    __syncthreads();
    if (v) atomicAdd(&tot, v);
    __syncthreads();
    if (threadIdx.x == 0 && tot) atomicAdd(out, tot);
}

// Non-zeros of the sparse rows of B (what the next E-step stages for the light words), added to *out.
__global__ void light_stats_kernel(const uint2 *wrec, int n, unsigned long long *out) {
    uint32_t nnz = 0;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) nnz += wrec[i].y;
    nnz = wave_sum(nnz);
    if (lane_id() == 0 && nnz) atomicAdd(out, (unsigned long long)nnz);
}

// ---------------------------------------------------------------------------------------------
// Log-likelihood reduction (the per-token log-likelihood is the quality metric of Sec. 4): binary64 sums in a
// fixed order, so the result is the same in every run.  kReduceBlocks workgroups of kReduceThreads threads: thread
// i of workgroup b adds the elements b * kReduceThreads + i, + kReduceBlocks * kReduceThreads, ...; lanes are
// combined by a DPP scan, wavefronts and workgroups in index order.
// ---------------------------------------------------------------------------------------------
constexpr int kReduceBlocks = 256, kReduceThreads = 256;

__device__ __forceinline__ double block_sum_f64(double v, double *wave_part) {
    const double w = readlane_f64(wave_incl_scan(v), 63);
    if (lane_id() == 0) wave_part[threadIdx.x / kWave] = w;
    __syncthreads();
    double sum = 0.0;
    for (int i = 0; i < (int)(blockDim.x / kWave); i++) sum += wave_part[i];
    __syncthreads();
    return sum;
}

// block_part[b] = sum of workgroup b's share of in[0..n)
__global__ void __launch_bounds__(kReduceThreads) reduce_partials_kernel(const double *in, int64_t n, double *block_part) {
    __shared__ double wave_part[kReduceThreads / kWave];
    double v = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kReduceThreads + threadIdx.x; i < n; i += (int64_t)kReduceBlocks * kReduceThreads) v += in[i];
    const double sum = block_sum_f64(v, wave_part);
    if (threadIdx.x == 0) block_part[blockIdx.x] = sum;
}

// block_part[b] = workgroup b's share of sum_d w_d ln(len_d + K alpha), w_d = wptr[d+1] - wptr[d] and
// len_d = lptr[d+1] - lptr[d]: the normaliser of theta_d, once per token that is scored in document d.
__global__ void __launch_bounds__(kReduceThreads) doc_norm_kernel(const int64_t *wptr, const int64_t *lptr, int64_t D,
                                                                   double k_alpha, double *block_part) {
    __shared__ double wave_part[kReduceThreads / kWave];
    double v = 0.0;
    for (int64_t d = (int64_t)blockIdx.x * kReduceThreads + threadIdx.x; d < D; d += (int64_t)kReduceBlocks * kReduceThreads) {
        const int64_t w = wptr[d + 1] - wptr[d];
        if (w > 0) v += (double)w * log((double)(lptr[d + 1] - lptr[d]) + k_alpha);
    }
    const double sum = block_sum_f64(v, wave_part);
    if (threadIdx.x == 0) block_part[blockIdx.x] = sum;
}

// *acc = (add ? *acc : 0) + sum of block_part[0..kReduceBlocks); one workgroup
__global__ void __launch_bounds__(kReduceThreads) reduce_final_kernel(const double *block_part, double *acc, int add) {
    __shared__ double wave_part[kReduceThreads / kWave];
    const double sum = block_sum_f64(threadIdx.x < kReduceBlocks ? block_part[threadIdx.x] : 0.0, wave_part);
    if (threadIdx.x == 0) *acc = (add ? *acc : 0.0) + sum;
}

// *out = (*sum_ln - *norm) / tokens: the per-token log-likelihood
__global__ void loglik_finish_kernel(const double *sum_ln, const double *norm, double tokens, double *out) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *out = (*sum_ln - *norm) / tokens;
}

// Plain streaming copy (16 bytes per lane per step): the yardstick for achievable HBM bandwidth and the
// calibration kernel for the profiler's FETCH_SIZE / WRITE_SIZE counters.
__global__ void copy_probe_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace saber
