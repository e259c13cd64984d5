// Ablation variants of two steps (the decomposition G0..G3 of Sec. 4.2, re-measured on this GPU).  They compute
// the same results as the regular kernels with the design decision in question taken the other way:
//   * estep_docmajor_kernel: tokens sampled in document order (the order before PDOW, Sec. 3.1.3): a document's row
//     of A is fetched once, but every token gathers from the Bhat row of another word, out of global memory;
//   * key / mark / count kernels: A rebuilt by sorting all (document, topic) pairs (the rebuild before the
//     shuffle-and-segmented-count of Sec. 3.3); the sort itself is rocPRIM's radix sort.
// Selected by saber_options.ablation; not on the default path.
#pragma once
#include "saber_kernels.hpp"

namespace saber {

struct DocMajorParams {
    const int64_t *doc_ptr;     // [D+1]
    const int32_t *word_ids;    // [T] canonical order
    const int32_t *word_row;    // [V] row of the word in phi / cwk (every word keeps a dense row in this variant)
    const uint2 *docrec;
    const uint32_t *cd_ent;
    const float *phi, *l3, *sumphi;
    const double *l3_64;
    void *z;
    unsigned long long *n_dense;
    int64_t D;
    int K, Kpad, n3, n3pad;
    uint32_t topic_bits, topic_mask;
    float alpha;
    uint32_t seed_lo, seed_hi, iter;
};

// One wavefront per document, the document's tokens one after another in their canonical order.  The arithmetic
// of a token is that of estep_kernel (same helpers, same order of additions), so the assignments are the same;
// only where the operands come from differs.
template <typename ZT>
__global__ void __launch_bounds__(256) estep_docmajor_kernel(DocMajorParams p) {
    const int lane = lane_id();
    const int64_t d = (int64_t)blockIdx.x * (int64_t)(blockDim.x / kWave) + (int64_t)(threadIdx.x / kWave);
    if (d >= p.D) return;                         // wave-uniform
    const int64_t begin = p.doc_ptr[d], end = p.doc_ptr[d + 1];
    if (end <= begin) return;
    const uint2 rec = p.docrec[d];
    const int kd = (int)rec.y;
    const uint32_t *row = p.cd_ent + (size_t)rec.x * 32u;
    const int nblk = (kd + 4 * kWave - 1) / (4 * kWave);
    const uint32_t bits = p.topic_bits, tmask = p.topic_mask;
    const uint4 e0 = load_block(row, kd, lane);   // first 256 entries of the document's row stay in registers
    uint4 e1 = make_uint4(0u, 0u, 0u, 0u);
    if (nblk >= 2) e1 = load_block(row + 4 * kWave, kd - 4 * kWave, lane);
    uint32_t dense_count = 0;

    for (int64_t b = begin; b < end; b += kWave) {
        const int n = (int)((end - b) < (int64_t)kWave ? (end - b) : (int64_t)kWave);
        const bool act = lane < n;
        const int64_t t = b + lane;
        const int v = act ? p.word_ids[t] : 0;
        const int my_row = act ? p.word_row[v] : 0;
        const float my_sum = act ? p.sumphi[v] : 0.f;
        const Rand2 r = philox_token(p.seed_lo, p.seed_hi, (uint64_t)t, p.iter);
        const float u0 = unit24(r.r0), u1 = unit24(r.r1);
        uint32_t my_z = 0;
        unsigned long long dense_mask = 0ull;

        for (int j = 0; j < n; j++) {
            const float *__restrict__ phi_row = p.phi + (size_t)readlane_u32((uint32_t)my_row, j) * (size_t)p.Kpad;
            const float Q = p.alpha * readlane_f32(my_sum, j);
            RowBlock b0, b1;
            block_products<false, false>(e0, bits, tmask, nullptr, phi_row, b0);
            const float t0 = readlane_f32(b0.incl, 63);
            float t1 = 0.f, S = t0;
            if (nblk >= 2) {
                block_products<false, false>(e1, bits, tmask, nullptr, phi_row, b1);
                t1 = readlane_f32(b1.incl, 63);
                S = t0 + t1;
                for (int blk = 2; blk < nblk; blk++) {
                    RowBlock bb;
                    block_products<false, false>(load_block(row + blk * 4 * kWave, kd - blk * 4 * kWave, lane), bits, tmask,
                                                 nullptr, phi_row, bb);
                    S = S + readlane_f32(bb.incl, 63);
                }
            }
            const float u0j = readlane_f32(u0, j), u1j = readlane_f32(u1, j);
            if (u0j * (S + Q) < S) {
                const float x = u1j * S;
                uint32_t topic;
                if (nblk == 1 || t0 >= x) topic = search_block(e0, b0, 0.f, x, kd, tmask);
                else if (nblk == 2 || t0 + t1 >= x) topic = search_block(e1, b1, t0, x, kd - 4 * kWave, tmask);
                else {
                    float carry = t0 + t1;
                    topic = 0u;
                    for (int blk = 2; blk < nblk; blk++) {
                        const int rel = kd - blk * 4 * kWave;
                        const uint4 e = load_block(row + blk * 4 * kWave, rel, lane);
                        RowBlock bb;
                        block_products<false, false>(e, bits, tmask, nullptr, phi_row, bb);
                        const float tot = readlane_f32(bb.incl, 63);
                        if (blk == nblk - 1 || carry + tot >= x) { topic = search_block(e, bb, carry, x, rel, tmask); break; }
                        carry = carry + tot;
                    }
                }
                my_z = llvm_amdgcn_writelane_u32(topic, (unsigned)j, my_z);
            } else {
                dense_mask |= 1ull << j;
            }
        }

        if (dense_mask) {
            // the dense term, four tokens at a time: the 16 lanes of DPP row g serve the g-th of them, each row with
            // the Bhat row and tree level of its own token's word
            dense_count += (uint32_t)__builtin_popcountll(dense_mask);
            const float xd = u1 * my_sum;
            const int g = lane >> 4, li = lane & 15;
            while (dense_mask) {
                int tl[4];
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    tl[q] = dense_mask ? (int)__builtin_ctzll(dense_mask) : -1;
                    if (dense_mask) dense_mask &= dense_mask - 1ull;
                }
                const int mine = g == 0 ? tl[0] : g == 1 ? tl[1] : g == 2 ? tl[2] : tl[3];
                const int src = (mine < 0 ? lane : mine) << 2;
                const float x = __int_as_float(__builtin_amdgcn_ds_bpermute(src, __float_as_int(xd)));
                const int vrow = __builtin_amdgcn_ds_bpermute(src, my_row);
                const int vword = __builtin_amdgcn_ds_bpermute(src, v);
                const uint32_t k = dense_query4(p.phi + (size_t)vrow * (size_t)p.Kpad, p.Kpad,
                                                p.l3 + (size_t)vword * (size_t)p.n3pad,
                                                p.l3_64 + (size_t)vword * (size_t)p.n3, p.n3, p.K, x, li);
#pragma unroll
                for (int q = 0; q < 4; q++)
                    if (tl[q] >= 0) my_z = llvm_amdgcn_writelane_u32(readlane_u32(k, 16 * q), (unsigned)tl[q], my_z);
            }
        }
        if (act) reinterpret_cast<ZT *>(p.z)[t] = (ZT)my_z;
    }
    if (lane == 0 && dense_count)
        atomicAdd(p.n_dense + (blockIdx.x & (kDenseSlots - 1)), (unsigned long long)dense_count);
}

// ---- A by sorting: keys (document << topic_bits | topic) of all tokens, one wavefront per document ----
template <typename ZT>
__global__ void __launch_bounds__(256) sort_keys_kernel(const int64_t *doc_ptr, const ZT *z, int64_t D,
                                                        uint32_t topic_bits, uint64_t *keys) {
    const int lane = lane_id();
    const int64_t d = (int64_t)blockIdx.x * (int64_t)(blockDim.x / kWave) + (int64_t)(threadIdx.x / kWave);
    if (d >= D) return;
    const int64_t begin = doc_ptr[d], end = doc_ptr[d + 1];
    for (int64_t t = begin + lane; t < end; t += kWave) keys[t] = ((uint64_t)d << topic_bits) | (uint64_t)(uint32_t)z[t];
}

// After the sort a document's keys are its segment [doc_ptr[d], doc_ptr[d+1]) again, ascending by topic.  One
// wavefront per document: every first key of a topic opens an entry (topic, count 0) at its rank in the row, every
// token notes the rank of its entry; the row's length and padding are written as CountByDZ does.
__global__ void __launch_bounds__(256) sort_mark_kernel(const int64_t *doc_ptr, const uint64_t *keys, int64_t D,
                                                        uint32_t topic_mask, uint2 *docrec, uint32_t *cd_ent,
                                                        uint32_t *rank_of) {
    const int lane = lane_id();
    const int64_t d = (int64_t)blockIdx.x * (int64_t)(blockDim.x / kWave) + (int64_t)(threadIdx.x / kWave);
    if (d >= D) return;
    const int64_t begin = doc_ptr[d], end = doc_ptr[d + 1];
    if (end <= begin) { if (lane == 0) docrec[d].y = 0u; return; }
    uint32_t *row = cd_ent + (size_t)docrec[d].x * 32u;
    uint32_t carry = 0;            // entries opened so far
    uint32_t prev_last = 0xffffffffu, last_topic = 0u;
    for (int64_t b = begin; b < end; b += kWave) {
        const int64_t t = b + lane;
        const bool act = t < end;
        const uint32_t topic = act ? (uint32_t)keys[t] & topic_mask : 0xffffffffu;
        uint32_t prev = (uint32_t)__builtin_amdgcn_update_dpp((int)0, (int)topic, 0x138, 0xf, 0xf, false);   // wave_shr:1
        if (lane == 0) prev = prev_last;
        const uint32_t flag = (act && topic != prev) ? 1u : 0u;
        const uint32_t incl = wave_incl_scan(flag);
        const uint32_t rank = carry + incl - 1u;          // entry of this token (incl >= 1 for every active lane after the first key)
        if (flag) row[rank] = topic;
        if (act) rank_of[t] = rank;
        carry += readlane_u32(incl, kWave - 1);
        const int n = (int)((end - b) < (int64_t)kWave ? (end - b) : (int64_t)kWave);
        prev_last = readlane_u32(topic, n - 1);
        last_topic = prev_last;
    }
    const int kd = (int)carry;
    if (lane < 4) {
        const int r = kd + lane;
        if (r < ((kd + 3) & ~3)) row[r] = last_topic;
    }
    if (lane == 0) docrec[d].y = (uint32_t)kd;
}

// one count per token into the entry marked for it
__global__ void __launch_bounds__(256) sort_count_kernel(const int64_t *doc_ptr, const uint32_t *rank_of, int64_t D,
                                                         const uint2 *docrec, uint32_t *cd_ent, uint32_t topic_bits) {
    const int lane = lane_id();
    const int64_t d = (int64_t)blockIdx.x * (int64_t)(blockDim.x / kWave) + (int64_t)(threadIdx.x / kWave);
    if (d >= D) return;
    const int64_t begin = doc_ptr[d], end = doc_ptr[d + 1];
    uint32_t *row = cd_ent + (size_t)docrec[d].x * 32u;
    for (int64_t t = begin + lane; t < end; t += kWave) atomicAdd(&row[rank_of[t]], 1u << topic_bits);
}

// ---- alias tables (the alternative to the tree that Sec. 3.2.3 weighs) ----
// Vose's construction for the Bhat rows of the words with dense rows, one thread per row: the pairing of an
// under-full with an over-full bucket is a chain in which every step needs the previous one's remainder, which is
// what keeps it from using a wavefront's lanes.  Bucket k keeps topic k with probability prob[k] and hands the
// rest to alias[k].  Arrays are laid out [K][nrows] so that the lanes of a wavefront (neighbouring rows) touch
// neighbouring addresses as long as they walk in step.  scaled: K * p_k in binary64 while the row is worked on;
// stack: under-full buckets from the bottom, over-full ones from the top.
__global__ void __launch_bounds__(256) alias_build_kernel(const float *__restrict__ phi, int nrows, int K, int Kpad,
                                                          double *scaled, int32_t *stack, float *prob, int32_t *alias) {
    const int r = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (r >= nrows) return;
    const float *row = phi + (size_t)r * (size_t)Kpad;
    const size_t n = (size_t)nrows;
    double tot = 0.0;
    for (int k = 0; k < K; k++) tot += (double)row[k];
    const double scale = (double)K / tot;
    int ns = 0, nl = 0;                           // stack[ns-1] .. under-full, stack[K-nl] .. over-full
    for (int k = 0; k < K; k++) {
        const double q = (double)row[k] * scale;
        scaled[(size_t)k * n + r] = q;
        if (q < 1.0) stack[(size_t)(ns++) * n + r] = k;
        else stack[(size_t)(K - 1 - nl++) * n + r] = k;
    }
    while (ns > 0 && nl > 0) {
        const int s = stack[(size_t)(--ns) * n + r];
        const int l = stack[(size_t)(K - nl) * n + r];        // top of the over-full stack
        const double qs = scaled[(size_t)s * n + r];
        prob[(size_t)s * n + r] = (float)qs;
        alias[(size_t)s * n + r] = l;
        const double ql = scaled[(size_t)l * n + r] + qs - 1.0;
        scaled[(size_t)l * n + r] = ql;
        if (ql < 1.0) {                                       // the over-full bucket became under-full: move it
            nl--;
            stack[(size_t)(ns++) * n + r] = l;
        }
    }
    // what is left is full up to rounding
    while (ns > 0) { const int s = stack[(size_t)(--ns) * n + r]; prob[(size_t)s * n + r] = 1.f; alias[(size_t)s * n + r] = s; }
    while (nl > 0) { const int l = stack[(size_t)(K - nl) * n + r]; nl--; prob[(size_t)l * n + r] = 1.f; alias[(size_t)l * n + r] = l; }
}

// the tables of the rows listed, as [m][K]
__global__ void alias_export_kernel(const int32_t *rows, int m, int nrows, int K, const float *prob, const int32_t *alias,
                                    float *out_prob, int32_t *out_alias) {
    const int64_t total = (int64_t)m * K;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int w = (int)(i / K), k = (int)(i % K);
        out_prob[i] = prob[(size_t)k * (size_t)nrows + (size_t)rows[w]];
        out_alias[i] = alias[(size_t)k * (size_t)nrows + (size_t)rows[w]];
    }
}

}  // namespace saber
