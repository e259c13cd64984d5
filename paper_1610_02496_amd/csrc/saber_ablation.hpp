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

// ---- alias tables built by a whole workgroup, and sampled from (saber_options.ablation bit 2) ----
// The sweep construction visits light items (K p_k / sum p <= 1) and heavy items in index order: the current heavy
// item fills light buckets until less than one bucket of it is left, then takes its own bucket and the next heavy
// item makes up the shortfall.  Written with prefix sums it needs no chain: with l_a = what the first a light items
// lack of a full bucket and h_b = what the first b heavy items have beyond one,
//   light item a is filled by the first heavy item b with h_(b+1) > l_a;
//   heavy item b keeps 1 + h_(b+1) - l_a of its own bucket, a = the first a with l_a >= h_(b+1), and hands the
//   rest to heavy item b + 1 (the last heavy item keeps a full bucket).
// So every item finds its partner by a binary search in the other kind's prefix sums, all items at once: the
// "vectorised" construction, against the serial pairing chain of Vose's algorithm above.
// One workgroup of 1,024 threads per row (the LDS it needs leaves room for one workgroup per CU); thread t owns the
// items [t c, (t+1) c), c = ceil(K / 1024), so that both
// kinds keep their index order.  LDS: K + 1 binary64 prefix sums (l_0..l_nL, then h_1..h_nH) and K item numbers
// (light ones first).  table[row][k] = {prob as binary32 bits, alias}: bucket k yields k with probability prob.
constexpr int kAliasThreads = 1024, kAliasWaves = kAliasThreads / kWave;
__device__ __forceinline__ void block_excl_scan2(double &a, double &b, uint32_t &n, double (*sd)[kAliasWaves + 1], uint32_t *su) {
    // exclusive scan of (a, b, n) over the workgroup's threads; totals come back in sd[0..1][kAliasWaves], su[kAliasWaves]
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const double ia = wave_incl_scan(a), ib = wave_incl_scan(b);
    const uint32_t in = wave_incl_scan(n);
    if (lane == kWave - 1) { sd[0][wave] = ia; sd[1][wave] = ib; su[wave] = in; }
    __syncthreads();
    double oa = 0.0, ob = 0.0, ta = 0.0, tb = 0.0; uint32_t on = 0u, tn = 0u;
    for (int w = 0; w < kAliasWaves; w++) {
        if (w < wave) { oa += sd[0][w]; ob += sd[1][w]; on += su[w]; }
        ta += sd[0][w]; tb += sd[1][w]; tn += su[w];
    }
    __syncthreads();
    if (threadIdx.x == 0) { sd[0][kAliasWaves] = ta; sd[1][kAliasWaves] = tb; su[kAliasWaves] = tn; }
    __syncthreads();
    a = oa + ia - a; b = ob + ib - b; n = on + in - n;
}

__global__ void __launch_bounds__(kAliasThreads) alias_sweep_kernel(const float *__restrict__ phi, int K, int Kpad, uint2 *table) {
    extern __shared__ double lds_pre[];
    __shared__ double sd[2][kAliasWaves + 1];
    __shared__ uint32_t su[kAliasWaves + 1];
    double *pre = lds_pre;
    uint32_t *idx = reinterpret_cast<uint32_t *>(lds_pre + K + 1);
    const float *__restrict__ row = phi + (size_t)blockIdx.x * (size_t)Kpad;
    uint2 *__restrict__ out = table + (size_t)blockIdx.x * (size_t)K;
    const int tid = (int)threadIdx.x, c = (K + kAliasThreads - 1) / kAliasThreads;
    const int k0 = min(K, tid * c), k1 = min(K, k0 + c);
    double part = 0.0, zero = 0.0; uint32_t none = 0u;
    for (int k = k0; k < k1; k++) part += (double)row[k];
    block_excl_scan2(part, zero, none, sd, su);
    const double scale = (double)K / sd[0][kAliasWaves];
    __syncthreads();                                   // sd is reused below
    double lack = 0.0, extra = 0.0; uint32_t nlight = 0u;
    for (int k = k0; k < k1; k++) {
        const double q = (double)row[k] * scale;
        if (q > 1.0) extra += q - 1.0; else { lack += 1.0 - q; nlight++; }
    }
    block_excl_scan2(lack, extra, nlight, sd, su);     // now: what the items before this thread's lack / have beyond
    const int nL = (int)su[kAliasWaves], nH = K - nL;
    int a = (int)nlight, b = k0 - (int)nlight;
    for (int k = k0; k < k1; k++) {
        const double q = (double)row[k] * scale;
        if (q > 1.0) { extra += q - 1.0; idx[nL + b] = (uint32_t)k; pre[nL + 1 + b] = extra; b++; }
        else { idx[a] = (uint32_t)k; pre[a] = lack; lack += 1.0 - q; a++; }
    }
    if (tid == 0) pre[nL] = sd[0][kAliasWaves];
    __syncthreads();
    for (int i = tid; i < nL; i += kAliasThreads) {              // light items
        const int k = (int)idx[i];
        const double q = (double)row[k] * scale, l = pre[i];
        int lo = 0, hi = nH;
        while (lo < hi) { const int mid = (lo + hi) >> 1; if (pre[nL + 1 + mid] > l) hi = mid; else lo = mid + 1; }
        if (lo >= nH) lo = nH - 1;                     // rounding used up every heavy item: the last one
        out[k] = nH > 0 ? make_uint2(__float_as_uint((float)q), idx[nL + lo]) : make_uint2(__float_as_uint(1.0f), (uint32_t)k);
    }
    for (int i = tid; i < nH; i += kAliasThreads) {              // heavy items
        const int k = (int)idx[nL + i];
        const double h = pre[nL + 1 + i];
        int lo = 0, hi = nL + 1;
        while (lo < hi) { const int mid = (lo + hi) >> 1; if (pre[mid] >= h) hi = mid; else lo = mid + 1; }
        if (lo <= nL && i + 1 < nH) {
            double r = 1.0 + h - pre[lo];
            r = r < 0.0 ? 0.0 : (r > 1.0 ? 1.0 : r);
            out[k] = make_uint2(__float_as_uint((float)r), idx[nL + i + 1]);
        } else {
            out[k] = make_uint2(__float_as_uint(1.0f), (uint32_t)k);
        }
    }
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
