// Hybrid-mask paged attention for the decode step (bf16 MFMA path) and its split-KV combine.
//
// Work item = (sequence, kv head, chunk of 32-row query tiles, split of the key range).  The query rows of a
// kv head are the rows of all query heads in its group, flattened (head-in-group major), so a K/V tile that
// is staged once in LDS serves every query head that shares it.  Four waves split the query tiles; each wave
// keeps its Q fragments, its O^T accumulators and its softmax state in registers for the whole key range.
//
// MFMA: v_mfma_f32_32x32x16_bf16 (on gfx950 twice the rate of the 16x16x32 form).  Scores are formed
// transposed, S^T[key][q] = K . Q^T, so that in the result layout a lane holds one query column and 16 of the
// 32 keys of a block: register i <-> key 8*(i/4) + 4*(lane/32) + i%4.  Registers 0-7 (keys of the first page of
// the pair) and 8-15 (second page) are, after exponentiation and without any data movement, the B operands
// (P^T) of two MFMAs O^T[d][q] += V^T[d][key] . P^T[key][q]; V is kept transposed in HBM ([head_dim][16
// tokens] per page) and its LDS rows are written with the four-key groups permuted so that the matching A
// operand is one 16-byte read.
//
// Softmax numerators are taken against an integral power-of-two reference (ceil of the running maximum in
// log2 units): their bf16 rounding is then independent of the reference in force, i.e. of tiling and splits,
// every rescale is exact, and the reference moves so rarely that the rescale of O^T is skipped almost always.
//
// Keys come in units of 16: cache pages 0 .. ceil((L+nc)/16)-1, then the mask rows' scratch tiles.  Pages that
// lie wholly below L need no mask at all (every row sees the whole prefix); everything else goes through the
// (row, key) predicate and a per-(query tile, key pair) skip when nothing is visible.
#include <stdlib.h>

#include "tidar_internal.h"

namespace {

constexpr int HD = 128;
constexpr int K_STRIDE = HD + 8;        // bf16 per key row in LDS (+16 B: conflict-free 16-byte reads)
constexpr int V_STRIDE = 32 + 8;        // bf16 per head-dim row in LDS: 32 keys + pad
constexpr int OOB = 0x7ffffff0;

__device__ inline __amdgpu_buffer_rsrc_t attn_rsrc(const void *base, size_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)(bytes > 0x7fffffe0ull ? 0x7fffffe0ull : bytes),
                                             0x00020000);
}
__device__ inline bf16x8 attn_buf_load(__amdgpu_buffer_rsrc_t r, int byte_off) {
    return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0));
}

struct AttnArgs {
    const bf16_t *q;
    KvView kv;
    const bf16_t *k_scr, *v_scr;
    const int32_t *prefix_len;
    RowDesc d;
    int n_q, group;
    int n_chunks, tiles_per_chunk, splits, per;
    int n_pages;               // physical pages per layer (bounds of the page buffers)
    float scale_log2e;
    float *opart, *mpart, *lpart;
    bf16_t *out;               // single split only: [rows][n_q][HD], or the A-fragment layout (out_af)
    int out_af;
    ActLayout lay;
};

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// One 32-query x 32-key block: S^T = K.Q^T, online softmax against the integral reference, O^T += V^T.P^T.
// c = softmax scale * log2(e).  VIS: bit e set = register e's key is visible to this lane's query row (only read
// when MASKED).  Kept lean: per score one max, one fma, one v_exp_f32, half a pack and half a dot2.
template <bool MASKED>
__device__ inline void attn_block(const bf16_t *k_lds, const bf16_t *v_lds, int lq, int lh, const bf16x8 (&qf)[8],
                                  f32x16 (&acc)[4], float &m_run, float &l_run, float c, unsigned vis) {
    // K as A operand (lane = key, hd half of the k step); fragments are consumed as they arrive.  One
    // accumulation chain: a second one costs 16 registers, and the other resident wave covers the dependency
    f32x16 s;
#pragma unroll
    for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 kf0 = *(const bf16x8 *)(k_lds + lq * K_STRIDE + 16 * ks + 8 * lh);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf0, qf[ks], s, 0, 0, 0);
    }
    // V^T as A operand (lane = d, key chunk): the first half is issued now and is needed after the softmax
    // arithmetic; the second half is read once the scores are dead and takes over their registers
    bf16x8 vf[2][2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int u = 0; u < 2; ++u)
            vf[dt][u] = *(const bf16x8 *)(v_lds + (32 * dt + lq) * V_STRIDE + 16 * u + 8 * lh);
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        if (MASKED) s[e] = ((vis >> e) & 1u) ? s[e] : -INFINITY;
        mx = fmaxf(mx, s[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, ceilf(mx * c));
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    if (__any(m_new != m_run)) {                    // rare after the first blocks: rescale by the exact 2^(old-new)
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[dt][e] *= alpha;
        m_run = m_new;
    }
    const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
    float psum = 0.f;
    bf16x8 pf[2];
#pragma unroll
    for (int e = 0; e < 16; e += 2) {
        bf16x2 pk = {(bf16_t)__builtin_amdgcn_exp2f(fmaf(s[e], c, -m_safe)),
                     (bf16_t)__builtin_amdgcn_exp2f(fmaf(s[e + 1], c, -m_safe))};
        psum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, psum, false);   // the denominator sums the rounded values
        pf[e >> 3][e & 7] = pk[0];
        pf[e >> 3][(e & 7) + 1] = pk[1];
    }
    l_run += psum;
    bf16x8 vg[2][2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int u = 0; u < 2; ++u)
            vg[dt][u] = *(const bf16x8 *)(v_lds + (32 * (dt + 2) + lq) * V_STRIDE + 16 * u + 8 * lh);
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int u = 0; u < 2; ++u)
            acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][u], pf[u], acc[dt], 0, 0, 0);
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int u = 0; u < 2; ++u)
            acc[dt + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vg[dt][u], pf[u], acc[dt + 2], 0, 0, 0);
}

// QT: 32-row query tiles per wave.
template <int QT>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) bf16_t k_lds[2][32 * K_STRIDE];
    __shared__ __attribute__((aligned(16))) bf16_t v_lds[2][HD * V_STRIDE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, lh = lane >> 5;
    int bx = blockIdx.x;
    const int chunk = bx % a.n_chunks;
    bx /= a.n_chunks;
    const int g = bx % a.kv.n_kv;
    const int b = bx / a.kv.n_kv;
    const int split = blockIdx.y;
    const RowDesc d = a.d;
    const int L = a.prefix_len[d.seq_base + b];
    const int n_mask = d.nm;
    const int n_cache_units = (L + d.nc + 15) >> 4;
    const int n_pure = L >> 4;
    const int n_mt = (n_mask + 15) >> 4;
    const int U = n_cache_units + n_mt;
    const int n_it = (U + 1) >> 1;
    // Split s takes key-pair iterations [s*per, (s+1)*per) with per fixed by the host from its bound on the key
    // count: which split a key falls into does not depend on how long the sequence is right now, so the same
    // query over the same keys is reduced in the same grouping at every step (the last split takes whatever a
    // loose bound leaves over; splits past the end write an empty partial).
    const int per = a.per;
    const int it0 = min(n_it, split * per);
    const int it1 = (split == a.splits - 1) ? n_it : min(n_it, it0 + per);
    const int F = a.group * d.R;                     // flattened query rows of this kv head
    const int TQ = (F + 31) >> 5;
    const int t0 = chunk * a.tiles_per_chunk;
    const int t1 = min(TQ, t0 + a.tiles_per_chunk);
    // Key-pair iterations this workgroup can need at all: cache units up to the furthest key any of its rows
    // sees, then the mask units of its rows' own blocks.  (Rows of one query head only; a workgroup that straddles
    // two heads keeps the whole range.)  Inside a prefill or scoring pass most of the range falls away: causal
    // rows see neither the later rows of the pass nor any mask row, a mask block only the text before it and
    // itself.  Iterations are dropped whole, so the pairing of keys into iterations and splits is untouched.
    int itA1 = n_it, itB0 = n_it, itB1 = n_it;       // [it0, itA1) and [itB0, itB1), itA1 <= itB0
    {
        const int f_lo = t0 * 32, f_hi = min(F, t1 * 32) - 1;
        const int h_lo = f_lo / d.R, h_hi = f_hi / d.R;
        if (h_lo == h_hi) {
            const int r_lo = f_lo - h_lo * d.R, r_hi = f_hi - h_lo * d.R;
            int vis_max = min(r_hi, d.nc - 1) + 1;                       // the causal rows among them
            int um0 = 0, um1 = 0;                                        // mask units [um0, um1)
            if (r_hi >= d.nc) {
                const int j_lo = (max(r_lo, d.nc) - d.nc) / d.bl, j_hi = (r_hi - d.nc) / d.bl;
                if (r_lo >= d.nc) vis_max = 0;
                vis_max = max(vis_max, d.cond0 + j_hi * d.cstride);
                um0 = (j_lo * d.bl) >> 4;
                um1 = (min((j_hi + 1) * d.bl, n_mask) + 15) >> 4;
            }
            const int uc1 = min(n_cache_units, (L + min(vis_max, d.nc) + 15) >> 4);
            itA1 = (uc1 + 1) >> 1;
            itB0 = max(itA1, (n_cache_units + um0) >> 1);
            itB1 = um1 > um0 ? max(itB0, (n_cache_units + um1 + 1) >> 1) : itB0;
        } else {
            itB0 = itB1 = n_it;
        }
    }
    // this split's share of the two ranges, walked as one sequence of nA + nB iterations
    const int a0 = it0, a1 = max(a0, min(it1, itA1));
    const int b0 = max(it0, itB0), b1 = max(b0, min(it1, itB1));
    const int nA = a1 - a0, n_seq = nA + (b1 - b0);
    auto seq_it = [&](int n) { return n < nA ? a0 + n : b0 + (n - nA); };

    // ---- this wave's query tiles: Q fragments (B operand: lane = (q row, hd half of the k step)), row info
    bf16x8 qf[QT][8];
    int r_vis[QT], r_blk[QT];
    f32x16 acc[QT][4];
    float m_run[QT], l_run[QT];
#pragma unroll
    for (int i = 0; i < QT; ++i) {
        const int tile = t0 + wave + 4 * i;
        const int f = tile * 32 + lq;
        const bool ok = tile < t1 && f < F;
        const int hq = ok ? f / d.R : 0;
        const int r = ok ? f - hq * d.R : 0;
        const RowInfo ri = row_info(d, r, L);
        r_vis[i] = ok ? ri.vis : 0;
        r_blk[i] = ok ? ri.blk : -2;
        const bf16_t *qp = a.q + (((size_t)b * d.R + r) * a.n_q + (g * a.group + hq)) * HD + 8 * lh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (ok) v = *(const bf16x8 *)(qp + 16 * ks);
            qf[i][ks] = v;
        }
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][dt][e] = 0.f;
        m_run[i] = -INFINITY;
        l_run[i] = 0.f;
    }

    // ---- K/V staging through buffer loads (an absent unit reads as zeros, no branch): per iteration each thread
    // moves one 16-byte piece of K and of V^T for both units of the pair
    const size_t page_elems = (size_t)a.kv.n_kv * 16 * HD;
    const __amdgpu_buffer_rsrc_t rk = attn_rsrc(a.kv.k_pages, (size_t)a.n_pages * page_elems * 2);
    const __amdgpu_buffer_rsrc_t rv = attn_rsrc(a.kv.v_pages, (size_t)a.n_pages * page_elems * 2);
    const size_t scr_elems = (size_t)gridDim.x / a.n_chunks * (n_mt > 0 ? n_mt : 1) * 16 * HD;   // B * n_kv tiles
    const __amdgpu_buffer_rsrc_t rks = attn_rsrc(a.k_scr, scr_elems * 2);
    const __amdgpu_buffer_rsrc_t rvs = attn_rsrc(a.v_scr, scr_elems * 2);
    bf16x8 st_k[2], st_v[2];
    const int k_key = tid >> 4, k_piece = tid & 15;
    const int v_d = tid >> 1, v_half = tid & 1;
    const int k_in = (k_key * HD + k_piece * 8) * 2, v_in = (v_d * 16 + v_half * 8) * 2;   // byte offsets in a unit
    const int32_t *pt = a.kv.page_table + (size_t)(d.seq_base + b) * a.kv.pages_per_seq;
    auto load_kv = [&](int n) {                         // n: position in this workgroup's iteration sequence
        const int it = seq_it(n);
        const bool live = n < n_seq;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int uu = 2 * it + u;
            const bool in_cache = uu < n_cache_units, in_mask = !in_cache && uu < U && live;
            int base = OOB, valid = 0;
            if (in_cache && live) {                     // scalar (uniform) selects, no vector branch
                const int page = pt[uu];
                base = (int)((((size_t)page * a.kv.n_kv + g) * 16 * HD) * 2);
                valid = min(16, L + d.nc - 16 * uu);
            } else if (in_mask) {
                const int mt = uu - n_cache_units;
                base = (int)(((((size_t)b * a.kv.n_kv + g) * n_mt + mt) * 16 * HD) * 2);
                valid = min(16, n_mask - 16 * mt);
            }
            const int ko = base == OOB ? OOB : base + k_in, vo = base == OOB ? OOB : base + v_in;
            bf16x8 kk = in_mask ? attn_buf_load(rks, ko) : attn_buf_load(rk, ko);
            bf16x8 vv = in_mask ? attn_buf_load(rvs, vo) : attn_buf_load(rv, vo);
            if (valid < 16) {                           // uniform; slots past the data may hold anything
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (v_half * 8 + j >= valid) vv[j] = (bf16_t)0.f;
            }
            st_k[u] = kk;
            st_v[u] = vv;
        }
    };
    auto store_kv = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            *(bf16x8 *)(&k_lds[buf][(16 * u + k_key) * K_STRIDE + k_piece * 8]) = st_k[u];
            // V^T row layout: four-key groups g0..g7 of the pair stored as [g0 g2 | g1 g3 | g4 g6 | g5 g7]
            typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
            bf16x4 lo = {st_v[u][0], st_v[u][1], st_v[u][2], st_v[u][3]};
            bf16x4 hi = {st_v[u][4], st_v[u][5], st_v[u][6], st_v[u][7]};
            bf16_t *row = &v_lds[buf][v_d * V_STRIDE];
            // this thread holds groups 2*half and 2*half+1 of unit u: half 0 -> positions 0 and 2, half 1 -> 1 and 3
            *(bf16x4 *)(row + 4 * (4 * u + v_half)) = lo;
            *(bf16x4 *)(row + 4 * (4 * u + 2 + v_half)) = hi;
        }
    };

    load_kv(0);
    store_kv(0);
    __syncthreads();

    for (int n = 0; n < n_seq; ++n) {
        const int it = seq_it(n);
        const int buf = n & 1;
        load_kv(n + 1);

        const bool pure = (2 * it + 1) < n_pure;
#pragma unroll
        for (int i = 0; i < QT; ++i) {
            const int tile = t0 + wave + 4 * i;
            if (tile >= t1) continue;                       // wave-uniform
            if (pure) {
                attn_block<false>(k_lds[buf], v_lds[buf], lq, lh, qf[i], acc[i], m_run[i], l_run[i], a.scale_log2e,
                                  0xffffu);
            } else {
                // A row sees a contiguous key range of each unit: cache positions below L + vis, or the mask rows
                // of its own block.  The range becomes a 16-bit mask over the unit's keys, from which the lane
                // picks its eight: register e of unit u <-> key 8*((e/4)%2) + 4*lh + e%4 of that unit.
                unsigned vis_bits = 0;                      // bit 8u+e: visible to this lane's query row
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int uu = 2 * it + u;
                    unsigned m16 = 0;
                    if (uu < n_cache_units) {               // uniform
                        const int lim = min(max(L + r_vis[i] - 16 * uu, 0), 16);
                        m16 = (1u << lim) - 1u;
                    } else if (uu < U) {
                        const int m0 = 16 * (uu - n_cache_units);
                        const int lo = min(max(r_blk[i] * d.bl - m0, 0), 16);
                        const int hi = min(max(min((r_blk[i] + 1) * d.bl, n_mask) - m0, 0), 16);
                        m16 = (r_blk[i] >= 0 && hi > lo) ? (((1u << hi) - 1u) & ~((1u << lo) - 1u)) : 0u;
                    }
                    const unsigned v8 = ((m16 >> (4 * lh)) & 0xfu) | (((m16 >> (8 + 4 * lh)) & 0xfu) << 4);
                    vis_bits |= v8 << (8 * u);
                }
                if (!__any(vis_bits != 0)) continue;        // nothing of this pair is visible to this tile
                attn_block<true>(k_lds[buf], v_lds[buf], lq, lh, qf[i], acc[i], m_run[i], l_run[i], a.scale_log2e,
                                 vis_bits);
            }
        }

        store_kv(buf ^ 1);
        __syncthreads();
    }

    // ---- a single split is the whole answer: normalise in registers and store it (a lane holds, for its query
    // row, 16 runs of four consecutive head-dim values), no partial results and no combine launch
    if (a.splits == 1) {
#pragma unroll
        for (int i = 0; i < QT; ++i) {
            const int tile = t0 + wave + 4 * i;
            if (tile >= t1) continue;
            float l = l_run[i];
            l += __shfl_xor(l, 32);
            const int f = tile * 32 + lq;
            if (f >= F) continue;
            const float inv = 1.f / l;
            const int hq = f / d.R, r = f - hq * d.R;
            const int row = b * d.R + r, col0 = (g * a.group + hq) * HD + 4 * lh;
            typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const bf16x4 o = {(bf16_t)(acc[i][dt][4 * r4] * inv), (bf16_t)(acc[i][dt][4 * r4 + 1] * inv),
                                      (bf16_t)(acc[i][dt][4 * r4 + 2] * inv), (bf16_t)(acc[i][dt][4 * r4 + 3] * inv)};
                    const int col = col0 + 32 * dt + 8 * r4;
                    const size_t idx = a.out_af ? af_index(row, col, a.lay) : (size_t)row * a.n_q * HD + col;
                    *(bf16x4 *)(a.out + idx) = o;
                }
        }
        return;
    }

    // ---- write this split's partial (unnormalised O, reference in log2 units, denominator)
    const size_t pbase = (((size_t)b * a.kv.n_kv + g) * a.splits + split) * F;
#pragma unroll
    for (int i = 0; i < QT; ++i) {
        const int tile = t0 + wave + 4 * i;
        if (tile >= t1) continue;
        float l = l_run[i];
        l += __shfl_xor(l, 32);
        const int f = tile * 32 + lq;
        if (f < F) {
            float *op = a.opart + (pbase + f) * HD;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    f32x4 v = {acc[i][dt][4 * r4], acc[i][dt][4 * r4 + 1], acc[i][dt][4 * r4 + 2],
                               acc[i][dt][4 * r4 + 3]};
                    *(f32x4 *)(op + 32 * dt + 8 * r4 + 4 * lh) = v;
                }
            if (lh == 0) {
                a.mpart[pbase + f] = m_run[i];
                a.lpart[pbase + f] = l;
            }
        }
    }
}

// out[row][head][d] = sum_s w_s O_s / sum_s w_s l_s,  w_s = 2^(m_s - max m): exact powers of two, since every
// split keeps an integral reference.  One wave per (row, head): lane = (8-value head-dim chunk, one of 4 split
// lanes); the split lanes share the splits between them and are folded with two shuffles.  The 16-byte result
// goes out row-major or in the A-fragment layout of the O projection's input.
__global__ __launch_bounds__(64) void attn_combine_kernel(const float *__restrict__ opart,
                                                          const float *__restrict__ mpart,
                                                          const float *__restrict__ lpart, int R, int n_q, int n_kv,
                                                          int splits, bf16_t *__restrict__ out, int out_af,
                                                          ActLayout lay) {
    const int row = blockIdx.x;                 // b * R + r
    const int head = blockIdx.y;
    const int b = row / R, r = row - b * R;
    const int group = n_q / n_kv;
    const int F = group * R;
    const int g = head / group, hq = head - g * group;
    const int f = hq * R + r;
    const int lane = threadIdx.x, d0 = 8 * (lane & 15), sl = lane >> 4;
    const size_t base = ((size_t)b * n_kv + g) * splits;
    // reference of the whole row: lane s reads split s's (there are at most 64 splits), then a wave-wide maximum
    float mmax = lane < splits ? mpart[(base + lane) * F + f] : -INFINITY;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) mmax = fmaxf(mmax, __shfl_xor(mmax, o));
    float num[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, den = 0.f;
    // four splits of this split lane at a time: all their loads are issued before the first is used (an absent
    // split re-reads the last one and is given the weight of an empty split)
    for (int sp0 = sl; sp0 < splits; sp0 += 16) {
        float m[4], l[4];
        float4 a[4], c[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int sp = sp0 + 4 * j;
            const size_t pi = (base + min(sp, splits - 1)) * F + f;
            m[j] = mpart[pi];
            l[j] = lpart[pi];
            const float *op = opart + pi * HD + d0;
            a[j] = *(const float4 *)op;
            c[j] = *(const float4 *)(op + 4);
            if (sp >= splits) m[j] = -INFINITY;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (m[j] == -INFINITY) continue;
            const float wgt = exp2f(m[j] - mmax);
            num[0] += wgt * a[j].x; num[1] += wgt * a[j].y; num[2] += wgt * a[j].z; num[3] += wgt * a[j].w;
            num[4] += wgt * c[j].x; num[5] += wgt * c[j].y; num[6] += wgt * c[j].z; num[7] += wgt * c[j].w;
            den += wgt * l[j];
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        num[e] += __shfl_xor(num[e], 16);
        num[e] += __shfl_xor(num[e], 32);
    }
    den += __shfl_xor(den, 16);
    den += __shfl_xor(den, 32);
    if (sl == 0) {
        const float inv = 1.f / den;
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (bf16_t)(num[e] * inv);
        const size_t idx = out_af ? af_index(row, head * HD + d0, lay) : ((size_t)row * n_q + head) * HD + d0;
        *(bf16x8 *)(out + idx) = o;
    }
}

}  // namespace

AttnPlan plan_attention(int B, int n_kv, int group, int R, int max_keys) {
    AttnPlan p;
    int TQ = (group * R + 31) / 32;           // 32-row query tiles per kv head
    p.tiles_per_chunk = TQ < 4 ? TQ : 4;      // four waves x one query tile each
    p.n_chunks = (TQ + p.tiles_per_chunk - 1) / p.tiles_per_chunk;
    int base = B * n_kv * p.n_chunks;
    int iters = (max_keys + 31) / 32;
    // Two workgroups are resident per CU (512 slots).  A split costs about eight key-pair iterations of prologue
    // and partial-sum epilogue; a grid of w slot-fulls takes about w + 1/2 workgroup times (the last round is
    // ragged).  The split count with the least estimated time wins, the smaller one on a near tie (fewer partial
    // sums for the combine kernel): 7 at batch 1 and 4096 keys (one full round), 5 at batch 4 and 8192 keys
    // (where one split left 44 % of the slots idle for the whole launch), 1 once the batch alone fills the chip
    // several times over.
    // No more than 64 splits (the combine kernel reads one per lane) and, beyond two, no more than four slot-fulls
    // of workgroups: that bound depends on the row structure alone, and the workspace is sized by it, so the
    // partial-sum area does not depend on the key bound of a particular call.
    p.splits_bound = 2048 / base < 2 ? 2 : 2048 / base > 64 ? 64 : 2048 / base;
    int cap = (iters + 3) / 4;                // at least four key pairs per split
    if (cap > p.splits_bound) cap = p.splits_bound;
    int s = 1;
    double best = 0.0;
    for (int c = 1; c <= cap; ++c) {
        const double waves = (double)base * c / 512.0;
        const double cost = (waves <= 1.0 ? 1.0 : waves + 0.5) * ((iters + c - 1) / c + 8);
        if (c == 1 || cost < 0.97 * best) {
            best = cost;
            s = c;
        }
    }
    p.splits = s < 1 ? 1 : s;
    if (const char *e = getenv("TIDAR_ATTN_SPLITS")) {     // tuning override for sweeps (unset in normal use)
        int v = atoi(e);
        if (v >= 1 && v <= 64) p.splits = v < cap ? v : (cap < 1 ? 1 : cap);
    }
    p.per = (iters + 1 + p.splits - 1) / p.splits;   // +1: the kernel counts cache and scratch units separately
    return p;
}

size_t attn_partial_floats(int B, int n_kv, int group, int R, int hd, int splits) {
    return (size_t)B * n_kv * splits * group * R * (hd + 2);
}

void launch_attention_bf16(const bf16_t *q, KvView kv, int n_pages, const bf16_t *k_scr, const bf16_t *v_scr,
                           const int32_t *prefix_len, RowDesc d, int B, int n_q, const AttnPlan &p, float *part,
                           bf16_t *out, int out_af, hipStream_t st) {
    AttnArgs a;
    a.out = out;
    a.out_af = out_af;
    a.lay = act_layout(B * d.R);
    a.q = q;
    a.kv = kv;
    a.k_scr = k_scr;
    a.v_scr = v_scr;
    a.prefix_len = prefix_len;
    a.d = d;
    a.n_q = n_q;
    a.group = n_q / kv.n_kv;
    a.n_chunks = p.n_chunks;
    a.tiles_per_chunk = p.tiles_per_chunk;
    a.splits = p.splits;
    a.per = p.per;
    a.n_pages = n_pages;
    a.scale_log2e = 1.4426950408889634f / sqrtf((float)kv.hd);
    size_t F = (size_t)a.group * d.R;
    size_t rows = (size_t)B * kv.n_kv * p.splits * F;
    a.opart = part;
    a.mpart = part + rows * HD;
    a.lpart = a.mpart + rows;
    dim3 grid(B * kv.n_kv * p.n_chunks, p.splits);
    attn_bf16_kernel<1><<<grid, 256, 0, st>>>(a);
}

void launch_attention_combine(const float *part, int B, int R, int n_q, int n_kv, int hd, int splits, bf16_t *out,
                              int out_af, hipStream_t st) {
    if (splits == 1) return;                  // the attention kernel has written the result itself
    size_t F = (size_t)(n_q / n_kv) * R;
    size_t rows = (size_t)B * n_kv * splits * F;
    attn_combine_kernel<<<dim3(B * R, n_q), 64, 0, st>>>(part, part + rows * hd, part + rows * hd + rows, R, n_q, n_kv,
                                                         splits, out, out_af, act_layout(B * R));
}
