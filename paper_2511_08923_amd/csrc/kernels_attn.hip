// Hybrid-mask paged attention for the decode step (bf16 MFMA path) and its split-KV combine.
//
// Work item = (sequence, kv head, chunk of 16-row query tiles, split of the key range).  The query rows of a
// kv head are the rows of all query heads in its group, flattened (head-in-group major), so a K/V tile that
// is staged once in LDS serves every query head that shares it.  Four waves split the query tiles; each wave
// keeps its Q fragments, its O^T accumulators and its softmax state in registers for the whole key range.
//
// Softmax numerators are taken against an integral power-of-two reference (ceil of the running maximum in
// log2 units): their bf16 rounding is then independent of the reference in force, i.e. of tiling and splits.
//
// Orientation: scores are formed transposed, S^T[key][q] = K . Q^T, so that in the MFMA result layout a lane
// holds one query column and four keys per 16-key tile.  Exponentials of two such tiles are, without any data
// movement, the B operand (P^T) of O^T[d][q] += V^T[d][key] . P^T[key][q].  V is kept transposed in HBM
// ([head_dim][16 tokens] per page) so its A-operand fragments are plain 16-byte LDS reads.
//
// Keys come in units of 16: cache pages 0 .. ceil((L+nc)/16)-1, then the mask rows' scratch tiles.  Pages that
// lie wholly below L need no mask at all (every row sees the whole prefix); everything else goes through the
// (row, key) predicate and a per-(query tile, key pair) skip when nothing is visible.
#include "tidar_internal.h"

namespace {

constexpr int HD = 128;
constexpr int K_STRIDE = HD + 8;        // bf16 per key row in LDS (+16 B: conflict-free 16-byte reads)
constexpr int V_STRIDE = 32 + 8;        // bf16 per head-dim row in LDS: 32 keys + pad

struct AttnArgs {
    const bf16_t *q;
    KvView kv;
    const bf16_t *k_scr, *v_scr;
    const int32_t *prefix_len;
    RowDesc d;
    int n_q, group;
    int n_chunks, tiles_per_chunk, splits;
    int inv_bl;                // ceil(65536 / bl)
    float scale_log2e;
    float *opart, *mpart, *lpart;
};

struct UnitAddr {
    const bf16_t *k;   // [16][128]
    const bf16_t *v;   // [128][16]
    int valid;         // number of keys that hold data (0..16)
};

__device__ inline UnitAddr unit_addr(const AttnArgs &a, int b, int g, int uu, int L, int n_cache_units, int n_mt) {
    UnitAddr u;
    u.k = nullptr;
    u.v = nullptr;
    u.valid = 0;
    if (uu < n_cache_units) {
        int page = a.kv.page_table[(size_t)(a.d.seq_base + b) * a.kv.pages_per_seq + uu];
        size_t base = ((size_t)page * a.kv.n_kv + g) * 16 * HD;
        u.k = (const bf16_t *)a.kv.k_pages + base;
        u.v = (const bf16_t *)a.kv.v_pages + base;
        u.valid = min(16, L + a.d.nc - 16 * uu);
    } else if (uu < n_cache_units + n_mt) {
        int mt = uu - n_cache_units;
        size_t base = (((size_t)b * a.kv.n_kv + g) * n_mt + mt) * 16 * HD;
        u.k = a.k_scr + base;
        u.v = a.v_scr + base;
        u.valid = min(16, a.d.nb * a.d.bl - 16 * mt);
    }
    return u;
}

template <int QT>
__global__ __launch_bounds__(256) void attn_bf16_kernel(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) bf16_t k_lds[2][2][16 * K_STRIDE];
    __shared__ __attribute__((aligned(16))) bf16_t v_lds[2][HD * V_STRIDE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 15, lg = lane >> 4;
    int bx = blockIdx.x;
    const int chunk = bx % a.n_chunks;
    bx /= a.n_chunks;
    const int g = bx % a.kv.n_kv;
    const int b = bx / a.kv.n_kv;
    const int split = blockIdx.y;
    const RowDesc d = a.d;
    const int L = a.prefix_len[d.seq_base + b];
    const int n_mask = d.nb * d.bl;
    const int n_cache_units = (L + d.nc + 15) >> 4;
    const int n_pure = L >> 4;
    const int n_mt = (n_mask + 15) >> 4;
    const int U = n_cache_units + n_mt;
    const int n_it = (U + 1) >> 1;
    const int per = (n_it + a.splits - 1) / a.splits;
    const int it0 = split * per;
    const int it1 = min(n_it, it0 + per);
    const int F = a.group * d.R;                     // flattened query rows of this kv head
    const int TQ = (F + 15) >> 4;
    const int t0 = chunk * a.tiles_per_chunk;
    const int t1 = min(TQ, t0 + a.tiles_per_chunk);

    // ---- this wave's query tiles: Q fragments (B operand), row info, accumulators
    bf16x8 qf[QT][4];
    int r_vis[QT], r_blk[QT];
    f32x4 acc[QT][8];
    float m_run[QT], l_run[QT];
#pragma unroll
    for (int i = 0; i < QT; ++i) {
        int tile = t0 + wave + 4 * i;
        int f = tile * 16 + lq;
        bool ok = tile < t1 && f < F;
        int hq = ok ? f / d.R : 0;
        int r = ok ? f - hq * d.R : 0;
        RowInfo ri = row_info(d, r, L);
        r_vis[i] = ok ? ri.vis : 0;
        r_blk[i] = ok ? ri.blk : -2;
        const bf16_t *qp = a.q + (((size_t)b * d.R + r) * a.n_q + (g * a.group + hq)) * HD + 8 * lg;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (ok) v = *(const bf16x8 *)(qp + 32 * ks);
            qf[i][ks] = v;
        }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) acc[i][dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
        m_run[i] = -INFINITY;
        l_run[i] = 0.f;
    }

    // ---- K/V staging: per iteration each thread moves one 16-byte piece of K and of V^T for both units
    bf16x8 st_k[2], st_v[2];
    const int k_key = tid >> 4, k_piece = tid & 15;
    const int v_d = tid >> 1, v_half = tid & 1;
    auto load_kv = [&](int it) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            UnitAddr ua = unit_addr(a, b, g, 2 * it + u, L, n_cache_units, n_mt);
            bf16x8 kk = {0, 0, 0, 0, 0, 0, 0, 0}, vv = {0, 0, 0, 0, 0, 0, 0, 0};
            if (ua.valid > 0) {
                kk = *(const bf16x8 *)(ua.k + k_key * HD + k_piece * 8);
                vv = *(const bf16x8 *)(ua.v + v_d * 16 + v_half * 8);
                if (ua.valid < 16) {        // slots past the data may hold anything: keep them out of P.V
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (v_half * 8 + j >= ua.valid) vv[j] = (bf16_t)0.f;
                }
            }
            st_k[u] = kk;
            st_v[u] = vv;
        }
    };
    auto store_kv = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            *(bf16x8 *)(&k_lds[buf][u][k_key * K_STRIDE + k_piece * 8]) = st_k[u];
            // V^T row layout: four-key groups of the two units interleaved: [A0-3 B0-3 A4-7 B4-7 ...]
            typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
            bf16x4 lo = {st_v[u][0], st_v[u][1], st_v[u][2], st_v[u][3]};
            bf16x4 hi = {st_v[u][4], st_v[u][5], st_v[u][6], st_v[u][7]};
            bf16_t *row = &v_lds[buf][v_d * V_STRIDE];
            *(bf16x4 *)(row + 8 * (2 * v_half) + 4 * u) = lo;
            *(bf16x4 *)(row + 8 * (2 * v_half + 1) + 4 * u) = hi;
        }
    };

    if (it0 < it1) {
        load_kv(it0);
        store_kv(0);
    }
    __syncthreads();

    for (int it = it0; it < it1; ++it) {
        const int buf = (it - it0) & 1;
        if (it + 1 < it1) load_kv(it + 1);

        // fragments of this key pair
        bf16x8 kf[2][4], vf[8];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                kf[u][ks] = *(const bf16x8 *)(&k_lds[buf][u][lq * K_STRIDE + 32 * ks + 8 * lg]);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) vf[dt] = *(const bf16x8 *)(&v_lds[buf][(16 * dt + lq) * V_STRIDE + 8 * lg]);

        const bool pure = (2 * it + 1) < n_pure;
        // per-key facts for the masked path (independent of the query tile)
        int key_kind[2];        // 0: cache unit, 1: mask unit, 2: nothing
        int key_base[2];        // cache: absolute position of this lane's first key; mask: mask-row index
        int key_blk[2][4];
        if (!pure) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                int uu = 2 * it + u;
                if (uu < n_cache_units) {
                    key_kind[u] = 0;
                    key_base[u] = 16 * uu + 4 * lg;
                } else if (uu < U) {
                    key_kind[u] = 1;
                    key_base[u] = 16 * (uu - n_cache_units) + 4 * lg;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        int m = key_base[u] + j;
                        key_blk[u][j] = (m < n_mask) ? ((m * a.inv_bl) >> 16) : -3;
                    }
                } else {
                    key_kind[u] = 2;
                    key_base[u] = 0;
                }
            }
        }

#pragma unroll
        for (int i = 0; i < QT; ++i) {
            const int tile = t0 + wave + 4 * i;
            if (tile >= t1) continue;                       // wave-uniform
            bool vis[2][4];
            if (!pure) {
                bool any = false;
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        bool v;
                        if (key_kind[u] == 0) {
                            int p = key_base[u] + j;
                            v = (p < L) || (p - L < r_vis[i]);
                        } else if (key_kind[u] == 1) {
                            v = key_blk[u][j] == r_blk[i];
                        } else {
                            v = false;
                        }
                        vis[u][j] = v;
                        any |= v;
                    }
                if (!__any(any)) continue;                  // nothing of this pair is visible to this tile
            }
            f32x4 s[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                s[u] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    s[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[u][ks], qf[i][ks], s[u], 0, 0, 0);
            }
            float mx = -INFINITY;
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float v = s[u][j] * a.scale_log2e;
                    if (!pure && !vis[u][j]) v = -INFINITY;
                    s[u][j] = v;
                    mx = fmaxf(mx, v);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // the reference exponent is kept integral: numerators 2^(s - ref) then round to bf16 the same way
            // whichever reference is current, so the result does not depend on tile order or split count,
            // and every rescale below is by an exact power of two
            const float m_new = fmaxf(m_run[i], ceilf(mx));
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = exp2f(m_run[i] - m_safe);
            m_run[i] = m_new;
            float psum = 0.f;
            bf16x8 pf;
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float p = exp2f(s[u][j] - m_safe);
                    bf16_t pb = (bf16_t)p;
                    psum += (float)pb;                      // the denominator sums what P.V really uses
                    pf[4 * u + j] = pb;
                }
            l_run[i] = l_run[i] * alpha + psum;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                f32x4 o = acc[i][dt];
                o[0] *= alpha; o[1] *= alpha; o[2] *= alpha; o[3] *= alpha;
                acc[i][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pf, o, 0, 0, 0);
            }
        }

        if (it + 1 < it1) store_kv(buf ^ 1);
        __syncthreads();
    }

    // ---- write this split's partial (unnormalised O, running max in log2 units, denominator)
    const size_t pbase = (((size_t)b * a.kv.n_kv + g) * a.splits + split) * F;
#pragma unroll
    for (int i = 0; i < QT; ++i) {
        const int tile = t0 + wave + 4 * i;
        if (tile >= t1) continue;
        float l = l_run[i];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        int f = tile * 16 + lq;
        if (f < F) {
            float *op = a.opart + (pbase + f) * HD;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) *(f32x4 *)(op + 16 * dt + 4 * lg) = acc[i][dt];
            if (lg == 0) {
                a.mpart[pbase + f] = m_run[i];
                a.lpart[pbase + f] = l;
            }
        }
    }
}

// out[row][head][d] = sum_s w_s O_s / sum_s w_s l_s,  w_s = 2^(m_s - max m): exact powers of two, since every
// split keeps an integral reference.  One block per row; a thread owns 8 head-dim values of one head and writes
// them as one 16-byte piece, either row-major or in the A-fragment layout of the O projection's input.
__global__ __launch_bounds__(256) void attn_combine_kernel(const float *__restrict__ opart,
                                                           const float *__restrict__ mpart,
                                                           const float *__restrict__ lpart, int R, int n_q, int n_kv,
                                                           int splits, bf16_t *__restrict__ out, int out_af,
                                                           ActLayout lay) {
    const int row = blockIdx.x;                 // b * R + r
    const int b = row / R, r = row - b * R;
    const int group = n_q / n_kv;
    const int F = group * R;
    for (int item = threadIdx.x; item < n_q * (HD / 8); item += blockDim.x) {
        const int head = item / (HD / 8), d0 = 8 * (item % (HD / 8));
        const int g = head / group, hq = head - g * group;
        const int f = hq * R + r;
        const size_t base = ((size_t)b * n_kv + g) * splits;
        float mmax = -INFINITY;
        for (int sp = 0; sp < splits; ++sp) mmax = fmaxf(mmax, mpart[(base + sp) * F + f]);
        float num[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, den = 0.f;
        for (int sp = 0; sp < splits; ++sp) {
            const float m = mpart[(base + sp) * F + f];
            if (m == -INFINITY) continue;
            const float wgt = exp2f(m - mmax);
            const float *op = opart + ((base + sp) * F + f) * HD + d0;
            const float4 a = *(const float4 *)op, c = *(const float4 *)(op + 4);
            num[0] += wgt * a.x; num[1] += wgt * a.y; num[2] += wgt * a.z; num[3] += wgt * a.w;
            num[4] += wgt * c.x; num[5] += wgt * c.y; num[6] += wgt * c.z; num[7] += wgt * c.w;
            den += wgt * lpart[(base + sp) * F + f];
        }
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
    int TQ = (group * R + 15) / 16;
    p.tiles_per_chunk = TQ < 16 ? TQ : 16;    // four waves x at most four query tiles each
    p.n_chunks = (TQ + p.tiles_per_chunk - 1) / p.tiles_per_chunk;
    int base = B * n_kv * p.n_chunks;
    int iters = (max_keys + 31) / 32;
    int s = (256 + base - 1) / base;
    if (s > 64) s = 64;
    int cap = (iters + 3) / 4;                // at least four key pairs per split
    if (s > cap) s = cap;
    p.splits = s < 1 ? 1 : s;
    return p;
}

size_t attn_partial_floats(int B, int n_kv, int group, int R, int hd, int splits) {
    return (size_t)B * n_kv * splits * group * R * (hd + 2);
}

void launch_attention_bf16(const bf16_t *q, KvView kv, const bf16_t *k_scr, const bf16_t *v_scr,
                           const int32_t *prefix_len, RowDesc d, int B, int n_q, const AttnPlan &p, float *part,
                           hipStream_t st) {
    AttnArgs a;
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
    a.inv_bl = d.bl > 0 ? (65536 + d.bl - 1) / d.bl : 0;
    a.scale_log2e = 1.4426950408889634f / sqrtf((float)kv.hd);
    size_t F = (size_t)a.group * d.R;
    size_t rows = (size_t)B * kv.n_kv * p.splits * F;
    a.opart = part;
    a.mpart = part + rows * HD;
    a.lpart = a.mpart + rows;
    dim3 grid(B * kv.n_kv * p.n_chunks, p.splits);
    int qt = (p.tiles_per_chunk + 3) / 4;
    if (qt <= 1) attn_bf16_kernel<1><<<grid, 256, 0, st>>>(a);
    else if (qt <= 2) attn_bf16_kernel<2><<<grid, 256, 0, st>>>(a);
    else attn_bf16_kernel<4><<<grid, 256, 0, st>>>(a);
}

void launch_attention_combine(const float *part, int B, int R, int n_q, int n_kv, int hd, int splits, bf16_t *out,
                              int out_af, hipStream_t st) {
    size_t F = (size_t)(n_q / n_kv) * R;
    size_t rows = (size_t)B * n_kv * splits * F;
    attn_combine_kernel<<<B * R, 256, 0, st>>>(part, part + rows * hd, part + rows * hd + rows, R, n_q, n_kv, splits,
                                               out, out_af, act_layout(B * R));
}
