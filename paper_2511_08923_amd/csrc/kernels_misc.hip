// Small kernels of the decode step: weight packing, row assembly + embedding gather, RMSNorm with fused
// residual/split-K reduction, RoPE + K/V placement, SwiGLU, vocabulary argmax / Gumbel-max, verify/accept.
// Also the fp32-mode GEMM and attention (plain ALU kernels used by the fp32 configuration).
#include "tidar_internal.h"

namespace {

template <typename T> __device__ inline float to_f(T v);
template <> __device__ inline float to_f<float>(float v) { return v; }
template <> __device__ inline float to_f<bf16_t>(bf16_t v) { return (float)v; }
template <typename T> __device__ inline T from_f(float v);
template <> __device__ inline float from_f<float>(float v) { return v; }
template <> __device__ inline bf16_t from_f<bf16_t>(float v) { return (bf16_t)v; }   // round to nearest even

template <typename T> __device__ inline void store4(T *p, float a, float b, float c, float d);
template <> __device__ inline void store4<float>(float *p, float a, float b, float c, float d) {
    *(float4 *)p = make_float4(a, b, c, d);
}
template <> __device__ inline void store4<bf16_t>(bf16_t *p, float a, float b, float c, float d) {
    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
    bf16x4 v = {(bf16_t)a, (bf16_t)b, (bf16_t)c, (bf16_t)d};
    *(bf16x4 *)p = v;
}

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

// ------------------------------------------------------------------ weight packing
// bf16 destination: [k step of 16][32-row tile][lane][8], lane = (k/8 % 2) * 32 + row % 32: the register image
// of the 32x32x16 MFMA B operand.  The k step is outermost: all workgroups of a GEMM advance through K together,
// so at any moment they read one contiguous front of the matrix, which spreads over every HBM channel.
// Source row r lands in destination row 16 * (tile_off + (r / 16) * tile_stride) + r % 16.
__global__ void pack_bf16_kernel(const bf16_t *__restrict__ src, int rows, int K, bf16_t *__restrict__ dst,
                                 int dst_tiles32, int tile_off, int tile_stride) {
    const int k8 = K / 8;
    size_t n = (size_t)rows * k8;                               // one 16-byte piece per index
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n;
         idx += (size_t)gridDim.x * blockDim.x) {
        int r = (int)(idx / k8);
        int k = 8 * (int)(idx % k8);
        int rd = 16 * (tile_off + (r >> 4) * tile_stride) + (r & 15);
        size_t o = ((((size_t)(k >> 4) * dst_tiles32 + (rd >> 5)) * 64) + ((k >> 3) & 1) * 32 + (rd & 31)) * 8;
        *(bf16x8 *)(dst + o) = *(const bf16x8 *)(src + (size_t)r * K + k);
    }
}

// fp32: plain row-major; tile placement only.
__global__ void pack_f32_kernel(const float *__restrict__ src, int rows, int K, float *__restrict__ dst,
                                int tile_off, int tile_stride) {
    size_t n = (size_t)rows * K;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x) {
        int r = (int)(idx / K);
        int c = (int)(idx % K);
        size_t dr = (size_t)(tile_off + (r / 16) * tile_stride) * 16 + (r % 16);
        dst[dr * K + c] = src[idx];
    }
}

// ------------------------------------------------------------------ row assembly + embedding gather (+ RoPE table)
template <typename T>
__global__ void embed_rows_kernel(const T *__restrict__ embed, const int32_t *__restrict__ tokens, int tok_stride,
                                  const int32_t *__restrict__ prefix_len, RowDesc d, int d_model, int mask_id,
                                  int vocab, KvView kv, int hd, float rope_base, float *__restrict__ x,
                                  int32_t *__restrict__ pos_out, float *__restrict__ rope_cs) {
    int row = blockIdx.x;                 // b * R + r
    int b = row / d.R;
    int r = row - b * d.R;
    int L = clamp_prefix(kv, prefix_len[d.seq_base + b], d.nc);
    RowInfo ri = row_info(d, r, L);
    int tok = (r < d.nc) ? tokens[(size_t)b * tok_stride + r] : mask_id;
    if ((unsigned)tok >= (unsigned)vocab) tok = mask_id;      // an id outside the table is never dereferenced (the
                                                              // kernel that finishes the call reports it)
    if (threadIdx.x == 0) pos_out[row] = ri.pos;
    const T *e = embed + (size_t)tok * d_model;
    float *xo = x + (size_t)row * d_model;
    for (int c = threadIdx.x; c < d_model; c += blockDim.x) xo[c] = to_f<T>(e[c]);
    // cos/sin of pos * base^(-2i/hd), angle formed in double so that long contexts keep their phase
    int half = hd / 2;
    for (int i = threadIdx.x; i < half; i += blockDim.x) {
        double inv = exp2(-(double)(2 * i) / (double)hd * log2((double)rope_base));
        double ang = (double)ri.pos * inv;
        double s, c;
        sincos(ang, &s, &c);
        rope_cs[((size_t)row * half + i) * 2 + 0] = (float)c;
        rope_cs[((size_t)row * half + i) * 2 + 1] = (float)s;
    }
}

// ------------------------------------------------------------------ residual add (split-K partials) + RMSNorm
// One block per output row.  part: tiled GEMM output over M_all rows; out: A-fragment layout over the selected rows.
template <typename T>
__global__ __launch_bounds__(1024) void rmsnorm_kernel(float *__restrict__ x, const float *__restrict__ part, int S,
                                                      size_t split_stride, const T *__restrict__ gain, float eps,
                                                      int R, int row0, int d_model, int M_all, T *__restrict__ out,
                                                      ActLayout lay) {
    const int Rh = R - row0;
    const int b = blockIdx.x / Rh;
    const int o = blockIdx.x - b * Rh;
    const int row = b * R + row0 + o;
    float *xr = x + (size_t)row * d_model;
    float ss = 0.f;
    for (int c = 4 * threadIdx.x; c < d_model; c += 4 * blockDim.x) {
        float4 v = *(const float4 *)(xr + c);
        if (S > 0) {
            const float *pp = part + pt_index(c, row, M_all);
            int sp = 0;
            for (; sp + 4 <= S; sp += 4) {         // four independent loads at a time, summed in split order
                const float4 q0 = *(const float4 *)(pp + (size_t)sp * split_stride);
                const float4 q1 = *(const float4 *)(pp + (size_t)(sp + 1) * split_stride);
                const float4 q2 = *(const float4 *)(pp + (size_t)(sp + 2) * split_stride);
                const float4 q3 = *(const float4 *)(pp + (size_t)(sp + 3) * split_stride);
                v.x = (((v.x + q0.x) + q1.x) + q2.x) + q3.x;
                v.y = (((v.y + q0.y) + q1.y) + q2.y) + q3.y;
                v.z = (((v.z + q0.z) + q1.z) + q2.z) + q3.z;
                v.w = (((v.w + q0.w) + q1.w) + q2.w) + q3.w;
            }
            for (; sp < S; ++sp) {
                const float4 q = *(const float4 *)(pp + (size_t)sp * split_stride);
                v.x += q.x; v.y += q.y; v.z += q.z; v.w += q.w;
            }
            *(float4 *)(xr + c) = v;
        }
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    __shared__ float red[16];
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) tot += red[w];
    const float rs = rsqrtf(tot / (float)d_model + eps);
    for (int c = 4 * threadIdx.x; c < d_model; c += 4 * blockDim.x) {
        float4 v = *(const float4 *)(xr + c);          // this thread's own writes
        store4<T>(out + af_index(blockIdx.x, c, lay), v.x * rs * to_f<T>(gain[c]), v.y * rs * to_f<T>(gain[c + 1]),
                  v.z * rs * to_f<T>(gain[c + 2]), v.w * rs * to_f<T>(gain[c + 3]));
    }
}

// ------------------------------------------------------------------ RoPE + K/V placement
// blockIdx.x < rows: one row, blockIdx.y = slice of the row's work (Q rotation, K rotation and placement).
// blockIdx.x >= rows: one 16-key V tile of one sequence (a cache page the causal rows touch, or a scratch tile of
// the mask rows), blockIdx.y = slice of its (kv head, d) pairs.  V is kept transposed ([d][16 keys]); written row
// by row that is one 2-byte store per value, 32 bytes apart (measured: 2.8 times the bytes at the memory side and
// half of this kernel's time at batch 32), so the tile blocks gather by (head, d) and write whole pieces.
// qkv_part: tiled GEMM output, [S] x (q_dim + 2 kv_dim) columns.  Q rows -> q_out [M][q_dim];
// K/V of causal rows -> cache at position L + r; K/V of mask rows -> scratch tiles
// k_scr [B][n_kv][n_mtiles][16][hd], v_scr [B][n_kv][n_mtiles][hd][16].
template <typename T>
__global__ __launch_bounds__(256) void rope_kv_kernel(const float *__restrict__ part, int S, size_t split_stride,
                                                      const float *__restrict__ rope_cs,
                                                      const int32_t *__restrict__ prefix_len, RowDesc d, int n_q,
                                                      int M_all, KvView kv, T *__restrict__ q_out,
                                                      T *__restrict__ k_scr, T *__restrict__ v_scr) {
    const int hd = kv.hd, half = hd / 2, n_kv = kv.n_kv;
    const int q_dim = n_q * hd, kv_dim = n_kv * hd;
    if ((int)blockIdx.x >= M_all) {
        // item = (kv head, d, quarter of the tile's 16 keys): four keys gathered, 8 bytes (bf16) written; the four
        // quarters of a d are neighbouring lanes, so a wave still writes one contiguous run
        const int n_ct = (d.nc + 15) / 16 + 1;           // cache pages the causal rows can touch
        const int n_mtiles = (d.nm + 15) / 16;
        const int items = n_kv * hd * 4;
        const int per_blk = gridDim.y * blockDim.x;
        const int parts = (items + per_blk - 1) / per_blk;
        int vb = blockIdx.x - M_all;
        const int part_i = vb % parts;
        vb /= parts;
        const int b = vb / (n_ct + n_mtiles), t = vb - b * (n_ct + n_mtiles);
        const int idx = (part_i * gridDim.y + blockIdx.y) * blockDim.x + threadIdx.x;
        if (idx >= items) return;
        const int L_raw = prefix_len[d.seq_base + b];
        const int L = clamp_prefix(kv, L_raw, d.nc);
        int r0, lo, hi;                                  // the tile's key s is row r0 + s; keys [lo, hi) exist
        T *base;                                         // [n_kv][hd][16] of this tile, strided per head by hstride
        size_t hstride;
        if (t < n_ct) {
            if (!seq_fits(kv, L_raw, d.nc)) return;      // a sequence that does not fit stores nothing in the cache
            const int p = (L >> 4) + t;
            r0 = 16 * p - L;
            lo = max(0, -r0);
            hi = min(16, d.nc - r0);
            if (hi <= lo) return;
            const int page = kv.page_table[(size_t)(d.seq_base + b) * kv.pages_per_seq + p];
            if (!page_ok(kv, page)) return;
            base = (T *)kv.v_pages + v_page_offset(kv, page, 0, 0, 0);
            hstride = (size_t)hd * 16;
        } else {
            const int mt = t - n_ct;
            r0 = d.nc + 16 * mt;
            lo = 0;
            hi = min(16, d.nm - 16 * mt);
            base = v_scr + (size_t)b * n_kv * n_mtiles * hd * 16 + (size_t)mt * hd * 16;
            hstride = (size_t)n_mtiles * hd * 16;
        }
        const int qd = idx & 3, hdd = idx >> 2;
        const int h = hdd / hd, dd = hdd - h * hd;
        const int s0 = 4 * qd;
        T *dst = base + h * hstride + (size_t)dd * 16 + s0;
        const bool keep = t < n_ct && (s0 < lo || s0 + 4 > hi);     // slots of earlier or later tokens in this piece
        T vals[4];
        if (keep) {
#pragma unroll
            for (int e = 0; e < 4; ++e) vals[e] = dst[e];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) vals[e] = from_f<T>(0.f);
        }
        const float *pp[4];
        float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int s = min(max(s0 + e, lo), hi - 1);       // clamped: an existing row, value unused if outside
            pp[e] = part + pt_index(q_dim + kv_dim + h * hd + dd, b * d.R + r0 + s, M_all);
        }
#pragma unroll 4
        for (int sp = 0; sp < S; ++sp) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += pp[e][(size_t)sp * split_stride];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (s0 + e >= lo && s0 + e < hi) vals[e] = from_f<T>(v[e]);
        typedef T vec4 __attribute__((ext_vector_type(4)));
        *(vec4 *)dst = (vec4){vals[0], vals[1], vals[2], vals[3]};
        return;
    }
    const int row = blockIdx.x;
    const int b = row / d.R;
    const int r = row - b * d.R;
    const int per_head = half / 4;                   // groups of four rotation pairs
    const float *cs = rope_cs + (size_t)row * half * 2;
    auto val4 = [&](int col) {
        const float *pp = part + pt_index(col, row, M_all);
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
        for (int sp = 0; sp < S; ++sp) {
            float4 q = *(const float4 *)(pp + (size_t)sp * split_stride);
            v.x += q.x; v.y += q.y; v.z += q.z; v.w += q.w;
        }
        return v;
    };
    auto rotate = [&](float4 a, float4 bb, int i, float4 &lo, float4 &hi) {
        float4 c0 = *(const float4 *)(cs + 2 * i), c1 = *(const float4 *)(cs + 2 * i + 4);   // (cos,sin) x 4
        lo = make_float4(a.x * c0.x - bb.x * c0.y, a.y * c0.z - bb.y * c0.w, a.z * c1.x - bb.z * c1.y,
                         a.w * c1.z - bb.w * c1.w);
        hi = make_float4(bb.x * c0.x + a.x * c0.y, bb.y * c0.z + a.y * c0.w, bb.z * c1.x + a.z * c1.y,
                         bb.w * c1.z + a.w * c1.w);
    };
    // blockIdx.y: the first q_blocks workgroups of a row rotate Q (one item per thread), the rest place K/V
    const int q_blocks = (n_q * per_head + blockDim.x - 1) / blockDim.x;
    if ((int)blockIdx.y < q_blocks) {
        const int idx = blockIdx.y * blockDim.x + threadIdx.x;
        if (idx < n_q * per_head) {
            int h = idx / per_head, i = 4 * (idx - h * per_head);
            float4 lo, hi;
            rotate(val4(h * hd + i), val4(h * hd + i + half), i, lo, hi);
            T *qo = q_out + (size_t)row * q_dim + h * hd + i;
            store4<T>(qo, lo.x, lo.y, lo.z, lo.w);
            store4<T>(qo + half, hi.x, hi.y, hi.z, hi.w);
        }
        return;
    }
    // destination of this row's K/V
    const bool causal = r < d.nc;
    const int L_raw = prefix_len[d.seq_base + b];
    const int L = clamp_prefix(kv, L_raw, d.nc);
    int page = 0, slot = 0, mt = 0;
    const int n_mtiles = (d.nm + 15) / 16;
    if (causal) {
        int p = L + r;
        page = kv.page_table[(size_t)(d.seq_base + b) * kv.pages_per_seq + (p >> 4)];
        slot = p & 15;
        if (!seq_fits(kv, L_raw, d.nc) || !page_ok(kv, page)) return;     // nothing of this row reaches the cache
    } else {
        int m = r - d.nc;
        mt = m >> 4;
        slot = m & 15;
    }
    T *kp = (T *)kv.k_pages;
    for (int idx = (blockIdx.y - q_blocks) * blockDim.x + threadIdx.x; idx < n_kv * per_head;
         idx += (gridDim.y - q_blocks) * blockDim.x) {
        int h = idx / per_head, i = 4 * (idx - h * per_head);
        float4 lo, hi;
        rotate(val4(q_dim + h * hd + i), val4(q_dim + h * hd + i + half), i, lo, hi);
        T *kdst;                   // K: [slot][hd] contiguous in d (V goes by tiles, above)
        if (causal) {
            kdst = kp + k_page_offset(kv, page, h, slot, 0);
        } else {
            size_t tile = ((size_t)b * n_kv + h) * n_mtiles + mt;
            kdst = k_scr + (tile * 16 + slot) * hd;
        }
        store4<T>(kdst + i, lo.x, lo.y, lo.z, lo.w);
        store4<T>(kdst + i + half, hi.x, hi.y, hi.z, hi.w);
    }
}

// K/V given directly (attention entry point): same placement, no rotation.
template <typename T>
__global__ void place_kv_kernel(const T *__restrict__ k_new, const T *__restrict__ v_new,
                                const int32_t *__restrict__ prefix_len, RowDesc d, KvView kv, T *__restrict__ k_scr,
                                T *__restrict__ v_scr) {
    int row = blockIdx.x;
    int b = row / d.R;
    int r = row - b * d.R;
    int hd = kv.hd, n_kv = kv.n_kv;
    bool causal = r < d.nc;
    const int L_raw = prefix_len[d.seq_base + b];
    int L = clamp_prefix(kv, L_raw, d.nc);
    int page = 0, slot = 0, mt = 0;
    int n_mtiles = (d.nm + 15) / 16;
    if (causal) {
        int p = L + r;
        page = kv.page_table[(size_t)(d.seq_base + b) * kv.pages_per_seq + (p >> 4)];
        slot = p & 15;
        if (!seq_fits(kv, L_raw, d.nc) || !page_ok(kv, page)) return;
    } else {
        int m = r - d.nc;
        mt = m >> 4;
        slot = m & 15;
    }
    T *kp = (T *)kv.k_pages;
    T *vp = (T *)kv.v_pages;
    for (int idx = threadIdx.x; idx < n_kv * hd; idx += blockDim.x) {
        int h = idx / hd, i = idx - h * hd;
        T kk = k_new[(size_t)row * n_kv * hd + idx], vv = v_new[(size_t)row * n_kv * hd + idx];
        if (causal) {
            kp[k_page_offset(kv, page, h, slot, i)] = kk;
            vp[v_page_offset(kv, page, h, slot, i)] = vv;
        } else {
            size_t tile = ((size_t)b * n_kv + h) * n_mtiles + mt;
            k_scr[(tile * 16 + slot) * hd + i] = kk;
            v_scr[(tile * hd + i) * 16 + slot] = vv;
        }
    }
}

// ------------------------------------------------------------------ SwiGLU over interleaved gate/up columns
// part: tiled GEMM output with 2*d_ff columns (tile 2t = gate, 2t+1 = up); out: A-fragment layout, K = d_ff.
template <typename T>
__global__ void swiglu_kernel(const float *__restrict__ part, int S, size_t split_stride, int M, int d_ff,
                              T *__restrict__ out, ActLayout lay) {
    const int per_row = d_ff / 4;
    size_t n = (size_t)M * per_row;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x) {
        // consecutive threads walk down the rows of one column group: the tiled layout is row-contiguous
        int row = (int)(idx % M);
        int f = 4 * (int)(idx / M);
        const float *pg = part + pt_index(32 * (f >> 4) + (f & 15), row, M);
        const float *pu = part + pt_index(32 * (f >> 4) + 16 + (f & 15), row, M);
        float4 g = make_float4(0.f, 0.f, 0.f, 0.f), u = g;
        for (int sp = 0; sp < S; ++sp) {
            float4 a = *(const float4 *)(pg + (size_t)sp * split_stride);
            float4 c = *(const float4 *)(pu + (size_t)sp * split_stride);
            g.x += a.x; g.y += a.y; g.z += a.z; g.w += a.w;
            u.x += c.x; u.y += c.y; u.z += c.z; u.w += c.w;
        }
        store4<T>(out + af_index(row, f, lay), g.x / (1.f + __expf(-g.x)) * u.x, g.y / (1.f + __expf(-g.y)) * u.y,
                  g.z / (1.f + __expf(-g.z)) * u.z, g.w / (1.f + __expf(-g.w)) * u.w);
    }
}

// ------------------------------------------------------------------ vocabulary argmax / Gumbel-max
// One block per (sequence, row o < n_rows) over materialised logits with Rh rows per sequence.
__global__ void argmax_rows_kernel(const float *__restrict__ logits, int Rh, int n_rows, int vocab, int n_choose,
                                   const int32_t *__restrict__ pos_rows, int pos_stride, int pos_row0, int seq_base,
                                   int sample, float temperature, uint64_t seed, float beta, int mix_base,
                                   int mix_stride, int32_t *__restrict__ y, int y_stride) {
    int b = blockIdx.x / n_rows;
    int o = blockIdx.x - b * n_rows;
    const float *lg = logits + ((size_t)b * Rh + o) * vocab;
    bool choose = o < n_choose;            // a row whose token is *taken* (causal logits)
    const float *mix = nullptr;
    if (choose && beta != 1.0f) mix = logits + ((size_t)b * Rh + mix_base + (size_t)o * mix_stride) * vocab;
    bool noisy = choose && sample;
    uint64_t key = 0;
    float inv_t = 1.f;
    if (noisy) {
        int pos_pred = pos_rows[(size_t)b * pos_stride + pos_row0 + o] + 1;      // causal rows are label shifted
        key = noise_key(seed, seq_base + b, pos_pred);
        inv_t = 1.f / temperature;
    }
    float best = -INFINITY;
    int best_i = 0x7fffffff;
    for (int v = threadIdx.x; v < vocab; v += blockDim.x) {
        float val = lg[v];
        if (mix) val = beta * val + (1.f - beta) * mix[v];
        if (noisy) val = perturbed_logit(val, inv_t, key, (uint32_t)v);
        if (val > best || (val == best && v < best_i)) { best = val; best_i = v; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        float ob = __shfl_xor(best, off);
        int oi = __shfl_xor(best_i, off);
        if (ob > best || (ob == best && oi < best_i)) { best = ob; best_i = oi; }
    }
    __shared__ float sb[16];
    __shared__ int si[16];
    if ((threadIdx.x & 63) == 0) { sb[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = best_i; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < (int)(blockDim.x >> 6); ++w)
            if (sb[w] > best || (sb[w] == best && si[w] < best_i)) { best = sb[w]; best_i = si[w]; }
        y[(size_t)b * y_stride + o] = best_i == 0x7fffffff ? -1 : best_i;     // a row without a single number
                                                                              // (all NaN) has no token
    }
}

// ------------------------------------------------------------------ log-probability of a label under a row of logits
// One block per row of one scoring pass over text positions [c0, c0 + nc) of a sequence of `len` tokens.  Causal row
// r is label shifted (Section 3.1): it scores token c0 + r + 1 into ar_out[c0 + r] (0 when the text ends there);
// mask row m is scored against the token it stands in for, c0 + m, into diff_out[c0 + m].
// log p = logit[label] - (max + ln sum exp(logit - max)), two passes over the row.
__global__ __launch_bounds__(1024) void score_rows_kernel(const float *__restrict__ logits, int vocab,
                                                         const int32_t *__restrict__ text, int len, int c0, int nc,
                                                         float *__restrict__ ar_out, float *__restrict__ diff_out) {
    const int r = blockIdx.x;
    const float *lg = logits + (size_t)r * vocab;
    const bool causal = r < nc;
    const int i = c0 + (causal ? r : r - nc);
    const int li = causal ? i + 1 : i;
    float *dst = (causal ? ar_out : diff_out) + i;
    if (li >= len) {                       // uniform over the block
        if (threadIdx.x == 0) *dst = 0.f;
        return;
    }
    const int label = text[li];
    if ((unsigned)label >= (unsigned)vocab) {     // uniform over the block: an id outside the vocabulary scores NaN
        if (threadIdx.x == 0) *dst = __builtin_nanf("");
        return;
    }
    __shared__ float red[16];
    __shared__ float bc;
    const int nw = blockDim.x >> 6;
    float mx = -INFINITY;
    for (int v = 4 * threadIdx.x; v < vocab; v += 4 * blockDim.x) {        // vocab is a multiple of 16
        const float4 q = *(const float4 *)(lg + v);
        mx = fmaxf(fmaxf(mx, fmaxf(q.x, q.y)), fmaxf(q.z, q.w));
    }
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        float m = red[0];
        for (int w = 1; w < nw; ++w) m = fmaxf(m, red[w]);
        bc = m;
    }
    __syncthreads();
    mx = bc;
    float sum = 0.f;
    for (int v = 4 * threadIdx.x; v < vocab; v += 4 * blockDim.x) {
        const float4 q = *(const float4 *)(lg + v);
        sum += (expf(q.x - mx) + expf(q.y - mx)) + (expf(q.z - mx) + expf(q.w - mx));
    }
    sum = wave_sum(sum);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int w = 0; w < nw; ++w) t += red[w];
        *dst = lg[label] - (mx + logf(t));
    }
}

// Section 3.1 objective of one sequence from its per-token log-probabilities: both sums run over the first len-1
// entries and are divided by len-1; the causal one is weighted by alpha, the total by 1/(1+alpha).  Without a mask
// section (diff == nullptr) the result is the plain mean negative log-likelihood.  One block, fixed summation order;
// n = len - 1.
__global__ __launch_bounds__(256) void score_loss_kernel(const float *__restrict__ ar, const float *__restrict__ diff,
                                                        int n, float alpha, float *__restrict__ loss) {
    float sa = 0.f, sd = 0.f;
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        sa += ar[i];
        if (diff) sd += diff[i];
    }
    sa = wave_sum(sa);
    sd = wave_sum(sd);
    __shared__ float ra[4], rd[4];
    if ((threadIdx.x & 63) == 0) { ra[threadIdx.x >> 6] = sa; rd[threadIdx.x >> 6] = sd; }
    __syncthreads();
    if (threadIdx.x == 0) {
        const float ta = ((ra[0] + ra[1]) + ra[2]) + ra[3], td = ((rd[0] + rd[1]) + rd[2]) + rd[3];
        float v = 0.f;
        if (n > 0) v = diff ? (alpha * (-ta / n) + (-td / n)) / (1.f + alpha) : -ta / n;
        *loss = v;
    }
}

// ------------------------------------------------------------------ verify / accept / commit / next-draft select
// y: [B][k(k+1)] chosen token per row (rows: c_0..c_{k-1}, blk_0[0..k), ...).  One wavefront per sequence: lane i
// holds draft i, the token its causal row chose and the answer to "is draft i what row i-1 chose"; the acceptance
// length is the position of the first lane that says no.  The same wavefront is the call's device-side checker:
// a sequence that did not fit the page table, that wrote through a page id outside the pool, that was fed a token
// id outside the vocabulary or whose needed rows chose no token (all NaN) is reported with accepted_len 0, its
// tokens -1 and its prefix length untouched (the forward stored nothing of it where the store was unsafe).
__global__ __launch_bounds__(64) void verify_step_kernel(const int32_t *__restrict__ y,
                                                         const int32_t *__restrict__ drafts, int k, int vocab,
                                                         KvView kv, int seq_base, int32_t *__restrict__ prefix_len,
                                                         int32_t *__restrict__ accepted_len,
                                                         int32_t *__restrict__ accepted_tokens,
                                                         int32_t *__restrict__ next_drafts) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int R = k * (k + 1);
    const int32_t *yb = y + (size_t)b * R;
    const int L = prefix_len[b];
    const bool fits = seq_fits(kv, L, k);
    const bool mine = lane < k;
    const int c = mine ? drafts[(size_t)b * k + lane] : 0;
    const int y_prev = (mine && lane > 0) ? yb[lane - 1] : 0;            // causal row i-1 judges draft i
    bool bad = mine && (unsigned)c >= (unsigned)vocab;
    if (mine && fits) {
        const int page = kv.page_table[(size_t)(seq_base + b) * kv.pages_per_seq + ((L + lane) >> 4)];
        bad = bad || !page_ok(kv, page);
    }
    const unsigned long long no = __ballot(mine && lane > 0 && c != y_prev) | (1ull << k);
    const int a = __ffsll((long long)no) - 1;                            // first rejected draft = tokens accepted, 1..k
    const int nxt = !mine ? 0 : lane == 0 ? yb[a - 1] : yb[k + (a - 1) * k + lane];
    bad = bad || (mine && nxt < 0);
    const bool err = !fits || __ballot(bad) != 0ull;
    if (mine) {
        accepted_tokens[(size_t)b * k + lane] = (!err && lane < a) ? c : -1;
        next_drafts[(size_t)b * k + lane] = err ? -1 : nxt;
    }
    if (lane == 0) {
        accepted_len[b] = err ? 0 : a;
        if (!err) prefix_len[b] = L + a;           // commit: rejected drafts' K/V fall behind the frontier
    }
}

__global__ __launch_bounds__(64) void finish_ar_kernel(const int32_t *__restrict__ y,
                                                       const int32_t *__restrict__ token_in, int B, int vocab,
                                                       KvView kv, int32_t *__restrict__ prefix_len,
                                                       int32_t *__restrict__ token_out) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int L = prefix_len[b];
    bool err = !seq_fits(kv, L, 1) || (unsigned)token_in[b] >= (unsigned)vocab || y[b] < 0;
    if (!err) err = !page_ok(kv, kv.page_table[(size_t)b * kv.pages_per_seq + (L >> 4)]);
    token_out[b] = err ? -1 : y[b];
    if (!err) prefix_len[b] = L + 1;
}

// One wavefront per prefill pass over prompt positions [L, L + add_len) of sequence `seq`.  A pass that was fed a
// token id outside the vocabulary or met a page id outside the pool marks the sequence: prefix_len = -1, which
// keeps every later pass from storing anything for it, and first_drafts = -1.
__global__ __launch_bounds__(64) void finish_prefill_kernel(const int32_t *__restrict__ y,
                                                            const int32_t *__restrict__ tokens, int k, int seq,
                                                            int add_len, int last, int vocab, KvView kv,
                                                            int32_t *__restrict__ prefix_len,
                                                            int32_t *__restrict__ first_drafts) {
    const int lane = threadIdx.x;
    const int L = prefix_len[seq];
    bool bad = !seq_fits(kv, L, add_len);
    if (!bad) {
        for (int i = lane; i < add_len; i += 64) bad = bad || (unsigned)tokens[i] >= (unsigned)vocab;
        for (int p = (L >> 4) + lane; p <= ((L + add_len - 1) >> 4); p += 64)
            bad = bad || !page_ok(kv, kv.page_table[(size_t)seq * kv.pages_per_seq + p]);
    }
    // y rows: last prompt row, then mask slots 0..k-1; slot 0 of the block is superseded by the causal token
    int tok = 0;
    if (last && lane < k) {
        tok = (lane == 0) ? y[0] : y[1 + lane];
        bad = bad || tok < 0;
    }
    const bool err = __ballot(bad) != 0ull;
    if (lane == 0) prefix_len[seq] = err ? -1 : L + add_len;
    if ((last || err) && lane < k) first_drafts[(size_t)seq * k + lane] = err ? -1 : tok;
}

// plain row-major [M][K] -> A-fragment layout (8 elements per thread)
template <typename T>
__global__ void pack_act_kernel(const T *__restrict__ src, int M, int K, T *__restrict__ dst, ActLayout lay) {
    size_t n = (size_t)M * (K / 8);
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x) {
        int row = (int)(idx / (K / 8));
        int k = 8 * (int)(idx % (K / 8));
        const T *sp = src + (size_t)row * K + k;
        T *dp = dst + af_index(row, k, lay);
#pragma unroll
        for (int j = 0; j < 8; ++j) dp[j] = sp[j];
    }
}

// tiled partial sums [S][N/32][M][32] -> plain row-major [M][N]
__global__ void untile_sum_kernel(const float *__restrict__ part, int S, int M, int N, float *__restrict__ out) {
    size_t n = (size_t)M * N, stride = pt_split_stride(M, N);
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x) {
        int row = (int)(idx / N), col = (int)(idx % N);
        float v = 0.f;
        for (int sp = 0; sp < S; ++sp) v += part[(size_t)sp * stride + pt_index(col, row, M)];
        out[idx] = v;
    }
}

// Fold of the LM head's per-group maxima ([G][M] values, then [G][M] columns).  A block takes RB rows (a power
// of two, at most 16) and splits the groups over 1024 / RB slices; the slices are folded by a tree in LDS.  The
// order (larger value, then lower column) is total, so the result does not depend on how the fold is grouped.
__global__ __launch_bounds__(1024) void argmax_groups_kernel(const float *__restrict__ part, int M, int G, int RB,
                                                             int32_t *__restrict__ y) {
    const int r = threadIdx.x & (RB - 1), sl = threadIdx.x / RB, SL = 1024 / RB;
    const int row = blockIdx.x * RB + r;
    const float *pmax = part;
    const int *pidx = (const int *)(part + (size_t)G * M);
    float best = -INFINITY;
    int bi = 0x7fffffff;
    auto take = [&](float v, int i) {
        if (v > best || (v == best && i < bi)) {
            best = v;
            bi = i;
        }
    };
    if (row < M) {
        int g = sl;
        for (; g + 3 * SL < G; g += 4 * SL) {      // four independent loads at a time
            const float v0 = pmax[(size_t)g * M + row], v1 = pmax[(size_t)(g + SL) * M + row];
            const float v2 = pmax[(size_t)(g + 2 * SL) * M + row], v3 = pmax[(size_t)(g + 3 * SL) * M + row];
            const int i0 = pidx[(size_t)g * M + row], i1 = pidx[(size_t)(g + SL) * M + row];
            const int i2 = pidx[(size_t)(g + 2 * SL) * M + row], i3 = pidx[(size_t)(g + 3 * SL) * M + row];
            take(v0, i0);
            take(v1, i1);
            take(v2, i2);
            take(v3, i3);
        }
        for (; g < G; g += SL) take(pmax[(size_t)g * M + row], pidx[(size_t)g * M + row]);
    }
    __shared__ float sv[1024];
    __shared__ int si[1024];
    sv[threadIdx.x] = best;
    si[threadIdx.x] = bi;
    __syncthreads();
    for (int half = SL >> 1; half >= 1; half >>= 1) {
        if (sl < half) {
            take(sv[threadIdx.x + half * RB], si[threadIdx.x + half * RB]);
            sv[threadIdx.x] = best;
            si[threadIdx.x] = bi;
        }
        __syncthreads();
    }
    if (sl == 0 && row < M) y[row] = bi == 0x7fffffff ? -1 : bi;      // same rule as argmax_rows_kernel
}

__global__ void set_i32_kernel(int32_t *p, int n, int32_t v) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// ------------------------------------------------------------------ fp32 GEMM (plain ALU)
// a: A-fragment layout (fp32 elements), w: row-major [N][K], out: tiled or row-major.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ a, const float *__restrict__ w,
                                                       float *__restrict__ out, int M, int N, int K,
                                                       int out_row_major) {
    __shared__ float As[16][33];
    __shared__ float Ws[64][33];
    const int n0 = blockIdx.x * 64, m0 = blockIdx.y * 16;
    const int tc = threadIdx.x & 63, tr = threadIdx.x >> 6;      // column, row group (4 rows each)
    const ActLayout lay = act_layout(M);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < K; k0 += 32) {
        for (int i = threadIdx.x; i < 16 * 32; i += 256) {
            int r = i >> 5, c = i & 31;
            As[r][c] = (m0 + r < M && k0 + c < K) ? a[af_index(m0 + r, k0 + c, lay)] : 0.f;
        }
        for (int i = threadIdx.x; i < 64 * 32; i += 256) {
            int r = i >> 5, c = i & 31;
            Ws[r][c] = (n0 + r < N && k0 + c < K) ? w[(size_t)(n0 + r) * K + k0 + c] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int c = 0; c < 32; ++c) {
            float wv = Ws[tc][c];
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = fmaf(As[tr * 4 + i][c], wv, acc[i]);
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i) {
        int m = m0 + tr * 4 + i, n = n0 + tc;
        if (m < M && n < N) out[out_row_major ? (size_t)m * N + n : pt_index(n, m, M)] = acc[i];
    }
}

// ------------------------------------------------------------------ fp32 hybrid-mask attention (plain ALU)
// One wave per (sequence, query head, row).  Keys: cache positions [0, L + nc) then the mask rows' scratch tiles.
__global__ __launch_bounds__(64) void attention_f32_kernel(const float *__restrict__ q, KvView kv,
                                                           const float *__restrict__ k_scr,
                                                           const float *__restrict__ v_scr,
                                                           const int32_t *__restrict__ prefix_len, RowDesc d, int n_q,
                                                           float *__restrict__ out, int out_af, ActLayout lay) {
    int row = blockIdx.x;                  // b * R + r
    int head = blockIdx.y;
    int b = row / d.R, r = row - b * d.R;
    int hd = kv.hd, n_kv = kv.n_kv;
    int g = head / (n_q / n_kv);
    int L = clamp_prefix(kv, prefix_len[d.seq_base + b], d.nc);
    RowInfo ri = row_info(d, r, L);
    int n_cache = L + d.nc, n_mask = d.nm, n_mtiles = (n_mask + 15) / 16;
    int T = n_cache + n_mask;
    const float *kp = (const float *)kv.k_pages;
    const float *vp = (const float *)kv.v_pages;
    const int32_t *pt = kv.page_table + (size_t)(d.seq_base + b) * kv.pages_per_seq;
    __shared__ float qs[128];
    __shared__ float ps[64];
    int lane = threadIdx.x;
    for (int i = lane; i < hd; i += 64) qs[i] = q[((size_t)row * n_q + head) * hd + i];
    __syncthreads();
    float scale = rsqrtf((float)hd);
    float m_run = -INFINITY, l_run = 0.f;
    float o0 = 0.f, o1 = 0.f;              // this lane's output dims: lane, lane + 64
    for (int t0 = 0; t0 < T; t0 += 64) {
        int t = t0 + lane;
        bool vis = false;
        const float *krow = nullptr;
        if (t < n_cache) {
            vis = (t < L) || (t - L < ri.vis);
            const int page = pt[t >> 4];
            krow = kp + k_page_offset(kv, page_ok(kv, page) ? page : 0, g, t & 15, 0);
        } else if (t < T) {
            int m = t - n_cache;
            vis = (ri.blk >= 0) && (m / d.bl == ri.blk);
            krow = k_scr + ((((size_t)b * n_kv + g) * n_mtiles + (m >> 4)) * 16 + (m & 15)) * hd;
        }
        float s = -INFINITY;
        if (vis) {
            float acc = 0.f;
            for (int i = 0; i < hd; ++i) acc = fmaf(qs[i], krow[i], acc);
            s = acc * scale;
        }
        float mx = wave_max(s);
        if (mx == -INFINITY) continue;     // nothing visible in this chunk (uniform across the wave)
        float m_new = fmaxf(m_run, mx);
        float alpha = __expf(m_run - m_new);
        float p = vis ? __expf(s - m_new) : 0.f;
        l_run = l_run * alpha + wave_sum(p);
        o0 *= alpha;
        o1 *= alpha;
        m_run = m_new;
        ps[lane] = p;
        __syncthreads();
        int lim = min(64, T - t0);
        for (int j = 0; j < lim; ++j) {
            float pj = ps[j];
            if (pj == 0.f) continue;
            int tj = t0 + j;
            const float *vbase;
            size_t stride_d;
            if (tj < n_cache) {
                const int page = pt[tj >> 4];
                vbase = vp + v_page_offset(kv, page_ok(kv, page) ? page : 0, g, tj & 15, 0);
                stride_d = 16;
            } else {
                int m = tj - n_cache;
                vbase = v_scr + (((size_t)b * n_kv + g) * n_mtiles + (m >> 4)) * hd * 16 + (m & 15);
                stride_d = 16;
            }
            if (lane < hd) o0 = fmaf(pj, vbase[(size_t)lane * stride_d], o0);
            if (lane + 64 < hd) o1 = fmaf(pj, vbase[(size_t)(lane + 64) * stride_d], o1);
        }
        __syncthreads();
    }
    float inv = 1.f / l_run;
    auto oidx = [&](int dd) {
        return out_af ? af_index(row, head * hd + dd, lay) : ((size_t)row * n_q + head) * hd + dd;
    };
    if (lane < hd) out[oidx(lane)] = o0 * inv;
    if (lane + 64 < hd) out[oidx(lane + 64)] = o1 * inv;
}

inline int grid_for(size_t n, int block, int cap = 4096) {
    size_t g = (n + block - 1) / block;
    return (int)(g < 1 ? 1 : (g > (size_t)cap ? cap : g));
}

}  // namespace

void launch_pack_weight(int dtype, const void *src, int rows, int cols, void *dst, int dst_rows, int tile_off,
                        int tile_stride, hipStream_t st) {
    if (dtype == TIDAR_BF16) {
        size_t n = (size_t)rows * (cols / 8);
        pack_bf16_kernel<<<grid_for(n, 256, 65536), 256, 0, st>>>((const bf16_t *)src, rows, cols, (bf16_t *)dst,
                                                                   (dst_rows + 31) / 32, tile_off, tile_stride);
    } else {
        size_t n = (size_t)rows * cols;
        pack_f32_kernel<<<grid_for(n, 256, 65536), 256, 0, st>>>((const float *)src, rows, cols, (float *)dst,
                                                                  tile_off, tile_stride);
    }
}

void launch_embed_rows(int dtype, const void *embed, const int32_t *tokens, int tok_stride, const int32_t *prefix_len,
                       RowDesc d, int B, int d_model, int mask_id, int vocab, KvView kv, float rope_base, float *x,
                       int32_t *pos_out, float *rope_cs, hipStream_t st) {
    int rows = B * d.R;
    if (dtype == TIDAR_BF16)
        embed_rows_kernel<bf16_t><<<rows, 256, 0, st>>>((const bf16_t *)embed, tokens, tok_stride, prefix_len, d,
                                                         d_model, mask_id, vocab, kv, kv.hd, rope_base, x, pos_out,
                                                         rope_cs);
    else
        embed_rows_kernel<float><<<rows, 256, 0, st>>>((const float *)embed, tokens, tok_stride, prefix_len, d,
                                                        d_model, mask_id, vocab, kv, kv.hd, rope_base, x, pos_out,
                                                        rope_cs);
}

void launch_rmsnorm(int dtype, float *x, const float *part, int S, const void *gain, float eps, int B, int R, int row0,
                    int d_model, void *out, hipStream_t st) {
    int rows = B * (R - row0), M_all = B * R;
    ActLayout mt_out = act_layout(rows);
    size_t stride = pt_split_stride(M_all, d_model);
    // a row is one workgroup's only work: with few rows the chip is empty anyway, so a row gets as many threads
    // as it has 4-column pieces (all of its loads in flight at once); with many rows the count measured no difference
    int threads = 256;
    if (rows <= 64) {
        threads = ((d_model / 4 + 63) / 64) * 64;
        threads = threads > 1024 ? 1024 : threads < 64 ? 64 : threads;
    }
    if (dtype == TIDAR_BF16)
        rmsnorm_kernel<bf16_t><<<rows, threads, 0, st>>>(x, part, S, stride, (const bf16_t *)gain, eps, R, row0,
                                                          d_model, M_all, (bf16_t *)out, mt_out);
    else
        rmsnorm_kernel<float><<<rows, threads, 0, st>>>(x, part, S, stride, (const float *)gain, eps, R, row0, d_model,
                                                         M_all, (float *)out, mt_out);
}

void launch_gemm_f32(const float *a, const float *w, float *out, int M, int N, int K, int out_row_major,
                     hipStream_t st) {
    dim3 grid((N + 63) / 64, (M + 15) / 16);
    gemm_f32_kernel<<<grid, 256, 0, st>>>(a, w, out, M, N, K, out_row_major);
}

void launch_pack_act(int dtype, const void *src, int M, int K, void *dst, hipStream_t st) {
    size_t n = (size_t)M * (K / 8);
    ActLayout mt = act_layout(M);
    if (dtype == TIDAR_BF16)
        pack_act_kernel<bf16_t><<<grid_for(n, 256, 8192), 256, 0, st>>>((const bf16_t *)src, M, K, (bf16_t *)dst, mt);
    else
        pack_act_kernel<float><<<grid_for(n, 256, 8192), 256, 0, st>>>((const float *)src, M, K, (float *)dst, mt);
}

void launch_untile_sum(const float *part, int S, int M, int N, float *out, hipStream_t st) {
    untile_sum_kernel<<<grid_for((size_t)M * N, 256, 8192), 256, 0, st>>>(part, S, M, N, out);
}

void launch_rope_kv(int dtype, const float *qkv_part, int S, const float *rope_cs, const int32_t *prefix_len, RowDesc d,
                    int B, int n_q, KvView kv, void *q_out, void *k_scr, void *v_scr, hipStream_t st) {
    int rows = B * d.R;
    size_t stride = pt_split_stride(rows, (n_q + 2 * kv.n_kv) * kv.hd);
    const int per_head = kv.hd / 8;                  // items (four rotation pairs) per head
    const int gy = (n_q * per_head + 255) / 256 + (kv.n_kv * per_head + 255) / 256;
    const int v_parts = (kv.n_kv * kv.hd * 4 + gy * 256 - 1) / (gy * 256);      // see the kernel's V-tile branch
    const int v_tiles = B * ((d.nc + 15) / 16 + 1 + (d.nm + 15) / 16);
    dim3 grid(rows + v_tiles * v_parts, gy);
    if (dtype == TIDAR_BF16)
        rope_kv_kernel<bf16_t><<<grid, 256, 0, st>>>(qkv_part, S, stride, rope_cs, prefix_len, d, n_q, rows, kv,
                                                      (bf16_t *)q_out, (bf16_t *)k_scr, (bf16_t *)v_scr);
    else
        rope_kv_kernel<float><<<grid, 256, 0, st>>>(qkv_part, S, stride, rope_cs, prefix_len, d, n_q, rows, kv,
                                                     (float *)q_out, (float *)k_scr, (float *)v_scr);
}

void launch_place_kv(int dtype, const void *k_new, const void *v_new, const int32_t *prefix_len, RowDesc d, int B,
                     KvView kv, void *k_scr, void *v_scr, hipStream_t st) {
    int rows = B * d.R;
    if (dtype == TIDAR_BF16)
        place_kv_kernel<bf16_t><<<rows, 256, 0, st>>>((const bf16_t *)k_new, (const bf16_t *)v_new, prefix_len, d, kv,
                                                       (bf16_t *)k_scr, (bf16_t *)v_scr);
    else
        place_kv_kernel<float><<<rows, 256, 0, st>>>((const float *)k_new, (const float *)v_new, prefix_len, d, kv,
                                                      (float *)k_scr, (float *)v_scr);
}

void launch_attention_f32(const float *q, KvView kv, const float *k_scr, const float *v_scr,
                          const int32_t *prefix_len, RowDesc d, int B, int n_q, float *out, int out_af,
                          hipStream_t st) {
    dim3 grid(B * d.R, n_q);
    attention_f32_kernel<<<grid, 64, 0, st>>>(q, kv, k_scr, v_scr, prefix_len, d, n_q, out, out_af,
                                              act_layout(B * d.R));
}

void launch_swiglu(int dtype, const float *part, int S, int M, int d_ff, void *out, hipStream_t st) {
    size_t n = (size_t)M * (d_ff / 4);
    size_t stride = pt_split_stride(M, 2 * d_ff);
    ActLayout mt = act_layout(M);
    if (dtype == TIDAR_BF16)
        swiglu_kernel<bf16_t><<<grid_for(n, 256, 8192), 256, 0, st>>>(part, S, stride, M, d_ff, (bf16_t *)out, mt);
    else
        swiglu_kernel<float><<<grid_for(n, 256, 8192), 256, 0, st>>>(part, S, stride, M, d_ff, (float *)out, mt);
}

void launch_argmax_groups(const float *part, int M, int G, int32_t *y, hipStream_t st) {
    int RB = 16;
    while (RB > 1 && RB / 2 >= M) RB /= 2;       // smallest power of two that holds the rows, at most 16
    argmax_groups_kernel<<<(M + RB - 1) / RB, 1024, 0, st>>>(part, M, G, RB, y);
}

void launch_argmax_rows(const float *logits, int B, int Rh, int n_rows, int vocab, int n_choose,
                        const int32_t *pos_rows, int pos_stride, int pos_row0, int seq_base, int sample,
                        float temperature, uint64_t seed, float beta, int mix_base, int mix_stride, int32_t *y,
                        int y_stride, hipStream_t st) {
    argmax_rows_kernel<<<B * n_rows, 1024, 0, st>>>(logits, Rh, n_rows, vocab, n_choose, pos_rows, pos_stride, pos_row0,
                                                    seq_base, sample, temperature, seed, beta, mix_base, mix_stride, y,
                                                    y_stride);
}

void launch_score_rows(const float *logits, int rows, int vocab, const int32_t *text, int len, int c0, int nc,
                       float *ar_out, float *diff_out, hipStream_t st) {
    score_rows_kernel<<<rows, 1024, 0, st>>>(logits, vocab, text, len, c0, nc, ar_out, diff_out);
}

void launch_score_loss(const float *ar, const float *diff, int n, float alpha, float *loss, hipStream_t st) {
    score_loss_kernel<<<1, 256, 0, st>>>(ar, diff, n, alpha, loss);
}

void launch_verify_step(const int32_t *y, const int32_t *drafts, int k, int B, int vocab, KvView kv, int seq_base,
                        int32_t *prefix_len, int32_t *accepted_len, int32_t *accepted_tokens, int32_t *next_drafts,
                        hipStream_t st) {
    verify_step_kernel<<<B, 64, 0, st>>>(y, drafts, k, vocab, kv, seq_base, prefix_len, accepted_len, accepted_tokens,
                                         next_drafts);
}

void launch_finish_ar(const int32_t *y, const int32_t *token_in, int B, int vocab, KvView kv, int32_t *prefix_len,
                      int32_t *token_out, hipStream_t st) {
    finish_ar_kernel<<<(B + 63) / 64, 64, 0, st>>>(y, token_in, B, vocab, kv, prefix_len, token_out);
}

void launch_finish_prefill(const int32_t *y, const int32_t *tokens, int k, int seq, int add_len, int last, int vocab,
                           KvView kv, int32_t *prefix_len, int32_t *first_drafts, hipStream_t st) {
    finish_prefill_kernel<<<1, 64, 0, st>>>(y, tokens, k, seq, add_len, last, vocab, kv, prefix_len, first_drafts);
}

void launch_set_i32(int32_t *p, int n, int32_t v, hipStream_t st) {
    set_i32_kernel<<<(n + 255) / 256, 256, 0, st>>>(p, n, v);
}
