// Skinny bf16 GEMM of the decode step: out = A[M][K] (bf16) x W[N][K]^T (bf16), fp32 accumulation.
//
// M is the step's row count (1 .. 272 at batch 1; more rows run as row passes), N and K are model dimensions: every weight byte is used once
// per step, so the kernel is a weight streamer with MFMA attached.
//   * W lives in HBM as the register image of the 32x32x16 MFMA B operand
//     ([k step of 16][32-column tile][lane][8]); a wave's load of one fragment is one fully coalesced 1 KiB read
//     that goes straight to VGPRs through a ring many k steps deep.  Weights never pass through LDS.  The k
//     step is the outer index so that the workgroups, which all advance through K at the same pace, read one
//     contiguous front of the matrix.
//   * A lives in memory as the register image of the MFMA A operand (see ActLayout): the slice a workgroup
//     needs for a chunk of K is one contiguous block and its LDS image reads back conflict-free.
//   * every load is a raw buffer load: out-of-range tiles, rows and k steps are steered to an out-of-bounds
//     offset, which the hardware answers with zeros and no memory traffic.  The steady-state loop therefore
//     has no branches, and the compiler can keep exact in-flight counts (vmcnt(n), not vmcnt(0)) on the ring;
//     sched_barrier pins each reload right behind the MFMAs that free its slot.
//   * M <= 32: 16x16x32 MFMA (fewer pad rows), no LDS, no barriers; a wave streams its 32 columns and the A
//     fragments through two register rings.  M > 32: 32x32x16 MFMA (on gfx950 it issues at twice the rate of
//     16x16x32: measured 2.2 vs 1.2 PFLOP/s), A staged through LDS once per workgroup and prefetched into
//     registers ahead of the MFMAs; 4 waves either as a 2 x 2 grid over 128 columns (two row halves x two
//     64-column groups: launches without a row split), or side by side, every wave over all row tiles of the pass
//     (no weight fragment is then loaded by two waves): over 256 columns with two column tiles per wave for
//     single-split grids that are resident all at once and for the many-row class, over 128 columns with one
//     column tile per wave for the two-pass launches of 33-480 rows (no padded tile slots; twice the LDS fragment
//     reads per MFMA, which the LDS has room for).  The weight fragment is the MFMA's first operand, so the
//     accumulators hold the output transposed (lane = row): every epilogue starts from that.
//   * split-K over blockIdx.y works in units of 512 k, row passes over blockIdx.z; up to 480 rows the split count
//     depends on (N, K) and the kernel class (M <= 32 or not) only, so the partial-sum grouping of a row does not
//     depend on how many rows travel with it (from 481 rows on it also follows the number of 256-row passes).  Splits fill about half the CUs, two row passes the other half: a split
//     costs an M x N partial sum written and read again, a row pass only a second read of W from L2.
//   * output: [split][32-column tile][row][32] fp32 partial sums (summed in fixed order by the consumer), or
//     row-major logits, or - fused epilogues - bf16 SwiGLU products in the next GEMM's A-fragment layout, or
//     per-column-group (maximum, column) pairs for the greedy vocabulary reduction.
// 16x16x32: A lane l = row l%16, k slots 8*(l/16)..+7; B lane l = column l%16, same k slots; D lane l register i
// = row 4*(l/16)+i, column l%16.   32x32x16: A lane l = row l%32, k slots 8*(l/32)..+7; B lane l = column l%32;
// D lane l register i = row 8*(i/4) + 4*(l/32) + i%4, column l%32.
#include "tidar_internal.h"

namespace {

constexpr int SPLIT_UNIT = 512;           // k elements
constexpr int OOB = 0x7ffffff0;           // byte offset beyond any buffer: the load returns zeros

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *base, size_t bytes) {
    // raw buffer (stride 0), 32-bit data format; num_records in bytes
    return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)(bytes > 0x7fffffe0ull ? 0x7fffffe0ull : bytes),
                                             0x00020000);
}
__device__ inline bf16x8 buf_load(__amdgpu_buffer_rsrc_t r, int byte_off) {
    return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0));
}

struct SplitRange {
    int q0, q1;   // k steps [q0, q1)
};
__device__ inline SplitRange split_range(int K, int splits, int split) {
    const int units = (K + SPLIT_UNIT - 1) / SPLIT_UNIT;
    const int per = (units + splits - 1) / splits;
    SplitRange r;
    r.q0 = split * per * (SPLIT_UNIT / 32);
    r.q1 = min(K >> 5, (split + 1) * per * (SPLIT_UNIT / 32));
    return r;
}

// What the fused vocabulary reduction does with output row `row`: perturb its values before the maximum is formed
// (key, inv_t when noisy) and/or also write its logits to the compact buffer (sel >= 0: row index there).
struct RowChoice {
    bool noisy;
    uint64_t key;
    float inv_t;
    int sel;
};
__device__ inline RowChoice row_choice(const ChooseArgs &ch, int row, int M) {
    RowChoice rc;
    rc.noisy = false;
    rc.key = 0;
    rc.inv_t = 1.f;
    rc.sel = -1;
    if (ch.n_choose <= 0 || row >= M) return rc;
    const int b = row / ch.Rh, o = row - b * ch.Rh;
    if (o < ch.n_choose) {
        if (ch.sample) {
            rc.noisy = true;                // causal rows are label shifted: they predict the position after theirs
            rc.key = noise_key(ch.seed, ch.seq_base + b, ch.pos_rows[(size_t)b * ch.pos_stride + ch.pos_row0 + o] + 1);
            rc.inv_t = ch.inv_t;
        }
        if (ch.sel_logits) rc.sel = b * 2 * ch.n_choose + o;
    } else if (ch.sel_logits) {
        const int m = o - ch.n_choose;
        if (m % ch.mix_stride == 0 && m / ch.mix_stride < ch.n_choose) rc.sel = b * 2 * ch.n_choose + ch.n_choose + m / ch.mix_stride;
    }
    return rc;
}

template <int MTW, int NT>
__device__ inline void store_tiles(const f32x4 (&acc)[MTW][NT], float *out, int split, int M, int N, int tile0,
                                   int n_tiles, int mt0, int lane, int out_row_major, const ChooseArgs &ch) {
    if (out_row_major == GEMM_EPI_ARGMAX) {
        // lane l holds rows 4*(l/16)+i of a 16-row tile and column l%16 of each of its NT 16-column tiles: the
        // larger of its columns per row, then the 16 lanes of a row group are folded (ties: lowest column)
        const int G = ((N >> 4) + 1) >> 1;
        float *pmax = out;
        int *pidx = (int *)(out + (size_t)G * M);
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float best = -INFINITY;
                int bi = (tile0 << 4) + (lane & 15);
                const int row_i = (mt0 + mt) * 16 + (lane >> 4) * 4 + i;
                const RowChoice rc = row_choice(ch, row_i, M);
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    float v = acc[mt][j][i];
                    const int col = ((tile0 + j) << 4) + (lane & 15);
                    if (rc.sel >= 0 && tile0 + j < n_tiles) ch.sel_logits[(size_t)rc.sel * N + col] = v;
                    if (rc.noisy) v = perturbed_logit(v, rc.inv_t, rc.key, (uint32_t)col);
                    if (tile0 + j < n_tiles && v > best) {
                        best = v;
                        bi = ((tile0 + j) << 4) + (lane & 15);
                    }
                }
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) {
                    const float ob = __shfl_xor(best, o);
                    const int oi = __shfl_xor(bi, o);
                    if (ob > best || (ob == best && oi < bi)) {
                        best = ob;
                        bi = oi;
                    }
                }
                const int row = (mt0 + mt) * 16 + (lane >> 4) * 4 + i;
                if ((lane & 15) == 0 && row < M) {
                    pmax[(size_t)(tile0 >> 1) * M + row] = best;
                    pidx[(size_t)(tile0 >> 1) * M + row] = bi;
                }
            }
        }
        return;
    }
    if (out_row_major == GEMM_EPI_SWIGLU) {
        // the wave's two 16-column tiles are gate and up of the same 16 features (tile0 is even): a lane holds both
        // values of (row, feature), so h = silu(gate) * up needs no data movement; it is stored as bf16 in the
        // A-fragment layout of the next GEMM
        bf16_t *ho = reinterpret_cast<bf16_t *>(out);
        const ActLayout lay = act_layout(M);
        if (tile0 + 1 < n_tiles) {
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int row = (mt0 + mt) * 16 + (lane >> 4) * 4 + i;
                    const float g = acc[mt][0][i], u = acc[mt][1][i];
                    const float h = g * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g)) * u;
                    if (row < M) ho[af_index(row, (tile0 >> 1) * 16 + (lane & 15), lay)] = (bf16_t)h;
                }
        }
        return;
    }
    float *o = out + (size_t)split * pt_split_stride(M, N);
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        const int row0 = (mt0 + mt) * 16 + (lane >> 4) * 4;
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int tile = tile0 + j;
            if (tile >= n_tiles) continue;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = row0 + i;
                if (row < M) {
                    size_t idx = out_row_major == GEMM_EPI_ROWMAJOR ? (size_t)row * N + tile * 16 + (lane & 15)
                                               : pt_index(tile * 16 + (lane & 15), row, M);
                    o[idx] = acc[mt][j][i];
                }
            }
        }
    }
}

// ------------------------------------------------------------------ M <= 32: register rings only
template <int MT, int PFK>
__global__ __launch_bounds__(256) void gemm_bf16_small_kernel(const bf16_t *__restrict__ a,
                                                              const bf16_t *__restrict__ w, float *__restrict__ out,
                                                              int M, int N, int K, int splits, int out_row_major,
                                                              ChooseArgs ch) {
    constexpr int NT = 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_tiles = N >> 4, m_tiles = (M + 15) >> 4;
    const SplitRange sr = split_range(K, splits, blockIdx.y);
    const int tile0 = (blockIdx.x * 4 + wave) * NT;
    if (tile0 >= n_tiles) return;                              // no barriers in this kernel
    const __amdgpu_buffer_rsrc_t ra = make_rsrc(a, (size_t)(K >> 5) * m_tiles * 1024);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(w, (size_t)((N + 31) / 32) * 32 * K * 2);
    // byte offsets at k step 0; one k step further is n_tiles (resp. m_tiles) KiB on
    // W is stored for the 32x32x16 form; two of its k steps hold the 32 k of one 16x16x32 step.  Lane (n, g)
    // of the B operand takes its 8 values from stored k step 2Q + g/2, stored lane (g%2)*32 + 16*half + n:
    // k slot g then covers k = 32Q + 8g .. +7, the same slots the narrow A layout gives lane group g.
    const int t32 = (N + 31) >> 5;
    const int n = lane & 15, g = lane >> 4;
    int w_off[NT], a_off[MT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
        w_off[j] = (tile0 + j < n_tiles)
                       ? ((((g >> 1) * t32 + ((tile0 + j) >> 1)) * 64) + (g & 1) * 32 + ((tile0 + j) & 1) * 16 + n) * 16
                       : OOB;
#pragma unroll
    for (int i = 0; i < MT; ++i) a_off[i] = (i < m_tiles) ? (i * 64 + lane) * 16 : OOB;
    const int w_step = 2 * t32 * 1024, a_step = m_tiles * 1024;
    auto ld_w = [&](int j, int q) {
        return buf_load(rw, (q < sr.q1 && w_off[j] != OOB) ? w_off[j] + q * w_step : OOB);
    };
    auto ld_a = [&](int i, int q) {
        return buf_load(ra, (q < sr.q1 && a_off[i] != OOB) ? a_off[i] + q * a_step : OOB);
    };

    f32x4 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
    bf16x8 wbuf[PFK][NT], abuf[PFK][MT];
#pragma unroll
    for (int s = 0; s < PFK; ++s) {
#pragma unroll
        for (int j = 0; j < NT; ++j) wbuf[s][j] = ld_w(j, sr.q0 + s);
#pragma unroll
        for (int i = 0; i < MT; ++i) abuf[s][i] = ld_a(i, sr.q0 + s);
    }
    for (int qb = sr.q0; qb < sr.q1; qb += PFK) {
#pragma unroll
        for (int s = 0; s < PFK; ++s) {
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(abuf[s][i], wbuf[s][j], acc[i][j], 0, 0, 0);
#pragma unroll
            for (int j = 0; j < NT; ++j) wbuf[s][j] = ld_w(j, qb + s + PFK);
#pragma unroll
            for (int i = 0; i < MT; ++i) abuf[s][i] = ld_a(i, qb + s + PFK);
            // keep each slot's reload right behind its use: hoisting or sinking it shortens the ring
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    store_tiles<MT, NT>(acc, out, blockIdx.y, M, N, tile0, n_tiles, 0, lane, out_row_major, ch);
}

// ------------------------------------------------------------------ M <= 4: the same, its producer folded in
// The A operand is built by the workgroup itself (see FuseArgs) into LDS as plain bf16 rows of its share of K; a
// lane's fragment is then one 16-byte LDS read (lanes of rows that do not exist take zeros).  W streams through the
// same register ring, whose first loads are in flight while the prologue runs.
template <int FUSE>
__global__ __launch_bounds__(256) void gemm_bf16_small_fused_kernel(FuseArgs f, const bf16_t *__restrict__ w,
                                                                    float *__restrict__ out, int M, int N, int K,
                                                                    int splits, int epi) {
    constexpr int NT = 2, PFK = 16, MT = 1;
    extern __shared__ __attribute__((aligned(16))) unsigned char fused_smem[];
    bf16_t *lds_a = reinterpret_cast<bf16_t *>(fused_smem);           // [M][kr]
    __shared__ float red[4][kFuseMaxRows];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_tiles = N >> 4;
    const SplitRange sr = split_range(K, splits, blockIdx.y);
    const int k0 = sr.q0 * 32, kr = max(sr.q1 - sr.q0, 0) * 32;
    const int tile0 = (blockIdx.x * 4 + wave) * NT;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(w, (size_t)((N + 31) / 32) * 32 * K * 2);
    const int t32 = (N + 31) >> 5;
    const int n = lane & 15, g = lane >> 4;
    int w_off[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
        w_off[j] = (tile0 + j < n_tiles)
                       ? ((((g >> 1) * t32 + ((tile0 + j) >> 1)) * 64) + (g & 1) * 32 + ((tile0 + j) & 1) * 16 + n) * 16
                       : OOB;
    const int w_step = 2 * t32 * 1024;
    auto ld_w = [&](int j, int q) {
        return buf_load(rw, (q < sr.q1 && w_off[j] != OOB) ? w_off[j] + q * w_step : OOB);
    };
    // Loads return in order: the ring's first loads (for a short share of K: all of the workgroup's weights) are
    // issued *behind* the prologue's loads, which come from L2 and the memory-side cache and are back long before
    // the weights; the prologue's arithmetic then runs while the weights stream in.
    bf16x8 wbuf[PFK][NT];
    auto fill_ring = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < PFK; ++s)
#pragma unroll
            for (int j = 0; j < NT; ++j) wbuf[s][j] = ld_w(j, sr.q0 + s);
        __builtin_amdgcn_sched_barrier(0);
    };

    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
    if (FUSE == GEMM_FUSE_NORM) {
        // thread t holds columns 4 (t + 256 j) .. +3 of every row.  All loads of a row (the residual piece and up
        // to eight partial sums per piece) are issued before the first is used: one round trip per row, not one
        // per split.
        constexpr int KP = kFuseMaxK / 1024, SB = 8;
        float4 v[kFuseMaxRows][KP];
        float ss[kFuseMaxRows];
#pragma unroll
        for (int r = 0; r < kFuseMaxRows; ++r) {
            ss[r] = 0.f;
#pragma unroll
            for (int j = 0; j < KP; ++j) v[r][j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r >= M) continue;
#pragma unroll
            for (int j = 0; j < KP; ++j) {
                const int c = 4 * (tid + 256 * j);
                if (c < K) v[r][j] = *(const float4 *)(f.x_in + (size_t)r * K + c);
            }
            for (int sp0 = 0; sp0 < f.S; sp0 += SB) {
                float4 q[SB][KP];
#pragma unroll
                for (int u = 0; u < SB; ++u)
#pragma unroll
                    for (int j = 0; j < KP; ++j) {
                        const int c = min(4 * (tid + 256 * j), K - 4);            // clamped: always a real address
                        q[u][j] = *(const float4 *)(f.part + pt_index(c, r, M) +
                                                    (size_t)min(sp0 + u, f.S - 1) * f.split_stride);
                    }
#pragma unroll
                for (int u = 0; u < SB; ++u)                  // in split order, as the stand-alone kernel sums
#pragma unroll
                    for (int j = 0; j < KP; ++j)
                        if (sp0 + u < f.S && 4 * (tid + 256 * j) < K) {
                            v[r][j].x += q[u][j].x; v[r][j].y += q[u][j].y;
                            v[r][j].z += q[u][j].z; v[r][j].w += q[u][j].w;
                        }
            }
#pragma unroll
            for (int j = 0; j < KP; ++j)
                ss[r] += v[r][j].x * v[r][j].x + v[r][j].y * v[r][j].y + v[r][j].z * v[r][j].z + v[r][j].w * v[r][j].w;
        }
        fill_ring();
#pragma unroll
        for (int r = 0; r < kFuseMaxRows; ++r) {
            float t = ss[r];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o);
            if (lane == 0) red[wave][r] = t;
        }
        __syncthreads();
        const bool writer = blockIdx.x == 0 && blockIdx.y == 0;
#pragma unroll
        for (int r = 0; r < kFuseMaxRows; ++r) {
            if (r >= M) continue;
            const float tot = ((red[0][r] + red[1][r]) + red[2][r]) + red[3][r];
            const float rs = rsqrtf(tot / (float)K + f.eps);
#pragma unroll
            for (int j = 0; j < KP; ++j) {
                const int c = 4 * (tid + 256 * j);
                if (c >= K) continue;
                const float4 a = v[r][j];
                if (writer) *(float4 *)(f.x_out + (size_t)r * K + c) = a;
                if (c >= k0 && c < k0 + kr) {
                    const bf16x4 gn = *(const bf16x4 *)(f.gain + c);
                    const bf16x4 o = {(bf16_t)(a.x * rs * (float)gn[0]), (bf16_t)(a.y * rs * (float)gn[1]),
                                      (bf16_t)(a.z * rs * (float)gn[2]), (bf16_t)(a.w * rs * (float)gn[3])};
                    *(bf16x4 *)(lds_a + (size_t)r * kr + (c - k0)) = o;
                }
            }
        }
    } else {
        // One item = four head-dim values of one (row, head) of this workgroup's share of K = n_q * 128.  The
        // threads that the items leave over share an item's splits (TPI threads per item, sixteen splits loaded
        // together: one or two round trips to memory instead of one per split).  The fold is the online form:
        // every split keeps an integral reference, so moving the running reference scales by an exact power of
        // two and the order of the rescales leaves no trace; partial folds of an item meet in LDS in thread order.
        constexpr int SB = 16;
        const int group = f.n_q / f.n_kv, F = group * f.R, per_row = kr >> 2;
        const int items = M * per_row;
        int tpi = 1;
        while (tpi < 8 && items * tpi * 2 <= 256) tpi *= 2;
        __shared__ float fold[256][6];
        const int part_i = tid % tpi;
        for (int it0 = 0; it0 < items; it0 += 256 / tpi) {               // one round when the items fit (uniform)
        const int item = it0 + tid / tpi;
        float mrun = -INFINITY, den = 0.f;
        float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
        int r = 0, kk = k0;
        if (item < items) {
            r = item / per_row;
            kk = k0 + 4 * (item - r * per_row);
            const int head = kk >> 7, d0 = kk & 127;
            const int b = r / f.R, rr = r - b * f.R;
            const int kvh = head / group, hq = head - kvh * group;
            const size_t base = ((size_t)b * f.n_kv + kvh) * f.a_splits;
            const int fr = hq * f.R + rr;
            const int per_t = (f.a_splits + tpi - 1) / tpi;
            const int s_lo = part_i * per_t, s_hi = min(f.a_splits, s_lo + per_t);
            for (int sp0 = s_lo; sp0 < s_hi; sp0 += SB) {
                float m[SB], l[SB];
                float4 o[SB];
#pragma unroll
                for (int u = 0; u < SB; ++u) {
                    const size_t pi = (base + min(sp0 + u, f.a_splits - 1)) * F + fr;
                    m[u] = f.mpart[pi];
                    l[u] = f.lpart[pi];
                    o[u] = *(const float4 *)(f.opart + pi * 128 + d0);
                }
                float mc = mrun;
#pragma unroll
                for (int u = 0; u < SB; ++u)
                    if (sp0 + u < s_hi) mc = fmaxf(mc, m[u]);
                if (mc == -INFINITY) continue;                              // nothing but empty splits so far
                const float sc = exp2f(mrun - mc);                          // 0 when mrun is still -inf
                num.x *= sc; num.y *= sc; num.z *= sc; num.w *= sc;
                den *= sc;
                mrun = mc;
#pragma unroll
                for (int u = 0; u < SB; ++u) {
                    if (sp0 + u >= s_hi || m[u] == -INFINITY) continue;     // absent or empty split
                    const float wgt = exp2f(m[u] - mrun);
                    num.x += wgt * o[u].x; num.y += wgt * o[u].y; num.z += wgt * o[u].z; num.w += wgt * o[u].w;
                    den += wgt * l[u];
                }
            }
        }
        if (it0 == 0) fill_ring();
        if (tpi > 1) {
            __syncthreads();                                               // the previous round's folds were read
            fold[tid][0] = mrun; fold[tid][1] = den;
            fold[tid][2] = num.x; fold[tid][3] = num.y; fold[tid][4] = num.z; fold[tid][5] = num.w;
            __syncthreads();
            if (item < items && part_i == 0) {
                for (int t = 1; t < tpi; ++t) {
                    const float *o = fold[tid + t];
                    if (o[0] == -INFINITY) continue;
                    const float mc = fmaxf(mrun, o[0]);
                    const float sa = exp2f(mrun - mc), sb = exp2f(o[0] - mc);
                    num.x = num.x * sa + o[2] * sb; num.y = num.y * sa + o[3] * sb;
                    num.z = num.z * sa + o[4] * sb; num.w = num.w * sa + o[5] * sb;
                    den = den * sa + o[1] * sb;
                    mrun = mc;
                }
            }
        }
        if (item < items && part_i == 0) {
            const float inv = 1.f / den;
            const bf16x4 o = {(bf16_t)(num.x * inv), (bf16_t)(num.y * inv), (bf16_t)(num.z * inv), (bf16_t)(num.w * inv)};
            *(bf16x4 *)(lds_a + (size_t)r * kr + (kk - k0)) = o;
        }
        }
    }
    __syncthreads();

    f32x4 acc[MT][NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[0][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // A fragment of k step q: lane (row n, k slots 8g .. 8g+7)
    const bf16_t *a_row = lds_a + (size_t)min(n, M - 1) * kr + 8 * g;
    const bool a_real = n < M;
    for (int qb = sr.q0; qb < sr.q1; qb += PFK) {
#pragma unroll
        for (int s = 0; s < PFK; ++s) {
            const int q = qb + s;
            bf16x8 af = {0, 0, 0, 0, 0, 0, 0, 0};
            if (a_real && q < sr.q1) af = *(const bf16x8 *)(a_row + (q - sr.q0) * 32);
#pragma unroll
            for (int j = 0; j < NT; ++j)
                acc[0][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, wbuf[s][j], acc[0][j], 0, 0, 0);
#pragma unroll
            for (int j = 0; j < NT; ++j) wbuf[s][j] = ld_w(j, q + PFK);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (tile0 >= n_tiles) return;
    ChooseArgs none = {};
    store_tiles<MT, NT>(acc, out, blockIdx.y, M, N, tile0, n_tiles, 0, lane, epi, none);
}

// ------------------------------------------------------------------ 32 < M: 32x32x16 MFMA, A through LDS
// MTA: 32-row tiles per wave.  2 x 2 waves (WIDE false): the workgroup pass covers CTL = 2*MTA row tiles (9 when
// MTA is 5: the second row half then repeats a tile whose results are dropped) of 128 columns.  WIDE: four waves
// side by side, each over all CTL = MTA row tiles and NT 32-column tiles of the workgroup's 128 * NT columns.
// Chunk of K = 128 (8 k steps); weight ring 16 k steps.
template <int MTA, bool WIDE, int NT = 2, int NW = 4>
__global__ __launch_bounds__(64 * NW) void gemm_bf16_large_kernel(const bf16_t *__restrict__ a,
                                                              const bf16_t *__restrict__ w, float *__restrict__ out,
                                                              int M, int N, int K, int splits, int epi,
                                                              int swz_p, int swz_c, int n_pass, int n_colblk,
                                                              ChooseArgs ch) {
    constexpr int KS = 8;
    static_assert(NT == 2 || (NT == 1 && WIDE), "one column tile per wave only with the waves side by side");
    static_assert(NW == 4 || (NW == 8 && WIDE && NT == 1), "eight waves only side by side with one column tile each");
    constexpr int THREADS = 64 * NW;
    constexpr bool BIG = WIDE && MTA >= 6 && NT == 2;   // the many-row variants: registers go to the accumulators
    constexpr int PFK = BIG ? KS : 2 * KS;       // weight ring depth in k steps: one chunk or two
    constexpr int CTL = WIDE ? MTA : (MTA == 5) ? 9 : 2 * MTA;
    // Many row passes: the (pass, column block) plane is cut into super-tiles of swz_p x swz_c workgroups, each
    // handed whole to one XCD (workgroup i of a launch runs on XCD i % 8), passes fastest: the workgroups that
    // are resident together on an XCD then share their A rows and W columns through its L2 instead of each
    // streaming a private W slice from HBM.
    int bx = blockIdx.x, bz = blockIdx.z;
    if (swz_p > 0) {
        const int i = blockIdx.x, xcd = i & 7, j = i >> 3;
        const int per = swz_p * swz_c;
        const int n_sp = (n_pass + swz_p - 1) / swz_p, n_sc = (n_colblk + swz_c - 1) / swz_c;
        const int st = (j / per) * 8 + xcd, within = j % per;
        if (st >= n_sp * n_sc) return;
        bz = (st % n_sp) * swz_p + within % swz_p;
        bx = (st / n_sp) * swz_c + within / swz_p;
        if (bz >= n_pass || bx >= n_colblk) return;
    }
    constexpr int PIECES = CTL * KS * 64;        // 16-byte pieces per chunk
    constexpr int STAGE = (PIECES + THREADS - 1) / THREADS;
    constexpr int FR = KS * MTA;                 // A fragments a wave consumes per chunk
    constexpr int AFD = NT == 1 ? 6 : 3;         // LDS -> register prefetch distance in fragments (NT MFMAs each)
    static_assert(2 * STAGE <= FR, "one staging piece is stored after every other fragment");
    extern __shared__ __attribute__((aligned(16))) unsigned char gemm_smem[];
    bf16x8 *lds = reinterpret_cast<bf16x8 *>(gemm_smem);      // [2][KS][CTL][64]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int mh = WIDE ? 0 : wave & 1, ng = WIDE ? wave : wave >> 1;
    const int t32 = (N + 31) >> 5, m_tiles = (M + 31) >> 5;
    const int mt_base = bz * CTL;
    const int ct_here = min(CTL, m_tiles - mt_base);
    const int q_total = K >> 4;                                // k steps of 16
    const SplitRange sr32 = split_range(K, splits, blockIdx.y);
    const int q0 = sr32.q0 * 2, q1 = min(sr32.q1 * 2, q_total);
    const int c0 = q0 / KS, c1 = (q1 + KS - 1) / KS;
    const int tile0 = (bx * (WIDE ? NW : 2) + ng) * NT;  // first 32-column tile of this wave
    const __amdgpu_buffer_rsrc_t ra = make_rsrc(a, (size_t)q_total * m_tiles * 1024);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(w, (size_t)t32 * 32 * K * 2);

    int w_off[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) w_off[j] = (tile0 + j < t32) ? ((tile0 + j) * 64 + lane) * 16 : OOB;
    const int w_step = t32 * 1024;
    auto ld_w = [&](int j, int q) {
        return buf_load(rw, (q < q1 && w_off[j] != OOB) ? w_off[j] + q * w_step : OOB);
    };

    // A staging: piece p = tid + s*THREADS of the chunk = lane `lane` of fragment (wave + NW*s) -> (k step, row tile).
    // The fragment index is wave-uniform, so its address lives in scalar registers (the buffer load's scalar
    // offset) and only lane*16, or the out-of-bounds offset for a fragment that does not exist, in a VGPR.
    const int wv = __builtin_amdgcn_readfirstlane(wave);
    const int a_chunk_step = KS * m_tiles * 1024;
    const int lane16 = lane * 16;
    // HALF (the many-row variants, which have no registers to spare): half as many staging registers, each
    // carrying two pieces per chunk; a piece is then in flight for half a chunk instead of a whole one.
    constexpr bool HALF = BIG;
    constexpr int SR = HALF ? STAGE / 2 : STAGE;
    static_assert(!HALF || (STAGE % 2 == 0 && 4 * STAGE <= FR), "two events per staging register and chunk");
    bf16x8 stage[SR];
    auto load_a1 = [&](int s, int c) {          // piece s of chunk c -> staging register s % SR
        const int i = wv + NW * s;
        const int ks = i / CTL, ct = i % CTL;
        const bool ok = i < CTL * KS && ct < ct_here && c < c1;
        stage[s % SR] = __builtin_bit_cast(
            bf16x8, __builtin_amdgcn_raw_buffer_load_b128(ra, ok ? lane16 : OOB,
                                                          (ks * m_tiles + mt_base + ct) * 1024 + c * a_chunk_step, 0));
    };
    auto store_a1 = [&](int s, int buf) {
        if (STAGE * THREADS == PIECES || tid + s * THREADS < PIECES) lds[buf * PIECES + tid + s * THREADS] = stage[s % SR];
    };

    f32x16 acc[MTA][NT];
#pragma unroll
    for (int i = 0; i < MTA; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    bf16x8 wbuf[PFK][NT];
    // The loads of the ring's second half and of the second chunk's A are issued in the order the loop issues
    // them, so that the in-flight counts the compiler derives at the loop entry equal those of the back edge.
#pragma unroll
    for (int s = 0; s < SR; ++s) load_a1(s, c0);
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int j = 0; j < NT; ++j) wbuf[s][j] = ld_w(j, q0 + s);
#pragma unroll
    for (int s = 0; s < SR; ++s) store_a1(s, 0);
    if (HALF) {
#pragma unroll
        for (int s = SR; s < STAGE; ++s) load_a1(s, c0);
#pragma unroll
        for (int s = SR; s < STAGE; ++s) store_a1(s, 0);
#pragma unroll
        for (int s = 0; s < SR; ++s) load_a1(s, c0 + 1);
    } else {
#pragma unroll
        for (int f = 0; f < FR; ++f) {
            if (f % MTA == MTA - 1) {
#pragma unroll
                for (int j = 0; j < NT; ++j) wbuf[KS + f / MTA][j] = ld_w(j, q0 + KS + f / MTA);
            }
            if ((f & 1) && (f >> 1) < STAGE) load_a1(f >> 1, c0 + 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    __syncthreads();

    // fragment f of a chunk = (k step f / MTA, row tile f % MTA of this wave's half, clamped to a real tile)
    int frag_off[MTA];
#pragma unroll
    for (int mt = 0; mt < MTA; ++mt) frag_off[mt] = min(mh * MTA + mt, CTL - 1) * 64 + lane;
    auto lds_frag = [&](int buf, int f) { return lds[buf * PIECES + (f / MTA) * CTL * 64 + frag_off[f % MTA]]; };

    for (int cb = c0; cb < c1; cb += 2) {
#pragma unroll
        for (int ci = 0; ci < 2; ++ci) {          // two chunks = one revolution of the weight ring
            const int c = cb + ci;
            const int buf = ci;                   // chunks alternate buffers starting from buffer 0 at c0
            bf16x8 af[AFD + 1];
#pragma unroll
            for (int f = 0; f < AFD; ++f) af[f] = lds_frag(buf, f);
#pragma unroll
            for (int f = 0; f < FR; ++f) {
                if (f + AFD < FR) af[(f + AFD) % (AFD + 1)] = lds_frag(buf, f + AFD);
                const int ks = f / MTA, mt = f % MTA;
                const int slot = (ci * KS + ks) % PFK;
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[mt][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wbuf[slot][j], af[f % (AFD + 1)], acc[mt][j],
                                                                         0, 0, 0);   // W first: acc = out^T
                if (mt == MTA - 1) {              // this k step's ring slot is free again
#pragma unroll
                    for (int j = 0; j < NT; ++j) wbuf[slot][j] = ld_w(j, c * KS + ks + PFK);
                }
                // the next chunk's A goes to the other LDS buffer one piece at a time between the MFMAs (a
                // burst of stores would sit in front of the fragment reads in the in-order LDS queue), and
                // the freed staging register at once takes the piece of the chunk after that
                if (HALF) {
                    // event e stores piece e of the next chunk and reloads its register with the piece that is
                    // stored half a chunk later: e + STAGE/2 of the next chunk, or e - STAGE/2 of the one after
                    if ((f & 3) == 1 && (f >> 2) < STAGE) {
                        const int e = f >> 2;
                        store_a1(e, buf ^ 1);
                        if (e < SR) load_a1(e + SR, c + 1);
                        else load_a1(e - SR, c + 2);
                    }
                } else if ((f & 1) && (f >> 1) < STAGE) {
                    store_a1(f >> 1, buf ^ 1);
                    load_a1(f >> 1, c + 2);
                }
                __builtin_amdgcn_sched_barrier(0);    // pin the order: LDS prefetch, MFMAs, ring reload
            }
            __syncthreads();
        }
    }

    // ---- epilogue.  The weight fragment is the MFMA's first operand, so the accumulator holds the output tile
    // transposed: lane l owns activation row l%32 of the row tile, and its register e is column
    // 8*(e/4) + 4*(l/32) + e%4 of the 32-column tile: four consecutive registers are four consecutive columns of
    // one row.
    const int lq = lane & 31, lh = lane >> 5;
    if (epi == GEMM_EPI_SWIGLU) {
        // columns 0-15 of a tile are gate, 16-31 up, of the same 16 features (tile T = features 16T..16T+15 =
        // exactly one k step of the next GEMM's A-fragment layout), so gate and up of a feature sit in the same
        // lane, 8 registers apart: h = silu(gate) * up needs no shuffle.  A lane then holds features 4*(l/32)+0..3
        // and 8+4*(l/32)+0..3 of its row; the fragment wants 8*(l/32)+0..7.  One half-wave swap fixes that: the
        // upper lanes hand their features 4-7 to the lower lanes and take the lower lanes' 8-11.
        bf16_t *ho = reinterpret_cast<bf16_t *>(out);
        typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int mt = 0; mt < MTA; ++mt) {
            const int tile_r = mh * MTA + mt;
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                unsigned pk[4];
#pragma unroll
                for (int i = 0; i < 8; i += 2) {
                    float h2[2];
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const float g = acc[mt][j][i + t], u = acc[mt][j][i + t + 8];
                        h2[t] = g * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g)) * u;
                    }
                    bf16x2 b;
                    b[0] = (bf16_t)h2[0];
                    b[1] = (bf16_t)h2[1];
                    pk[i >> 1] = __builtin_bit_cast(unsigned, b);
                }
                // pk[0..1]: features 4*lh + 0..3; pk[2..3]: features 8 + 4*lh + 0..3
                const auto s0 = __builtin_amdgcn_permlane32_swap(pk[0], pk[2], false, false);
                const auto s1 = __builtin_amdgcn_permlane32_swap(pk[1], pk[3], false, false);
                typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
                const u32x4 piece = {s0[0], s1[0], s0[1], s1[1]};
                if (tile_r < ct_here && tile0 + j < t32)
                    *(u32x4 *)(ho + (((size_t)(tile0 + j) * m_tiles + mt_base + tile_r) * 64 + lane) * 8) = piece;
            }
        }
        return;
    }
    if (epi == GEMM_EPI_ARGMAX) {
        // a lane walks its 16 columns of each of the wave's tiles in rising order (strict > keeps the lowest column
        // of a tie), then the two half-waves, which hold the same rows, are folded.  A column group is 64 columns:
        // the wave's two tiles, or (NT = 1) the tiles of two neighbouring waves, folded through LDS.
        const int G = (t32 + 1) >> 1;
        float *pmax = out;
        int *pidx = (int *)(out + (size_t)G * M);
        float bests[MTA];
        int bis[MTA];
#pragma unroll
        for (int mt = 0; mt < MTA; ++mt) {
            const int tile_r = mh * MTA + mt;
            float best = -INFINITY;
            int bi = tile0 * 32 + 4 * lh;
            bests[mt] = best;
            bis[mt] = bi;
            if (tile_r >= ct_here) continue;      // wave-uniform
            const RowChoice rc = row_choice(ch, (mt_base + tile_r) * 32 + lq, M);
            if (__any(rc.noisy || rc.sel >= 0)) {     // a tile that holds rows a token is taken from (wave-uniform)
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int col = (tile0 + j) * 32 + 8 * (e >> 2) + 4 * lh + (e & 3);
                        float v = acc[mt][j][e];
                        if (rc.sel >= 0 && col < N) ch.sel_logits[(size_t)rc.sel * N + col] = v;
                        if (rc.noisy) v = perturbed_logit(v, rc.inv_t, rc.key, (uint32_t)col);
                        if (col < N && v > best) {
                            best = v;
                            bi = col;
                        }
                    }
            } else {
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int col = (tile0 + j) * 32 + 8 * (e >> 2) + 4 * lh + (e & 3);
                        const float v = acc[mt][j][e];
                        if (col < N && v > best) {
                            best = v;
                            bi = col;
                        }
                    }
            }
            const float ob = __shfl_xor(best, 32);
            const int oi = __shfl_xor(bi, 32);
            if (ob > best || (ob == best && oi < bi)) {
                best = ob;
                bi = oi;
            }
            bests[mt] = best;
            bis[mt] = bi;
        }
        if constexpr (NT == 1) {
            // the odd wave of a pair hands its result to the even one (the staging buffers are free by now)
            float *rb = reinterpret_cast<float *>(gemm_smem);
            int *ri = reinterpret_cast<int *>(gemm_smem) + NW * MTA * 32;
            if (lh == 0) {
#pragma unroll
                for (int mt = 0; mt < MTA; ++mt) {
                    rb[(wave * MTA + mt) * 32 + lq] = bests[mt];
                    ri[(wave * MTA + mt) * 32 + lq] = bis[mt];
                }
            }
            __syncthreads();
            if (wave & 1) return;
#pragma unroll
            for (int mt = 0; mt < MTA; ++mt) {
                const float ob = rb[((wave + 1) * MTA + mt) * 32 + lq];
                const int oi = ri[((wave + 1) * MTA + mt) * 32 + lq];
                if (ob > bests[mt] || (ob == bests[mt] && oi < bis[mt])) {
                    bests[mt] = ob;
                    bis[mt] = oi;
                }
            }
        }
#pragma unroll
        for (int mt = 0; mt < MTA; ++mt) {
            const int tile_r = mh * MTA + mt;
            const int row = (mt_base + tile_r) * 32 + lq;
            if (tile_r < ct_here && lh == 0 && row < M && tile0 < t32) {
                pmax[(size_t)(tile0 >> 1) * M + row] = bests[mt];
                pidx[(size_t)(tile0 >> 1) * M + row] = bis[mt];
            }
        }
        return;
    }
    // Partial sums and logits: a lane's four consecutive columns are 16 bytes, but neighbouring lanes are
    // neighbouring rows, 128 bytes apart in the tiled layout.  Each tile is therefore turned through a per-wave
    // LDS patch (16-byte writes, 16-byte reads; the staging buffers are free after the last barrier) so that eight
    // lanes together store one whole row of the tile (128 bytes) and a store instruction covers 1 KiB in one run.
    float *scr = reinterpret_cast<float *>(gemm_smem) + wave * (32 * 36);
    float *o = out + (size_t)blockIdx.y * pt_split_stride(M, N);
#pragma unroll
    for (int mt = 0; mt < MTA; ++mt) {
        const int tile_r = mh * MTA + mt;
        if (tile_r >= ct_here) continue;          // also drops the repeated tile (wave-uniform)
#pragma unroll
        for (int j = 0; j < NT; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *(f32x4 *)(scr + lq * 36 + 8 * g + 4 * lh) = (f32x4){acc[mt][j][4 * g], acc[mt][j][4 * g + 1],
                                                                     acc[mt][j][4 * g + 2], acc[mt][j][4 * g + 3]};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int idx = lane + 64 * i;
                const int r = idx >> 3, c4 = idx & 7;
                const f32x4 v = *(const f32x4 *)(scr + r * 36 + 4 * c4);
                const int row = (mt_base + tile_r) * 32 + r;
                const int col = (tile0 + j) * 32 + 4 * c4;
                if (row < M && col < N) {
                    const size_t oi = (epi == GEMM_EPI_ROWMAJOR) ? (size_t)row * N + col : pt_index(col, row, M);
                    *(f32x4 *)(o + oi) = v;
                }
            }
        }
    }
}

template <int MT, int PFK>
void launch_small(const bf16_t *a, const bf16_t *w, float *out, int M, int N, int K, const GemmPlan &p, int row_major,
                  hipStream_t st, const ChooseArgs &ch) {
    dim3 grid((N + 127) / 128, p.splits, 1);
    gemm_bf16_small_kernel<MT, PFK><<<grid, 256, 0, st>>>(a, w, out, M, N, K, p.splits, row_major, ch);
}

template <int MTA, bool WIDE, int NT = 2, int NW = 4>
void launch_large(const bf16_t *a, const bf16_t *w, float *out, int M, int N, int K, const GemmPlan &p, int epi,
                  hipStream_t st, const ChooseArgs &ch) {
    constexpr int CTL = WIDE ? MTA : (MTA == 5) ? 9 : 2 * MTA;
    constexpr int BN = WIDE ? 32 * NW * NT : 128;
    int m_tiles = (M + 31) / 32;
    dim3 grid((N + BN - 1) / BN, p.splits, (m_tiles + CTL - 1) / CTL);
    const int n_colblk = grid.x, n_pass = grid.z;
    int swz_p = 0, swz_c = 0;
    if (p.swz > 0 && n_pass >= 2) {          // super-tiles of swz x swz workgroups, dealt to the XCDs in turn
        swz_p = p.swz < n_pass ? p.swz : n_pass;
        swz_c = p.swz;
        const int n_st = ((n_pass + swz_p - 1) / swz_p) * ((n_colblk + swz_c - 1) / swz_c);
        grid = dim3(8 * ((n_st + 7) / 8) * swz_p * swz_c, p.splits, 1);
    }
    // two staging buffers of a chunk's A tiles; the epilogue's per-wave transposition patches (4 x 32 x 36 floats)
    // reuse the same memory and need 18 KiB of it
    constexpr size_t PATCH = (size_t)NW * 32 * 36 * 4;
    constexpr size_t SMEM = (size_t)2 * CTL * 8 * 1024 > PATCH ? (size_t)2 * CTL * 8 * 1024 : PATCH;
    // LDS above 64 KiB has to be granted per kernel, on every device the kernel is launched on
    static bool attr_set[64] = {};
    int dev = 0;
    (void)hipGetDevice(&dev);
    if (dev < 0 || dev >= 64 || !attr_set[dev]) {
        (void)hipFuncSetAttribute((const void *)gemm_bf16_large_kernel<MTA, WIDE, NT, NW>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)SMEM);
        if (dev >= 0 && dev < 64) attr_set[dev] = true;
    }
    gemm_bf16_large_kernel<MTA, WIDE, NT, NW><<<grid, 64 * NW, SMEM, st>>>(a, w, out, M, N, K, p.splits, epi, swz_p, swz_c, n_pass,
                                                               n_colblk, ch);
}

}  // namespace

bool gemm_fuse_ok(int M, int N, int K) { return M >= 1 && M <= kFuseMaxRows && K <= kFuseMaxK && K % 32 == 0 && N % 16 == 0; }

void launch_gemm_bf16_fused(const FuseArgs &f, const bf16_t *w, float *out, int M, int N, int K, const GemmPlan &p,
                            int epi, hipStream_t st) {
    dim3 grid((N + 127) / 128, p.splits, 1);
    const int units = (K + SPLIT_UNIT - 1) / SPLIT_UNIT, per = (units + p.splits - 1) / p.splits;
    const size_t smem = (size_t)M * per * SPLIT_UNIT * 2;             // bf16 rows of the largest share of K
    if (f.kind == GEMM_FUSE_NORM)
        gemm_bf16_small_fused_kernel<GEMM_FUSE_NORM><<<grid, 256, smem, st>>>(f, w, out, M, N, K, p.splits, epi);
    else
        gemm_bf16_small_fused_kernel<GEMM_FUSE_COMBINE><<<grid, 256, smem, st>>>(f, w, out, M, N, K, p.splits, epi);
}

GemmPlan plan_gemm_bf16(int M, int N, int K, bool force_single_split) {
    GemmPlan p;
    p.nt = 2;
    p.bk = 128;
    p.wide = 0;
    p.nw = 4;
    p.swz = 0;
    const int wgs = (N + 127) / 128;
    const int units = (K + SPLIT_UNIT - 1) / SPLIT_UNIT;
    auto fit = [&](int want) {                   // clamp to the units there are and drop empty trailing splits
        want = want < 1 ? 1 : want > units ? units : want;
        int per = (units + want - 1) / want;
        return (units + per - 1) / per;
    };
    int splits = 1;
    if (M <= 32) {
        p.mt = M <= 16 ? 1 : 2;                  // 16-row tiles per wave (narrow kernel)
        p.m_chunks = 1;
        // nearest count that brings the grid to about one wave of CUs
        if (!force_single_split && wgs < 224) splits = fit((256 + wgs / 2) / wgs);
    } else {
        // Partial sums are the expensive part of a split (each one is M x N floats written and read again), so
        // the column blocks are split over K only until about half the CUs are busy; the rest of the chip is
        // filled by cutting the rows into two workgroup passes, which costs a second read of W from L2 and no
        // extra output.  The split count is a function of (N, K) alone: a row's sum is grouped the same way
        // whatever the batch size.
        if (!force_single_split) splits = fit(128 / wgs);
        const int t = (M + 31) / 32;             // 32-row tiles
        const bool row_split = !force_single_split && wgs * splits <= 128;
        const int per_pass = row_split ? (t + 1) / 2 : t;
        p.mt = per_pass <= 2 ? 1 : per_pass <= 4 ? 2 : per_pass <= 6 ? 3 : 5;      // per wave (wide kernel)
        int ctl = p.mt == 5 ? 9 : 2 * p.mt;
        // Two row passes of three to five tiles (129-320 rows): the four waves side by side, each over all row tiles of
        // the pass and one 32-column tile of the workgroup's 128 columns - at 272 rows five MFMAs per wave and k step
        // where the 2 x 2 arrangement runs six (two passes of six tile slots for nine tiles), and no weight fragment
        // is loaded twice
        if (row_split && t < 16) {
            p.wide = 1;
            p.nt = 1;
            p.mt = per_pass;
            ctl = per_pass;
        }
        // many column blocks, one split, more than five row tiles: 256-column workgroups over five row tiles
        // (four waves side by side, no weight fragment loaded twice) in two or more row passes.  Only when the
        // whole grid is resident at once: the passes of a column block then run together and the second read
        // of its weights hits L2 (measured on the LM head, whose grid takes several rounds: 30 % slower in
        // plain launch order)
        const int wide_wgs = ((N + 255) / 256) * ((t + 4) / 5);
        if (splits == 1 && wgs >= 128 && (t == 6 || t == 7)) {
            // Six or seven row tiles, one split, many column blocks (gate/up and the LM head at 161-224 rows): one
            // row pass of 128-column workgroups, every wave over all row tiles and one column tile - t MFMAs per
            // wave and k step where two passes of five tile slots ran ten, the weights read once.  Measured per
            // GEMM: -12 % at six tiles, -10 % at seven, nothing at eight, +5 % at nine (a workgroup then stages all
            // of A for half as many columns), so from eight tiles on the two passes stay.
            p.wide = 1;
            p.nt = 1;
            p.mt = t;
            ctl = t;
        } else if (splits == 1 && wgs >= 128 && t > 5 && wide_wgs <= 256) {
            p.wide = 1;
            p.nt = 1;
            p.nw = 8;
            p.mt = 5;
            ctl = 5;
        } else if (splits == 1 && wgs >= 512 && t > 5) {
            // The LM head: its grid takes several rounds either way.  With the (row pass, column block) plane
            // dealt to the XCDs in super-tiles the passes of a column block run on one XCD at about the same
            // time and share the weights through its L2: 436 -> 402 us at 272 rows.
            p.wide = 1;
            p.nt = 1;
            p.nw = 8;
            p.mt = 5;
            ctl = 5;
            p.swz = 4;
        }
        // 512 rows and more: the launch is bound by the compute units' L1 bandwidth, not by HBM (every workgroup
        // pulls its A rows and W columns through it), so the workgroup tile is made as square as the register
        // file allows: up to 256 rows x 256 columns, eight row tiles per wave.  Measured at 4096 rows of the 8B shape:
        // 0.65-0.95 PFLOP/s with 288 x 128 tiles, 0.88-1.28 with these.  Grids of many rounds (the LM head) are
        // also dealt to the XCDs in 4 x 4 super-tiles (+20 %; on grids of a few rounds the uneven deal costs more
        // than the sharing gains).
        if (t >= 16) {
            p.wide = 1;
            p.nt = 2;
            const int passes = (t + 7) / 8;
            p.mt = ctl = (t + passes - 1) / passes;      // 6, 7 or 8 row tiles per pass: the passes come out even
            p.swz = (N + 255) / 256 >= 256 ? 4 : 0;
            // With this many rows the row passes fill the chip by themselves, and a split costs M x N floats
            // written and read again (570 MB per launch at 8704 rows and N = 4096, four splits).  The count, never
            // above the (N, K) rule's, minimises an estimate in microseconds: rounds of 256 workgroups x (a
            // workgroup's share of K at the measured 22 ns per k of a 256 x 256 tile + 8 of prologue and
            // epilogue) + the partial sums through the fabric at 6 TB/s out and 4 TB/s back in.  It is a function
            // of the pass count (rows / 256, rounded up) alone, so within this class a row's sum is grouped the
            // same way for every row count with the same number of passes.
            const int base = ((N + 255) / 256) * passes, s_max = splits;
            double best = 0.0;
            for (int c = 1; c <= s_max; ++c) {
                const int sc = fit(c);
                const int rounds = (base * sc + 255) / 256;
                const double cost = rounds * (0.022 * K / sc + 8.0) + sc * (256.0 * passes) * N * 1.67e-6;
                if (c == 1 || cost < best) {
                    best = cost;
                    splits = sc;
                }
            }
        }
        p.m_chunks = (t + ctl - 1) / ctl;
    }
    p.splits = splits;
    return p;
}

void launch_gemm_bf16(const bf16_t *a, const bf16_t *w, float *out, int M, int N, int K, const GemmPlan &p,
                      int out_row_major, hipStream_t st, const ChooseArgs *choose) {
    ChooseArgs ch = {};
    if (choose && out_row_major == GEMM_EPI_ARGMAX) ch = *choose;
    if (M <= 32) {
        if (p.mt == 1) launch_small<1, 16>(a, w, out, M, N, K, p, out_row_major, st, ch);
        else launch_small<2, 8>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide && p.nt == 1 && p.nw == 8) {     // eight waves side by side, one column tile each
        launch_large<5, true, 1, 8>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide && p.nt == 1 && p.mt == 1) {
        launch_large<1, true, 1>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide && p.nt == 1 && p.mt == 2) {
        launch_large<2, true, 1>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide && p.nt == 1 && p.mt == 3) {
        launch_large<3, true, 1>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide && p.nt == 1 && p.mt == 4) {
        launch_large<4, true, 1>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide && p.nt == 1 && p.mt == 5) {
        launch_large<5, true, 1>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide && p.nt == 1 && p.mt == 6) {
        launch_large<6, true, 1>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide && p.nt == 1 && p.mt == 7) {
        launch_large<7, true, 1>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide && p.nt == 1) {
        launch_large<8, true, 1>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide && p.mt == 8) {
        launch_large<8, true>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide && p.mt == 7) {
        launch_large<7, true>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide && p.mt == 6) {
        launch_large<6, true>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.wide) {
        launch_large<5, true>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.mt == 1) {
        launch_large<1, false>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.mt == 2) {
        launch_large<2, false>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else if (p.mt == 3) {
        launch_large<3, false>(a, w, out, M, N, K, p, out_row_major, st, ch);
    } else {
        launch_large<5, false>(a, w, out, M, N, K, p, out_row_major, st, ch);
    }
}
