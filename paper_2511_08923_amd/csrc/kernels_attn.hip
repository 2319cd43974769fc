// Hybrid-mask paged attention for the decode step (bf16 MFMA path) and its split-KV combine.
//
// Work item = (sequence, kv head, chunk of 32-row query tiles, split of the key range).  The query rows of a
// kv head are the rows of all query heads in its group, flattened (head-in-group major), so a K/V tile that
// is brought into LDS once serves every query head that shares it.  Four waves split the query tiles; each wave
// keeps its Q fragments, its O^T accumulators and its softmax state in registers for the whole key range.
//
// MFMA: v_mfma_f32_32x32x16_bf16 (on gfx950 twice the rate of the 16x16x32 form).  Scores are formed
// transposed, S^T[key][q] = K . Q^T, so that in the result layout a lane holds one query column and 16 of the
// 32 keys of a block.  After exponentiation and without any data movement a lane's registers 0-7 (first page of
// the pair) and 8-15 (second page) are the B operands (P^T) of two MFMAs O^T[d][q] += V^T[d][key] . P^T[key][q];
// V is kept transposed in HBM ([head_dim][16 tokens] per page).
//
// K/V tiles go from HBM straight into LDS (buffer_load ... lds, 16 bytes per lane), three buffers deep, two
// key-pair iterations ahead of their use: no staging registers, no LDS stores, and the loads of a tile have two
// iterations to arrive.  A wave's lanes choose *which* 16 bytes they fetch, which is where the LDS layout comes
// from: K rows of 256 bytes whose 16-byte pieces are XOR-swizzled by the row (conflict-free fragment reads without
// padding), rows 4-7 and 8-11 of a unit exchanged so that a lane's score registers of a unit are eight consecutive
// keys, the same eight that one 16-byte piece of V^T holds.
//
// Softmax numerators are taken against an integral power-of-two reference (ceil of a running maximum in log2
// units): their bf16 rounding is then independent of the reference in force, i.e. of tiling and splits, and
// every rescale is exact.  The reference is lazy: a row's reference is set by its first visible block and moves
// only when the scores outgrow it by 2^60, which in practice is never; the loop over plain prefix keys therefore
// has no rescale arm at all (attn_block_fixed_ref), and leaves for the general loop if that ever happens.
//
// Keys come in units of 16: cache pages 0 .. ceil((L+nc)/16)-1, then the mask rows' scratch tiles.  Pages that
// lie wholly below L need no mask at all (every row sees the whole prefix); everything else goes through the
// (row, key) predicate and a per-(query tile, key pair) skip when nothing is visible.
#include <type_traits>

#include "tidar_internal.h"

namespace {

constexpr int HD = 128;
constexpr int TILE = 32 * HD;           // bf16 elements of one K tile (32 keys) and of one V^T tile

// 16 bytes per lane straight from a raw buffer into LDS at lds_addr + 16 * lane (the tile's wave-uniform base goes
// through M0).  Written as inline assembly so that only the explicit vmcnt waits of the kernel order these loads
// against the LDS reads: issued through the compiler's builtin, every LDS read waits for *all* loads in flight,
// which is exactly the prefetch this is meant to keep running.
typedef int int4v __attribute__((ext_vector_type(4)));
__device__ inline int4v raw_desc(const void *base, size_t bytes) {
    const unsigned long long p = (unsigned long long)base;
    return (int4v){(int)(p & 0xffffffffull), (int)((p >> 32) & 0xffffull),
                   (int)(bytes > 0x7fffffe0ull ? 0x7fffffe0ull : bytes), 0x00020000};
}
// (M0 is a reserved register that the compiler sets itself right before each of its own uses; this kernel has none.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ inline void dma16(unsigned lds_addr, int voff, int4v desc, int soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(desc), "s"(soff)
                 : "memory", "m0");
}
#pragma clang diagnostic pop
__device__ inline void lds_barrier() {       // workgroup barrier for LDS traffic only: global loads stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

struct AttnArgs {
    const bf16_t *q;
    KvView kv;
    const bf16_t *k_scr, *v_scr;
    const int32_t *prefix_len;
    RowDesc d;
    int n_q, group;
    int n_chunks, tiles_per_chunk, splits, per;
    int n_groups;                         // batch x kv heads
    int xcd_q;                            // 0: plain order; q >= 1: a group's chunks go to q XCDs (see the kernel)
    float scale_log2e;
    float *opart, *mpart, *lpart;
    bf16_t *out;               // single split only: [rows][n_q][HD], or the A-fragment layout (out_af)
    int out_af;
    ActLayout lay;
    AttnRope rp;               // ROPE kernels only
};

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// One 32-query x 32-key block: S^T = K.Q^T, online softmax against the integral reference, O^T += V^T.P^T.
// c = softmax scale * log2(e).  VIS: bit e set = register e's key is visible to this lane's query row (only read
// when MASKED).  Kept lean: per score one max, one fma, one v_exp_f32, half a pack and half a dot2.
// Tile layout in LDS (see the kernel): K rows of 256 bytes with the 16-byte pieces XOR-swizzled by the row, rows
// 4-7 and 8-11 of a unit exchanged so that score register e of unit u is key 8*(lane/32) + e%8; V^T as
// [unit][key half][d] 16-byte pieces in natural key order.
template <bool MASKED>
__device__ inline void attn_block(const bf16_t *k_lds, const bf16_t *v_lds, int lq, int lh, const bf16x8 (&qf)[8],
                                  f32x16 (&acc)[4], float &m_run, float &l_run, float c, unsigned vis) {
    const unsigned char *kb = reinterpret_cast<const unsigned char *>(k_lds);
    const unsigned char *vb = reinterpret_cast<const unsigned char *>(v_lds);
    // K as A operand: lane = (tile row, hd half of the k step); V^T as A operand: lane = (d, key half of the unit)
    auto k_frag = [&](int ks) { return *(const bf16x8 *)(kb + lq * 256 + (((2 * ks + lh) ^ (lq & 15)) << 4)); };
    auto v_frag = [&](int dt, int u) { return *(const bf16x8 *)(vb + (((u * 2 + lh) * 128 + 32 * dt + lq) << 4)); };
    // K as A operand (lane = key, hd half of the k step); fragments are consumed as they arrive.  One
    // accumulation chain: a second one costs 16 registers, and the other resident wave covers the dependency
    f32x16 s;
#pragma unroll
    for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 kf0 = k_frag(ks);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf0, qf[ks], s, 0, 0, 0);
    }
    // V^T as A operand (lane = d, key chunk): the first half is issued now and is needed after the softmax
    // arithmetic; the second half is read once the scores are dead and takes over their registers
    bf16x8 vf[2][2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int u = 0; u < 2; ++u)
            vf[dt][u] = v_frag(dt, u);
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        if (MASKED) s[e] = ((vis >> e) & 1u) ? s[e] : -INFINITY;
        mx = fmaxf(mx, s[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    // The reference of a row moves only when its scores outgrow it by 2^60 (or it is still -inf): the same rule
    // that makes attn_block_fixed_ref refuse a block, so that which of the two ran a block (that depends on how
    // much of the key range is plain prefix, i.e. on the sequence length) leaves no trace in the result.  (The
    // numerators' mantissas do not depend on the reference in exact arithmetic, but fma(s, c, -m) is rounded.)
    const bool grow = !(mx * c <= m_run + 60.f);
    const float m_new = grow ? fmaxf(m_run, ceilf(mx * c)) : m_run;
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
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
    // O^T += V^T.P^T.  The rescale by the exact 2^(old - new) is rare after the first blocks; it shares its arm of
    // the branch with a copy of the accumulation so that the common arm updates the accumulators in place (a
    // rescale arm that rejoined before the MFMAs made the compiler copy all 64 accumulator registers per block)
    auto accumulate = [&]() __attribute__((always_inline)) {
        bf16x8 vg[2][2];
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int u = 0; u < 2; ++u) vg[dt][u] = v_frag(dt + 2, u);
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
    };
    if (__builtin_expect(__any(m_new != m_run), 0)) {
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[dt][e] *= alpha;
        m_run = m_new;
        accumulate();
    } else {
        l_run += psum;
        accumulate();
    }
}

// The same block for keys that are all visible, without the arm that moves the reference: the numerators are
// 2^(s.c - m_run) with the reference of an earlier block, so they may exceed 1 (by less than 2^60, or the block
// is refused before it changes anything: the caller then runs attn_block, which moves the reference by the same
// rule).  bf16 rounding is a matter of the mantissa alone, and every quantity (numerators, denominator, O^T)
// carries the same power of two.  No rescale arm means no branch that rejoins around the accumulators: with one,
// the compiler copied all 64 accumulator registers twice per block.
template <bool PRIO>
__device__ inline bool attn_block_fixed_ref(const bf16_t *k_lds, const bf16_t *v_lds, int lq, int lh,
                                            const bf16x8 (&qf)[8], f32x16 (&acc)[4], float m_run, float &l_run,
                                            float c) {
    const unsigned char *kb = reinterpret_cast<const unsigned char *>(k_lds);
    const unsigned char *vb = reinterpret_cast<const unsigned char *>(v_lds);
    // K as A operand: lane = (tile row, hd half of the k step); V^T as A operand: lane = (d, key half of the unit)
    auto k_frag = [&](int ks) { return *(const bf16x8 *)(kb + lq * 256 + (((2 * ks + lh) ^ (lq & 15)) << 4)); };
    auto v_frag = [&](int dt, int u) { return *(const bf16x8 *)(vb + (((u * 2 + lh) * 128 + 32 * dt + lq) << 4)); };
    // all eight K fragments are asked for before the first MFMA: read one or two ahead of its MFMA, as the compiler
    // orders them by itself, every link of the score chain waits out a full LDS round trip
    bf16x8 kf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kf[ks] = k_frag(ks);
    __builtin_amdgcn_sched_barrier(0);
    f32x16 s;
#pragma unroll
    for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], s, 0, 0, 0);
    // PRIO (launches in which all four waves hold a query tile): the softmax section runs at a raised wave priority.
    // The SIMD's other wave is then the one that waits while it is in an MFMA chain of its own, and the two fall into
    // opposite phases more often (measured: -3 % at 272 rows, -1 % at batch 8; raising the priority of the MFMA
    // chains instead changes nothing).  Not for the few-row shapes, whose three other waves only move tiles: there
    // the raised wave holds up their loads (1-token step at batch 8: +2.6 %).
    if (PRIO) __builtin_amdgcn_s_setprio(3);
    bf16x8 vf[2][2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int u = 0; u < 2; ++u) vf[dt][u] = v_frag(dt, u);
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[e]);
    if (__any(!(mx * c <= m_run + 60.f))) {                       // also refuses a reference that is still -inf
        if (PRIO) __builtin_amdgcn_s_setprio(0);
        return false;
    }
    const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
    float psum = 0.f;
    bf16x8 pf[2];
#pragma unroll
    for (int e = 0; e < 16; e += 2) {
        bf16x2 pk = {(bf16_t)__builtin_amdgcn_exp2f(fmaf(s[e], c, -m_run)),
                     (bf16_t)__builtin_amdgcn_exp2f(fmaf(s[e + 1], c, -m_run))};
        psum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, psum, false);
        pf[e >> 3][e & 7] = pk[0];
        pf[e >> 3][(e & 7) + 1] = pk[1];
    }
    l_run += psum;
    if (PRIO) __builtin_amdgcn_s_setprio(0);
    bf16x8 vg[2][2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int u = 0; u < 2; ++u) vg[dt][u] = v_frag(dt + 2, u);
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
    return true;
}

// QT: 32-row query tiles per wave.
template <int QT, bool PRIO, bool ROPE>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(AttnArgs a) {
    constexpr int NBUF = 3, K_TILE = TILE, V_TILE = TILE;
    __shared__ __attribute__((aligned(16))) bf16_t k_lds[NBUF][K_TILE];
    __shared__ __attribute__((aligned(16))) bf16_t v_lds[NBUF][V_TILE];
    __shared__ __attribute__((aligned(16))) bf16_t q_lds[ROPE ? 32 * HD : 8];     // ROPE: the rotated Q rows of the group

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // known to be uniform: scalar registers
    const int lq = lane & 31, lh = lane >> 5;
    // Workgroup i of a launch runs on XCD i % 8 (the grid's x extent is then a multiple of 8, so the split index
    // does not change that).  Where the (sequence, kv head) groups divide evenly over the XCDs, or the XCDs over
    // the groups, the query chunks of one group are dealt to one XCD (or to 8 / groups of them), whose L2 then
    // fetches that head's K and V once instead of once per XCD that happens to run one of its chunks.
    int grp, chunk;
    if (a.xcd_q == 0) {
        chunk = blockIdx.x % a.n_chunks;
        grp = blockIdx.x / a.n_chunks;
    } else if (a.n_groups >= 8) {
        const int xj = blockIdx.x >> 3;
        grp = (xj / a.n_chunks) * 8 + (blockIdx.x & 7);
        chunk = xj % a.n_chunks;
    } else {
        const int xcd = blockIdx.x & 7;
        grp = xcd / a.xcd_q;
        chunk = (blockIdx.x >> 3) * a.xcd_q + xcd % a.xcd_q;
        if (chunk >= a.n_chunks) return;             // padding of the last round (whole workgroup)
    }
    const int g = grp % a.kv.n_kv;
    const int b = grp / a.kv.n_kv;
    const int split = blockIdx.y;
    const RowDesc d = a.d;
    const int L = clamp_prefix(a.kv, a.prefix_len[d.seq_base + b], d.nc);   // never walks past the page table
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

    if constexpr (ROPE) {
        // One row per sequence (R = 1): the group's query heads are the tile's rows.  A thread takes one rotation pair
        // (d, d + 64) of one head: it adds the split-K partial sums of the QKV projection and rotates by the row's
        // angles, exactly as the RoPE kernel does.  The workgroup whose key range holds the new row's position does
        // the same for K and copies V, and stores both into the cache page before any of its tile loads starts
        // (the stores are waited for, then a workgroup barrier: the loads that follow read them back from L2).
        const AttnRope &rp = a.rp;
        const int row = b;                                   // the call's row of this sequence
        const float *cs = rp.rope_cs + (size_t)row * (HD / 2) * 2;
        // sums of the splits in rising order (the RoPE kernel's order), two columns at a time and eight splits'
        // loads in flight for each: one load per trip would cost a memory round trip per split
        auto summed2 = [&](int col0, int col1, float &x, float &y) {
            const float *p0 = rp.part + pt_index(col0, row, rp.M_all), *p1 = rp.part + pt_index(col1, row, rp.M_all);
            x = 0.f;
            y = 0.f;
            for (int s0 = 0; s0 < rp.S; s0 += 8) {
                float t0[8], t1[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const size_t o = (size_t)min(s0 + j, rp.S - 1) * rp.split_stride;
                    t0[j] = p0[o];
                    t1[j] = p1[o];
                }
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (s0 + j < rp.S) {
                        x += t0[j];
                        y += t1[j];
                    }
            }
        };
        // The writing workgroup: its page id is asked for first, and every thread issues the loads of its K or V pair
        // together with those of its Q pair (a thread without a pair repeats a valid column and drops the sums), so
        // that the whole prologue is one memory round trip before the stores.
        const int L_raw = a.prefix_len[d.seq_base + b];
        const int it_new = (L >> 4) >> 1;                    // the key-pair iteration of position L
        const bool writes = it_new >= a0 && it_new < a1 && seq_fits(a.kv, L_raw, 1);
        int page = -1;
        if (writes) page = a.kv.page_table[(size_t)(d.seq_base + b) * a.kv.pages_per_seq + (L >> 4)];
        const int n_qp = a.group * (HD / 2);
        const int wi = tid & (HD / 2 - 1);
        const int wcol = (tid < HD / 2 ? rp.q_dim : rp.q_dim + rp.kv_dim) + g * HD + wi;
        float wx, wy;
        {
            const int idx = min(tid, n_qp - 1);
            const int hq = idx / (HD / 2), i = idx - hq * (HD / 2);
            const int col = (g * a.group + hq) * HD + i;
            float x, y;
            summed2(col, col + HD / 2, x, y);
            summed2(wcol, wcol + HD / 2, wx, wy);
            const float c = cs[2 * i], sn = cs[2 * i + 1];
            if (tid < n_qp) {
                q_lds[hq * HD + i] = (bf16_t)(x * c - y * sn);
                q_lds[hq * HD + i + HD / 2] = (bf16_t)(y * c + x * sn);
            }
        }
        for (int idx = tid + 256; idx < n_qp; idx += 256) {          // more than four query heads per kv head
            const int hq = idx / (HD / 2), i = idx - hq * (HD / 2);
            const int col = (g * a.group + hq) * HD + i;
            float x, y;
            summed2(col, col + HD / 2, x, y);
            const float c = cs[2 * i], sn = cs[2 * i + 1];
            q_lds[hq * HD + i] = (bf16_t)(x * c - y * sn);
            q_lds[hq * HD + i + HD / 2] = (bf16_t)(y * c + x * sn);
        }
        if (writes) {
            const int slot = L & 15;
            if (page_ok(a.kv, page) && tid < HD) {
                if (tid < HD / 2) {
                    const float c = cs[2 * wi], sn = cs[2 * wi + 1];
                    bf16_t *kdst = (bf16_t *)a.kv.k_pages + k_page_offset(a.kv, page, g, slot, 0);
                    kdst[wi] = (bf16_t)(wx * c - wy * sn);
                    kdst[wi + HD / 2] = (bf16_t)(wy * c + wx * sn);
                } else {
                    bf16_t *vp = (bf16_t *)a.kv.v_pages;
                    vp[v_page_offset(a.kv, page, g, slot, wi)] = (bf16_t)wx;
                    vp[v_page_offset(a.kv, page, g, slot, wi + HD / 2)] = (bf16_t)wy;
                }
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        __syncthreads();
    }

    // ---- this wave's query tiles: Q fragments (B operand: lane = (q row, hd half of the k step)), row info
    bf16x8 qf[QT][8];
    int r_vis[QT], r_blk[QT];
    int vis_min = 0x3fffffff;                        // fewest new keys any real row of this wave's tiles sees
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
        if (ok) vis_min = min(vis_min, ri.vis);
        const bf16_t *qp = ROPE ? q_lds + (ok ? f : 0) * HD + 8 * lh
                                : a.q + (((size_t)b * d.R + r) * a.n_q + (g * a.group + hq)) * HD + 8 * lh;
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

    const size_t page_elems = (size_t)a.kv.n_kv * 16 * HD;
    const size_t scr_elems = (size_t)a.n_groups * (n_mt > 0 ? n_mt : 1) * 16 * HD;   // B * n_kv tiles
    const int32_t *pt = a.kv.page_table + (size_t)(d.seq_base + b) * a.kv.pages_per_seq;

    // one key-pair iteration of every query tile of this wave against LDS buffer `buf`
    // (pure_c: both units lie wholly inside the prefix, no predicate.  The pure iterations are the leading ones of
    // the sequence and get a loop of their own: with both forms in one loop body the compiler copied all 64
    // accumulator registers back and forth at the point where the two paths meet, in every iteration.)
    auto compute = [&](auto pure_c, int it, int buf) __attribute__((always_inline)) {
        constexpr bool pure = decltype(pure_c)::value;
#pragma unroll
        for (int i = 0; i < QT; ++i) {
            const int tile = t0 + wave + 4 * i;
            if (tile >= t1) continue;                       // wave-uniform
            if constexpr (pure) {
                attn_block<false>(k_lds[buf], v_lds[buf], lq, lh, qf[i], acc[i], m_run[i], l_run[i],
                                       a.scale_log2e, 0xffffu);
            } else {
                // A row sees a contiguous key range of each unit: cache positions below L + vis, or the mask rows
                // of its own block.  The range becomes a 16-bit mask over the unit's keys, from which the lane
                // picks its eight: register e of unit u <-> key 8*lh + e%8 of that unit.
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
                    vis_bits |= ((m16 >> (8 * lh)) & 0xffu) << (8 * u);
                }
                if (!__any(vis_bits != 0)) continue;        // nothing of this pair is visible to this tile
                attn_block<true>(k_lds[buf], v_lds[buf], lq, lh, qf[i], acc[i], m_run[i], l_run[i],
                                      a.scale_log2e, vis_bits);
            }
        }
    };

    const std::true_type pure_c;
    const std::false_type masked_c;
    // Leading iterations whose two units every row of this wave's tiles sees in full: the prefix, and in a prefill
    // or scoring pass also the rows of the pass that lie before the tile (all but the diagonal of a causal pass).
    // The count differs from wave to wave; the loops below pass the same one barrier per iteration.
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) vis_min = min(vis_min, __shfl_xor(vis_min, o));
    const int n_pure_w = __builtin_amdgcn_readfirstlane(min(n_cache_units, max(n_pure, (L + min(vis_min, d.nc)) >> 4)));
    const int n_fast = min(max(min(a1, n_pure_w >> 1) - a0, 0), nA);
    {
        // Direct loads: wave w moves unit w/2 of the pair: for K the LDS rows 8*(w%2) .. +7 of that unit (two
        // instructions of 1 KiB: lane = (row, 16-byte slot), the slot holds piece slot ^ row%16 of the key the row
        // stands for), for V^T the key half w%2 of all 128 d (lane = d).  The tiles land in buffer n % 3 two
        // iterations ahead of their use; a wave waits for its own loads of iteration n (vmcnt), then the workgroup
        // barrier makes all four waves' parts visible and at the same time frees the buffer of iteration n-1 for
        // the loads of iteration n+2.
        const int u_w = wave >> 1, half_w = wave & 1;
        int k_voff[2], v_voff[2];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int row = 8 * half_w + 4 * jj + (lane >> 4);                    // LDS row within the unit
            const int key = (row & 3) | ((row & 4) << 1) | ((row & 8) >> 1);     // rows 4-7 <-> keys 8-11
            k_voff[jj] = key * (HD * 2) + (((lane & 15) ^ row) << 4);
            v_voff[jj] = (64 * jj + lane) * 32 + half_w * 16;
        }
        // An odd unit count leaves the second half of the last pair's tiles unwritten.  Its scores are masked by
        // a select, so stale K bits do no harm, but its V^T is multiplied by probabilities of exactly zero and
        // must not be NaN or Inf: the workgroup that runs that last pair clears the V^T tiles first.
        if ((U & 1) && n_seq > 0 && seq_it(n_seq - 1) == n_it - 1) {
            for (int i = tid; i < NBUF * V_TILE / 8; i += 256)
                reinterpret_cast<bf16x8 *>(&v_lds[0][0])[i] = (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
            __syncthreads();
        }
        // the Q fragments must have arrived before the loop: a wait for them inside it would be a vmcnt(0) and
        // drain the tile loads in flight
#pragma unroll
        for (int i = 0; i < QT; ++i)
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qf[i][ks]));
        const int4v dk = raw_desc(a.kv.k_pages, (size_t)a.kv.n_pages * page_elems * 2);
        const int4v dv = raw_desc(a.kv.v_pages, (size_t)a.kv.n_pages * page_elems * 2);
        const int4v dks = raw_desc(a.k_scr, scr_elems * 2), dvs = raw_desc(a.v_scr, scr_elems * 2);
        typedef __attribute__((address_space(3))) unsigned char lds_byte;
        const unsigned k_lds0 = (unsigned)(size_t)(lds_byte *)reinterpret_cast<unsigned char *>(&k_lds[0][0]);
        const unsigned v_lds0 = (unsigned)(size_t)(lds_byte *)reinterpret_cast<unsigned char *>(&v_lds[0][0]);
        // the page table does not change while the kernel runs: read through the constant address space, the page
        // ids come by scalar loads (no vector-memory traffic that the vmcnt bookkeeping below would have to count)
        const __attribute__((address_space(4))) int32_t *ptc = (const __attribute__((address_space(4))) int32_t *)pt;
        // V^T slots past the data of a unit (the page the sequence ends in, the last mask tile) may hold anything:
        // they are cleared in LDS before use (uniform, at most twice in a workgroup's life)
        auto clear_tail = [&](int it, int buf) __attribute__((always_inline)) {
            bool any = false;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int uu = 2 * it + u;
                int valid = 16;
                if (uu < n_cache_units) valid = min(16, L + d.nc - 16 * uu);
                else if (uu < U) valid = min(16, n_mask - 16 * (uu - n_cache_units));
                if (valid < 16) {
                    any = true;
                    if (tid < 128) {
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            bf16x8 *pv = reinterpret_cast<bf16x8 *>(&v_lds[buf][0]) + (u * 2 + h) * 128 + tid;
                            bf16x8 vv = *pv;
#pragma unroll
                            for (int j = 0; j < 8; ++j)
                                if (8 * h + j >= valid) vv[j] = (bf16_t)0.f;
                            *pv = vv;
                        }
                    }
                }
            }
            if (any) lds_barrier();
        };
        auto unit_of = [&](int m) { return 2 * seq_it(m) + u_w; };
        auto page_of = [&](int m) {                          // page id of this wave's unit in iteration m (or 0)
            const int uu = unit_of(m);
            return (m < n_seq && uu < n_cache_units) ? ptc[uu] : 0;
        };
        int b_cur = 0, b_nxt = 1, b_far = 2;                // buffers of iterations n, n+1, n+2
        int c_nxt = 0;                                      // loads this wave issued last (0 or 4)
        int page = page_of(0);                              // page id of the next loads to be issued
        auto issue = [&](int m, int buf) __attribute__((always_inline)) {      // this wave's loads of iteration m
            const int uu = unit_of(m);
            c_nxt = 0;
            if (m < n_seq && uu < U) {
                const unsigned kd = k_lds0 + buf * (K_TILE * 2) + (u_w * 16 + 8 * half_w) * 256;
                const unsigned vd = v_lds0 + buf * (V_TILE * 2) + (u_w * 2 + half_w) * 2048;
                if (uu < n_cache_units) {
                    const int base = (int)((((size_t)page * a.kv.n_kv + g) * 16 * HD) * 2);
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj) {
                        dma16(kd + 1024 * jj, k_voff[jj], dk, base);
                        dma16(vd + 1024 * jj, v_voff[jj], dv, base);
                    }
                } else {
                    const int mt = uu - n_cache_units;
                    const int base = (int)(((((size_t)b * a.kv.n_kv + g) * n_mt + mt) * 16 * HD) * 2);
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj) {
                        dma16(kd + 1024 * jj, k_voff[jj], dks, base);
                        dma16(vd + 1024 * jj, v_voff[jj], dvs, base);
                    }
                }
                c_nxt = 4;
            }
            page = page_of(m + 1);
        };
        // make the tiles of iteration n usable and start the loads of iteration n+2 into the buffer that the
        // barrier has just freed (every wave is past iteration n-1).  A wave's loads of iteration n have landed
        // once no more than those of n+1, its latest, are in flight.
        auto ready = [&](int n) __attribute__((always_inline)) {
            if (c_nxt == 4) __builtin_amdgcn_s_waitcnt(4 | (7 << 4) | (15 << 8));
            else __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));
            lds_barrier();
            issue(n + 2, b_far);
        };
        auto rotate = [&]() __attribute__((always_inline)) {
            const int t = b_cur;
            b_cur = b_nxt;
            b_nxt = b_far;
            b_far = t;
        };
        auto general = [&](int n) __attribute__((always_inline)) {
            const int it = seq_it(n);
            clear_tail(it, b_cur);
            compute(masked_c, it, b_cur);
        };
        issue(0, b_cur);
        issue(1, b_nxt);
        int n = 0;
        if (n_seq > 0) {
            ready(0);
            // the first iteration moves the references off -inf; the iterations that follow, while both their
            // units lie inside the prefix, keep them where they are (no rescale arm in that loop); a wave whose
            // scores outgrow its reference by 2^60 leaves for the general loop (the waves of a workgroup may
            // be in different loops: each iteration of either passes the same one barrier)
            if (n_fast > 0) compute(pure_c, seq_it(0), b_cur);
            else general(0);
            for (n = 1; n < n_fast; ++n) {
                rotate();
                ready(n);
                bool ok = true;
#pragma unroll
                for (int i = 0; i < QT; ++i) {
                    const int tile = t0 + wave + 4 * i;
                    if (tile < t1)
                        ok = ok && attn_block_fixed_ref<PRIO>(k_lds[b_cur], v_lds[b_cur], lq, lh, qf[i], acc[i], m_run[i],
                                                             l_run[i], a.scale_log2e);
                }
                if (!ok) break;
            }
            if (n < n_fast) {          // refused: this iteration's tiles are ready, only the block has to run
                general(n);
                ++n;
            }
            for (; n < n_seq; ++n) {
                rotate();
                ready(n);
                general(n);
            }
        }
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

AttnPlan plan_attention(int B, int n_kv, int group, int R, int nc, int max_keys) {
    AttnPlan p;
    int TQ = (group * R + 31) / 32;           // 32-row query tiles per kv head
    p.tiles_per_chunk = TQ < 4 ? TQ : 4;      // four waves x one query tile each
    p.n_chunks = (TQ + p.tiles_per_chunk - 1) / p.tiles_per_chunk;
    int base = B * n_kv * p.n_chunks;
    // the caller's bound is taken in steps of 256 keys: bounds that differ by less cut the keys alike, so results do
    // not change bit for bit because a caller's estimate of the final length moved a little
    max_keys = (max_keys + 255) & ~255;
    int iters = (max_keys + 31) / 32;
    // Two workgroups are resident per CU (512 slots).  A split costs about eight key-pair iterations of prologue
    // and partial-sum epilogue; a grid of w slot-fulls takes about w + 1/2 workgroup times (the last round is
    // ragged).  The split count with the least estimated time wins, the smaller one on a near tie (fewer partial
    // sums for the combine kernel): 7 at batch 1 and 4096 keys (one full round), 5 at batch 4 and 8192 keys
    // (where one split left 44 % of the slots idle for the whole launch), 1 once the batch alone fills the chip
    // several times over.  A pass with many causal rows (prefill, scoring) is another matter: its workgroups walk
    // key ranges of very different lengths, the rounds do not end together, and no ragged last round is charged
    // (measured on the training-layout pass of 4096 rows: two splits cost 6 ms per forward in partial sums and
    // their combine launch, against nothing gained in the attention kernel).
    // No more than 64 splits (the combine kernel reads one per lane) and, beyond two, no more than four slot-fulls
    // of workgroups: that bound depends on the row structure alone, and the workspace is sized by it, so the
    // partial-sum area does not depend on the key bound of a particular call.
    p.splits_bound = 2048 / base < 2 ? 2 : 2048 / base > 64 ? 64 : 2048 / base;
    int cap = (iters + 3) / 4;                // at least four key pairs per split
    if (cap > p.splits_bound) cap = p.splits_bound;
    // A single query tile per kv head and few sequences (the one-token step up to batch 4): every workgroup is mostly
    // prologue and epilogue, and its partial result is folded by each workgroup of the O projection.  No more splits
    // than give every CU one workgroup - a grid a little above 256 leaves some CUs with two (batch 1, 4096 keys:
    // 36 splits = 288 workgroups 3.75 ms per step, 32 splits 3.68; 12 288 keys: 3.94 -> 3.90) - as long as a split
    // then stays short (batch 4 at 8192 keys: 8 splits of 32 iterations lose to 16 of 16, 5.14 against 5.02 ms).
    if (TQ == 1 && base <= 32 && cap > 256 / base && iters <= 16 * (256 / base)) cap = 256 / base;
    int s = 1;
    double best = 0.0;
    for (int c = 1; c <= cap; ++c) {
        const double waves = (double)base * c / 512.0;
        const double cost = (waves <= 1.0 ? 1.0 : nc >= 64 ? waves : waves + 0.5) * ((iters + c - 1) / c + 8);
        if (c == 1 || cost < 0.97 * best) {
            best = cost;
            s = c;
        }
    }
    p.splits = s < 1 ? 1 : s;
    p.per = (iters + 1 + p.splits - 1) / p.splits;   // +1: the kernel counts cache and scratch units separately
    return p;
}

bool attention_rope_ok(RowDesc d, int group, int hd) {
    return d.R == 1 && d.nc == 1 && d.nm == 0 && group >= 1 && group <= 32 && hd == HD;
}

size_t attn_partial_floats(int B, int n_kv, int group, int R, int hd, int splits) {
    return (size_t)B * n_kv * splits * group * R * (hd + 2);
}

void launch_attention_bf16(const bf16_t *q, KvView kv, const bf16_t *k_scr, const bf16_t *v_scr,
                           const int32_t *prefix_len, RowDesc d, int B, int n_q, const AttnPlan &p, float *part,
                           bf16_t *out, int out_af, hipStream_t st, const AttnRope *rope) {
    AttnArgs a;
    a.rp = AttnRope{};
    const bool fused_rope = rope && rope->part && attention_rope_ok(d, n_q / kv.n_kv, kv.hd);
    if (fused_rope) a.rp = *rope;
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
    a.scale_log2e = 1.4426950408889634f / sqrtf((float)kv.hd);
    size_t F = (size_t)a.group * d.R;
    size_t rows = (size_t)B * kv.n_kv * p.splits * F;
    a.opart = part;
    a.mpart = part + rows * HD;
    a.lpart = a.mpart + rows;
    a.n_groups = B * kv.n_kv;
    a.xcd_q = a.n_groups % 8 == 0 ? 1 : (a.n_groups < 8 && 8 % a.n_groups == 0) ? 8 / a.n_groups : 0;
    dim3 grid(a.n_groups * p.n_chunks, p.splits);
    if (a.xcd_q > 1) grid.x = 8 * ((p.n_chunks + a.xcd_q - 1) / a.xcd_q);
    if (fused_rope) attn_bf16_kernel<1, false, true><<<grid, 256, 0, st>>>(a);
    else if (p.tiles_per_chunk == 4) attn_bf16_kernel<1, true, false><<<grid, 256, 0, st>>>(a);
    else attn_bf16_kernel<1, false, false><<<grid, 256, 0, st>>>(a);
}

void launch_attention_combine(const float *part, int B, int R, int n_q, int n_kv, int hd, int splits, bf16_t *out,
                              int out_af, hipStream_t st) {
    if (splits == 1) return;                  // the attention kernel has written the result itself
    size_t F = (size_t)(n_q / n_kv) * R;
    size_t rows = (size_t)B * n_kv * splits * F;
    attn_combine_kernel<<<dim3(B * R, n_q), 64, 0, st>>>(part, part + rows * hd, part + rows * hd + rows, R, n_q, n_kv,
                                                         splits, out, out_af, act_layout(B * R));
}
