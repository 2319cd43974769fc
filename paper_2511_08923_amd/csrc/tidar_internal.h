// Internal declarations shared by the library's translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tidar.h"

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// Row structure of one forward, identical for every sequence of the batch.
// Rows per sequence: nc causal rows, then nm mask rows in nb blocks of bl (the last block may be short).
// Block j is conditioned on the first cond0 + j * cstride causal rows and sits at the positions right after
// them: cstride 1 is the decode step (one block per possible acceptance length), cstride bl the training layout
// (block j stands in for causal rows [j*bl, (j+1)*bl), Section 3.1).
struct RowDesc {
    int nc, nb, bl, cond0;
    int cstride;
    int nm;         // mask rows: (nb - 1) * bl < nm <= nb * bl
    int R;          // nc + nm
    int seq_base;   // first sequence index (into prefix_len / page_table rows)
};

struct RowInfo {
    int pos;   // absolute position id
    int vis;   // number of new causal keys this row may see
    int blk;   // mask block index, -1 for causal rows
};

__host__ __device__ inline RowInfo row_info(const RowDesc &d, int r, int L) {
    RowInfo ri;
    if (r < d.nc) {
        ri.pos = L + r;
        ri.vis = r + 1;
        ri.blk = -1;
    } else {
        int m = r - d.nc;
        int j = m / d.bl;
        int s = m - j * d.bl;
        ri.vis = d.cond0 + j * d.cstride;
        ri.pos = L + ri.vis + s;
        ri.blk = j;
    }
    return ri;
}

// Activation layout of every GEMM input: the register image of the MFMA A operand, so that the slice a
// workgroup stages for a chunk of K is one contiguous block.  Two forms, chosen by the row count M:
//   M <= 32 ("narrow", 16x16x32 MFMA): [k step of 32][16-row tile][lane][8], lane = (k/8 % 4) * 16 + row % 16
//   M  > 32 ("wide",   32x32x16 MFMA): [k step of 16][32-row tile][lane][8], lane = (k/8 % 2) * 32 + row % 32
// Rows are padded to the tile height; pad rows are never written and results are never stored from them.
struct ActLayout {
    int wide;    // 0: narrow, 1: wide
    int tiles;   // row tiles
};
__host__ __device__ inline ActLayout act_layout(int M) {
    ActLayout a;
    a.wide = M > 32;
    a.tiles = a.wide ? (M + 31) / 32 : (M + 15) / 16;
    return a;
}
__host__ __device__ inline size_t af_index(int row, int k, ActLayout a) {
    if (a.wide)
        return ((((size_t)(k >> 4) * a.tiles + (row >> 5)) * 64) + ((k >> 3) & 1) * 32 + (row & 31)) * 8 + (k & 7);
    return ((((size_t)(k >> 5) * a.tiles + (row >> 4)) * 64) + ((k >> 3) & 3) * 16 + (row & 15)) * 8 + (k & 7);
}
__host__ __device__ inline size_t af_elems(int rows, int K) { return (size_t)((rows + 31) / 32) * 32 * K; }
// Layout of every GEMM output except the logits: [split][32-column tile][row][32] fp32.  A row's share of a tile
// is one 128-byte cache line, so a consumer that owns a row never fetches a line it shares with another row's
// consumer (with 16-column tiles every line was fetched twice, by two different XCDs).  N is padded to whole
// tiles; the pad columns are never written or read.
__host__ __device__ inline int pt_cols(int N) { return (N + 31) & ~31; }
__host__ __device__ inline size_t pt_index(int n, int row, int M) {
    return ((size_t)(n >> 5) * M + row) * 32 + (n & 31);
}
__host__ __device__ inline size_t pt_split_stride(int M, int N) { return (size_t)M * pt_cols(N); }

// Paged cache geometry of one layer.
struct KvView {
    void *k_pages;             // layer base
    void *v_pages;             // layer base
    const int32_t *page_table;
    int pages_per_seq;
    int n_pages;               // physical pages per layer: page ids outside [0, n_pages) are never dereferenced
    int n_kv, hd;
};

// Device-side guards.  The host checks capacity against the caller's length bound only; the kernels read the real
// prefix length and the page ids from device memory, which a stale bound or a corrupted table can put anywhere.
// Every kernel therefore works with a prefix length clamped into the table's range (no address is ever formed
// from the raw value), K/V of a sequence that does not fit or of a page id outside the pool are not stored, and
// the kernels that finish a call report such a sequence through its outputs (see tidar.h).
__host__ __device__ inline int kv_capacity(const KvView &kv) { return kv.pages_per_seq * 16; }
__host__ __device__ inline bool seq_fits(const KvView &kv, int L, int n_new) {
    return L >= 0 && (long long)L + n_new <= (long long)kv_capacity(kv);
}
__host__ __device__ inline int clamp_prefix(const KvView &kv, int L, int n_new) {
    const int hi = kv_capacity(kv) - n_new;
    return L < 0 ? 0 : L > hi ? (hi > 0 ? hi : 0) : L;
}
__host__ __device__ inline bool page_ok(const KvView &kv, int page) { return (unsigned)page < (unsigned)kv.n_pages; }

__device__ inline size_t k_page_offset(const KvView &kv, int page, int h, int slot, int d) {
    return (((size_t)page * kv.n_kv + h) * 16 + slot) * kv.hd + d;
}
__device__ inline size_t v_page_offset(const KvView &kv, int page, int h, int slot, int d) {
    return (((size_t)page * kv.n_kv + h) * kv.hd + d) * 16 + slot;
}

// Counter-based sampling noise (Section 3.2: tokens are *sampled* from the causal logits; the paper fixes no
// generator).  24 bits keyed by (seed, sequence, predicted absolute position, token id): a splitmix-style finaliser
// over a linear combination of the key fields; u = (bits + 1/2) / 2^24 in (0, 1); Gumbel noise -ln(-ln u).  Keyed
// by position, not by step, so one-token decoding and TiDAR decoding draw the same noise for the same token slot.
__host__ __device__ inline uint64_t noise_key(uint64_t seed, int seq, int pos_pred) {
    return seed ^ (0x9E3779B97F4A7C15ull * (uint64_t)(pos_pred + 1)) ^ (0xC2B2AE3D27D4EB4Full * (uint64_t)(seq + 1));
}
__host__ __device__ inline uint32_t hash_u24(uint64_t key, uint32_t v) {
    uint64_t z = key + (uint64_t)(v + 1) * 0xD6E8FEB86659FD93ull;
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (uint32_t)(z >> 40);
}
// logit / T + Gumbel(key, v): one expression for every kernel that samples, so that the fused vocabulary reduction
// and the reduction over materialised logits choose the same token bit for bit.
__device__ inline float perturbed_logit(float logit, float inv_t, uint64_t key, uint32_t v) {
    const float u = ((float)hash_u24(key, v) + 0.5f) * (1.0f / 16777216.0f);
    return __builtin_fmaf(logit, inv_t, -__logf(-__logf(u)));
}

// What the LM head's fused vocabulary reduction needs to know about its rows (row = b * Rh + o): the first
// n_choose rows of every sequence are the rows a token is *taken* from (causal logits); with `sample` their values
// are perturbed before the maximum is formed.  With sel_logits != nullptr (beta-mixed verification, Section 4.3.3)
// the logits of those rows and of their mix partners, rows n_choose + i * mix_stride, are also written, compactly:
// [b][2 * n_choose][N] floats, choose rows first; the mix needs two rows of logits side by side, everything else
// of the step still leaves the kernel as (maximum, column) pairs only.
struct ChooseArgs {
    int Rh, n_choose;
    const int32_t *pos_rows;      // position id of every row of the forward, [b][pos_stride]
    int pos_stride, pos_row0, seq_base;
    int sample;
    float inv_t;
    uint64_t seed;
    float *sel_logits;
    int mix_stride;
};

// Profiling hooks (defined in tidar_lib.hip).
enum KernelClass {
    KC_EMBED = 0, KC_RMSNORM, KC_GEMM, KC_ROPE_KV, KC_ATTN, KC_ATTN_COMBINE, KC_SWIGLU, KC_ARGMAX, KC_VERIFY,
    KC_PACK, KC_PLACE_KV, KC_SCORE, KC_COUNT
};

struct GemmPlan {
    int mt;        // 16-row tiles per workgroup pass
    int nt;        // 16-column tiles per wave
    int splits;    // split-K factor
    int bk;        // K elements staged per LDS chunk
    int m_chunks;  // passes over M (grid.z)
    int wide;      // the waves side by side, each over all row tiles of the pass (instead of 2 x 2 waves)
    int nw;        // waves per workgroup: 4, or 8 (side by side, one column tile each: two waves per SIMD)
    int swz;       // > 0: (row pass, column block) plane dealt to the XCDs in super-tiles of swz x swz workgroups
};

GemmPlan plan_gemm_bf16(int M, int N, int K, bool force_single_split);

// ---- launchers (each enqueues on `st`, checks nothing: callers validated shapes) ----
void launch_pack_weight(int dtype, const void *src, int rows, int cols, void *dst, int dst_rows, int tile_off,
                        int tile_stride, hipStream_t st);

void launch_embed_rows(int dtype, const void *embed, const int32_t *tokens, int tok_stride, const int32_t *prefix_len,
                       RowDesc d, int B, int d_model, int mask_id, int vocab, KvView kv, float rope_base,
                       float *x, int32_t *pos_out, float *rope_cs, hipStream_t st);

// x[row] += sum_s part[s][row]; out[row'] = rmsnorm(x[row]) * gain for rows [row0, R) of each sequence.
// part is in the tiled GEMM output layout over all B*R rows, out in the A-fragment layout over B*(R-row0) rows.
void launch_rmsnorm(int dtype, float *x, const float *part, int S, const void *gain, float eps,
                    int B, int R, int row0, int d_model, void *out, hipStream_t st);

// Epilogue forms of the bf16 GEMM: tiled fp32 partial sums (default), plain row-major fp32 (the logits), or, for the
// interleaved gate/up matrix with one split, SwiGLU applied in registers and h written as bf16 straight
// into the A-fragment layout of the down projection (out is then a bf16 buffer of af_elems(M, N/2)).
enum { GEMM_EPI_TILED = 0, GEMM_EPI_ROWMAJOR = 1, GEMM_EPI_SWIGLU = 2, GEMM_EPI_ARGMAX = 3 };
// GEMM_EPI_ARGMAX (single split): no output matrix; every wave reduces its columns to the largest value of each
// row and the lowest column that holds it.  out is then [G][M] floats (values) followed by [G][M] ints (columns),
// G = gemm_argmax_groups(M, N) column groups; launch_argmax_groups folds the groups (ties: lowest column).
inline int gemm_argmax_groups(int M, int N) { return M <= 32 ? (N + 31) / 32 : (N + 63) / 64; }
void launch_argmax_groups(const float *part, int M, int G, int32_t *y, hipStream_t st);
void launch_gemm_bf16(const bf16_t *a, const bf16_t *w_packed, float *out, int M, int N, int K, const GemmPlan &p,
                      int epi, hipStream_t st, const ChooseArgs *choose = nullptr);
void launch_gemm_f32(const float *a, const float *w, float *out, int M, int N, int K, int out_row_major,
                     hipStream_t st);

// The narrow GEMM (a handful of rows: the one-token step, very short blocks) with its producer folded in: instead
// of reading a ready bf16 operand, every workgroup builds the rows it multiplies itself.
//   GEMM_FUSE_NORM: A = rmsnorm(x_in + sum of the previous GEMM's split-K partial sums) * gain, rounded to bf16 (the
//     whole residual row is summed by every workgroup, in the same order, for the row's mean square; workgroup
//     (0, 0) also writes the updated residual stream to x_out, which must not be x_in);
//   GEMM_FUSE_COMBINE: A = the attention output folded from the attention kernel's per-split partial results (only
//     the heads of the workgroup's own share of K).
// Saves one launch each (a dependent launch costs more than either prologue at these row counts).
enum { GEMM_FUSE_NORM = 1, GEMM_FUSE_COMBINE = 2 };
constexpr int kFuseMaxRows = 4;        // rows up to which the fused forms are used
constexpr int kFuseMaxK = 4096;        // and the widest reduction they are built for
struct FuseArgs {
    int kind;
    // GEMM_FUSE_NORM
    const float *x_in;
    float *x_out;
    const float *part;         // tiled partial sums of the previous GEMM over the same rows, S copies
    int S;
    size_t split_stride;
    const bf16_t *gain;
    float eps;
    // GEMM_FUSE_COMBINE: partial results as the attention kernel lays them out
    const float *opart, *mpart, *lpart;
    int R, n_q, n_kv, a_splits;
};
bool gemm_fuse_ok(int M, int N, int K);
void launch_gemm_bf16_fused(const FuseArgs &f, const bf16_t *w_packed, float *out, int M, int N, int K,
                            const GemmPlan &p, int epi, hipStream_t st);
// plain row-major [M][K] -> A-fragment layout, and tiled partial sums -> plain row-major [M][N]
void launch_pack_act(int dtype, const void *src, int M, int K, void *dst, hipStream_t st);
void launch_untile_sum(const float *part, int S, int M, int N, float *out, hipStream_t st);

void launch_rope_kv(int dtype, const float *qkv_part, int S, const float *rope_cs,
                    const int32_t *prefix_len, RowDesc d, int B, int n_q, KvView kv,
                    void *q_out, void *k_scr, void *v_scr, hipStream_t st);

void launch_place_kv(int dtype, const void *k_new, const void *v_new, const int32_t *prefix_len, RowDesc d, int B,
                     KvView kv, void *k_scr, void *v_scr, hipStream_t st);

struct AttnPlan {
    int splits;
    int splits_bound;    // the most splits any key bound can give this row structure (sizes the workspace)
    int n_chunks;        // q-tile chunks per kv head
    int tiles_per_chunk;
    int per;             // key-pair iterations per split, from the caller's bound on the key count (not from the
                         // sequence's current length): a key's split then depends on its position alone
};
AttnPlan plan_attention(int B, int n_kv, int group, int R, int nc, int max_keys);
size_t attn_partial_floats(int B, int n_kv, int group, int R, int hd, int splits);

// The one-token step (R = 1, no mask rows) skips the RoPE launch: the attention workgroups take the new row's Q, K
// and V straight from the QKV projection's split-K partial sums (tiled layout, S splits), rotate Q and K by the
// row's angles, and the workgroup whose key range ends at the new row writes K and V into the cache before it
// reads that page.  part == nullptr: Q comes rotated from `q`, K/V are in place already.
struct AttnRope {
    const float *part;
    int S;
    size_t split_stride;
    const float *rope_cs;      // [row][hd/2][(cos, sin)]
    int M_all;                 // rows of the partial sums (= sequences of the call)
    int q_dim, kv_dim;
};

// With one split the kernel writes the result to out (row-major [rows][n_q][hd], or, out_af != 0, the A-fragment
// layout over B * R rows) and launch_attention_combine does nothing; with more it writes per-split partial
// results to part, which launch_attention_combine folds into out.
void launch_attention_bf16(const bf16_t *q, KvView kv, const bf16_t *k_scr, const bf16_t *v_scr,
                           const int32_t *prefix_len, RowDesc d, int B, int n_q, const AttnPlan &p, float *part,
                           bf16_t *out, int out_af, hipStream_t st, const AttnRope *rope = nullptr);
// whether launch_attention_bf16 can take the new row from the partial sums for this row structure
bool attention_rope_ok(RowDesc d, int group, int hd);
void launch_attention_combine(const float *part, int B, int R, int n_q, int n_kv, int hd, int splits, bf16_t *out,
                              int out_af, hipStream_t st);
void launch_attention_f32(const float *q, KvView kv, const float *k_scr, const float *v_scr,
                          const int32_t *prefix_len, RowDesc d, int B, int n_q, float *out, int out_af,
                          hipStream_t st);

void launch_swiglu(int dtype, const float *part, int S, int M, int d_ff, void *out, hipStream_t st);

// y[b * y_stride + o] = argmax over vocab of (logits or, for the first n_choose rows of each sequence, the sampled /
// beta-mixed value), for rows o < n_rows of each sequence.  Rows per sequence in `logits`: Rh; causal row i mixes
// with row mix_base + i*mix_stride when beta != 1.
void launch_argmax_rows(const float *logits, int B, int Rh, int n_rows, int vocab, int n_choose,
                        const int32_t *pos_rows, int pos_stride, int pos_row0, int seq_base, int sample,
                        float temperature, uint64_t seed, float beta, int mix_base, int mix_stride, int32_t *y,
                        int y_stride, hipStream_t st);

// Scoring (Section 3.1, Section 4.2.2): log-probability of each row's label under row-major logits of one pass over
// text positions [c0, c0 + nc) (nc causal rows, then the mask rows), and the objective of one sequence from its
// first n = len - 1 entries.
void launch_score_rows(const float *logits, int rows, int vocab, const int32_t *text, int len, int c0, int nc,
                       float *ar_out, float *diff_out, hipStream_t st);
void launch_score_loss(const float *ar, const float *diff, int n, float alpha, float *loss, hipStream_t st);

// The kernels that finish a call also check what only the device knows (real prefix lengths, page ids, token ids,
// rows without a token) and report a bad sequence through its outputs.  kv: any layer's view (table and bounds).
void launch_verify_step(const int32_t *y, const int32_t *drafts, int k, int B, int vocab, KvView kv, int seq_base,
                        int32_t *prefix_len, int32_t *accepted_len, int32_t *accepted_tokens, int32_t *next_drafts,
                        hipStream_t st);
void launch_finish_ar(const int32_t *y, const int32_t *token_in, int B, int vocab, KvView kv, int32_t *prefix_len,
                      int32_t *token_out, hipStream_t st);
void launch_finish_prefill(const int32_t *y, const int32_t *tokens, int k, int seq, int add_len, int last, int vocab,
                           KvView kv, int32_t *prefix_len, int32_t *first_drafts, hipStream_t st);
void launch_set_i32(int32_t *p, int n, int32_t v, hipStream_t st);
