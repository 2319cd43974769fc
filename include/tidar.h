/*
 * tidar.h — C ABI of the MI355X (gfx950) TiDAR decode-step library.
 *
 * One call = one transformer forward over
 *     [ KV-cached prefix ; the k tokens drafted last step ; k blocks of k mask tokens ]
 * with the paper's hybrid attention mask, followed by autoregressive
 * verification, the KV commit and the choice of the next draft
 * (paper Section 1 "at each generation step ...", Section 3.2, Section 3.3).
 *
 * Conventions that hold for every entry point unless it says otherwise:
 *   - "dev" pointers are device (HBM) addresses on the current HIP device,
 *     "host" pointers are ordinary host addresses.  All tensor memory is owned
 *     by the caller; the library allocates no device memory and keeps no
 *     pointer after a call returns.
 *   - Work is enqueued on `stream` (a hipStream_t of the current device passed
 *     as void*, NULL = the null stream) and the call returns without
 *     synchronising.
 *   - Argument and capacity errors are found on the host before anything is
 *     enqueued; a failing call has no effect on device memory.
 *   - What only the device knows is checked by the kernels, after the call has
 *     returned: a prefix_len[b] that is negative or, with the rows of the call,
 *     runs past pages_per_seq * 16 (the host saw only the caller's bound); a
 *     page-table entry outside [0, n_pages) under a position the call writes; a
 *     token id outside [0, vocab); a logits row without a single number (all
 *     NaN) where a token has to be chosen.  Such a sequence never makes the
 *     kernels touch memory outside the caller's buffers (lengths are clamped,
 *     bad ids replaced, unsafe K/V stores skipped) and is reported through its
 *     outputs, each entry point says how; the other sequences of the batch are
 *     not affected.
 *   - dtype 1 (bf16): activations, Q/K/V and weights are bf16, the residual
 *     stream and all accumulation are fp32.  dtype 0 (fp32): everything fp32.
 *   - Indices in comments are 0-based.
 */
#ifndef TIDAR_H
#define TIDAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tidar_ctx tidar_ctx;   /* opaque; host metadata, profiling events */

typedef enum {
    TIDAR_OK = 0,
    TIDAR_EINVAL = 1,      /* bad argument (null pointer, k out of range, unsupported shape) */
    TIDAR_ENOMEM = 2,      /* workspace too small */
    TIDAR_ECAPACITY = 3,   /* page table too short for prefix + new rows */
    TIDAR_EDEVICE = 4,     /* no gfx950 device / HIP error */
    TIDAR_ESTATE = 5       /* call order violated */
} tidar_status;

enum { TIDAR_F32 = 0, TIDAR_BF16 = 1 };
enum { TIDAR_PAGE_SIZE = 16, TIDAR_MAX_K = 16 };
enum { TIDAR_STATIC_SCRATCH_BYTES = 32 << 20 };   /* scratch of tidar_gemm_static, per GPU, for the life of the process */

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab;
    int32_t tied_embeddings;   /* informational: the caller passes lm_head explicitly either way */
    int32_t dtype;             /* TIDAR_F32 or TIDAR_BF16 */
    int32_t page_size;         /* must be 16 */
    int32_t max_k;             /* largest draft/block length that will be used, <= 16 */
    int32_t max_batch;
    int32_t mask_token_id;     /* id fed into every mask slot */
    float   rope_base;
    float   rms_eps;
} tidar_config;

/*
 * Weights, in the library's layout.  Norm gains are plain vectors of `dtype`.
 * `embed` is a plain row-major [vocab][d_model] table of `dtype`.
 * Every projection matrix must have been written by tidar_pack_weight into a
 * buffer of tidar_packed_weight_bytes(rows, cols):
 *     wqkv    : (n_q_heads + 2 n_kv_heads) * head_dim rows  x d_model   (Q rows, then K rows, then V rows)
 *     wo      : d_model rows x n_q_heads*head_dim
 *     w_gate_up: 2*d_ff rows x d_model, gate and up interleaved in groups of 16 rows
 *               (row tile 2t = gate rows 16t..16t+15, row tile 2t+1 = up rows 16t..16t+15)
 *     w_down  : d_model rows x d_ff
 *     lm_head : vocab rows x d_model (pack `embed` again when embeddings are tied)
 * Each per-layer field is a host array of n_layers device pointers.
 */
typedef struct {
    const void *embed;
    const void *lm_head;
    const void *final_norm;
    const void *const *attn_norm;
    const void *const *wqkv;
    const void *const *wo;
    const void *const *ffn_norm;
    const void *const *w_gate_up;
    const void *const *w_down;
} tidar_weights;

/*
 * Paged exact KV cache (paper Section 3.3: K/V of causally encoded tokens are
 * kept, never recomputed).  Element type = config dtype.
 *   k_pages : [n_layers][n_pages][n_kv_heads][16 tokens][head_dim]   (K after RoPE)
 *   v_pages : [n_layers][n_pages][n_kv_heads][head_dim][16 tokens]   (V, token index fastest)
 *   page_table : dev int32 [max_batch][pages_per_seq]; entry = physical page of
 *                logical page (token position / 16) of that sequence.
 * Token position p of sequence b lives in page page_table[b][p/16], slot p%16.
 * After a step, positions < prefix_len[b] hold exact causal K/V; anything at or
 * beyond prefix_len[b] is unspecified (rejected drafts are evicted by not
 * advancing prefix_len over them).  One layer's K (or V) pages may not exceed 2 GiB
 * (n_pages * n_kv_heads * 16 * head_dim * element size <= 0x7fffffe0: the kernels use
 * 32-bit byte offsets); larger caches are rejected with TIDAR_EINVAL.  The pages need not
 * be initialised: slots that hold no committed token are never read as data.
 */
typedef struct {
    void *k_pages;
    void *v_pages;
    const int32_t *page_table;
    int32_t pages_per_seq;
    int32_t n_pages;
} tidar_kv_cache;

typedef struct {
    int32_t  sample;        /* 0: greedy argmax (ties -> lowest id); 1: Gumbel-max sampling at the causal rows */
    float    temperature;   /* used when sample == 1, must be > 0 */
    uint64_t seed;          /* noise is keyed by (seed, sequence index, predicted absolute position, token id) */
    float    beta;          /* weight of the causal logits in verification (paper Section 4.3.3); 1 = trust AR */
} tidar_mode;

/* Create / destroy the host-side context.  Checks the shape against what the
 * kernels support (bf16: head_dim 128, d_model, d_ff and head products
 * multiples of 32; fp32: head_dim <= 128) and that device 0.. current is gfx950
 * when a device is present (a missing device is reported by the first launch). */
tidar_status tidar_create(const tidar_config *cfg, tidar_ctx **out);
void         tidar_destroy(tidar_ctx *ctx);
const char  *tidar_strerror(tidar_status s);

/* Bytes of a packed projection matrix with `rows` output features and `cols`
 * input features (rows multiple of 16, padded to 32; cols multiple of 32 in bf16 mode). */
size_t       tidar_packed_weight_bytes(int32_t dtype, int32_t rows, int32_t cols);

/*
 * Re-lay a plain row-major [rows][cols] matrix (dev, `dtype`) into the packed
 * buffer `dst` (dev).  Row tile t (16 rows) of `src` lands in row tile
 * dst_tile_offset + t * dst_tile_stride of the destination, so several source
 * matrices can share one destination (Q|K|V, interleaved gate/up).
 * `dst_rows` is the destination's total row count.
 * bf16 layout: [k step of 16][32-row tile][lane 0..63][8 values], lane = (k/8 % 2)*32 + row%32,
 * i.e. the register image of one 32x32x16 MFMA operand, k step outermost (destination rows are padded
 * to a multiple of 32); fp32 layout: plain row-major.
 */
tidar_status tidar_pack_weight(int32_t dtype, const void *src, int32_t rows, int32_t cols,
                               void *dst, int32_t dst_rows, int32_t dst_tile_offset, int32_t dst_tile_stride,
                               void *stream);

/* Workspace needed by tidar_prefill / tidar_step / tidar_ar_step /
 * tidar_hybrid_attention for up to `batch` sequences, block length `k` and
 * prefixes up to `max_prefix_len`. */
tidar_status tidar_workspace_bytes(const tidar_ctx *ctx, int32_t batch, int32_t k, int32_t max_prefix_len,
                                   size_t *bytes);

/*
 * Prefill (paper Section 3.2, Appendix B): encode each prompt causally, append
 * one bidirectional block of k mask tokens, fill the cache with the prompt's
 * K/V and return the first drafts.  Runs in causal chunks through the same
 * kernels as the step; untuned.
 *   prompt      dev int32 [batch][prompt_stride]
 *   prompt_len  host int32 [batch], each >= 1
 *   prefix_len  dev int32 [batch] out: set to prompt_len
 *   first_drafts dev int32 [batch][k] out: slot 0 = token chosen from the causal
 *               logits of the last prompt row (final), slots 1..k-1 = argmax of mask slots 1..k-1
 *   logits_out  optional dev fp32 [batch][1+k][vocab]: last prompt row, then the k mask rows
 * A sequence that fails a device-side check (token id, page id) gets prefix_len[b] = -1 and first_drafts[b][*] = -1.
 */
tidar_status tidar_prefill(tidar_ctx *ctx, const tidar_weights *w, const tidar_kv_cache *kv, int32_t batch,
                           const int32_t *prompt, int32_t prompt_stride, const int32_t *prompt_len, int32_t k,
                           const tidar_mode *mode, int32_t *prefix_len, int32_t *first_drafts, float *logits_out,
                           void *ws, size_t ws_bytes, void *stream);

/*
 * The decode step (paper Section 3.2; row count k(k+1) per Section 3.3).
 *   prefix_len  dev int32 [batch] in/out: L on entry, L + accepted_len on exit
 *   drafts      dev int32 [batch][k]: slot 0 is trusted (it is next_drafts[0] /
 *               first_drafts[0] of the previous call, already final); slots 1..k-1 are verified
 *   accepted_len    dev int32 [batch] out, in [1, k]
 *   accepted_tokens dev int32 [batch][k] out, first accepted_len valid (= drafts[0..a))
 *   next_drafts     dev int32 [batch][k] out: slot 0 = token from the causal logits at the first
 *               unverified position, slots 1..k-1 = argmax of slots 1..k-1 of mask block a-1
 *   logits_out  optional dev fp32 [batch][k(k+1)][vocab], rows in the order
 *               c_0..c_{k-1}, blk_0[0..k), ..., blk_{k-1}[0..k)
 *   max_prefix_len_hint  host upper bound of every prefix_len[b] on entry (capacity check, grid sizing).
 *               The attention kernel cuts the key range into equal splits of this bound (rounded up to a multiple
 *               of 256 keys, so that nearby bounds cut alike), so a key's split depends
 *               on its position and the bound, not on the current length: with one bound held over a run of calls
 *               (e.g. the length the generation may reach) a row with the same context gets bit-identical logits
 *               at every step; a bound far above the real length leaves the later splits empty (slower, still
 *               correct).
 * `drafts` may alias `next_drafts`.
 * A sequence that fails a device-side check (see the conventions above) gets accepted_len[b] = 0,
 * accepted_tokens[b][*] = next_drafts[b][*] = -1 and keeps its prefix_len[b].
 * The library keeps no per-sequence state: a call covers sequences 0..batch-1 of the arrays it is given, so a
 * run of sequences inside a larger batch is addressed by offsetting prefix_len, drafts, the outputs and
 * kv->page_table (by pages_per_seq entries per sequence).  That is how sequences with different k are stepped
 * (one call per run of equal k), join (tidar_prefill on their own slots) and leave.  (Sampling noise is keyed by
 * the sequence's index within the call: a sampled stream is reproducible only while that index stays the same.)
 */
tidar_status tidar_step(tidar_ctx *ctx, const tidar_weights *w, const tidar_kv_cache *kv, int32_t batch,
                        int32_t *prefix_len, const int32_t *drafts, int32_t k, const tidar_mode *mode,
                        int32_t *accepted_len, int32_t *accepted_tokens, int32_t *next_drafts, float *logits_out,
                        int32_t max_prefix_len_hint, void *ws, size_t ws_bytes, void *stream);

/*
 * The one-token autoregressive step the paper compares against (Section 1:
 * one token slot per forward): token_in[b] is appended at prefix_len[b], its
 * K/V committed, prefix_len += 1, token_out[b] = token chosen from its logits.
 *   logits_out optional dev fp32 [batch][vocab]
 * A sequence that fails a device-side check gets token_out[b] = -1 and keeps its prefix_len[b].
 */
tidar_status tidar_ar_step(tidar_ctx *ctx, const tidar_weights *w, const tidar_kv_cache *kv, int32_t batch,
                           int32_t *prefix_len, const int32_t *token_in, const tidar_mode *mode,
                           int32_t *token_out, float *logits_out, int32_t max_prefix_len_hint,
                           void *ws, size_t ws_bytes, void *stream);

/*
 * The hybrid-mask attention of one layer on its own (paper Figure 2 / Figure 3:
 * clean tokens causal, mask tokens bidirectional inside their block and
 * conditioned on the drafts their block stands for).
 * Rows per sequence R = n_causal + n_blocks*block_len, ordered causal rows
 * first, then block 0, block 1, ...  Block j sees the first cond0 + j causal
 * rows (cond0 = 1 for the decode step, = n_causal for the prefill block).
 *   q      dev [batch][R][n_q_heads][head_dim]  (already rotated)
 *   k_new, v_new dev [batch][R][n_kv_heads][head_dim]: K/V of the new rows; the causal rows'
 *          K/V are written into the cache of `layer` at positions prefix_len[b]+i,
 *          mask rows' K/V only into the workspace
 *   out    dev [batch][R][n_q_heads][head_dim]
 * Element type = config dtype.  prefix_len is read, not advanced.
 */
tidar_status tidar_hybrid_attention(tidar_ctx *ctx, const tidar_kv_cache *kv, int32_t layer, int32_t batch,
                                    const int32_t *prefix_len, const void *q, const void *k_new, const void *v_new,
                                    int32_t n_causal, int32_t n_blocks, int32_t block_len, int32_t cond0,
                                    void *out, int32_t max_prefix_len_hint, void *ws, size_t ws_bytes, void *stream);

/*
 * out[M][N] (dev fp32) = a[M][K] (dev, dtype) x packed weight (N rows, K cols)^T.
 * The skinny GEMM every projection of the step runs through, exposed for tests
 * and measurement.  ws must hold tidar_gemm_workspace_bytes(M, N, K) bytes.
 */
size_t       tidar_gemm_workspace_bytes(int32_t dtype, int32_t M, int32_t N, int32_t K);
tidar_status tidar_gemm(tidar_ctx *ctx, const void *a, const void *w_packed, float *out,
                        int32_t M, int32_t N, int32_t K, void *ws, size_t ws_bytes, void *stream);

/*
 * tidar_gemm for callers that cannot allocate or hand over a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same kernels and the same result as tidar_gemm, but the A-fragment copy
 * and the split-K partial sums live in a static device array of TIDAR_STATIC_SCRATCH_BYTES (32 MiB) that is part
 * of the library image on every GPU it runs on; the call allocates nothing, creates no events (the profiling
 * switch is ignored) and takes no workspace.  Shapes whose tidar_gemm_workspace_bytes exceed the array are rejected
 * with TIDAR_ENOMEM before anything is enqueued (272 x 4096 x 12288 in bf16 needs 24.5 MiB and fits; 4096 rows of
 * the same do not); TIDAR_EDEVICE when the current device cannot give the array's address.  All calls on one GPU
 * share the one array: calls that overlap in time on the same GPU (two streams, two threads) race; calls on one
 * stream are ordered.  Nothing in the array has to be cleared between calls, whatever an earlier call left there.
 */
tidar_status tidar_gemm_static(tidar_ctx *ctx, const void *a, const void *w_packed, float *out,
                               int32_t M, int32_t N, int32_t K, void *stream);

/*
 * Likelihood of a text in AR mode (paper Section 4.2.2: the causal section alone scores a text the way any
 * autoregressive model does, one forward) and, with block_len > 0, the forward over the doubled training sequence
 * (Section 3.1, Figure 3 left): the text followed by one mask token per text position, the text attended causally,
 * the masks of a block (block j covers positions [j*block_len, (j+1)*block_len), the last block may be short)
 * attending to each other in both directions and to the text before their block; a mask keeps the position id of
 * the token it stands in for.  Forward only: log-probabilities and the objective's value, no gradients.
 *   tokens   dev int32 [batch][stride]; len host int32 [batch], 1 <= len[b] <= stride
 *   block_len 0: causal section only (diff_logprob must be NULL); 1..16: both sections (diff_logprob required)
 *   ar_logprob   dev fp32 [batch][stride] out: entry i = ln p(tokens[i+1] | tokens[0..i]) from the causal row i
 *                (labels shifted by one), i < len-1; entry len-1 is set to 0, later entries are untouched
 *   diff_logprob dev fp32 [batch][stride] out: entry i = ln p(tokens[i] | text before the block of i, masks) from
 *                the mask row of position i (labels in place), i < len
 *   loss     optional dev fp32 [batch] out: the Section 3.1 objective of each sequence,
 *            (alpha * A + D) / (1 + alpha) with A = -mean of ar_logprob[0..len-1) and D = -mean of
 *            diff_logprob[0..len-1) (both sums printed with len-1 terms: the last mask position takes no part);
 *            with block_len = 0 it is A; 0 for a one-token text.  alpha in [0, 1].
 * The sequences are run one after another in passes of the prefill chunk's causal rows (rounded down to whole
 * blocks) through the step's kernels, every row through the LM head.  The K/V cache pages of sequences
 * 0..batch-1 are overwritten with the text's K/V (positions [0, len)); the caller's prefix_len array is not
 * involved.  ws must hold tidar_score_workspace_bytes(max over len, block_len) bytes.
 */
tidar_status tidar_score_workspace_bytes(const tidar_ctx *ctx, int32_t max_len, int32_t block_len, size_t *bytes);
tidar_status tidar_score(tidar_ctx *ctx, const tidar_weights *w, const tidar_kv_cache *kv, int32_t batch,
                         const int32_t *tokens, int32_t stride, const int32_t *len, int32_t block_len, float alpha,
                         float *ar_logprob, float *diff_logprob, float *loss, void *ws, size_t ws_bytes,
                         void *stream);

/* Causal rows per prefill pass (the prompt is prefilled in causal chunks through the step's kernels, the mask block
 * of Appendix B joins the last chunk).  Default 2048; 1..4096.  Larger passes stream the weights fewer times and
 * need a larger workspace: call before tidar_workspace_bytes / tidar_score_workspace_bytes.  Host only. */
tidar_status tidar_set_prefill_chunk(tidar_ctx *ctx, int32_t rows);

/* Block length for the coming steps (paper, Limitations, "Batch size": the block length can be changed between
 * decode steps without retraining; Section 1 / Figure 1: a step costs about as much as a 1-token step while its
 * rows fit the machine's free token slots).  Returns the largest k in {1, 2, 4, 8, 16} with
 * k <= min(cfg.max_k, k_cap) and batch * k * (k + 1) <= row_budget.  row_budget <= 0 takes the library's figure
 * for MI355X (160 rows: up to there the measured TiDAR step stays within about 1.4x of the 1-token step at the
 * 8B shape); k_cap <= 0 means no cap.  Host only, no device work.  Returns 1 when nothing larger fits and 0 on
 * invalid arguments (ctx NULL, batch < 1). */
int32_t tidar_select_block_len(const tidar_ctx *ctx, int32_t batch, int32_t k_cap, int32_t row_budget);

/*
 * Per-kernel timing with HIP events on the launch stream.  While enabled,
 * every kernel class the library launches is bracketed by events; reading
 * synchronises the recorded events.  `names`/`ms`/`launches` receive up to
 * `cap` entries; the return value is the number of kernel classes seen.
 * Timing a whole step should be done with profiling off.
 */
tidar_status tidar_profile_enable(tidar_ctx *ctx, int32_t on);
int32_t      tidar_profile_read(tidar_ctx *ctx, const char **names, double *ms, int64_t *launches, int32_t cap);
tidar_status tidar_profile_reset(tidar_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* TIDAR_H */
