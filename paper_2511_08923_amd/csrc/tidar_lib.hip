// Host side of the C ABI: argument validation, workspace carving, and the launch sequence of one forward.
// Nothing here synchronises the device; every kernel goes onto the caller's stream in program order.
#include <string.h>

#include <new>
#include <vector>

#include "tidar_internal.h"

namespace {

const char *kClassNames[KC_COUNT] = {"embed_rows", "rmsnorm", "gemm", "rope_kv", "attention", "attention_combine",
                                     "swiglu", "argmax_rows", "verify", "pack_weight", "place_kv",
                                     "score_rows"};

struct ProfEvent {
    int cls;
    hipEvent_t start, stop;
};

}  // namespace

// Scratch of tidar_gemm_static: device memory that belongs to the library image itself, so that the entry point
// needs no allocation and no workspace argument.  Every GPU the library runs on holds its own copy of the array at
// its own address for the life of the process.  In host code the array's name is only a handle for the symbol:
// the address kernels may use is asked for once per device (scratch_address) and kept.
static __device__ __align__(256) unsigned char scratch[TIDAR_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_addr[kMaxDevices] = {};

// Address of `scratch` on the current device; nullptr when there is no usable device.
void *scratch_address() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    if (!g_scratch_addr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_addr[dev] = p;
    }
    return g_scratch_addr[dev];
}
}  // namespace

struct tidar_ctx {
    tidar_config cfg;
    int prefill_chunk;
    bool profiling;
    std::vector<ProfEvent> events;
    double ms[KC_COUNT];
    int64_t launches[KC_COUNT];
};

namespace {

// Causal rows per prefill pass unless the caller sets another count: measured on the 8B shape, a 4096-token prompt
// takes 117 ms in passes of 256 rows, 93 ms in passes of 1024 and 92 ms in passes of 2048 (every pass streams all
// weights once, so fewer and larger passes win until the GEMMs are compute-bound).
constexpr int kDefaultPrefillChunk = 2048;
constexpr int kMaxPrefillChunk = 4096;

struct Prof {
    tidar_ctx *ctx;
    int cls;
    hipStream_t st;
    ProfEvent ev;
    bool on;
    Prof(tidar_ctx *c, int cls_, hipStream_t s) : ctx(c), cls(cls_), st(s), on(c && c->profiling) {
        if (on) {
            ev.cls = cls;
            on = hipEventCreate(&ev.start) == hipSuccess && hipEventCreate(&ev.stop) == hipSuccess;
            if (on) (void)hipEventRecord(ev.start, st);
        }
    }
    ~Prof() {
        if (on) {
            (void)hipEventRecord(ev.stop, st);
            ctx->events.push_back(ev);
        }
    }
};

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
inline size_t esize(int dtype) { return dtype == TIDAR_BF16 ? 2 : 4; }

struct Layout {
    size_t pos, rope_cs, x, x2, xn, gemm_out, gemm_out2, q, k_scr, v_scr, attn_part, o, h, xh, logits, logits_bytes,
        sel_logits, y, total;
    int attn_splits;
};

size_t gemm_out_floats(const tidar_config &c, int M, int N, int K) {
    if (c.dtype != TIDAR_BF16) return pt_split_stride(M, N);
    // the split count depends on the row-tile class of M (and, from 481 rows on, on the number of 256-row passes);
    // taking the maximum over the class boundaries below M keeps the size monotone in M and large enough for
    // every call with fewer rows (the passes of a prefill differ in length)
    size_t best = 0;
    auto consider = [&](int m) {
        m = m < M ? m : M;
        GemmPlan p = plan_gemm_bf16(m, N, K, false);
        size_t v = (size_t)p.splits * pt_split_stride(m, N);
        if (v > best) best = v;
    };
    const int bounds[5] = {16, 32, 80, 144, M};
    for (int i = 0; i < 5; ++i) consider(bounds[i]);
    for (int m = 512; m < M; m += 256) consider(m);      // the largest row count of each pass count
    return best;
}

// Workspace of one forward over B sequences of R rows (n_mask mask rows each), Mh rows through the LM head.
// n_mix: causal rows per sequence whose verification may mix two rows of logits (the decode step: k; else 0).
Layout make_layout(const tidar_config &c, int B, int R, int n_mask, int Mh, int max_keys, bool own_logits,
                   int n_mix = 0) {
    Layout l;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off += align_up(bytes);
        return o;
    };
    size_t es = esize(c.dtype);
    int M = B * R;
    int q_dim = c.n_q_heads * c.head_dim, kv_dim = c.n_kv_heads * c.head_dim;
    l.pos = take((size_t)M * 4);
    l.rope_cs = take((size_t)M * c.head_dim * 4);
    l.x = take((size_t)M * c.d_model * 4);
    // the fused chain of a few-row forward (see forward_rows) alternates between two residual buffers and two
    // partial-sum areas: a GEMM that folds its producer in reads one pair while it writes the other
    const bool fused_rows = c.dtype == TIDAR_BF16 && M <= kFuseMaxRows;
    l.x2 = take(fused_rows ? (size_t)M * c.d_model * 4 : 0);
    l.xn = take(af_elems(M, c.d_model) * es);
    size_t g = gemm_out_floats(c, M, q_dim + 2 * kv_dim, c.d_model);
    size_t g2 = gemm_out_floats(c, M, c.d_model, q_dim);
    size_t g3 = gemm_out_floats(c, M, 2 * c.d_ff, c.d_model);
    size_t g4 = gemm_out_floats(c, M, c.d_model, c.d_ff);
    g = g > g2 ? g : g2;
    g = g > g3 ? g : g3;
    g = g > g4 ? g : g4;
    l.gemm_out = take(g * 4);
    l.gemm_out2 = take(fused_rows ? g * 4 : 0);
    l.q = take((size_t)M * q_dim * es);
    int n_mt = (n_mask + 15) / 16;
    l.k_scr = take((size_t)B * c.n_kv_heads * (n_mt > 0 ? n_mt : 1) * 16 * c.head_dim * es);
    l.v_scr = take((size_t)B * c.n_kv_heads * (n_mt > 0 ? n_mt : 1) * 16 * c.head_dim * es);
    l.attn_splits = 1;
    size_t pf = 0;
    if (c.dtype == TIDAR_BF16) {
        AttnPlan ap = plan_attention(B, c.n_kv_heads, c.n_q_heads / c.n_kv_heads, R, R - n_mask, max_keys);
        l.attn_splits = ap.splits;
        pf = attn_partial_floats(B, c.n_kv_heads, c.n_q_heads / c.n_kv_heads, R, c.head_dim, ap.splits_bound);
    }
    l.attn_part = take(pf * 4);
    l.o = take(af_elems(M, q_dim) * es);
    l.h = take(af_elems(M, c.d_ff) * es);
    l.xh = take(af_elems(Mh > 0 ? Mh : 1, c.d_model) * es);
    l.logits_bytes = own_logits ? (size_t)(Mh > 0 ? Mh : 1) * c.vocab * 4 : 0;
    l.logits = take(l.logits_bytes);
    // beta-mixed verification through the fused reduction: logits of the k causal rows and their k mix partners only
    l.sel_logits = take(own_logits && c.dtype == TIDAR_BF16 ? (size_t)B * 2 * n_mix * c.vocab * 4 : 0);
    l.y = take((size_t)(Mh > 0 ? Mh : 1) * 4);
    l.total = off;
    return l;
}

bool shape_ok(const tidar_config &c) {
    if (c.n_layers < 1 || c.d_model < 1 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.head_dim < 2 || c.d_ff < 1 ||
        c.vocab < 2)
        return false;
    if (c.n_q_heads % c.n_kv_heads) return false;
    if (c.page_size != TIDAR_PAGE_SIZE) return false;
    if (c.max_k < 1 || c.max_k > TIDAR_MAX_K || c.max_batch < 1) return false;
    if (c.mask_token_id < 0 || c.mask_token_id >= c.vocab) return false;
    if (c.head_dim % 2 || c.head_dim > 128) return false;
    int q_dim = c.n_q_heads * c.head_dim, kv_dim = c.n_kv_heads * c.head_dim;
    if (q_dim % 16 || kv_dim % 16 || c.d_ff % 16 || c.d_model % 16 || c.vocab % 16) return false;
    if (c.dtype == TIDAR_BF16) {
        if (c.head_dim != 128) return false;
        if (c.d_model % 32 || c.d_ff % 32 || q_dim % 32) return false;
    } else if (c.dtype != TIDAR_F32) {
        return false;
    }
    if (!(c.rope_base > 1.f) || !(c.rms_eps >= 0.f)) return false;
    if ((int64_t)c.vocab * c.d_model * 2 > 0x7fff0000ll || (int64_t)c.d_ff * c.d_model * 4 > 0x7fff0000ll)
        return false;                          // buffer-load offsets are 32-bit
    return true;
}

bool mode_ok(const tidar_mode *m) {
    if (!m) return false;
    if (m->sample != 0 && m->sample != 1) return false;
    if (m->sample && !(m->temperature > 0.f)) return false;
    if (!(m->beta >= 0.f && m->beta <= 1.f)) return false;
    return true;
}

bool weights_ok(const tidar_weights *w) {
    return w && w->embed && w->lm_head && w->final_norm && w->attn_norm && w->wqkv && w->wo && w->ffn_norm &&
           w->w_gate_up && w->w_down;
}

// The kernels address a layer's pages with 32-bit byte offsets (raw buffer loads): a layer's K (or V) pages may
// not exceed 2 GiB, i.e. 65 535 pages of the 8B shape = one million tokens per layer buffer.
bool kv_ok(const tidar_config &c, const tidar_kv_cache *kv) {
    if (!(kv && kv->k_pages && kv->v_pages && kv->page_table && kv->pages_per_seq > 0 && kv->n_pages > 0))
        return false;
    return (int64_t)kv->n_pages * c.n_kv_heads * 16 * c.head_dim * (int64_t)esize(c.dtype) <= 0x7fffffe0ll;
}

KvView layer_view(const tidar_config &c, const tidar_kv_cache *kv, int layer) {
    KvView v;
    size_t per_layer = (size_t)kv->n_pages * c.n_kv_heads * 16 * c.head_dim * esize(c.dtype);
    v.k_pages = (char *)kv->k_pages + per_layer * layer;
    v.v_pages = (char *)kv->v_pages + per_layer * layer;
    v.page_table = kv->page_table;
    v.pages_per_seq = kv->pages_per_seq;
    v.n_pages = kv->n_pages;
    v.n_kv = c.n_kv_heads;
    v.hd = c.head_dim;
    return v;
}

// `head` selects the LM-head form: one split, plain row-major output (the logits the caller may ask for)
void gemm(tidar_ctx *ctx, const void *a, const void *w, float *out, int M, int N, int K, bool head, int *S,
          hipStream_t st) {
    Prof p(ctx, KC_GEMM, st);
    if (ctx->cfg.dtype == TIDAR_BF16) {
        GemmPlan gp = plan_gemm_bf16(M, N, K, head);
        *S = gp.splits;
        launch_gemm_bf16((const bf16_t *)a, (const bf16_t *)w, out, M, N, K, gp,
                         head ? GEMM_EPI_ROWMAJOR : GEMM_EPI_TILED, st);
    } else {
        *S = 1;
        launch_gemm_f32((const float *)a, (const float *)w, out, M, N, K, head ? 1 : 0, st);
    }
}

// Returns the number of key splits whose partial results wait in the workspace (1: o_out holds the result).  With
// defer_combine the partial results are left for the consumer to fold.
int attention(tidar_ctx *ctx, const Layout &l, char *ws, KvView kvv, const int32_t *prefix_len,
              RowDesc d, int B, int max_keys, void *o_out, hipStream_t st, bool defer_combine = false,
              const AttnRope *rope = nullptr) {
    const tidar_config &c = ctx->cfg;
    if (c.dtype == TIDAR_BF16) {
        AttnPlan ap = plan_attention(B, c.n_kv_heads, c.n_q_heads / c.n_kv_heads, d.R, d.nc, max_keys);
        {
            Prof p(ctx, KC_ATTN, st);
            launch_attention_bf16((const bf16_t *)(ws + l.q), kvv, (const bf16_t *)(ws + l.k_scr),
                                  (const bf16_t *)(ws + l.v_scr), prefix_len, d, B, c.n_q_heads, ap,
                                  (float *)(ws + l.attn_part), (bf16_t *)o_out, 1, st, rope);
        }
        if (ap.splits > 1 && !defer_combine) {
            Prof p(ctx, KC_ATTN_COMBINE, st);
            launch_attention_combine((const float *)(ws + l.attn_part), B, d.R, c.n_q_heads, c.n_kv_heads, c.head_dim,
                                     ap.splits, (bf16_t *)o_out, 1, st);
        }
        return ap.splits;
    }
    Prof p(ctx, KC_ATTN, st);
    launch_attention_f32((const float *)(ws + l.q), kvv, (const float *)(ws + l.k_scr),
                         (const float *)(ws + l.v_scr), prefix_len, d, B, c.n_q_heads, (float *)o_out, 1, st);
    return 1;
}

// What a scoring pass does with its logits instead of choosing tokens: rows cover text positions [c0, c0 + nc).
struct ScorePass {
    const int32_t *text;   // device, the sequence's tokens
    int len, c0;
    float *ar_out, *diff_out;
};

// One forward over B sequences with row structure d.  head_row0 < 0: no LM head.  Otherwise rows
// [head_row0, R) of every sequence go through the final norm, the LM head and the vocabulary reduction;
// the chosen tokens land in ws + layout.y.
void forward_rows(tidar_ctx *ctx, const tidar_weights *w, const tidar_kv_cache *kv, int B, RowDesc d,
                  const int32_t *tokens, int tok_stride, const int32_t *prefix_len, int max_keys, int head_row0,
                  int n_choose, const tidar_mode *mode, int mix_base, int mix_stride, float *logits_dst,
                  const Layout &l, char *ws, hipStream_t st, const ScorePass *score = nullptr) {
    const tidar_config &c = ctx->cfg;
    const int M = B * d.R;
    const int q_dim = c.n_q_heads * c.head_dim, kv_dim = c.n_kv_heads * c.head_dim;
    float *x = (float *)(ws + l.x);
    float *gout = (float *)(ws + l.gemm_out);
    {
        Prof p(ctx, KC_EMBED, st);
        launch_embed_rows(c.dtype, w->embed, tokens, tok_stride, prefix_len, d, B, c.d_model, c.mask_token_id,
                          c.vocab, layer_view(c, kv, 0), c.rope_base, x, (int32_t *)(ws + l.pos),
                          (float *)(ws + l.rope_cs), st);
    }
    int S_prev = 0;   // split count of the partial sums still waiting to be added to the residual stream
    // A forward of a few rows (the one-token step, very short blocks) is a chain of dependent launches whose kernels
    // are much shorter than the hand-over between them: there the RMSNorms and the split-KV combine are folded into
    // the GEMMs that consume them (6 launches per layer instead of 9; 5 for the one-token step, see below).
    const bool fuse = c.dtype == TIDAR_BF16 && gemm_fuse_ok(M, q_dim + 2 * kv_dim, c.d_model) &&
                      gemm_fuse_ok(M, c.d_model, q_dim) && gemm_fuse_ok(M, 2 * c.d_ff, c.d_model);
    float *x_alt = (float *)(ws + l.x2);
    float *g_cur = gout, *g_alt = (float *)(ws + l.gemm_out2);      // g_cur: where the pending partial sums are
    auto fused_norm_gemm = [&](const void *gain, const void *wmat, int N, float *dst, int epi, int *S_out) {
        Prof p(ctx, KC_GEMM, st);
        GemmPlan gp = plan_gemm_bf16(M, N, c.d_model, epi == GEMM_EPI_SWIGLU);
        FuseArgs f = {};
        f.kind = GEMM_FUSE_NORM;
        f.x_in = x;
        f.x_out = x_alt;
        f.part = g_cur;
        f.S = S_prev;
        f.split_stride = pt_split_stride(M, c.d_model);
        f.gain = (const bf16_t *)gain;
        f.eps = c.rms_eps;
        launch_gemm_bf16_fused(f, (const bf16_t *)wmat, dst, M, N, c.d_model, gp, epi, st);
        *S_out = gp.splits;
        float *t = x;          // the residual stream now lives in the other buffer
        x = x_alt;
        x_alt = t;
    };
    for (int layer = 0; layer < c.n_layers; ++layer) {
        KvView kvv = layer_view(c, kv, layer);
        int S = 1;
        if (fuse) {
            // reads (x, g_cur), writes the other residual buffer and the other partial-sum area
            fused_norm_gemm(w->attn_norm[layer], w->wqkv[layer], q_dim + 2 * kv_dim, g_alt, GEMM_EPI_TILED, &S);
            float *t = g_cur;
            g_cur = g_alt;
            g_alt = t;
        } else {
            {
                Prof p(ctx, KC_RMSNORM, st);
                launch_rmsnorm(c.dtype, x, g_cur, S_prev, w->attn_norm[layer], c.rms_eps, B, d.R, 0, c.d_model,
                               ws + l.xn, st);
            }
            gemm(ctx, ws + l.xn, w->wqkv[layer], g_cur, M, q_dim + 2 * kv_dim, c.d_model, false, &S, st);
        }
        // The one-token step has no RoPE launch either: its attention workgroups rotate the new row themselves
        AttnRope rope = {};
        if (fuse && attention_rope_ok(d, c.n_q_heads / c.n_kv_heads, c.head_dim)) {
            rope.part = g_cur;
            rope.S = S;
            rope.split_stride = pt_split_stride(M, q_dim + 2 * kv_dim);
            rope.rope_cs = (const float *)(ws + l.rope_cs);
            rope.M_all = M;
            rope.q_dim = q_dim;
            rope.kv_dim = kv_dim;
        } else {
            Prof p(ctx, KC_ROPE_KV, st);
            launch_rope_kv(c.dtype, g_cur, S, (const float *)(ws + l.rope_cs), prefix_len, d, B, c.n_q_heads, kvv,
                           ws + l.q, ws + l.k_scr, ws + l.v_scr, st);
        }
        const int a_splits = attention(ctx, l, ws, kvv, prefix_len, d, B, max_keys, ws + l.o, st, fuse,
                                       rope.part ? &rope : nullptr);
        if (fuse && a_splits > 1) {
            Prof p(ctx, KC_GEMM, st);
            GemmPlan gp = plan_gemm_bf16(M, c.d_model, q_dim, false);
            const size_t rows = (size_t)B * c.n_kv_heads * a_splits * (c.n_q_heads / c.n_kv_heads) * d.R;
            FuseArgs f = {};
            f.kind = GEMM_FUSE_COMBINE;
            f.opart = (const float *)(ws + l.attn_part);
            f.mpart = f.opart + rows * c.head_dim;
            f.lpart = f.mpart + rows;
            f.R = d.R;
            f.n_q = c.n_q_heads;
            f.n_kv = c.n_kv_heads;
            f.a_splits = a_splits;
            launch_gemm_bf16_fused(f, (const bf16_t *)w->wo[layer], g_cur, M, c.d_model, q_dim, gp, GEMM_EPI_TILED, st);
            S = gp.splits;
        } else {
            gemm(ctx, ws + l.o, w->wo[layer], g_cur, M, c.d_model, q_dim, false, &S, st);
        }
        S_prev = S;
        bool fused_swiglu = false;
        if (fuse) {
            // gate/up of a few rows always runs as one split, so SwiGLU lives in its epilogue
            fused_norm_gemm(w->ffn_norm[layer], w->w_gate_up[layer], 2 * c.d_ff, (float *)(ws + l.h), GEMM_EPI_SWIGLU,
                            &S);
            fused_swiglu = true;
        } else {
            {
                Prof p(ctx, KC_RMSNORM, st);
                launch_rmsnorm(c.dtype, x, g_cur, S, w->ffn_norm[layer], c.rms_eps, B, d.R, 0, c.d_model, ws + l.xn,
                               st);
            }
            if (c.dtype == TIDAR_BF16) {
                GemmPlan gp = plan_gemm_bf16(M, 2 * c.d_ff, c.d_model, false);
                if (gp.splits == 1 && gp.m_chunks >= 1) {       // nothing to reduce: SwiGLU can live in the epilogue
                    Prof p(ctx, KC_GEMM, st);
                    launch_gemm_bf16((const bf16_t *)(ws + l.xn), (const bf16_t *)w->w_gate_up[layer],
                                     (float *)(ws + l.h), M, 2 * c.d_ff, c.d_model, gp, GEMM_EPI_SWIGLU, st);
                    fused_swiglu = true;
                }
            }
        }
        if (!fused_swiglu) {
            gemm(ctx, ws + l.xn, w->w_gate_up[layer], g_cur, M, 2 * c.d_ff, c.d_model, false, &S, st);
            Prof p(ctx, KC_SWIGLU, st);
            launch_swiglu(c.dtype, g_cur, S, M, c.d_ff, ws + l.h, st);
        }
        gemm(ctx, ws + l.h, w->w_down[layer], g_cur, M, c.d_model, c.d_ff, false, &S, st);
        S_prev = S;
    }
    gout = g_cur;
    if (head_row0 < 0) return;
    const int Rh = d.R - head_row0;
    const int Mh = B * Rh;
    {
        Prof p(ctx, KC_RMSNORM, st);
        launch_rmsnorm(c.dtype, x, gout, S_prev, w->final_norm, c.rms_eps, B, d.R, head_row0, c.d_model, ws + l.xh, st);
    }
    float *logits = logits_dst ? logits_dst : (float *)(ws + l.logits);
    if (score) {               // one sequence; every row's label is scored, no token is chosen
        int S1 = 1;
        gemm(ctx, ws + l.xh, w->lm_head, logits, Mh, c.vocab, c.d_model, true, &S1, st);
        Prof p(ctx, KC_SCORE, st);
        launch_score_rows(logits, Mh, c.vocab, score->text, score->len, score->c0, d.nc, score->ar_out,
                          score->diff_out, st);
        return;
    }
    // Nobody asked for the logits: they are never written.  The LM head's epilogue forms, per row and column group,
    // the largest value and the lowest column that holds it; for the rows a token is sampled from it perturbs the
    // values first (same noise, same expression as the reduction over materialised logits).  Beta-mixed
    // verification needs two rows of logits side by side: the epilogue then also writes the logits of the k causal
    // rows and of their k mix partners (2k of the k(k+1) rows), which argmax_rows mixes, perturbs and reduces.
    // (The per-group pairs fit the logits area: 8 bytes per row and 32 or 64 columns.)
    if (c.dtype == TIDAR_BF16 && !logits_dst && l.logits_bytes > 0) {
        const int G = gemm_argmax_groups(Mh, c.vocab);
        const bool mix = mode->beta != 1.0f && n_choose > 0 && mix_stride > 0;
        ChooseArgs ch = {};
        ch.Rh = Rh;
        ch.n_choose = n_choose;
        ch.pos_rows = (const int32_t *)(ws + l.pos);
        ch.pos_stride = d.R;
        ch.pos_row0 = head_row0;
        ch.seq_base = d.seq_base;
        ch.sample = mix ? 0 : mode->sample;          // mixed rows are perturbed after the mix, by argmax_rows
        ch.inv_t = 1.f / mode->temperature;
        ch.seed = mode->seed;
        ch.sel_logits = mix ? (float *)(ws + l.sel_logits) : nullptr;
        ch.mix_stride = mix_stride;
        {
            Prof p(ctx, KC_GEMM, st);
            GemmPlan gp = plan_gemm_bf16(Mh, c.vocab, c.d_model, true);
            launch_gemm_bf16((const bf16_t *)(ws + l.xh), (const bf16_t *)w->lm_head, logits, Mh, c.vocab, c.d_model,
                             gp, GEMM_EPI_ARGMAX, st, &ch);
        }
        Prof p(ctx, KC_ARGMAX, st);
        launch_argmax_groups(logits, Mh, G, (int32_t *)(ws + l.y), st);
        if (mix)       // compact rows per sequence: causal row i at i, its partner at n_choose + i
            launch_argmax_rows(ch.sel_logits, B, 2 * n_choose, n_choose, c.vocab, n_choose, ch.pos_rows, d.R, head_row0,
                               d.seq_base, mode->sample, mode->temperature, mode->seed, mode->beta, n_choose, 1,
                               (int32_t *)(ws + l.y), Rh, st);
        return;
    }
    int S = 1;
    gemm(ctx, ws + l.xh, w->lm_head, logits, Mh, c.vocab, c.d_model, true, &S, st);
    {
        Prof p(ctx, KC_ARGMAX, st);
        launch_argmax_rows(logits, B, Rh, Rh, c.vocab, n_choose, (const int32_t *)(ws + l.pos), d.R, head_row0,
                           d.seq_base, mode->sample, mode->temperature, mode->seed, mode->beta, mix_base, mix_stride,
                           (int32_t *)(ws + l.y), Rh, st);
    }
}

RowDesc step_desc(int k) {
    RowDesc d;
    d.nc = k;
    d.nb = k;
    d.bl = k;
    d.cond0 = 1;
    d.cstride = 1;
    d.nm = k * k;
    d.R = k * (k + 1);
    d.seq_base = 0;
    return d;
}
RowDesc ar_desc() {
    RowDesc d;
    d.nc = 1;
    d.nb = 0;
    d.bl = 1;
    d.cond0 = 1;
    d.cstride = 1;
    d.nm = 0;
    d.R = 1;
    d.seq_base = 0;
    return d;
}
RowDesc prefill_desc(int nc, int k, bool last, int seq) {
    RowDesc d;
    d.nc = nc;
    d.nb = last ? 1 : 0;
    d.bl = k;
    d.cond0 = nc;
    d.cstride = 1;
    d.nm = last ? k : 0;
    d.R = nc + (last ? k : 0);
    d.seq_base = seq;
    return d;
}

// Scoring pass over text positions [c0, c0 + nc): the causal rows, and with block_len > 0 one mask row per
// position, in blocks that start at multiples of block_len (c0 is one) and see the text before them.
RowDesc score_desc(int nc, int block_len, int seq) {
    RowDesc d;
    d.nc = nc;
    d.bl = block_len > 0 ? block_len : 1;
    d.nb = block_len > 0 ? (nc + block_len - 1) / block_len : 0;
    d.cond0 = 0;
    d.cstride = d.bl;
    d.nm = block_len > 0 ? nc : 0;
    d.R = nc + d.nm;
    d.seq_base = seq;
    return d;
}

int score_chunk(const tidar_ctx *ctx, int block_len) {
    int chunk = ctx->prefill_chunk;
    if (block_len > 0) {
        chunk -= chunk % block_len;
        if (chunk < block_len) chunk = block_len;
    }
    return chunk;
}

size_t score_header_bytes(const tidar_config &c) { return align_up((size_t)c.max_batch * 4); }

}  // namespace

extern "C" {

const char *tidar_strerror(tidar_status s) {
    switch (s) {
        case TIDAR_OK: return "ok";
        case TIDAR_EINVAL: return "invalid argument";
        case TIDAR_ENOMEM: return "workspace too small (or, for tidar_gemm_static, the shape needs more than the static scratch)";
        case TIDAR_ECAPACITY: return "KV page table too short for prefix plus new rows";
        case TIDAR_EDEVICE: return "no gfx950 device or HIP error";
        case TIDAR_ESTATE: return "call order violated";
    }
    return "unknown status";
}

tidar_status tidar_create(const tidar_config *cfg, tidar_ctx **out) {
    if (!cfg || !out) return TIDAR_EINVAL;
    *out = nullptr;
    if (!shape_ok(*cfg)) return TIDAR_EINVAL;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) == hipSuccess && n_dev > 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return TIDAR_EDEVICE;
        if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return TIDAR_EDEVICE;
    } else {
        (void)hipGetLastError();
    }
    tidar_ctx *c = new (std::nothrow) tidar_ctx();
    if (!c) return TIDAR_ENOMEM;
    if (n_dev > 0) (void)scratch_address();     // set-up time is the place for the symbol lookup of this device
    c->cfg = *cfg;
    c->prefill_chunk = kDefaultPrefillChunk;
    c->profiling = false;
    for (int i = 0; i < KC_COUNT; ++i) {
        c->ms[i] = 0.0;
        c->launches[i] = 0;
    }
    *out = c;
    return TIDAR_OK;
}

void tidar_destroy(tidar_ctx *ctx) {
    if (!ctx) return;
    for (auto &e : ctx->events) {
        (void)hipEventDestroy(e.start);
        (void)hipEventDestroy(e.stop);
    }
    delete ctx;
}

size_t tidar_packed_weight_bytes(int32_t dtype, int32_t rows, int32_t cols) {
    if (rows <= 0 || cols <= 0) return 0;
    return (size_t)((rows + 31) / 32) * 32 * cols * esize(dtype);      // rows padded to the 32-row tile
}

tidar_status tidar_pack_weight(int32_t dtype, const void *src, int32_t rows, int32_t cols, void *dst,
                               int32_t dst_rows, int32_t dst_tile_offset, int32_t dst_tile_stride, void *stream) {
    if (!src || !dst || rows <= 0 || cols <= 0 || dst_rows <= 0) return TIDAR_EINVAL;
    if (dtype != TIDAR_F32 && dtype != TIDAR_BF16) return TIDAR_EINVAL;
    if (rows % 16 || dst_rows % 16 || dst_tile_offset < 0 || dst_tile_stride < 1) return TIDAR_EINVAL;
    if (dtype == TIDAR_BF16 && cols % 32) return TIDAR_EINVAL;
    int last_tile = dst_tile_offset + (rows / 16 - 1) * dst_tile_stride;
    if (last_tile >= dst_rows / 16) return TIDAR_EINVAL;
    launch_pack_weight(dtype, src, rows, cols, dst, dst_rows, dst_tile_offset, dst_tile_stride, (hipStream_t)stream);
    return TIDAR_OK;
}

tidar_status tidar_workspace_bytes(const tidar_ctx *ctx, int32_t batch, int32_t k, int32_t max_prefix_len,
                                   size_t *bytes) {
    if (!ctx || !bytes) return TIDAR_EINVAL;
    const tidar_config &c = ctx->cfg;
    if (batch < 1 || batch > c.max_batch || k < 1 || k > c.max_k || max_prefix_len < 0) return TIDAR_EINVAL;
    int R = k * (k + 1);
    Layout a = make_layout(c, batch, R, k * k, batch * R, max_prefix_len + R, true, k);
    Layout b = make_layout(c, batch, 1, 0, batch, max_prefix_len + 1, true);
    size_t t = a.total > b.total ? a.total : b.total;
    // prefill passes: a full causal chunk, or a last pass of 1..chunk causal rows plus the mask block
    Layout full = make_layout(c, 1, ctx->prefill_chunk, 0, 0, max_prefix_len + ctx->prefill_chunk, true);
    if (full.total > t) t = full.total;
    for (int nc = 1; nc <= ctx->prefill_chunk; ++nc) {
        Layout p = make_layout(c, 1, nc + k, k, 1 + k, max_prefix_len + k, true);
        if (p.total > t) t = p.total;
    }
    *bytes = t;
    return TIDAR_OK;
}

tidar_status tidar_step(tidar_ctx *ctx, const tidar_weights *w, const tidar_kv_cache *kv, int32_t batch,
                        int32_t *prefix_len, const int32_t *drafts, int32_t k, const tidar_mode *mode,
                        int32_t *accepted_len, int32_t *accepted_tokens, int32_t *next_drafts, float *logits_out,
                        int32_t max_prefix_len_hint, void *ws, size_t ws_bytes, void *stream) {
    if (!ctx || !weights_ok(w) || !kv_ok(ctx->cfg, kv) || !prefix_len || !drafts || !mode_ok(mode) || !accepted_len ||
        !accepted_tokens || !next_drafts || !ws)
        return TIDAR_EINVAL;
    const tidar_config &c = ctx->cfg;
    if (batch < 1 || batch > c.max_batch || k < 1 || k > c.max_k || max_prefix_len_hint < 0) return TIDAR_EINVAL;
    if ((int64_t)max_prefix_len_hint + k > (int64_t)kv->pages_per_seq * TIDAR_PAGE_SIZE) return TIDAR_ECAPACITY;
    RowDesc d = step_desc(k);
    Layout l = make_layout(c, batch, d.R, k * k, batch * d.R, max_prefix_len_hint + d.R, logits_out == nullptr, k);
    if (l.total > ws_bytes) return TIDAR_ENOMEM;
    hipStream_t st = (hipStream_t)stream;
    // causal row i is label shifted and judges draft i+1; with beta != 1 it is mixed with slot 0 of block i
    forward_rows(ctx, w, kv, batch, d, drafts, k, prefix_len, max_prefix_len_hint + d.R, 0, k, mode, k, k, logits_out,
                 l, (char *)ws, st);
    {
        Prof p(ctx, KC_VERIFY, st);
        launch_verify_step((const int32_t *)((char *)ws + l.y), drafts, k, batch, c.vocab, layer_view(c, kv, 0), 0,
                           prefix_len, accepted_len, accepted_tokens, next_drafts, st);
    }
    return TIDAR_OK;
}

tidar_status tidar_ar_step(tidar_ctx *ctx, const tidar_weights *w, const tidar_kv_cache *kv, int32_t batch,
                           int32_t *prefix_len, const int32_t *token_in, const tidar_mode *mode, int32_t *token_out,
                           float *logits_out, int32_t max_prefix_len_hint, void *ws, size_t ws_bytes, void *stream) {
    if (!ctx || !weights_ok(w) || !kv_ok(ctx->cfg, kv) || !prefix_len || !token_in || !mode_ok(mode) || !token_out || !ws)
        return TIDAR_EINVAL;
    const tidar_config &c = ctx->cfg;
    if (batch < 1 || batch > c.max_batch || max_prefix_len_hint < 0) return TIDAR_EINVAL;
    if ((int64_t)max_prefix_len_hint + 1 > (int64_t)kv->pages_per_seq * TIDAR_PAGE_SIZE) return TIDAR_ECAPACITY;
    RowDesc d = ar_desc();
    Layout l = make_layout(c, batch, 1, 0, batch, max_prefix_len_hint + 1, logits_out == nullptr);
    if (l.total > ws_bytes) return TIDAR_ENOMEM;
    hipStream_t st = (hipStream_t)stream;
    tidar_mode m = *mode;
    m.beta = 1.f;                 // a one-token step has no diffusion row to mix with
    forward_rows(ctx, w, kv, batch, d, token_in, 1, prefix_len, max_prefix_len_hint + 1, 0, 1, &m, 0, 0, logits_out,
                 l, (char *)ws, st);
    {
        Prof p(ctx, KC_VERIFY, st);
        launch_finish_ar((const int32_t *)((char *)ws + l.y), token_in, batch, c.vocab, layer_view(c, kv, 0),
                         prefix_len, token_out, st);
    }
    return TIDAR_OK;
}

tidar_status tidar_prefill(tidar_ctx *ctx, const tidar_weights *w, const tidar_kv_cache *kv, int32_t batch,
                           const int32_t *prompt, int32_t prompt_stride, const int32_t *prompt_len, int32_t k,
                           const tidar_mode *mode, int32_t *prefix_len, int32_t *first_drafts, float *logits_out,
                           void *ws, size_t ws_bytes, void *stream) {
    if (!ctx || !weights_ok(w) || !kv_ok(ctx->cfg, kv) || !prompt || !prompt_len || !mode_ok(mode) || !prefix_len ||
        !first_drafts || !ws)
        return TIDAR_EINVAL;
    const tidar_config &c = ctx->cfg;
    if (batch < 1 || batch > c.max_batch || k < 1 || k > c.max_k || prompt_stride < 1) return TIDAR_EINVAL;
    int max_len = 0;
    for (int b = 0; b < batch; ++b) {
        if (prompt_len[b] < 1 || prompt_len[b] > prompt_stride) return TIDAR_EINVAL;
        if ((int64_t)prompt_len[b] + k > (int64_t)kv->pages_per_seq * TIDAR_PAGE_SIZE) return TIDAR_ECAPACITY;
        if (prompt_len[b] > max_len) max_len = prompt_len[b];
    }
    for (int b = 0; b < batch; ++b) {      // size every pass before anything is enqueued
        const int P = prompt_len[b];
        for (int c0 = 0; c0 < P; c0 += ctx->prefill_chunk) {
            const int nc = (P - c0 < ctx->prefill_chunk) ? P - c0 : ctx->prefill_chunk;
            const bool last = c0 + nc >= P;
            Layout l = make_layout(c, 1, nc + (last ? k : 0), last ? k : 0, last ? 1 + k : 0,
                                   c0 + nc + (last ? k : 0), true);
            if (l.total > ws_bytes) return TIDAR_ENOMEM;
        }
    }
    hipStream_t st = (hipStream_t)stream;
    tidar_mode pm = *mode;
    pm.beta = 1.f;                // the first token comes from the causal logits alone
    launch_set_i32(prefix_len, batch, 0, st);
    for (int b = 0; b < batch; ++b) {
        const int P = prompt_len[b];
        for (int c0 = 0; c0 < P; c0 += ctx->prefill_chunk) {
            const int nc = (P - c0 < ctx->prefill_chunk) ? P - c0 : ctx->prefill_chunk;
            const bool last = c0 + nc >= P;
            RowDesc d = prefill_desc(nc, k, last, b);
            Layout l = make_layout(c, 1, d.R, last ? k : 0, last ? 1 + k : 0, c0 + d.R, true);
            float *lg = (last && logits_out) ? logits_out + (size_t)b * (1 + k) * c.vocab : nullptr;
            // the last pass sends the final prompt row and the k mask rows through the LM head
            forward_rows(ctx, w, kv, 1, d, prompt + (size_t)b * prompt_stride + c0, prompt_stride, prefix_len,
                         c0 + d.R, last ? nc - 1 : -1, 1, &pm, 1, 0, lg, l, (char *)ws, st);
            {
                Prof p(ctx, KC_VERIFY, st);
                launch_finish_prefill((const int32_t *)((char *)ws + l.y), prompt + (size_t)b * prompt_stride + c0, k,
                                      b, nc, last ? 1 : 0, c.vocab, layer_view(c, kv, 0), prefix_len, first_drafts,
                                      st);
            }
        }
    }
    return TIDAR_OK;
}

tidar_status tidar_score_workspace_bytes(const tidar_ctx *ctx, int32_t max_len, int32_t block_len, size_t *bytes) {
    if (!ctx || !bytes || max_len < 1 || block_len < 0 || block_len > TIDAR_MAX_K) return TIDAR_EINVAL;
    const tidar_config &c = ctx->cfg;
    const int chunk = score_chunk(ctx, block_len);
    size_t t = 0;
    // the workspace grows with the key bound for a given pass shape, and no pass ends beyond max_len
    for (int nc = 1; nc <= chunk && nc <= max_len; ++nc) {
        RowDesc d = score_desc(nc, block_len, 0);
        Layout l = make_layout(c, 1, d.R, d.nm, d.R, max_len + d.nm, true);
        if (l.total > t) t = l.total;
    }
    *bytes = score_header_bytes(c) + t;
    return TIDAR_OK;
}

tidar_status tidar_score(tidar_ctx *ctx, const tidar_weights *w, const tidar_kv_cache *kv, int32_t batch,
                         const int32_t *tokens, int32_t stride, const int32_t *len, int32_t block_len, float alpha,
                         float *ar_logprob, float *diff_logprob, float *loss, void *ws, size_t ws_bytes,
                         void *stream) {
    if (!ctx || !weights_ok(w) || !kv_ok(ctx->cfg, kv) || !tokens || !len || !ar_logprob || !ws) return TIDAR_EINVAL;
    const tidar_config &c = ctx->cfg;
    if (batch < 1 || batch > c.max_batch || stride < 1 || block_len < 0 || block_len > TIDAR_MAX_K)
        return TIDAR_EINVAL;
    if ((block_len > 0) != (diff_logprob != nullptr)) return TIDAR_EINVAL;
    if (!(alpha >= 0.f && alpha <= 1.f)) return TIDAR_EINVAL;
    const int chunk = score_chunk(ctx, block_len);
    const size_t hdr = score_header_bytes(c);
    for (int b = 0; b < batch; ++b) {      // size every pass before anything is enqueued
        if (len[b] < 1 || len[b] > stride) return TIDAR_EINVAL;
        if ((int64_t)len[b] > (int64_t)kv->pages_per_seq * TIDAR_PAGE_SIZE) return TIDAR_ECAPACITY;
        for (int c0 = 0; c0 < len[b]; c0 += chunk) {
            RowDesc d = score_desc(len[b] - c0 < chunk ? len[b] - c0 : chunk, block_len, b);
            Layout l = make_layout(c, 1, d.R, d.nm, d.R, c0 + d.R, true);
            if (hdr + l.total > ws_bytes) return TIDAR_ENOMEM;
        }
    }
    hipStream_t st = (hipStream_t)stream;
    int32_t *cur = (int32_t *)ws;          // the passes' own prefix lengths, one entry per sequence
    char *wsb = (char *)ws + hdr;
    tidar_mode gm;
    gm.sample = 0;
    gm.temperature = 1.f;
    gm.seed = 0;
    gm.beta = 1.f;
    for (int b = 0; b < batch; ++b) {
        const int32_t *text = tokens + (size_t)b * stride;
        for (int c0 = 0; c0 < len[b]; c0 += chunk) {
            RowDesc d = score_desc(len[b] - c0 < chunk ? len[b] - c0 : chunk, block_len, b);
            Layout l = make_layout(c, 1, d.R, d.nm, d.R, c0 + d.R, true);
            launch_set_i32(cur + b, 1, c0, st);
            ScorePass sp;
            sp.text = text;
            sp.len = len[b];
            sp.c0 = c0;
            sp.ar_out = ar_logprob + (size_t)b * stride;
            sp.diff_out = diff_logprob ? diff_logprob + (size_t)b * stride : nullptr;
            forward_rows(ctx, w, kv, 1, d, text + c0, stride, cur, c0 + d.R, 0, 0, &gm, 0, 0, nullptr, l, wsb, st, &sp);
        }
        if (loss) {
            Prof p(ctx, KC_SCORE, st);
            launch_score_loss(ar_logprob + (size_t)b * stride, diff_logprob ? diff_logprob + (size_t)b * stride : nullptr,
                              len[b] - 1, alpha, loss + b, st);
        }
    }
    return TIDAR_OK;
}

tidar_status tidar_hybrid_attention(tidar_ctx *ctx, const tidar_kv_cache *kv, int32_t layer, int32_t batch,
                                    const int32_t *prefix_len, const void *q, const void *k_new, const void *v_new,
                                    int32_t n_causal, int32_t n_blocks, int32_t block_len, int32_t cond0, void *out,
                                    int32_t max_prefix_len_hint, void *ws, size_t ws_bytes, void *stream) {
    if (!ctx || !kv_ok(ctx->cfg, kv) || !prefix_len || !q || !k_new || !v_new || !out || !ws) return TIDAR_EINVAL;
    const tidar_config &c = ctx->cfg;
    if (layer < 0 || layer >= c.n_layers || batch < 1 || batch > c.max_batch) return TIDAR_EINVAL;
    if (n_causal < 1 || n_blocks < 0 || block_len < 1 || block_len > TIDAR_MAX_K || cond0 < 0 ||
        max_prefix_len_hint < 0)
        return TIDAR_EINVAL;
    if (n_blocks > 0 && cond0 + n_blocks - 1 > n_causal) return TIDAR_EINVAL;
    if ((int64_t)max_prefix_len_hint + n_causal > (int64_t)kv->pages_per_seq * TIDAR_PAGE_SIZE)
        return TIDAR_ECAPACITY;
    RowDesc d;
    d.nc = n_causal;
    d.nb = n_blocks;
    d.bl = block_len;
    d.cond0 = cond0;
    d.cstride = 1;
    d.nm = n_blocks * block_len;
    d.R = n_causal + n_blocks * block_len;
    d.seq_base = 0;
    size_t es = esize(c.dtype);
    int n_mask = n_blocks * block_len;
    int n_mt = (n_mask + 15) / 16;
    if (n_mt < 1) n_mt = 1;
    size_t scr = align_up((size_t)batch * c.n_kv_heads * n_mt * 16 * c.head_dim * es);
    int max_keys = max_prefix_len_hint + d.R;
    AttnPlan ap = plan_attention(batch, c.n_kv_heads, c.n_q_heads / c.n_kv_heads, d.R, d.nc, max_keys);
    size_t pf = c.dtype == TIDAR_BF16
                    ? attn_partial_floats(batch, c.n_kv_heads, c.n_q_heads / c.n_kv_heads, d.R, c.head_dim,
                                          ap.splits_bound)
                    : 0;
    if (2 * scr + align_up(pf * 4) > ws_bytes) return TIDAR_ENOMEM;
    char *wsb = (char *)ws;
    hipStream_t st = (hipStream_t)stream;
    KvView kvv = layer_view(c, kv, layer);
    {
        Prof p(ctx, KC_PLACE_KV, st);
        launch_place_kv(c.dtype, k_new, v_new, prefix_len, d, batch, kvv, wsb, wsb + scr, st);
    }
    if (c.dtype == TIDAR_BF16) {
        {
            Prof p(ctx, KC_ATTN, st);
            launch_attention_bf16((const bf16_t *)q, kvv, (const bf16_t *)wsb,
                                  (const bf16_t *)(wsb + scr), prefix_len, d, batch, c.n_q_heads, ap,
                                  (float *)(wsb + 2 * scr), (bf16_t *)out, 0, st);
        }
        if (ap.splits == 1) return TIDAR_OK;
        Prof p(ctx, KC_ATTN_COMBINE, st);
        launch_attention_combine((const float *)(wsb + 2 * scr), batch, d.R, c.n_q_heads, c.n_kv_heads, c.head_dim,
                                 ap.splits, (bf16_t *)out, 0, st);
    } else {
        Prof p(ctx, KC_ATTN, st);
        launch_attention_f32((const float *)q, kvv, (const float *)wsb, (const float *)(wsb + scr), prefix_len, d,
                             batch, c.n_q_heads, (float *)out, 0, st);
    }
    return TIDAR_OK;
}

size_t tidar_gemm_workspace_bytes(int32_t dtype, int32_t M, int32_t N, int32_t K) {
    if (M < 1 || N < 16 || K < 8) return 256;
    int splits = dtype == TIDAR_BF16 ? plan_gemm_bf16(M, N, K, false).splits : 1;
    return align_up(af_elems(M, K) * esize(dtype)) + align_up((size_t)splits * pt_split_stride(M, N) * 4);
}

tidar_status tidar_gemm(tidar_ctx *ctx, const void *a, const void *w_packed, float *out, int32_t M, int32_t N,
                        int32_t K, void *ws, size_t ws_bytes, void *stream) {
    if (!ctx || !a || !w_packed || !out || !ws || M < 1 || N < 1 || K < 1) return TIDAR_EINVAL;
    if (N % 16 || K % 8) return TIDAR_EINVAL;
    const int dtype = ctx->cfg.dtype;
    if (dtype == TIDAR_BF16 && K % 32) return TIDAR_EINVAL;
    if (ws_bytes < tidar_gemm_workspace_bytes(dtype, M, N, K)) return TIDAR_ENOMEM;
    hipStream_t st = (hipStream_t)stream;
    char *a_frag = (char *)ws;
    float *part = (float *)((char *)ws + align_up(af_elems(M, K) * esize(dtype)));
    launch_pack_act(dtype, a, M, K, a_frag, st);       // the step's producers write this layout directly
    int S = 1;
    gemm(ctx, a_frag, w_packed, part, M, N, K, false, &S, st);
    launch_untile_sum(part, S, M, N, out, st);
    return TIDAR_OK;
}

tidar_status tidar_gemm_static(tidar_ctx *ctx, const void *a, const void *w_packed, float *out, int32_t M, int32_t N,
                               int32_t K, void *stream) {
    if (!ctx || !a || !w_packed || !out || M < 1 || N < 1 || K < 1) return TIDAR_EINVAL;
    if (N % 16 || K % 8) return TIDAR_EINVAL;
    const int dtype = ctx->cfg.dtype;
    if (dtype == TIDAR_BF16 && K % 32) return TIDAR_EINVAL;
    if (tidar_gemm_workspace_bytes(dtype, M, N, K) > (size_t)TIDAR_STATIC_SCRATCH_BYTES) return TIDAR_ENOMEM;
    char *base = (char *)scratch_address();     // first call on this device: one symbol lookup, no allocation
    if (!base) return TIDAR_EDEVICE;
    hipStream_t st = (hipStream_t)stream;
    float *part = (float *)(base + align_up(af_elems(M, K) * esize(dtype)));
    // Nothing in the scratch has to start at zero: pack_act writes every A element of the M real rows, the pad
    // rows of the last row tile only feed output rows that are never stored, and untile_sum reads exactly the
    // partial sums this call's GEMM wrote.  What an earlier, larger call left behind is never read as data.
    launch_pack_act(dtype, a, M, K, base, st);
    if (dtype == TIDAR_BF16) {
        GemmPlan gp = plan_gemm_bf16(M, N, K, false);
        launch_gemm_bf16((const bf16_t *)base, (const bf16_t *)w_packed, part, M, N, K, gp, GEMM_EPI_TILED, st);
        launch_untile_sum(part, gp.splits, M, N, out, st);
    } else {
        launch_gemm_f32((const float *)base, (const float *)w_packed, part, M, N, K, 0, st);
        launch_untile_sum(part, 1, M, N, out, st);
    }
    return TIDAR_OK;
}

tidar_status tidar_set_prefill_chunk(tidar_ctx *ctx, int32_t rows) {
    if (!ctx || rows < 1 || rows > kMaxPrefillChunk) return TIDAR_EINVAL;
    ctx->prefill_chunk = rows;
    return TIDAR_OK;
}

int32_t tidar_select_block_len(const tidar_ctx *ctx, int32_t batch, int32_t k_cap, int32_t row_budget) {
    if (!ctx || batch < 1) return 0;
    const int budget = row_budget > 0 ? row_budget : 160;
    int cap = ctx->cfg.max_k;
    if (k_cap > 0 && k_cap < cap) cap = k_cap;
    int best = 1;
    for (int k = 2; k <= 16 && k <= cap; k *= 2)
        if ((int64_t)batch * k * (k + 1) <= budget) best = k;
    return best;
}

tidar_status tidar_profile_enable(tidar_ctx *ctx, int32_t on) {
    if (!ctx) return TIDAR_EINVAL;
    ctx->profiling = on != 0;
    return TIDAR_OK;
}

static void drain_events(tidar_ctx *ctx) {
    for (auto &e : ctx->events) {
        float ms = 0.f;
        if (hipEventSynchronize(e.stop) == hipSuccess && hipEventElapsedTime(&ms, e.start, e.stop) == hipSuccess) {
            ctx->ms[e.cls] += ms;
            ctx->launches[e.cls] += 1;
        }
        (void)hipEventDestroy(e.start);
        (void)hipEventDestroy(e.stop);
    }
    ctx->events.clear();
}

int32_t tidar_profile_read(tidar_ctx *ctx, const char **names, double *ms, int64_t *launches, int32_t cap) {
    if (!ctx) return 0;
    drain_events(ctx);
    int n = 0;
    for (int i = 0; i < KC_COUNT; ++i) {
        if (ctx->launches[i] == 0) continue;
        if (n < cap) {
            if (names) names[n] = kClassNames[i];
            if (ms) ms[n] = ctx->ms[i];
            if (launches) launches[n] = ctx->launches[i];
        }
        ++n;
    }
    return n;
}

tidar_status tidar_profile_reset(tidar_ctx *ctx) {
    if (!ctx) return TIDAR_EINVAL;
    drain_events(ctx);
    for (int i = 0; i < KC_COUNT; ++i) {
        ctx->ms[i] = 0.0;
        ctx->launches[i] = 0;
    }
    return TIDAR_OK;
}

}  // extern "C"
