// C ABI layer: argument validation, workspace, the forward pass wiring, the
// step (forward + selector) and the host-side stage controller of Algorithm 1.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <string>
#include <vector>

#include "internal.h"

using namespace dllm;

namespace {

thread_local std::string g_err;

struct Workspace {
    float *x = nullptr;          // residual stream fp32 [M][d]
    uint16_t *h = nullptr;       // normalised activations bf16 [M][d]
    uint16_t *qkv = nullptr;     // [M][3d]
    uint16_t *att = nullptr;     // [M][d]
    uint16_t *act = nullptr;     // [M][f]
    float *partials = nullptr;   // split-K slabs fp32 [splits][rows][d], partials_cap floats
    size_t partials_cap = 0;
    float *ssq = nullptr;        // per row, partial sums of squares of the residual stream: [M][ssq_stride]
    int ssq_stride = 0;
    int32_t *tickets = nullptr;  // one counter per output tile of a split-K residual product, zero between launches
    int n_tickets = 0;
    uint16_t *logits = nullptr;  // [M][V]
    float *rowstats = nullptr;   // [3][gemm_rowstats_max_parts(V)][M]: per-slice (max, sum of exp, argmax) of the fused selector
    int32_t *pred = nullptr;     // [M]
    float *conf = nullptr;       // [M]
    float2 *rope = nullptr;      // [max_seq][dh/2]
    // decode-only state
    int32_t *prev_pred = nullptr;  // [M]
    int32_t *cl_ints = nullptr;    // n_commit, e_cand, first_masked, n_masked_after: 4 x [max_batch], then bad_token
    int32_t *bad_token = nullptr;  // = cl_ints + 4 * max_batch: set by the embedding kernel on an id outside [0, vocab)
    int32_t *cl_pos = nullptr, *cl_tok = nullptr;
    float *cl_conf = nullptr;      // [max_batch][max_seq]
    // pinned host memory: mask [M] | step results [4 * max_batch + 1] | confidences [M] | 2 x (rows [M], pos [M])
    uint8_t *host_pinned = nullptr;
    int32_t *host_ints = nullptr;
    float *host_conf = nullptr;
    int32_t *host_rows[2] = {nullptr, nullptr};  // row / position lists of cached steps, double-buffered
    hipEvent_t rows_copied[2] = {nullptr, nullptr};
    int rows_slot = 0;
    // out-of-span caching: per-layer qkv rows of every position (k and v thirds are the cached features)
    std::vector<uint16_t *> kv_cache;
    int32_t *rows_d = nullptr, *pos_d = nullptr;  // recomputed rows of a step and their positions, [M]
    bool cache_valid = false;
    int cache_B = 0, cache_L = 0;  // batch shape the cache rows belong to
};

}  // namespace

struct dllm_handle {
    dllm_config cfg;
    hipStream_t stream;
    const void *embed, *lm_head, *final_norm;
    std::vector<const void *> attn_norm, wqkv, wo, ffn_norm, w_gate_up, w_down;
    // panel-major copies of the projection weights (see GemmLayout), made at create; null where the reduction
    // length is not a multiple of 64 (those products run on the register-staged kernel from the caller's rows)
    const void *lm_head_p = nullptr;
    std::vector<const void *> wqkv_p, wo_p, w_gate_up_p, w_down_p;
    bool packed_d = false, packed_f = false;  // weights with K = d_model / K = d_ffn have panel-major copies
    Workspace ws;
    std::vector<void *> allocs;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    std::string err;
    int last_B = 0, last_L = 0;
    bool fused_selector = true;  // dllm_set_fused_selector
    bool fused_norm = true;      // RMSNorm folded into the projections (off: environment DLLM_NO_FUSED_NORM at create)
    bool fused_splitk = false;   // also where the O / down projection runs K splits (environment DLLM_FUSED_SPLITK)
    // measurement hook: event pairs around the gate/up GEMM launches
    std::vector<hipEvent_t> prof_ev;
    int prof_cap = 0, prof_used = 0;
    bool prof_on = false;
};

namespace {

int fail(dllm_handle *h, int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (h) h->err = buf; else g_err = buf;
    return code;
}

#define HIP_TRY(h, call)                                                                          \
    do {                                                                                          \
        hipError_t e_ = (call);                                                                   \
        if (e_ != hipSuccess) return fail(h, DLLM_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <class T>
int dev_alloc(dllm_handle *h, T **p, size_t count)
{
    void *q = nullptr;
    if (hipMalloc(&q, count * sizeof(T) + 256) != hipSuccess) {
        (void)hipGetLastError();
        return fail(h, DLLM_ENOMEM, "device allocation of %zu bytes failed", count * sizeof(T));
    }
    h->allocs.push_back(q);
    *p = static_cast<T *>(q);
    return DLLM_OK;
}

// How many fp32 split-K slabs of `rows` rows the slab workspace holds (0: not even one).  The planner
// is given this as its limit, so every row count up to max_batch * max_seq gets a plan that fits.
int slab_limit(const dllm_handle *h, int rows)
{
    const size_t n = h->ws.partials_cap / ((size_t)rows * h->cfg.d_model);
    return n > (size_t)kGemmMaxSplits ? kGemmMaxSplits : (int)n;
}

// The bf16 logits [max_batch * max_seq][vocab] are by far the largest buffer and only dllm_forward and
// steps with the fused selector off need them: allocated on first use.
int ensure_logits(dllm_handle *h)
{
    if (h->ws.logits) return DLLM_OK;
    const size_t M = (size_t)h->cfg.max_batch * h->cfg.max_seq;
    return dev_alloc(h, &h->ws.logits, M * (size_t)h->cfg.vocab);
}

// Checks the per-sequence parameters and turns them into kernel windows.
int build_select_args(dllm_handle *h, int B, int L, const dllm_stage_params *sp, int capacity, SelectArgs *out,
                      const int32_t *cache_mode = nullptr)
{
    if (B < 1 || B > DLLM_MAX_BATCH) return fail(h, DLLM_EINVAL, "batch %d outside [1, %d]", B, DLLM_MAX_BATCH);
    if (L < 1 || L > 8192) return fail(h, DLLM_EINVAL, "sequence length %d outside [1, 8192]", L);
    int longest = 0;
    for (int b = 0; b < B; ++b) {
        const dllm_stage_params &p = sp[b];
        SeqWindow &w = out->w[b];
        w.stage = p.stage; w.top_k = p.top_k; w.tau_min = p.tau_min_conf; w.tau_high = p.tau_high_conf;
        w.conv_mode = p.conv_mode;
        const int cm = cache_mode ? cache_mode[b] : DLLM_CACHE_OFF;
        if (cm != DLLM_CACHE_OFF && cm != DLLM_CACHE_REFRESH && cm != DLLM_CACHE_REUSE)
            return fail(h, DLLM_EINVAL, "sequence %d: unknown cache mode %d", b, cm);
        if (p.stage == DLLM_STAGE_IDLE) { w.lo = 0; w.hi = -1; w.eval_hi = -1; continue; }

        if (p.stage != DLLM_STAGE_SLOW && p.stage != DLLM_STAGE_FAST)
            return fail(h, DLLM_EINVAL, "sequence %d: unknown stage %d", b, p.stage);
        if (p.gen_start < 0 || p.gen_end > L || p.gen_start > p.gen_end)
            return fail(h, DLLM_EINVAL, "sequence %d: generated region [%d, %d) outside [0, %d]", b, p.gen_start,
                        p.gen_end, L);
        if (p.top_k < 1) return fail(h, DLLM_EINVAL, "sequence %d: top_k %d < 1", b, p.top_k);
        if (p.conv_mode != 0 && p.conv_mode != 1)
            return fail(h, DLLM_EINVAL, "sequence %d: conv_mode %d is not 0 or 1", b, p.conv_mode);
        w.lo = p.s_cycle;
        w.hi = p.stage == DLLM_STAGE_SLOW ? p.gen_end - 1 : p.e_cycle;
        // a refresh step of the fast stage also rates what lies right of the span
        w.eval_hi = (cm == DLLM_CACHE_REFRESH && p.stage == DLLM_STAGE_FAST) ? p.gen_end - 1 : w.hi;
        if (p.stage == DLLM_STAGE_FAST && p.e_cycle < p.s_cycle)
            return fail(h, DLLM_EINVAL, "sequence %d: fast stage with e_cycle %d < s_cycle %d", b, p.e_cycle,
                        p.s_cycle);
        if (w.lo < p.gen_start || w.hi >= p.gen_end)
            return fail(h, DLLM_EINVAL, "sequence %d: window [%d, %d] outside the generated region [%d, %d)", b, w.lo,
                        w.hi, p.gen_start, p.gen_end);
        if (w.eval_hi < w.hi) w.eval_hi = w.hi;
        if (w.hi - w.lo + 1 > longest) longest = w.hi - w.lo + 1;
    }
    if (capacity < longest)
        return fail(h, DLLM_ECAPACITY, "commit list capacity %d below the longest window %d", capacity, longest);
    return DLLM_OK;
}

int check_commit_list(dllm_handle *h, const dllm_commit_list *o, CommitOut *c)
{
    if (!o) return fail(h, DLLM_EINVAL, "commit list is null");
    if (!o->n_commit || !o->pos || !o->tok || !o->conf || !o->e_cand || !o->first_masked || !o->n_masked_after)
        return fail(h, DLLM_EINVAL, "commit list has a null member");
    if (o->capacity < 0) return fail(h, DLLM_EINVAL, "commit list capacity %d < 0", o->capacity);
    *c = CommitOut{o->capacity, o->n_commit, o->pos, o->tok, o->conf, o->e_cand, o->first_masked, o->n_masked_after};
    return DLLM_OK;
}

// Vocabulary projection over n consecutive rows of the normalised hidden states, starting at row
// h_row of ws.h; abs_row is the batch row (b * L + i) of the first of them.  With the fused selector
// and a mask, the projection leaves per-slice row statistics instead of logits and the merge
// kernel turns them into ws.pred / ws.conf at the masked rows of the windows.
// h_panel_rows: 0, or the rows per panel of a panel-major ws.h.
int vocab_rows(dllm_handle *h, long h_row, long abs_row, int n, int L, const uint8_t *mask, const SelectArgs *win,
               int h_panel_rows, RowScale scale)
{
    if (scale.ssq) scale.ssq += h_row * scale.stride;
    const dllm_config &c = h->cfg;
    Workspace &w = h->ws;
    // the first of the n rows: 64 bytes per row inside panel 0, or d_model elements per row
    const uint16_t *A = h_panel_rows ? w.h + h_row * 32 : w.h + h_row * c.d_model;
    const void *W = h_panel_rows ? h->lm_head_p : h->lm_head;
    const GemmLayout lay{h_panel_rows, h_panel_rows ? c.vocab : 0, 0};
    if (h->fused_selector && mask && win) {
        int parts = 0;
        HIP_TRY(h, launch_gemm_rowstats(h->stream, A, W, w.rowstats, n, c.vocab, c.d_model, c.mask_id, &parts, lay, scale));
        HIP_TRY(h, launch_rowstats_merge(h->stream, w.rowstats, parts, n, (int)abs_row, L, mask, *win, w.pred, w.conf));
    } else {
        if (int rc = ensure_logits(h)) return rc;
        HIP_TRY(h, launch_gemm(h->stream, kEpiBf16, A, W, w.logits + abs_row * (long)c.vocab, n, c.vocab, c.d_model,
                               kGemmMaxSplits, lay, scale));
    }
    return DLLM_OK;
}

// Which activations of a forward over `rows` rows are kept panel-major: those that feed products with
// reduction length d_model (normalised hidden states, attention output) and d_ffn (SwiGLU output), each only
// if the handle has panel-major weights for them and every such product runs on the asynchronous-copy kernel.
struct PanelChoice {
    int d_rows, f_rows;  // rows per panel, 0 = row-major
};
PanelChoice pick_panels(const dllm_handle *h, int rows)
{
    const dllm_config &c = h->cfg;
    const int d = c.d_model, f = c.d_ffn;
    const int qkv_epi = gemm_qkv_rope_supported(rows, d, c.head_dim) ? (c.head_dim == 128 ? 4 : 3) : (int)kEpiBf16;
    const bool pd = h->packed_d && gemm_async_copy_path(qkv_epi, rows, 3 * d, d) &&
                    gemm_async_copy_path(kEpiPartial, rows, d, d) && gemm_async_copy_path(kEpiSwiglu, rows, 2 * f, d) &&
                    gemm_async_copy_path(kEpiBf16, rows, c.vocab, d) && gemm_async_copy_path(5, rows, c.vocab, d);
    const bool pf = h->packed_f && gemm_async_copy_path(kEpiPartial, rows, d, f);
    return PanelChoice{pd ? rows : 0, pf ? rows : 0};
}

// Embedding, all layers and the final norm over `rows` rows (all B * L of them, or the gathered subset of a
// cached step), leaving in ws.h what the vocabulary projection multiplies.
//   rows_d / pos_d (device, nullable): batch row and position of every row of a gathered subset
//   kv_rows (nullable): cached step: queries of sequence b are rows [first, first + count) and attend to the
//                       layer's key/value cache; to_cache: the QKV projection writes straight into the cache
// The RMSNorm in front of a projection is applied in one of two ways, chosen per product.  Folded: whoever
// produced the residual stream left bf16(x * gain) and per-row partial sums of squares, and the projection
// scales its output rows (*scale / sc say how).  Separate: ws.h holds normalised rows and sc is empty.
// The embedding kernel always leaves the folded form.  An O or down projection that the planner runs
// without K splits adds the residual and leaves the folded form in its own epilogue; with K splits it leaves
// fp32 slabs and the residual-add + RMSNorm kernel sums them into the separate form (summing them inside the
// projection, by the last workgroup of each tile to arrive, is built and tested, environment
// DLLM_FUSED_SPLITK=1, but measured slower: 93 vs 54 + 10.7 us for the down projection at M = 512, the
// device-scope release / acquire around the tickets costs more than the kernel it saves).
struct LayerRun {
    int rows, B, L;
    const int32_t *rows_d = nullptr, *pos_d = nullptr;
    const SeqRows *kv_rows = nullptr;
    bool to_cache = false;
};
int run_layers(dllm_handle *h, const int32_t *tokens, const LayerRun &r, int *h_panel_rows, RowScale *scale)
{
    const dllm_config &c = h->cfg;
    const int M = r.rows, d = c.d_model, f = c.d_ffn;
    Workspace &w = h->ws;
    hipStream_t st = h->stream;
    const int slabs = slab_limit(h, M);
    if (slabs < 1) return fail(h, DLLM_ESTATE, "the split-K workspace does not hold one slab of %d rows", M);
    const PanelChoice pc = pick_panels(h, M);
    const int pd = pc.d_rows, pf = pc.f_rows;
    const bool fused = h->fused_norm;
    const bool fused_rope = gemm_qkv_rope_supported(M, d, c.head_dim);
    *h_panel_rows = pd;
    RowScale sc;  // how the rows currently in ws.h still have to be scaled (empty: they are normalised)
    const void *first_gain = c.n_layers > 0 ? h->attn_norm[0] : h->final_norm;
    if (fused) {
        HIP_TRY(h, launch_embed(st, tokens, r.rows_d, h->embed, w.x, M, d, c.vocab, w.bad_token, first_gain, w.h, pd, w.ssq,
                                w.ssq_stride));
        sc = RowScale{w.ssq, 1, w.ssq_stride, c.rms_eps};
    } else {
        HIP_TRY(h, launch_embed(st, tokens, r.rows_d, h->embed, w.x, M, d, c.vocab, w.bad_token));
        HIP_TRY(h, launch_add_rmsnorm(st, w.x, w.partials, 0, first_gain, w.h, M, d, c.rms_eps, pd));
    }
    ResidualOut ro;
    ro.x = w.x; ro.h = w.h; ro.h_panel_rows = pd; ro.ssq = w.ssq; ro.ssq_stride = w.ssq_stride; ro.slabs = w.partials;
    ro.tickets = w.tickets; ro.n_tickets = w.n_tickets;
    // x += A W^T and the operand of the next projection (whose norm has gain `gain`), one way or the other
    auto residual_product = [&](const void *A, const void *W, int K, const GemmLayout &lay, const void *gain) -> int {
        const int splits = gemm_num_splits(M, d, K, slabs);
        if (fused && (splits == 1 || h->fused_splitk)) {
            ro.gain = gain;
            sc = RowScale{w.ssq, 0, w.ssq_stride, c.rms_eps};
            HIP_TRY(h, launch_gemm_residual(st, A, W, ro, M, d, K, h->fused_splitk ? slabs : 1, lay, &sc.parts));
        } else {
            HIP_TRY(h, launch_gemm(st, kEpiPartial, A, W, w.partials, M, d, K, slabs, lay));
            HIP_TRY(h, launch_add_rmsnorm(st, w.x, w.partials, splits, gain, w.h, M, d, c.rms_eps, pd));
            sc = RowScale();
        }
        return DLLM_OK;
    };
    for (int l = 0; l < c.n_layers; ++l) {
        const void *wqkv = pd ? h->wqkv_p[l] : h->wqkv[l];
        const GemmLayout lq{pd, pd ? 3 * d : 0, 0};
        void *qkv_out = r.to_cache ? (void *)w.kv_cache[l] : (void *)w.qkv;
        // a forward over gathered rows: the rotary epilogue puts keys and values at their rows of the cache
        const bool scatter_in_epilogue = fused_rope && r.kv_rows && !r.to_cache;
        if (fused_rope) {
            HIP_TRY(h, launch_gemm_qkv_rope(st, w.h, wqkv, qkv_out, M, d, c.head_dim, w.rope, r.L, r.pos_d, lq, sc,
                                            scatter_in_epilogue ? (void *)w.kv_cache[l] : nullptr,
                                            scatter_in_epilogue ? r.rows_d : nullptr));
        } else {
            HIP_TRY(h, launch_gemm(st, kEpiBf16, w.h, wqkv, qkv_out, M, 3 * d, d, kGemmMaxSplits, lq, sc));
            HIP_TRY(h, launch_rope(st, qkv_out, w.rope, r.B, r.L, c.n_heads, c.head_dim, c.rope_theta));
        }
        if (r.kv_rows) {
            if (!r.to_cache && !scatter_in_epilogue) HIP_TRY(h, launch_scatter_kv(st, w.qkv, w.kv_cache[l], r.rows_d, M, d));
            HIP_TRY(h, launch_attention_rows(st, qkv_out, w.kv_cache[l], w.att, r.B, r.L, c.n_heads, c.head_dim, *r.kv_rows, pd));
        } else {
            HIP_TRY(h, launch_attention(st, w.qkv, w.att, r.B, r.L, c.n_heads, c.head_dim, pd));
        }
        if (int rc = residual_product(w.att, pd ? h->wo_p[l] : h->wo[l], d, GemmLayout{pd, pd ? d : 0, 0}, h->ffn_norm[l])) return rc;
        const bool prof = h->prof_on && h->prof_used < h->prof_cap;
        if (prof) HIP_TRY(h, hipEventRecord(h->prof_ev[2 * h->prof_used], st));
        HIP_TRY(h, launch_gemm(st, kEpiSwiglu, w.h, pd ? h->w_gate_up_p[l] : h->w_gate_up[l], w.act, M, 2 * f, d,
                               kGemmMaxSplits, GemmLayout{pd, pd ? 2 * f : 0, pf}, sc));
        if (prof) HIP_TRY(h, hipEventRecord(h->prof_ev[2 * h->prof_used++ + 1], st));
        if (int rc = residual_product(w.act, pf ? h->w_down_p[l] : h->w_down[l], f, GemmLayout{pf, pf ? d : 0, 0},
                                      l + 1 < c.n_layers ? h->attn_norm[l + 1] : h->final_norm)) return rc;
    }
    *scale = sc;
    return DLLM_OK;
}

// `win` (nullable): per-sequence windows; the vocabulary projection then only
// covers the rows lo..hi of each sequence (the rows the selector reads).
// `mask` (nullable): see vocab_rows.
int forward_impl(dllm_handle *h, int B, int L, const int32_t *tokens, const SelectArgs *win, const uint8_t *mask = nullptr)
{
    const int M = B * L;
    LayerRun r;
    r.rows = M; r.B = B; r.L = L;
    int pd = 0;
    RowScale sc;
    if (int rc = run_layers(h, tokens, r, &pd, &sc)) return rc;
    if (!win) {
        if (int rc = vocab_rows(h, 0, 0, M, L, nullptr, nullptr, pd, sc)) return rc;
    } else {
        // merge sequences whose windows make one contiguous run of rows (always true for B = 1)
        int b = 0;
        while (b < B) {
            if (win->w[b].hi < win->w[b].lo) { ++b; continue; }
            const long first = (long)b * L + win->w[b].lo;
            long last = (long)b * L + win->w[b].hi;
            int e = b + 1;
            while (e < B && win->w[e].hi >= win->w[e].lo && (long)e * L + win->w[e].lo == last + 1) {
                last = (long)e * L + win->w[e].hi;
                ++e;
            }
            if (int rc = vocab_rows(h, first, first, (int)(last - first + 1), L, mask, win, pd, sc)) return rc;
            b = e;
        }
    }
    h->last_B = B;
    h->last_L = L;
    return DLLM_OK;
}

// Forward with out-of-span caching (Section 3.3).  skip (host, [B][L], nullable): positions that are
// not recomputed; every other position is recomputed from the current tokens, attends to all L positions
// of its sequence (cached keys/values for the skipped ones) and refreshes its own cache rows.  The
// vocabulary projection covers rows lo..eval_hi of each window; none of them may be skipped.
int forward_cached_impl(dllm_handle *h, int B, int L, const int32_t *tokens, const SelectArgs &win, const uint8_t *skip,
                        const uint8_t *mask)
{
    const dllm_config &c = h->cfg;
    const int d = c.d_model;
    Workspace &w = h->ws;
    hipStream_t st = h->stream;
    if (!gemm_qkv_rope_supported(B * L, d, c.head_dim))
        return fail(h, DLLM_EINVAL, "cached steps need the fused QKV + RoPE kernel (d_model %% 64 == 0)");
    const size_t Mmax = (size_t)c.max_batch * c.max_seq;
    if (w.kv_cache.empty()) {
        int rc = DLLM_OK;
        std::vector<uint16_t *> bufs(c.n_layers, nullptr);
        for (int l = 0; l < c.n_layers && rc == DLLM_OK; ++l) rc = dev_alloc(h, &bufs[l], Mmax * 3 * d);
        if (rc == DLLM_OK) rc = dev_alloc(h, &w.rows_d, Mmax);
        if (rc == DLLM_OK) rc = dev_alloc(h, &w.pos_d, Mmax);
        if (rc != DLLM_OK) return rc;
        w.kv_cache = bufs;
    }
    // the recomputed rows, in order, and where each sequence's rows start; the lists are built in pinned
    // memory (two slots in turn: the copy of the step before may still be waiting for its turn on the stream)
    const int slot = w.rows_slot;
    w.rows_slot ^= 1;
    HIP_TRY(h, hipEventSynchronize(w.rows_copied[slot]));
    int32_t *rows = w.host_rows[slot], *pos = rows + Mmax;
    SeqRows sr;
    bool any_skip = false;
    int Ma = 0;
    for (int b = 0; b < B; ++b) {
        sr.first[b] = Ma;
        for (int i = 0; i < L; ++i) {
            if (skip && skip[(size_t)b * L + i]) { any_skip = true; continue; }
            rows[Ma] = b * L + i;
            pos[Ma] = i;
            ++Ma;
        }
        sr.count[b] = Ma - sr.first[b];
    }
    if (any_skip && !(w.cache_valid && w.cache_B == B && w.cache_L == L))
        return fail(h, DLLM_ESTATE, "positions are skipped but no step has filled the cache for this batch shape yet");
    if (Ma == 0) return fail(h, DLLM_EINVAL, "every position is skipped");
    HIP_TRY(h, hipMemcpyAsync(w.rows_d, rows, (size_t)Ma * sizeof(int32_t), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipMemcpyAsync(w.pos_d, pos, (size_t)Ma * sizeof(int32_t), hipMemcpyHostToDevice, st));
    HIP_TRY(h, hipEventRecord(w.rows_copied[slot], st));

    LayerRun r;
    r.rows = Ma; r.B = B; r.L = L; r.rows_d = w.rows_d; r.pos_d = w.pos_d; r.kv_rows = &sr;
    r.to_cache = !any_skip;   // everything is recomputed: the QKV projection writes straight into the layer's cache
    int pd = 0;
    RowScale sc;
    if (int rc = run_layers(h, tokens, r, &pd, &sc)) return rc;
    // logits stay indexed by absolute row; the rows of a window are consecutive among the recomputed ones
    for (int b = 0; b < B; ++b) {
        const SeqWindow &sw = win.w[b];
        if (sw.eval_hi < sw.lo) continue;
        const long first_abs = (long)b * L + sw.lo, n = sw.eval_hi - sw.lo + 1;
        long first_cmp = sr.first[b];
        for (int i = 0; i < sw.lo; ++i) first_cmp += !(skip && skip[(size_t)b * L + i]);
        for (int i = sw.lo; i <= sw.eval_hi; ++i)
            if (skip && skip[(size_t)b * L + i]) return fail(h, DLLM_EINVAL, "sequence %d: position %d is skipped but inside the window", b, i);
        if (int rc = vocab_rows(h, first_cmp, first_abs, (int)n, L, mask, &win, pd, sc)) return rc;
    }
    if (!any_skip) { w.cache_valid = true; w.cache_B = B; w.cache_L = L; }
    h->last_B = B;
    h->last_L = L;
    return DLLM_OK;
}

// The embedding kernel met a token id outside [0, vocab) (it used a row of zeros instead): clear the
// flag and report it.  Called after a synchronisation that brought the flag to the host.
int bad_token_seen(dllm_handle *h)
{
    (void)hipMemsetAsync(h->ws.bad_token, 0, sizeof(int32_t), h->stream);
    return fail(h, DLLM_EINVAL, "a token id outside [0, %d) was passed in `tokens`; the steps that read it used an "
                                "all-zero embedding, so their results are not meaningful", h->cfg.vocab);
}

int check_batch(dllm_handle *h, int B, int L)
{
    if (!h) return fail(nullptr, DLLM_EINVAL, "handle is null");
    if (B < 1 || B > h->cfg.max_batch) return fail(h, DLLM_EINVAL, "batch %d outside [1, %d]", B, h->cfg.max_batch);
    if (L < 1 || L > h->cfg.max_seq) return fail(h, DLLM_EINVAL, "sequence length %d outside [1, %d]", L, h->cfg.max_seq);
    return DLLM_OK;
}

// ---- stage controller (Algorithm 1, outer loop) as a per-sequence state machine
struct Controller {
    int gen_start, gen_end;
    const dllm_decode_params *p;
    int s_cycle, e_cycle, stage = DLLM_STAGE_SLOW;
    int step_count = 0, steps = 0;
    std::vector<int> hist;
    int fast_steps = 0;           // steps taken in the current fast stage
    std::vector<uint8_t> skip;    // cached set of the current fast stage ([L], empty: none)

    Controller(int gs, int ge, const dllm_decode_params *pp)
        : gen_start(gs), gen_end(ge), p(pp), s_cycle(gs), e_cycle(ge - 1) {}

    static bool any_mask(const uint8_t *m, int lo, int hi)
    {
        for (int i = lo; i <= hi; ++i)
            if (m[i]) return true;
        return false;
    }
    // false: the sequence is finished (or out of steps)
    bool next(const uint8_t *mask, int L, dllm_stage_params *sp) const
    {
        sp->tau_min_conf = p->tau_min_conf; sp->tau_high_conf = p->tau_high_conf; sp->conv_mode = p->conv_mode;
        sp->gen_start = gen_start; sp->gen_end = gen_end;
        if (steps >= p->max_steps || !any_mask(mask, 0, L - 1)) {
            sp->stage = DLLM_STAGE_IDLE; sp->s_cycle = 0; sp->e_cycle = -1; sp->top_k = 1;
            return false;
        }
        sp->stage = stage;
        sp->s_cycle = s_cycle;
        sp->e_cycle = stage == DLLM_STAGE_SLOW ? gen_end - 1 : e_cycle;
        sp->top_k = stage == DLLM_STAGE_SLOW ? p->k_slow : p->k_fast;
        return true;
    }
    void start_slow() { stage = DLLM_STAGE_SLOW; hist.clear(); step_count = 0; fast_steps = 0; skip.clear(); }
    // cache mode of the step `next` describes
    int cache_mode() const
    {
        if (stage != DLLM_STAGE_FAST || !p->out_of_span_cache) return DLLM_CACHE_OFF;
        return fast_steps == 0 ? DLLM_CACHE_REFRESH : DLLM_CACHE_REUSE;
    }
    void enter_fast(int e, const uint8_t *mask)
    {
        if (e < s_cycle) e = s_cycle;
        if (e > gen_end - 1) e = gen_end - 1;
        e_cycle = e;
        if (any_mask(mask, s_cycle, e)) {
            stage = DLLM_STAGE_FAST;
            fast_steps = 0;
            skip.clear();
        } else {  // nothing left in the span: the next cycle starts behind it
            s_cycle = e + 1;
            start_slow();
        }
    }
    // conf: the step's confidences of this sequence (read after a refresh step only, may be null otherwise)
    void observe(int e_cand, int first_masked, const uint8_t *mask_after, const float *conf = nullptr)
    {
        ++steps;
        if (stage == DLLM_STAGE_SLOW) {
            ++step_count;
            const int e_k = e_cand >= 0 ? e_cand : first_masked;
            hist.push_back(e_k);
            if ((int)hist.size() > p->w_hist) hist.erase(hist.begin());
            double mean = 0.0, var = 0.0;
            long sum = 0;
            for (int v : hist) { mean += v; sum += v; }
            mean /= (double)hist.size();
            for (int v : hist) var += ((double)v - mean) * ((double)v - mean);
            var /= (double)hist.size();  // population variance (eq. 7)
            if ((int)hist.size() >= p->w_hist && var < (double)p->sigma2_stable)
                enter_fast((int)(sum / (long)hist.size()), mask_after);  // floor of the mean (eq. 8)
            else if (step_count >= p->k_max)
                enter_fast(e_k, mask_after);  // no convergence: last candidate
        } else {
            if (p->out_of_span_cache && fast_steps == 0 && conf) {
                // Out-of-span caching: masked, right of the span, below tau_min in this complete step
                skip.assign(gen_end, 0);
                for (int i = e_cycle + 1; i < gen_end; ++i)
                    skip[i] = mask_after[i] && conf[i] < p->tau_min_conf;
            }
            ++fast_steps;
            if (!any_mask(mask_after, s_cycle, e_cycle)) {
                s_cycle = e_cycle + 1;
                start_slow();
            }
        }
    }
};

}  // namespace

// ---- built-in scratch of the entry point that allocates nothing --------------------------------
// One rotary table, (cos, sin) for up to 8192 positions x 64 pairs (head_dim 128) = 4 MiB, resident
// on every GPU the library runs on until the process ends.  `scratch` names the symbol, not a device
// address: host code uses only the address that hipGetSymbolAddress returns for the current device.
constexpr size_t kStaticRopeEntries = (size_t)8192 * 64;
static __device__ __align__(256) float2 scratch[kStaticRopeEntries];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static float2 *g_scratch_ptr[kMaxDevices] = {};  // per device, set on the first call with that device current

namespace {
int static_scratch(float2 **out)
{
    int dev = -1;
    HIP_TRY(nullptr, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, DLLM_EINVAL, "device index %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(nullptr, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(nullptr, DLLM_EHIP, "hipGetSymbolAddress returned a null address for the built-in scratch");
        g_scratch_ptr[dev] = static_cast<float2 *>(p);
    }
    *out = g_scratch_ptr[dev];
    return DLLM_OK;
}
}  // namespace

extern "C" {

const char *dllm_last_error(const dllm_handle *h) { return h ? h->err.c_str() : g_err.c_str(); }

int dllm_create(const dllm_config *cfg, const dllm_weights *w, void *hip_stream, dllm_handle **out)
{
    if (!cfg || !w || !out) return fail(nullptr, DLLM_EINVAL, "dllm_create: null argument");
    *out = nullptr;
    const dllm_config &c = *cfg;
    if (c.n_layers < 0 || c.d_model < 8 || c.n_heads < 1 || c.d_ffn < 8 || c.vocab < 8)
        return fail(nullptr, DLLM_EINVAL, "dllm_create: non-positive model dimension");
    if (c.head_dim != 64 && c.head_dim != 128)
        return fail(nullptr, DLLM_EINVAL, "dllm_create: head_dim %d is not 64 or 128", c.head_dim);
    if ((long)c.n_heads * c.head_dim != c.d_model)
        return fail(nullptr, DLLM_EINVAL, "dllm_create: n_heads * head_dim = %ld differs from d_model %d",
                    (long)c.n_heads * c.head_dim, c.d_model);
    if (c.d_model % 8 || c.d_ffn % 8 || c.vocab % 8)
        return fail(nullptr, DLLM_EINVAL, "dllm_create: d_model, d_ffn and vocab must be multiples of 8");
    if (c.mask_id < 0 || c.mask_id >= c.vocab)
        return fail(nullptr, DLLM_EINVAL, "dllm_create: mask_id %d outside [0, %d)", c.mask_id, c.vocab);
    if (c.max_batch < 1 || c.max_batch > DLLM_MAX_BATCH)
        return fail(nullptr, DLLM_EINVAL, "dllm_create: max_batch %d outside [1, %d]", c.max_batch, DLLM_MAX_BATCH);
    if (c.max_seq < 1 || c.max_seq > 8192)
        return fail(nullptr, DLLM_EINVAL, "dllm_create: max_seq %d outside [1, 8192]", c.max_seq);
    if (!(c.rms_eps >= 0.0f) || !(c.rope_theta > 0.0f))
        return fail(nullptr, DLLM_EINVAL, "dllm_create: rms_eps must be >= 0 and rope_theta > 0");
    if (!w->embed || !w->lm_head || !w->final_norm)
        return fail(nullptr, DLLM_EINVAL, "dllm_create: null embed / lm_head / final_norm");
    if (c.n_layers > 0 && (!w->attn_norm || !w->wqkv || !w->wo || !w->ffn_norm || !w->w_gate_up || !w->w_down))
        return fail(nullptr, DLLM_EINVAL, "dllm_create: null per-layer weight array");
    if (!aligned16(w->embed) || !aligned16(w->lm_head) || !aligned16(w->final_norm))
        return fail(nullptr, DLLM_EINVAL, "dllm_create: weights must be 16-byte aligned");

    dllm_handle *h = new (std::nothrow) dllm_handle();
    if (!h) return fail(nullptr, DLLM_ENOMEM, "dllm_create: host allocation failed");
    h->cfg = c;
    h->stream = static_cast<hipStream_t>(hip_stream);
    h->embed = w->embed; h->lm_head = w->lm_head; h->final_norm = w->final_norm;
    for (int l = 0; l < c.n_layers; ++l) {
        const void *ptrs[6] = {w->attn_norm[l], w->wqkv[l], w->wo[l], w->ffn_norm[l], w->w_gate_up[l], w->w_down[l]};
        for (const void *p : ptrs)
            if (!p || !aligned16(p)) {
                delete h;
                return fail(nullptr, DLLM_EINVAL, "dllm_create: layer %d has a null or misaligned weight", l);
            }
        h->attn_norm.push_back(ptrs[0]); h->wqkv.push_back(ptrs[1]); h->wo.push_back(ptrs[2]);
        h->ffn_norm.push_back(ptrs[3]); h->w_gate_up.push_back(ptrs[4]); h->w_down.push_back(ptrs[5]);
    }

    const size_t M = (size_t)c.max_batch * c.max_seq, d = c.d_model, f = c.d_ffn;
    Workspace &s = h->ws;
    int rc = DLLM_OK;
    auto A = [&](int r) { if (rc == DLLM_OK) rc = r; };
    A(dev_alloc(h, &s.x, M * d));
    A(dev_alloc(h, &s.h, M * d));
    A(dev_alloc(h, &s.qkv, M * 3 * d));
    A(dev_alloc(h, &s.att, M * d));
    A(dev_alloc(h, &s.act, M * f));
    // slabs: every split count fits up to 4096 rows, two slabs beyond (once the row tiles alone fill the chip
    // the planner wants few or no splits); each launch hands the planner the number of slabs that fit
    size_t slab_rows = (size_t)kGemmMaxSplits * (M < 4096 ? M : 4096);
    if (2 * M > slab_rows) slab_rows = 2 * M;
    s.partials_cap = slab_rows * d;
    A(dev_alloc(h, &s.partials, s.partials_cap));
    s.ssq_stride = gemm_residual_max_parts((int)d);
    A(dev_alloc(h, &s.ssq, M * (size_t)s.ssq_stride));
    s.n_tickets = (int)(((M + 63) / 64) * ((d + 63) / 64));
    A(dev_alloc(h, &s.tickets, (size_t)s.n_tickets));
    if (rc == DLLM_OK && hipMemsetAsync(s.tickets, 0, (size_t)s.n_tickets * sizeof(int32_t), h->stream) != hipSuccess)
        rc = fail(h, DLLM_EHIP, "dllm_create: hipMemsetAsync failed");
    A(dev_alloc(h, &s.rowstats, 3 * gemm_rowstats_max_parts(c.vocab) * M));
    A(dev_alloc(h, &s.pred, M));
    A(dev_alloc(h, &s.conf, M));
    A(dev_alloc(h, &s.rope, (size_t)c.max_seq * (c.head_dim / 2)));
    A(dev_alloc(h, &s.prev_pred, M));
    A(dev_alloc(h, &s.cl_ints, (size_t)4 * c.max_batch + 1));
    if (rc == DLLM_OK) {
        s.bad_token = s.cl_ints + 4 * c.max_batch;
        if (hipMemsetAsync(s.cl_ints, 0, ((size_t)4 * c.max_batch + 1) * sizeof(int32_t), h->stream) != hipSuccess)
            rc = fail(h, DLLM_EHIP, "dllm_create: hipMemsetAsync failed");
    }
    A(dev_alloc(h, &s.cl_pos, M));
    A(dev_alloc(h, &s.cl_tok, M));
    A(dev_alloc(h, &s.cl_conf, M));
    const size_t m64 = (M + 63) & ~(size_t)63, ints64 = (((size_t)4 * c.max_batch + 1) * 4 + 63) & ~(size_t)63;
    if (rc == DLLM_OK && hipHostMalloc(reinterpret_cast<void **>(&s.host_pinned), m64 + ints64 + 5 * M * 4 + 64,
                                       hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        rc = fail(h, DLLM_ENOMEM, "dllm_create: pinned host allocation failed");
    }
    if (rc == DLLM_OK) {
        s.host_ints = reinterpret_cast<int32_t *>(s.host_pinned + m64);
        s.host_conf = reinterpret_cast<float *>(s.host_pinned + m64 + ints64);
        s.host_rows[0] = reinterpret_cast<int32_t *>(s.host_conf + M);
        s.host_rows[1] = s.host_rows[0] + 2 * M;
    }
    if (rc == DLLM_OK && (hipEventCreate(&h->ev0) != hipSuccess || hipEventCreate(&h->ev1) != hipSuccess ||
                          hipEventCreateWithFlags(&s.rows_copied[0], hipEventDisableTiming) != hipSuccess ||
                          hipEventCreateWithFlags(&s.rows_copied[1], hipEventDisableTiming) != hipSuccess))
        rc = fail(h, DLLM_EHIP, "dllm_create: hipEventCreate failed");
    if (rc == DLLM_OK && launch_rope_table(h->stream, s.rope, c.max_seq, c.head_dim, c.rope_theta) != hipSuccess)
        rc = fail(h, DLLM_EHIP, "dllm_create: rope table launch failed");
    h->fused_norm = getenv("DLLM_NO_FUSED_NORM") == nullptr;
    h->fused_splitk = getenv("DLLM_FUSED_SPLITK") != nullptr;
    // panel-major copies of the weights (the caller's stay in use for shapes the asynchronous-copy kernel does not take)
    if (rc == DLLM_OK && getenv("DLLM_NO_PACK") == nullptr) {
        auto pack = [&](const void *src, size_t rows, size_t K, const void **dst) {
            uint16_t *p = nullptr;
            if (rc == DLLM_OK) rc = dev_alloc(h, &p, rows * K);
            if (rc == DLLM_OK && launch_pack_panels(h->stream, src, p, rows, (int)K) != hipSuccess)
                rc = fail(h, DLLM_EHIP, "dllm_create: weight packing launch failed");
            *dst = p;
        };
        h->packed_d = d % 64 == 0;
        h->packed_f = f % 64 == 0;
        if (h->packed_d) {
            pack(h->lm_head, c.vocab, d, &h->lm_head_p);
            h->wqkv_p.assign(c.n_layers, nullptr); h->wo_p.assign(c.n_layers, nullptr); h->w_gate_up_p.assign(c.n_layers, nullptr);
            for (int l = 0; l < c.n_layers; ++l) {
                pack(h->wqkv[l], 3 * d, d, &h->wqkv_p[l]);
                pack(h->wo[l], d, d, &h->wo_p[l]);
                pack(h->w_gate_up[l], 2 * f, d, &h->w_gate_up_p[l]);
            }
        }
        if (h->packed_f) {
            h->w_down_p.assign(c.n_layers, nullptr);
            for (int l = 0; l < c.n_layers; ++l) pack(h->w_down[l], d, f, &h->w_down_p[l]);
        }
    }
    if (rc == DLLM_OK && hipStreamSynchronize(h->stream) != hipSuccess)
        rc = fail(h, DLLM_EHIP, "dllm_create: stream synchronize failed");
    if (rc != DLLM_OK) {
        g_err = h->err;
        dllm_destroy(h);
        return rc;
    }
    *out = h;
    return DLLM_OK;
}

void dllm_destroy(dllm_handle *h)
{
    if (!h) return;
    (void)hipStreamSynchronize(h->stream);
    for (void *p : h->allocs) (void)hipFree(p);
    if (h->ws.host_pinned) (void)hipHostFree(h->ws.host_pinned);
    for (hipEvent_t e : h->prof_ev) (void)hipEventDestroy(e);
    if (h->ev0) (void)hipEventDestroy(h->ev0);
    if (h->ev1) (void)hipEventDestroy(h->ev1);
    for (hipEvent_t e : h->ws.rows_copied)
        if (e) (void)hipEventDestroy(e);
    delete h;
}

int dllm_forward(dllm_handle *h, int32_t B, int32_t L, const int32_t *tokens)
{
    int rc = check_batch(h, B, L);
    if (rc) return rc;
    if (!tokens) return fail(h, DLLM_EINVAL, "dllm_forward: tokens is null");
    return forward_impl(h, B, L, tokens, nullptr);
}

int dllm_step(dllm_handle *h, int32_t B, int32_t L, int32_t *tokens, uint8_t *mask, int32_t *prev_pred,
              const dllm_stage_params *sp, const dllm_commit_list *out)
{
    int rc = check_batch(h, B, L);
    if (rc) return rc;
    if (!tokens || !mask || !prev_pred || !sp) return fail(h, DLLM_EINVAL, "dllm_step: null argument");
    CommitOut co;
    if ((rc = check_commit_list(h, out, &co))) return rc;
    SelectArgs args;
    if ((rc = build_select_args(h, B, L, sp, out->capacity, &args))) return rc;
    if ((rc = forward_impl(h, B, L, tokens, &args, mask))) return rc;
    if (!h->fused_selector)
        HIP_TRY(h, launch_row_phase(h->stream, h->ws.logits, B, L, h->cfg.vocab, h->cfg.mask_id, mask, args, h->ws.pred,
                                    h->ws.conf));
    HIP_TRY(h, launch_seq_phase(h->stream, B, L, tokens, mask, prev_pred, h->ws.pred, h->ws.conf, args, co));
    return DLLM_OK;
}

int dllm_sync_status(dllm_handle *h)
{
    if (!h) return fail(nullptr, DLLM_EINVAL, "dllm_sync_status: handle is null");
    int32_t *flag = h->ws.host_ints + 4 * h->cfg.max_batch;
    HIP_TRY(h, hipMemcpyAsync(flag, h->ws.bad_token, sizeof(int32_t), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    if (*flag != 0) return bad_token_seen(h);
    return DLLM_OK;
}

int dllm_set_fused_selector(dllm_handle *h, int32_t enable)
{
    if (!h) return fail(nullptr, DLLM_EINVAL, "dllm_set_fused_selector: null handle");
    h->fused_selector = enable != 0;
    return DLLM_OK;
}

int dllm_step_cached(dllm_handle *h, int32_t B, int32_t L, int32_t *tokens, uint8_t *mask, int32_t *prev_pred,
                     const dllm_stage_params *sp, const int32_t *cache_mode, const uint8_t *skip,
                     const dllm_commit_list *out)
{
    int rc = check_batch(h, B, L);
    if (rc) return rc;
    if (!tokens || !mask || !prev_pred || !sp || !cache_mode) return fail(h, DLLM_EINVAL, "dllm_step_cached: null argument");
    CommitOut co;
    if ((rc = check_commit_list(h, out, &co))) return rc;
    SelectArgs args;
    if ((rc = build_select_args(h, B, L, sp, out->capacity, &args, cache_mode))) return rc;
    bool any_cache = false, any_reuse = false;
    for (int b = 0; b < B; ++b) {
        any_cache |= cache_mode[b] != DLLM_CACHE_OFF;
        any_reuse |= cache_mode[b] == DLLM_CACHE_REUSE;
    }
    if (any_reuse && !skip) return fail(h, DLLM_EINVAL, "dllm_step_cached: a sequence reuses the cache but skip is null");
    if (!any_cache) {
        if ((rc = forward_impl(h, B, L, tokens, &args, mask))) return rc;
    } else {
        // only sequences in reuse mode skip anything
        std::vector<uint8_t> eff;
        if (any_reuse) {
            eff.assign((size_t)B * L, 0);
            for (int b = 0; b < B; ++b) {
                if (cache_mode[b] != DLLM_CACHE_REUSE) continue;
                for (int i = 0; i < L; ++i) {
                    const uint8_t v = skip[(size_t)b * L + i];
                    if (v && i >= args.w[b].lo && i <= args.w[b].eval_hi)
                        return fail(h, DLLM_EINVAL, "dllm_step_cached: sequence %d skips position %d, which is inside its window", b, i);
                    eff[(size_t)b * L + i] = v != 0;
                }
            }
        }
        if ((rc = forward_cached_impl(h, B, L, tokens, args, any_reuse ? eff.data() : nullptr, mask))) return rc;
    }
    if (!h->fused_selector)
        HIP_TRY(h, launch_row_phase(h->stream, h->ws.logits, B, L, h->cfg.vocab, h->cfg.mask_id, mask, args, h->ws.pred,
                                    h->ws.conf));
    HIP_TRY(h, launch_seq_phase(h->stream, B, L, tokens, mask, prev_pred, h->ws.pred, h->ws.conf, args, co));
    return DLLM_OK;
}

int dllm_select(void *hip_stream, const void *logits, int32_t B, int32_t L, int32_t V, int32_t mask_id,
                int32_t *tokens, uint8_t *mask, int32_t *prev_pred, const dllm_stage_params *sp, int32_t *pred,
                float *conf, const dllm_commit_list *out)
{
    if (!logits || !tokens || !mask || !prev_pred || !sp || !pred || !conf)
        return fail(nullptr, DLLM_EINVAL, "dllm_select: null argument");
    if (V < 1) return fail(nullptr, DLLM_EINVAL, "dllm_select: vocab %d < 1", V);
    if (mask_id < 0 || mask_id >= V) return fail(nullptr, DLLM_EINVAL, "dllm_select: mask_id %d outside [0, %d)", mask_id, V);
    if ((reinterpret_cast<uintptr_t>(logits) & 1) != 0) return fail(nullptr, DLLM_EINVAL, "dllm_select: misaligned logits");
    CommitOut co;
    int rc;
    if ((rc = check_commit_list(nullptr, out, &co))) return rc;
    SelectArgs args;
    if ((rc = build_select_args(nullptr, B, L, sp, out->capacity, &args))) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    HIP_TRY(nullptr, launch_row_phase(st, logits, B, L, V, mask_id, mask, args, pred, conf));
    HIP_TRY(nullptr, launch_seq_phase(st, B, L, tokens, mask, prev_pred, pred, conf, args, co));
    return DLLM_OK;
}

int dllm_decode(dllm_handle *h, int32_t B, int32_t L, int32_t gen_start, int32_t *tokens, uint8_t *mask,
                const dllm_decode_params *p, int32_t *steps_taken, dllm_step_stat *stats, int32_t stats_capacity)
{
    int rc = check_batch(h, B, L);
    if (rc) return rc;
    if (!tokens || !mask || !p || !steps_taken) return fail(h, DLLM_EINVAL, "dllm_decode: null argument");
    if (gen_start < 0 || gen_start > L) return fail(h, DLLM_EINVAL, "dllm_decode: gen_start %d outside [0, %d]", gen_start, L);
    if (p->max_steps < 0 || p->k_max < 1 || p->w_hist < 1 || p->k_slow < 1 || p->k_fast < 1)
        return fail(h, DLLM_EINVAL, "dllm_decode: max_steps >= 0, k_max, w_hist, k_slow, k_fast >= 1 required");
    if (p->conv_mode != 0 && p->conv_mode != 1) return fail(h, DLLM_EINVAL, "dllm_decode: conv_mode must be 0 or 1");
    if (p->out_of_span_cache != 0 && p->out_of_span_cache != 1)
        return fail(h, DLLM_EINVAL, "dllm_decode: out_of_span_cache must be 0 or 1");
    if (p->prompt_cache_interval < 0) return fail(h, DLLM_EINVAL, "dllm_decode: prompt_cache_interval must be >= 0");
    if (p->response_cache_interval < 0) return fail(h, DLLM_EINVAL, "dllm_decode: response_cache_interval must be >= 0");
    if (stats && stats_capacity < 0) return fail(h, DLLM_EINVAL, "dllm_decode: negative stats_capacity");

    Workspace &w = h->ws;
    const int mb = h->cfg.max_batch;
    hipStream_t st = h->stream;
    // prev_pred <- -1 (all bytes 0xff)
    HIP_TRY(h, hipMemsetAsync(w.prev_pred, 0xff, (size_t)B * L * sizeof(int32_t), st));
    uint8_t *hmask = w.host_pinned;
    int32_t *hints = w.host_ints;
    HIP_TRY(h, hipMemcpyAsync(hmask, mask, (size_t)B * L, hipMemcpyDeviceToHost, st));
    HIP_TRY(h, hipStreamSynchronize(st));

    dllm_commit_list cl;
    cl.capacity = L;
    cl.n_commit = w.cl_ints; cl.e_cand = w.cl_ints + mb; cl.first_masked = w.cl_ints + 2 * mb;
    cl.n_masked_after = w.cl_ints + 3 * mb;
    cl.pos = w.cl_pos; cl.tok = w.cl_tok; cl.conf = w.cl_conf;

    std::vector<Controller> ctl;
    for (int b = 0; b < B; ++b) ctl.emplace_back(gen_start, L, p);
    std::vector<dllm_stage_params> sps(B);
    std::vector<int32_t> modes(B, DLLM_CACHE_OFF);
    std::vector<uint8_t> skip((size_t)B * L, 0);
    float *hconf = w.host_conf;
    int steps = 0;
    for (;;) {
        bool live = false;
        int n_slow = 0, n_fast = 0, n_idle = 0;
        for (int b = 0; b < B; ++b) {
            live |= ctl[b].next(hmask + (size_t)b * L, L, &sps[b]);
            n_slow += sps[b].stage == DLLM_STAGE_SLOW;
            n_fast += sps[b].stage == DLLM_STAGE_FAST;
            n_idle += sps[b].stage == DLLM_STAGE_IDLE;
        }
        if (!live) break;
        const bool timed = stats && steps < stats_capacity;
        bool any_cache = false, any_refresh = false;
        // interval caches: every K_p-th step recomputes the prompt, every K_r-th the whole response; the
        // others leave the prompt / the response outside each sequence's rated range out
        const int kp = p->prompt_cache_interval, kr = p->response_cache_interval;
        const bool prompt_refresh = kp > 0 && steps % kp == 0, response_refresh = kr > 0 && steps % kr == 0;
        for (int b = 0; b < B; ++b) {
            uint8_t *sk = skip.data() + (size_t)b * L;
            const int oos = sps[b].stage == DLLM_STAGE_IDLE ? DLLM_CACHE_OFF : ctl[b].cache_mode();
            any_refresh |= oos == DLLM_CACHE_REFRESH;
            if (oos == DLLM_CACHE_REUSE && !ctl[b].skip.empty())
                memcpy(sk, ctl[b].skip.data(), L);
            else
                memset(sk, 0, L);
            modes[b] = oos;
            if ((kp > 0 || kr > 0) && oos != DLLM_CACHE_REFRESH) {
                if (kp > 0 && !prompt_refresh) memset(sk, 1, gen_start);
                if (kr > 0 && !response_refresh) {
                    const bool idle = sps[b].stage == DLLM_STAGE_IDLE;
                    const int lo = idle ? L : sps[b].s_cycle;
                    const int hi = idle ? -1 : sps[b].stage == DLLM_STAGE_SLOW ? L - 1 : sps[b].e_cycle;
                    for (int i = gen_start; i < L; ++i)
                        if (i < lo || i > hi) sk[i] = 1;
                }
                // through the cached path without the wider rated range of an out-of-span refresh step: an
                // all-zero skip set recomputes every position and refreshes its cache rows
                modes[b] = DLLM_CACHE_REUSE;
            }
            any_cache |= modes[b] != DLLM_CACHE_OFF;
        }
        if (timed) HIP_TRY(h, hipEventRecord(h->ev0, st));
        if (any_cache) {
            if ((rc = dllm_step_cached(h, B, L, tokens, mask, w.prev_pred, sps.data(), modes.data(), skip.data(), &cl))) return rc;
        } else {
            if ((rc = dllm_step(h, B, L, tokens, mask, w.prev_pred, sps.data(), &cl))) return rc;
        }
        if (timed) HIP_TRY(h, hipEventRecord(h->ev1, st));
        HIP_TRY(h, hipMemcpyAsync(hmask, mask, (size_t)B * L, hipMemcpyDeviceToHost, st));
        HIP_TRY(h, hipMemcpyAsync(hints, w.cl_ints, ((size_t)4 * mb + 1) * sizeof(int32_t), hipMemcpyDeviceToHost, st));
        if (any_refresh)  // the confidences decide what is cached for the rest of the stage
            HIP_TRY(h, hipMemcpyAsync(hconf, w.conf, (size_t)B * L * sizeof(float), hipMemcpyDeviceToHost, st));
        HIP_TRY(h, hipStreamSynchronize(st));
        if (hints[4 * mb] != 0) return bad_token_seen(h);
        int committed = 0;
        for (int b = 0; b < B; ++b) {
            if (sps[b].stage == DLLM_STAGE_IDLE) continue;
            committed += hints[b];
            ctl[b].observe(hints[mb + b], hints[2 * mb + b], hmask + (size_t)b * L,
                           any_refresh ? hconf + (size_t)b * L : nullptr);
        }
        if (timed) {
            float ms = 0.0f;
            HIP_TRY(h, hipEventElapsedTime(&ms, h->ev0, h->ev1));
            stats[steps] = dllm_step_stat{n_slow, n_fast, n_idle, committed, ms};
        }
        ++steps;
    }
    *steps_taken = steps;
    return DLLM_OK;
}

int dllm_decode_low_confidence(dllm_handle *h, int32_t B, int32_t L, int32_t gen_start, int32_t *tokens,
                               uint8_t *mask, int32_t n_steps, int32_t block_len, int32_t *steps_taken,
                               dllm_step_stat *stats, int32_t stats_capacity)
{
    int rc = check_batch(h, B, L);
    if (rc) return rc;
    if (!tokens || !mask || !steps_taken) return fail(h, DLLM_EINVAL, "dllm_decode_low_confidence: null argument");
    if (gen_start < 0 || gen_start > L)
        return fail(h, DLLM_EINVAL, "dllm_decode_low_confidence: gen_start %d outside [0, %d]", gen_start, L);
    if (stats && stats_capacity < 0) return fail(h, DLLM_EINVAL, "dllm_decode_low_confidence: negative stats_capacity");
    const int G = L - gen_start;
    *steps_taken = 0;
    if (G == 0) return DLLM_OK;
    const int lb = block_len <= 0 ? G : block_len;
    if (G % lb) return fail(h, DLLM_EINVAL, "dllm_decode_low_confidence: block_len %d does not divide the %d generated positions", lb, G);
    const int n_blocks = G / lb;
    if (n_steps < n_blocks || n_steps % n_blocks)
        return fail(h, DLLM_EINVAL, "dllm_decode_low_confidence: n_steps %d is not a positive multiple of the %d blocks", n_steps, n_blocks);
    const int per_block = n_steps / n_blocks;

    Workspace &w = h->ws;
    const int mb = h->cfg.max_batch;
    hipStream_t st = h->stream;
    HIP_TRY(h, hipMemsetAsync(w.prev_pred, 0xff, (size_t)B * L * sizeof(int32_t), st));
    uint8_t *hmask = w.host_pinned;
    int32_t *hints = w.host_ints;
    HIP_TRY(h, hipMemcpyAsync(hmask, mask, (size_t)B * L, hipMemcpyDeviceToHost, st));
    HIP_TRY(h, hipStreamSynchronize(st));

    dllm_commit_list cl;
    cl.capacity = L;
    cl.n_commit = w.cl_ints; cl.e_cand = w.cl_ints + mb; cl.first_masked = w.cl_ints + 2 * mb;
    cl.n_masked_after = w.cl_ints + 3 * mb;
    cl.pos = w.cl_pos; cl.tok = w.cl_tok; cl.conf = w.cl_conf;

    std::vector<dllm_stage_params> sps(B);
    int steps = 0;
    for (int blk = 0; blk < n_blocks; ++blk) {
        const int lo = gen_start + blk * lb, hi = lo + lb;  // [lo, hi)
        for (int j = 1; j <= per_block; ++j) {
            const long target = (long)lb * j / per_block;  // tokens of the block unmasked after this step
            int n_live = 0;
            for (int b = 0; b < B; ++b) {
                int masked = 0;
                for (int i = lo; i < hi; ++i) masked += hmask[(size_t)b * L + i] != 0;
                const long k = target - (lb - masked);
                dllm_stage_params &sp = sps[b];
                sp.tau_min_conf = 0.0f; sp.tau_high_conf = 1.0f; sp.conv_mode = 0;
                sp.gen_start = gen_start; sp.gen_end = hi;
                if (k >= 1) {
                    sp.stage = DLLM_STAGE_SLOW; sp.s_cycle = lo; sp.e_cycle = hi - 1; sp.top_k = (int)k;
                    ++n_live;
                } else {
                    sp.stage = DLLM_STAGE_IDLE; sp.s_cycle = 0; sp.e_cycle = -1; sp.top_k = 1;
                }
            }
            if (n_live == 0) continue;
            const bool timed = stats && steps < stats_capacity;
            if (timed) HIP_TRY(h, hipEventRecord(h->ev0, st));
            if ((rc = dllm_step(h, B, L, tokens, mask, w.prev_pred, sps.data(), &cl))) return rc;
            if (timed) HIP_TRY(h, hipEventRecord(h->ev1, st));
            HIP_TRY(h, hipMemcpyAsync(hmask, mask, (size_t)B * L, hipMemcpyDeviceToHost, st));
            HIP_TRY(h, hipMemcpyAsync(hints, w.cl_ints, ((size_t)4 * mb + 1) * sizeof(int32_t), hipMemcpyDeviceToHost, st));
            HIP_TRY(h, hipStreamSynchronize(st));
            if (hints[4 * mb] != 0) return bad_token_seen(h);
            if (timed) {
                int committed = 0;
                for (int b = 0; b < B; ++b)
                    if (sps[b].stage != DLLM_STAGE_IDLE) committed += hints[b];
                float ms = 0.0f;
                HIP_TRY(h, hipEventElapsedTime(&ms, h->ev0, h->ev1));
                stats[steps] = dllm_step_stat{n_live, 0, B - n_live, committed, ms};
            }
            ++steps;
        }
    }
    *steps_taken = steps;
    return DLLM_OK;
}

int dllm_profile_begin(dllm_handle *h, int32_t max_launches)
{
    if (!h) return fail(nullptr, DLLM_EINVAL, "dllm_profile_begin: handle is null");
    if (max_launches < 1 || max_launches > (1 << 20)) return fail(h, DLLM_EINVAL, "dllm_profile_begin: max_launches outside [1, 2^20]");
    while ((int)h->prof_ev.size() < 2 * max_launches) {
        hipEvent_t e;
        HIP_TRY(h, hipEventCreate(&e));
        h->prof_ev.push_back(e);
    }
    h->prof_cap = max_launches;
    h->prof_used = 0;
    h->prof_on = true;
    return DLLM_OK;
}

int dllm_profile_end(dllm_handle *h, float *total_ms, int32_t *launches)
{
    if (!h || !total_ms || !launches) return fail(h, DLLM_EINVAL, "dllm_profile_end: null argument");
    if (!h->prof_on) return fail(h, DLLM_ESTATE, "dllm_profile_end: profiling is not enabled");
    h->prof_on = false;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    float tot = 0.0f;
    for (int i = 0; i < h->prof_used; ++i) {
        float ms = 0.0f;
        HIP_TRY(h, hipEventElapsedTime(&ms, h->prof_ev[2 * i], h->prof_ev[2 * i + 1]));
        tot += ms;
    }
    *total_ms = tot;
    *launches = h->prof_used;
    return DLLM_OK;
}

void dllm_debug_reload_env(void) { gemm_reload_env(); }

int dllm_debug_gemm_plan(int32_t epilogue, int32_t M, int32_t N, int32_t K, int32_t split_limit, int32_t *out8)
{
    if (!out8) return fail(nullptr, DLLM_EINVAL, "dllm_debug_gemm_plan: out8 is null");
    if (epilogue < 0 || epilogue > 5 || M < 1 || N < 1 || K < 8 || K % 8)
        return fail(nullptr, DLLM_EINVAL, "dllm_debug_gemm_plan: epilogue in [0, 5], M, N >= 1, K a positive multiple of 8");
    const GemmPlanInfo p = gemm_plan_info(epilogue, M, N, K, split_limit);
    const int32_t v[8] = {p.bm, p.bn, p.bk, p.stages, p.waves_m, p.waves_n, p.splits, p.async_copy};
    memcpy(out8, v, sizeof v);
    return DLLM_OK;
}

int dllm_debug_mfma_rate(void *hip_stream, const void *operands, int32_t n_operands, float *sink, int32_t workgroups,
                         int32_t iters)
{
    if (!operands || !sink) return fail(nullptr, DLLM_EINVAL, "dllm_debug_mfma_rate: null pointer");
    if (n_operands < 1 || workgroups < 1 || workgroups > (1 << 20) || iters < 1 || iters > (1 << 20))
        return fail(nullptr, DLLM_EINVAL, "dllm_debug_mfma_rate: n_operands >= 1, workgroups and iters in [1, 2^20]");
    HIP_TRY(nullptr, launch_mfma_rate(static_cast<hipStream_t>(hip_stream), operands, n_operands, sink, workgroups, iters));
    return DLLM_OK;
}

int dllm_debug_logits(dllm_handle *h, const void **logits)
{
    if (!h || !logits) return fail(h, DLLM_EINVAL, "dllm_debug_logits: null argument");
    if (h->last_B == 0 || !h->ws.logits)
        return fail(h, DLLM_ESTATE, "dllm_debug_logits: no call on this handle has written logits");
    *logits = h->ws.logits;
    return DLLM_OK;
}

int dllm_debug_rows(dllm_handle *h, const int32_t **pred, const float **conf)
{
    if (!h || !pred || !conf) return fail(h, DLLM_EINVAL, "dllm_debug_rows: null argument");
    if (h->last_B == 0) return fail(h, DLLM_ESTATE, "dllm_debug_rows: no step has run");
    *pred = h->ws.pred;
    *conf = h->ws.conf;
    return DLLM_OK;
}

// ---- building blocks --------------------------------------------------------

static int check_linear(const void *A, const void *W, const void *C, int M, int N, int K, const char *who)
{
    if (!A || !W || !C) return fail(nullptr, DLLM_EINVAL, "%s: null argument", who);
    if (M < 1 || N < 1 || K < 8 || K % 8) return fail(nullptr, DLLM_EINVAL, "%s: need M, N >= 1 and K a positive multiple of 8", who);
    if (!aligned16(A) || !aligned16(W) || !aligned16(C)) return fail(nullptr, DLLM_EINVAL, "%s: pointers must be 16-byte aligned", who);
    return DLLM_OK;
}

int dllm_op_linear(void *hip_stream, const void *A, const void *W, void *C, int32_t M, int32_t N, int32_t K)
{
    int rc = check_linear(A, W, C, M, N, K, "dllm_op_linear");
    if (rc) return rc;
    HIP_TRY(nullptr, launch_gemm(static_cast<hipStream_t>(hip_stream), kEpiBf16, A, W, C, M, N, K));
    return DLLM_OK;
}

int dllm_op_linear_swiglu(void *hip_stream, const void *A, const void *W, void *out, int32_t M, int32_t f, int32_t K)
{
    int rc = check_linear(A, W, out, M, f, K, "dllm_op_linear_swiglu");
    if (rc) return rc;
    HIP_TRY(nullptr, launch_gemm(static_cast<hipStream_t>(hip_stream), kEpiSwiglu, A, W, out, M, 2 * f, K));
    return DLLM_OK;
}

int dllm_op_pack_panels(void *hip_stream, const void *src, void *dst, int64_t rows, int32_t K)
{
    if (!src || !dst || !aligned16(src) || !aligned16(dst)) return fail(nullptr, DLLM_EINVAL, "dllm_op_pack_panels: null or misaligned pointer");
    if (rows < 1 || K < 32 || K % 32) return fail(nullptr, DLLM_EINVAL, "dllm_op_pack_panels: need rows >= 1 and K a positive multiple of 32");
    HIP_TRY(nullptr, launch_pack_panels(static_cast<hipStream_t>(hip_stream), src, dst, (size_t)rows, K));
    return DLLM_OK;
}

int dllm_op_linear_panels(void *hip_stream, const void *A, const void *W, void *C, int32_t M, int32_t N, int32_t K,
                          int32_t swiglu, int32_t a_panel_rows, int32_t w_panels, int32_t c_panel_rows)
{
    int rc = check_linear(A, W, C, M, N, K, "dllm_op_linear_panels");
    if (rc) return rc;
    if (a_panel_rows < 0 || c_panel_rows < 0 || (a_panel_rows && a_panel_rows < M) || (c_panel_rows && c_panel_rows < M))
        return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_panels: panel rows must be 0 or >= M");
    if (c_panel_rows && !swiglu) return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_panels: only the SwiGLU output can be panel-major");
    if (swiglu && (N % 2)) return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_panels: SwiGLU needs an even number of W rows");
    if (c_panel_rows && (N / 2) % 32) return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_panels: a panel-major output needs N / 2 %% 32 == 0");
    const GemmEpilogue epi = swiglu ? kEpiSwiglu : kEpiBf16;
    if ((a_panel_rows || w_panels || c_panel_rows) && !gemm_async_copy_path(epi, M, N, K))
        return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_panels: panel-major operands need the asynchronous-copy kernel "
                                          "(K %% 64 == 0, operands below 4 GB, DLLM_GEMM_FALLBACK unset)");
    HIP_TRY(nullptr, launch_gemm(static_cast<hipStream_t>(hip_stream), epi, A, W, C, M, N, K, kGemmMaxSplits,
                                 GemmLayout{a_panel_rows, w_panels ? N : 0, c_panel_rows}));
    return DLLM_OK;
}

int dllm_op_add_rmsnorm(void *hip_stream, float *x, const float *partials, int32_t n_partials, const void *gain,
                        void *hout, int32_t M, int32_t d, float eps)
{
    if (!x || !gain || !hout || (n_partials > 0 && !partials)) return fail(nullptr, DLLM_EINVAL, "dllm_op_add_rmsnorm: null argument");
    if (M < 1 || d < 4 || d % 4 || n_partials < 0 || n_partials > kGemmMaxSplits)
        return fail(nullptr, DLLM_EINVAL, "dllm_op_add_rmsnorm: need M >= 1, d a positive multiple of 4, 0 <= n_partials <= %d", kGemmMaxSplits);
    if (!aligned16(x) || !aligned16(gain) || !aligned16(hout) || !aligned16(partials)) return fail(nullptr, DLLM_EINVAL, "dllm_op_add_rmsnorm: pointers must be 16-byte aligned");
    HIP_TRY(nullptr, launch_add_rmsnorm(static_cast<hipStream_t>(hip_stream), x, partials, n_partials, gain, hout, M, d, eps));
    return DLLM_OK;
}

int dllm_op_rope(void *hip_stream, void *qkv, int32_t B, int32_t L, int32_t H, int32_t dh, float theta)
{
    if (!qkv || !aligned16(qkv)) return fail(nullptr, DLLM_EINVAL, "dllm_op_rope: null or misaligned qkv");
    if (B < 1 || L < 1 || H < 1 || (dh != 64 && dh != 128) || !(theta > 0.0f)) return fail(nullptr, DLLM_EINVAL, "dllm_op_rope: bad shape");
    HIP_TRY(nullptr, launch_rope(static_cast<hipStream_t>(hip_stream), qkv, nullptr, B, L, H, dh, theta));
    return DLLM_OK;
}

int dllm_op_linear_qkv_rope(void *hip_stream, const void *A, const void *W, void *qkv, float *table, int32_t B,
                            int32_t L, int32_t H, int32_t dh, float theta)
{
    if (!A || !W || !qkv || !table) return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_qkv_rope: null argument");
    if (!aligned16(A) || !aligned16(W) || !aligned16(qkv) || !aligned16(table))
        return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_qkv_rope: pointers must be 16-byte aligned");
    if (B < 1 || L < 1 || H < 1 || !(theta > 0.0f) || (long)B * L > (1L << 24) || (long)H * dh > (1L << 20))
        return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_qkv_rope: bad shape");
    const int M = B * L, d = H * dh;
    if (!gemm_qkv_rope_supported(M, d, dh))
        return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_qkv_rope: shape not covered by the fused kernel");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    HIP_TRY(nullptr, launch_rope_table(st, reinterpret_cast<float2 *>(table), L, dh, theta));
    HIP_TRY(nullptr, launch_gemm_qkv_rope(st, A, W, qkv, M, d, dh, reinterpret_cast<const float2 *>(table), L));
    return DLLM_OK;
}

int dllm_op_linear_qkv_rope_static(void *hip_stream, const void *A, const void *W, void *qkv, int32_t B, int32_t L,
                                   int32_t H, int32_t dh, float theta)
{
    if (!A || !W || !qkv) return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_qkv_rope_static: null argument");
    if (!aligned16(A) || !aligned16(W) || !aligned16(qkv))
        return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_qkv_rope_static: pointers must be 16-byte aligned");
    if (B < 1 || L < 1 || H < 1 || !(theta > 0.0f) || (long)B * L > (1L << 24) || (long)H * dh > (1L << 20))
        return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_qkv_rope_static: bad shape");
    const int M = B * L, d = H * dh;
    if (!gemm_qkv_rope_supported(M, d, dh))
        return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_qkv_rope_static: shape not covered by the fused kernel");
    if ((size_t)L * (size_t)(dh / 2) > kStaticRopeEntries)
        return fail(nullptr, DLLM_EINVAL, "dllm_op_linear_qkv_rope_static: the rotary table of L = %d positions x %d pairs "
                                          "exceeds the built-in scratch of %zu entries (L <= %zu at this head_dim)",
                    L, dh / 2, kStaticRopeEntries, kStaticRopeEntries / (size_t)(dh / 2));
    float2 *table = nullptr;
    if (int rc = static_scratch(&table)) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    HIP_TRY(nullptr, launch_rope_table(st, table, L, dh, theta));
    HIP_TRY(nullptr, launch_gemm_qkv_rope(st, A, W, qkv, M, d, dh, table, L));
    return DLLM_OK;
}

int dllm_op_attention(void *hip_stream, const void *qkv, void *out, int32_t B, int32_t L, int32_t H, int32_t dh)
{
    if (!qkv || !out || !aligned16(qkv) || !aligned16(out)) return fail(nullptr, DLLM_EINVAL, "dllm_op_attention: null or misaligned pointer");
    if (B < 1 || L < 1 || H < 1 || (dh != 64 && dh != 128)) return fail(nullptr, DLLM_EINVAL, "dllm_op_attention: bad shape");
    if ((long)B > 65535 || (long)H > 65535) return fail(nullptr, DLLM_EINVAL, "dllm_op_attention: B and H must be <= 65535");
    if ((double)L * 3.0 * H * dh * 2.0 >= 4.0e9)
        return fail(nullptr, DLLM_EINVAL, "dllm_op_attention: one sequence of qkv must stay below 4 GB (32-bit offsets)");
    HIP_TRY(nullptr, launch_attention(static_cast<hipStream_t>(hip_stream), qkv, out, B, L, H, dh));
    return DLLM_OK;
}

}  // extern "C"
