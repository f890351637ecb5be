/*
 * CPU oracle for one denoising step of a masked-diffusion LLM: the mask
 * predictor's forward pass and the per-position greedy decode + confidence.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a slow, plain, fp64 statement of
 * what the GPU library must compute.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may load it; the product never does.  It shares
 * no code with the HIP kernels.
 *
 * Everything is written as the definition: triple-loop contractions, softmax
 * by explicit max / exp / sum, attention over every (query, key) pair.  No
 * blocking, no fusion.  OpenMP "parallel for" over independent rows is the
 * only parallelism.
 *
 * What the paper fixes (Section 3.1): the predictor returns a distribution
 * over the vocabulary at every position in one pass; the greedy estimate is
 * the arg max of that distribution (eq. 3) and the confidence is the
 * probability of that arg max (the confidence equation of "Low-Confidence
 * Remasking", repeated in the Certainty Principle).  The paper only says the
 * predictor is a bidirectional Transformer; the operator list (RMSNorm, RoPE,
 * non-causal multi-head attention, SwiGLU, vocabulary projection) is the
 * LLaDA-style stack this build targets.
 *
 * Layouts (all row-major):
 *   weights are bf16 bit patterns (uint16_t), a linear map is W[N][K] and
 *   y = x W^T;  wqkv rows are [q features | k features | v features], each
 *   head-major (h * head_dim + j);  w_gate_up rows are [gate | up].
 *   activations are double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab, mask_id;
    double rms_eps, rope_theta;
} orc_config;

typedef struct {
    const uint16_t *embed;      /* [vocab][d_model]  */
    const uint16_t *lm_head;    /* [vocab][d_model]  */
    const uint16_t *final_norm; /* [d_model]         */
    const uint16_t **attn_norm; /* n_layers x [d_model]            */
    const uint16_t **wqkv;      /* n_layers x [3 d_model][d_model] */
    const uint16_t **wo;        /* n_layers x [d_model][d_model]   */
    const uint16_t **ffn_norm;  /* n_layers x [d_model]            */
    const uint16_t **w_gate_up; /* n_layers x [2 d_ffn][d_model]   */
    const uint16_t **w_down;    /* n_layers x [d_model][d_ffn]     */
} orc_weights;

/* ---- bf16 <-> double ---------------------------------------------------- */

/* bf16 is the upper half of an IEEE binary32. Widening is exact. */
double orc_bf16_to_f64(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Round a double to the nearest bf16 (ties to even) in one rounding: bf16
 * keeps 8 significant bits, so a value in [2^e, 2^(e+1)) is a multiple of
 * 2^(e-7); below the normal range the spacing is fixed at 2^-133. */
uint16_t orc_f64_to_bf16(double x)
{
    if (isnan(x)) return 0x7fc0;
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    if (a == 0.0) return sign;
    if (isinf(a)) return sign | 0x7f80;
    int e;
    (void)frexp(a, &e); /* a = m * 2^e, m in [0.5,1)  ->  a in [2^(e-1), 2^e) */
    int ulp_exp = (e - 1) - 7;
    if (ulp_exp < -133) ulp_exp = -133;
    double q = nearbyint(ldexp(a, -ulp_exp)); /* default mode: ties to even */
    double r = ldexp(q, ulp_exp);
    if (r >= ldexp(1.0, 128)) return sign | 0x7f80;
    float f = (float)r; /* exact: r has at most 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return sign | (uint16_t)(u >> 16);
}

void orc_round_to_bf16(const double *x, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_f64_to_bf16(x[i]);
}

/* ---- the operators of the predictor ------------------------------------- */

/* RMSNorm: out = x / sqrt(mean(x^2) + eps) * g, per row. */
void orc_rmsnorm(const double *x, const uint16_t *g, int64_t rows, int d, double eps, double *out)
{
#pragma omp parallel for
    for (int64_t r = 0; r < rows; ++r) {
        double ss = 0.0;
        for (int j = 0; j < d; ++j) ss += x[r * d + j] * x[r * d + j];
        double inv = 1.0 / sqrt(ss / d + eps);
        for (int j = 0; j < d; ++j) out[r * d + j] = x[r * d + j] * inv * orc_bf16_to_f64(g[j]);
    }
}

/* y[r][n] = sum_k x[r][k] * W[n][k] */
void orc_linear(const double *x, const uint16_t *W, int64_t rows, int K, int N, double *y)
{
#pragma omp parallel for
    for (int n = 0; n < N; ++n) {
        double *wn = (double *)malloc(sizeof(double) * K); /* row n of W, widened once */
        for (int k = 0; k < K; ++k) wn[k] = orc_bf16_to_f64(W[(int64_t)n * K + k]);
        for (int64_t r = 0; r < rows; ++r) {
            const double *xr = x + r * K;
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int k = 0; k < K; ++k) acc += xr[k] * wn[k];
            y[r * (int64_t)N + n] = acc;
        }
        free(wn);
    }
}

/* Rotary position embedding, "rotate-half" pairing: inside each head the
 * coordinate pair (j, j + dh/2) at position p is rotated by the angle
 * p * theta^(-2j/dh).  x is [rows][n_heads][dh]; pos[r] is the position of row r. */
void orc_rope(double *x, const int32_t *pos, int64_t rows, int n_heads, int dh, double theta)
{
    int half = dh / 2;
#pragma omp parallel for
    for (int64_t r = 0; r < rows; ++r) {
        for (int h = 0; h < n_heads; ++h) {
            double *v = x + (r * n_heads + h) * dh;
            for (int j = 0; j < half; ++j) {
                double ang = (double)pos[r] * pow(theta, -2.0 * j / dh);
                double c = cos(ang), s = sin(ang);
                double a = v[j], b = v[j + half];
                v[j] = a * c - b * s;
                v[j + half] = a * s + b * c;
            }
        }
    }
}

/* Non-causal multi-head attention for one sequence: every query attends to
 * all L keys.  q, k, v, out are [L][n_heads][dh]. */
void orc_attention(const double *q, const double *k, const double *v, int L, int n_heads, int dh, double *out)
{
    double scale = 1.0 / sqrt((double)dh);
#pragma omp parallel for collapse(2)
    for (int i = 0; i < L; ++i) {
        for (int h = 0; h < n_heads; ++h) {
            double *p = (double *)malloc(sizeof(double) * L);
            const double *qi = q + ((int64_t)i * n_heads + h) * dh;
            double m = -INFINITY;
            for (int j = 0; j < L; ++j) {
                const double *kj = k + ((int64_t)j * n_heads + h) * dh;
                double s = 0.0;
                for (int t = 0; t < dh; ++t) s += qi[t] * kj[t];
                p[j] = s * scale;
                if (p[j] > m) m = p[j];
            }
            double z = 0.0;
            for (int j = 0; j < L; ++j) {
                p[j] = exp(p[j] - m);
                z += p[j];
            }
            double *o = out + ((int64_t)i * n_heads + h) * dh;
            for (int t = 0; t < dh; ++t) o[t] = 0.0;
            for (int j = 0; j < L; ++j) {
                const double *vj = v + ((int64_t)j * n_heads + h) * dh;
                double w = p[j] / z;
                for (int t = 0; t < dh; ++t) o[t] += w * vj[t];
            }
            free(p);
        }
    }
}

/* SwiGLU gate: out = silu(gate) * up,  silu(a) = a / (1 + exp(-a)). */
void orc_swiglu(const double *gate, const double *up, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = gate[i] / (1.0 + exp(-gate[i])) * up[i];
}

/* Full forward of the mask predictor (Section 3.1, eq. 2): token ids
 * [B][L] -> logits [B*L][vocab] in double.  Pre-norm residual blocks, no
 * biases, positions 0..L-1 inside each sequence, no attention mask.
 * If rows != NULL only the n_rows listed rows (indices into B*L) get a
 * vocabulary projection and logits is [n_rows][vocab]; the layers always run
 * on every position. */
int orc_forward(const orc_config *c, const orc_weights *w, const int32_t *tokens, int B, int L,
                const int32_t *rows, int n_rows, double *logits)
{
    const int d = c->d_model, H = c->n_heads, dh = c->head_dim, f = c->d_ffn;
    if (H * dh != d) return -1;
    const int64_t M = (int64_t)B * L;
    double *x = malloc(sizeof(double) * M * d);
    double *h = malloc(sizeof(double) * M * d);
    double *qkv = malloc(sizeof(double) * M * 3 * d);
    double *q = malloc(sizeof(double) * M * d);
    double *k = malloc(sizeof(double) * M * d);
    double *v = malloc(sizeof(double) * M * d);
    double *att = malloc(sizeof(double) * M * d);
    double *proj = malloc(sizeof(double) * M * d);
    double *gu = malloc(sizeof(double) * M * 2 * f);
    double *gate = malloc(sizeof(double) * M * f);
    double *up = malloc(sizeof(double) * M * f);
    double *act = malloc(sizeof(double) * M * f);
    int32_t *pos = malloc(sizeof(int32_t) * M);
    if (!x || !h || !qkv || !q || !k || !v || !att || !proj || !gu || !gate || !up || !act || !pos) return -2;

    for (int64_t r = 0; r < M; ++r) {
        int32_t t = tokens[r];
        if (t < 0 || t >= c->vocab) return -3;
        for (int j = 0; j < d; ++j) x[r * d + j] = orc_bf16_to_f64(w->embed[(int64_t)t * d + j]);
        pos[r] = (int32_t)(r % L);
    }
    for (int l = 0; l < c->n_layers; ++l) {
        /* attention block */
        orc_rmsnorm(x, w->attn_norm[l], M, d, c->rms_eps, h);
        orc_linear(h, w->wqkv[l], M, d, 3 * d, qkv);
        for (int64_t r = 0; r < M; ++r)
            for (int j = 0; j < d; ++j) {
                q[r * d + j] = qkv[r * 3 * d + j];
                k[r * d + j] = qkv[r * 3 * d + d + j];
                v[r * d + j] = qkv[r * 3 * d + 2 * d + j];
            }
        orc_rope(q, pos, M, H, dh, c->rope_theta);
        orc_rope(k, pos, M, H, dh, c->rope_theta);
        for (int b = 0; b < B; ++b) {
            int64_t o = (int64_t)b * L * d;
            orc_attention(q + o, k + o, v + o, L, H, dh, att + o);
        }
        orc_linear(att, w->wo[l], M, d, d, proj);
        for (int64_t i = 0; i < M * d; ++i) x[i] += proj[i];
        /* feed-forward block */
        orc_rmsnorm(x, w->ffn_norm[l], M, d, c->rms_eps, h);
        orc_linear(h, w->w_gate_up[l], M, d, 2 * f, gu);
        for (int64_t r = 0; r < M; ++r)
            for (int j = 0; j < f; ++j) {
                gate[r * f + j] = gu[r * 2 * f + j];
                up[r * f + j] = gu[r * 2 * f + f + j];
            }
        orc_swiglu(gate, up, M * f, act);
        orc_linear(act, w->w_down[l], M, f, d, proj);
        for (int64_t i = 0; i < M * d; ++i) x[i] += proj[i];
    }
    orc_rmsnorm(x, w->final_norm, M, d, c->rms_eps, h);
    if (rows) {
        for (int i = 0; i < n_rows; ++i) {
            if (rows[i] < 0 || rows[i] >= M) return -4;
            memcpy(x + (int64_t)i * d, h + (int64_t)rows[i] * d, sizeof(double) * d);
        }
        orc_linear(x, w->lm_head, n_rows, d, c->vocab, logits);
    } else {
        orc_linear(h, w->lm_head, M, d, c->vocab, logits);
    }

    free(x); free(h); free(qkv); free(q); free(k); free(v); free(att); free(proj);
    free(gu); free(gate); free(up); free(act); free(pos);
    return 0;
}

/* Attention of Lq queries over Lk keys (one sequence, no mask): q, out are
 * [Lq][n_heads][dh]; k, v are [Lk][n_heads][dh]. */
static void orc_attention_qk(const double *q, int Lq, const double *k, const double *v, int Lk, int n_heads, int dh,
                             double *out)
{
    double scale = 1.0 / sqrt((double)dh);
#pragma omp parallel for collapse(2)
    for (int i = 0; i < Lq; ++i) {
        for (int h = 0; h < n_heads; ++h) {
            double *p = (double *)malloc(sizeof(double) * Lk);
            const double *qi = q + ((int64_t)i * n_heads + h) * dh;
            double m = -INFINITY;
            for (int j = 0; j < Lk; ++j) {
                const double *kj = k + ((int64_t)j * n_heads + h) * dh;
                double s = 0.0;
                for (int t = 0; t < dh; ++t) s += qi[t] * kj[t];
                p[j] = s * scale;
                if (p[j] > m) m = p[j];
            }
            double z = 0.0;
            for (int j = 0; j < Lk; ++j) {
                p[j] = exp(p[j] - m);
                z += p[j];
            }
            double *o = out + ((int64_t)i * n_heads + h) * dh;
            for (int t = 0; t < dh; ++t) o[t] = 0.0;
            for (int j = 0; j < Lk; ++j) {
                const double *vj = v + ((int64_t)j * n_heads + h) * dh;
                double w = p[j] / z;
                for (int t = 0; t < dh; ++t) o[t] += w * vj[t];
            }
            free(p);
        }
    }
}

/* Forward with out-of-span caching (Section 3.3, "Out-of-Span Caching"; the
 * "cache features for position i" branch of Algorithm 1's fast phase).  The
 * features kept per position are, for every layer, its key (after the rotary
 * embedding) and its value: all that other positions ever read from it.
 *   kcache, vcache  [n_layers][B*L][d_model], in/out
 *   skip            [B*L] or NULL; skip[r] != 0: position r is not recomputed,
 *                   its cached keys/values of every layer are used as they are
 * Every other position is recomputed from the current tokens, attends to all
 * L positions of its sequence (fresh keys/values of recomputed positions,
 * cached ones of skipped positions), and overwrites its own cache rows.  With
 * skip == NULL this is the full forward that also fills the cache.
 *   rows / n_rows   rows (indices into B*L, none of them skipped) that get a
 *                   vocabulary projection; logits is [n_rows][vocab]. */
int orc_forward_cached(const orc_config *c, const orc_weights *w, const int32_t *tokens, int B, int L,
                       const uint8_t *skip, double *kcache, double *vcache, const int32_t *rows, int n_rows,
                       double *logits)
{
    const int d = c->d_model, H = c->n_heads, dh = c->head_dim, f = c->d_ffn;
    if (H * dh != d || !kcache || !vcache || !rows) return -1;
    const int64_t M = (int64_t)B * L;
    /* the positions that are recomputed, in order; cidx maps a row to its index among them */
    int32_t *act = malloc(sizeof(int32_t) * M), *cidx = malloc(sizeof(int32_t) * M);
    int32_t *first = malloc(sizeof(int32_t) * (B + 1));
    if (!act || !cidx || !first) return -2;
    int64_t Ma = 0;
    for (int b = 0; b < B; ++b) {
        first[b] = (int32_t)Ma;
        for (int i = 0; i < L; ++i) {
            int64_t r = (int64_t)b * L + i;
            cidx[r] = -1;
            if (!skip || !skip[r]) { cidx[r] = (int32_t)Ma; act[Ma++] = (int32_t)r; }
        }
    }
    first[B] = (int32_t)Ma;
    if (Ma == 0) { free(act); free(cidx); free(first); return n_rows == 0 ? 0 : -4; }
    double *x = malloc(sizeof(double) * Ma * d);
    double *h = malloc(sizeof(double) * Ma * d);
    double *qkv = malloc(sizeof(double) * Ma * 3 * d);
    double *q = malloc(sizeof(double) * Ma * d);
    double *k = malloc(sizeof(double) * Ma * d);
    double *v = malloc(sizeof(double) * Ma * d);
    double *att = malloc(sizeof(double) * Ma * d);
    double *proj = malloc(sizeof(double) * Ma * d);
    double *gu = malloc(sizeof(double) * Ma * 2 * f);
    double *gate = malloc(sizeof(double) * Ma * f);
    double *up = malloc(sizeof(double) * Ma * f);
    double *actv = malloc(sizeof(double) * Ma * f);
    int32_t *pos = malloc(sizeof(int32_t) * Ma);
    if (!x || !h || !qkv || !q || !k || !v || !att || !proj || !gu || !gate || !up || !actv || !pos) return -2;

    for (int64_t a = 0; a < Ma; ++a) {
        int32_t t = tokens[act[a]];
        if (t < 0 || t >= c->vocab) return -3;
        for (int j = 0; j < d; ++j) x[a * d + j] = orc_bf16_to_f64(w->embed[(int64_t)t * d + j]);
        pos[a] = act[a] % L;
    }
    for (int l = 0; l < c->n_layers; ++l) {
        double *kc = kcache + (int64_t)l * M * d, *vc = vcache + (int64_t)l * M * d;
        orc_rmsnorm(x, w->attn_norm[l], Ma, d, c->rms_eps, h);
        orc_linear(h, w->wqkv[l], Ma, d, 3 * d, qkv);
        for (int64_t a = 0; a < Ma; ++a)
            for (int j = 0; j < d; ++j) {
                q[a * d + j] = qkv[a * 3 * d + j];
                k[a * d + j] = qkv[a * 3 * d + d + j];
                v[a * d + j] = qkv[a * 3 * d + 2 * d + j];
            }
        orc_rope(q, pos, Ma, H, dh, c->rope_theta);
        orc_rope(k, pos, Ma, H, dh, c->rope_theta);
        /* recomputed positions refresh their cache rows; skipped ones keep theirs */
        for (int64_t a = 0; a < Ma; ++a) {
            memcpy(kc + (int64_t)act[a] * d, k + a * d, sizeof(double) * d);
            memcpy(vc + (int64_t)act[a] * d, v + a * d, sizeof(double) * d);
        }
        for (int b = 0; b < B; ++b) {
            int Lq = first[b + 1] - first[b];
            if (Lq == 0) continue;
            int64_t qo = (int64_t)first[b] * d, ko = (int64_t)b * L * d;
            orc_attention_qk(q + qo, Lq, kc + ko, vc + ko, L, H, dh, att + qo);
        }
        orc_linear(att, w->wo[l], Ma, d, d, proj);
        for (int64_t i = 0; i < Ma * d; ++i) x[i] += proj[i];
        orc_rmsnorm(x, w->ffn_norm[l], Ma, d, c->rms_eps, h);
        orc_linear(h, w->w_gate_up[l], Ma, d, 2 * f, gu);
        for (int64_t a = 0; a < Ma; ++a)
            for (int j = 0; j < f; ++j) {
                gate[a * f + j] = gu[a * 2 * f + j];
                up[a * f + j] = gu[a * 2 * f + f + j];
            }
        orc_swiglu(gate, up, Ma * f, actv);
        orc_linear(actv, w->w_down[l], Ma, f, d, proj);
        for (int64_t i = 0; i < Ma * d; ++i) x[i] += proj[i];
    }
    orc_rmsnorm(x, w->final_norm, Ma, d, c->rms_eps, h);
    for (int i = 0; i < n_rows; ++i) {
        if (rows[i] < 0 || rows[i] >= M || cidx[rows[i]] < 0) return -4;
        memcpy(x + (int64_t)i * d, h + (int64_t)cidx[rows[i]] * d, sizeof(double) * d);
    }
    if (n_rows > Ma) return -4;
    orc_linear(x, w->lm_head, n_rows, d, c->vocab, logits);

    free(x); free(h); free(qkv); free(q); free(k); free(v); free(att); free(proj);
    free(gu); free(gate); free(up); free(actv); free(pos); free(act); free(cidx); free(first);
    return 0;
}

/* ---- per-position greedy decode and confidence (eq. 3, confidence eq.) --- */

/* Softmax of one logits row by definition, with the [MASK] id removed from
 * the support (its probability is 0).  prob may be NULL. Returns the arg max
 * (lowest id among equal maxima) and writes the arg max's probability. */
int32_t orc_softmax_row(const uint16_t *logits, int V, int mask_id, double *prob, double *conf)
{
    double m = -INFINITY;
    int32_t arg = -1;
    for (int v = 0; v < V; ++v) {
        if (v == mask_id) continue;
        double x = orc_bf16_to_f64(logits[v]);
        if (x > m) { m = x; arg = v; }
    }
    double z = 0.0;
    for (int v = 0; v < V; ++v) {
        if (v == mask_id) continue;
        z += exp(orc_bf16_to_f64(logits[v]) - m);
    }
    if (prob)
        for (int v = 0; v < V; ++v)
            prob[v] = (v == mask_id) ? 0.0 : exp(orc_bf16_to_f64(logits[v]) - m) / z;
    *conf = 1.0 / z; /* exp(m - m) / z */
    return arg;
}

/* Row phase over a [rows][V] bf16 logits matrix.  Rows with active[r] == 0
 * are skipped (pred = -1, conf = 0).  conf is returned rounded to binary32,
 * the precision in which every later threshold and ranking decision is taken. */
void orc_row_phase(const uint16_t *logits, int64_t rows, int V, int mask_id, const uint8_t *active,
                   int32_t *pred, float *conf)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t r = 0; r < rows; ++r) {
        if (active && !active[r]) { pred[r] = -1; conf[r] = 0.0f; continue; }
        double c;
        pred[r] = orc_softmax_row(logits + r * (int64_t)V, V, mask_id, NULL, &c);
        conf[r] = (float)c;
    }
}
