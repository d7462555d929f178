/*
 * CPU oracle for the block-decode step of SDLM's Next Sequence Prediction
 * inference ("Sequential Diffusion Language Models", Sec. 3.2-3.4).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU library and
 * must never be linked, imported or called by it.
 *
 * Arithmetic: weights are read as given (fp32, or bf16 bit patterns widened
 * exactly); every sum, product, exponential and square root is IEEE double.
 * The only single-precision arithmetic is the acceptance decision (the
 * confidence is rounded to float, the cumulative product of Eq. (gamma_tau)
 * is a float product taken left to right, the comparison is >= on floats),
 * because that is the precision in which the GPU takes the same integer
 * decision.
 *
 * What is computed (paper notation):
 *   - block input  X_T = [x_last, [m] x (D-1)]            (training objective, Sec. 3.2)
 *   - attention mask A_uv = 1{v<=u} OR 1{u>=s and v>=s}    (Sec. 3.3; the printed
 *     operator is a circled plus, read as OR because the following sentence
 *     demands full mutual attention inside the block)
 *   - logits Z in R^{D x |V|} of the D block rows            (Sec. 3.2)
 *   - logit confidence  p = softmax(z)_argmax                (Sec. 3.4, item (1))
 *   - entropy confidence p = 1 - H/log|V|                    (Sec. 3.4, item (2))
 *   - gamma_tau = max({j : prod_{k<=j} p_k >= tau} U {1})    (Sec. 3.4, greedy decoding)
 *   - Decode(Z, gamma): first gamma argmax tokens            (Sec. 3.2)
 * The decoder itself is the Qwen-2.5 architecture the paper fine-tunes
 * (Sec. 4.1): pre-norm RMSNorm, rotary embedding (rotate-half), grouped-query
 * attention with 1/sqrt(d) scaling, SwiGLU feed-forward, untied LM head.
 *
 * Three independent routes to the same logits are provided so that they can
 * be checked against one another:
 *   orc_brute_step   - no cache: full forward over [x^0..x^{n-1}, m..m] with the
 *                      dense mask A written out as a matrix;
 *   orc_seq_*        - incremental: a cache that only ever holds K/V of real
 *                      tokens computed under causal attention, "pending" rows
 *                      for the tokens accepted last step, D block rows;
 *   orc_ntp_logits   - a textbook causal next-token decoder (block size 1).
 *
 * Parity pins: tests/test_oracle_*.py (closed forms, a hand-worked micro model,
 * a library cross-check, brute == cached == textbook).  End-to-end agreement
 * with a *trained* SDLM checkpoint is unpinned: no weights are available.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    int32_t mask_token_id, has_qkv_bias;
    int32_t wdtype;              /* 0: float32 arrays, 1: bf16 bit patterns (uint16) */
    double rope_theta, rms_eps, logit_scale;
    int32_t bf16_points;         /* 1: round activations to bf16 at the points where a bf16 pipeline does (see round_rows) */
    int32_t block_causal;        /* 1: the ablation of Sec. 4.4 "Causal Attention": causal instead of mutual attention inside the block */
} orc_cfg;

typedef struct {
    const void *embed, *lm_head, *final_norm;          /* [V,h] [V,h] [h] */
    const void *const *attn_norm, *const *wq, *const *wk, *const *wv, *const *wo;
    const void *const *bq, *const *bk, *const *bv;    /* entries may be NULL */
    const void *const *ffn_norm, *const *w_gate, *const *w_up, *const *w_down;
} orc_weights;

/* Threads the OpenMP loops use (for reporting only). */
int32_t orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- helpers */

static double wget(const void *p, int wdtype, size_t i)
{
    if (wdtype == 0)
        return (double)((const float *)p)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}

/*
 * Optional model of a bf16 pipeline's rounding points.  The plain oracle (bf16_points = 0) keeps every
 * intermediate in double.  With bf16_points = 1 the tensors that a bf16 matrix-core implementation has to hand to
 * its contractions are rounded to bf16 (nearest even) where such an implementation rounds them: the output of
 * every RMSNorm, the rotated queries and keys and the values, the softmax weights entering the weighted sum of
 * values (their normaliser stays unrounded), the attention output, and the SwiGLU activation.  Nothing else
 * changes.  This separates rounding noise, which no bf16 implementation can avoid, from errors.
 */
static double round_bf16(double v)
{
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return v;
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

static void round_rows(const orc_cfg *c, double *x, size_t n)
{
    if (!c->bf16_points) return;
    for (size_t i = 0; i < n; ++i) x[i] = round_bf16(x[i]);
}

/* y[r][o] = sum_k x[r][k] * W[o][k] (+ b[o]);  W is [n_out, n_in] row-major. */
static void dense(double *y, const double *x, const void *W, const void *b,
                  int wdtype, int rows, int n_in, int n_out)
{
#pragma omp parallel
    {
        double *wr = malloc(sizeof(double) * (size_t)n_in);   /* row o of W, widened */
#pragma omp for schedule(static)
        for (int o = 0; o < n_out; ++o) {
            double bias = b ? wget(b, wdtype, (size_t)o) : 0.0;
            for (int k = 0; k < n_in; ++k) wr[k] = wget(W, wdtype, (size_t)o * n_in + k);
            for (int r = 0; r < rows; ++r) {
                const double *xr = x + (size_t)r * n_in;
                double acc = 0.0;
#pragma omp simd reduction(+ : acc)
                for (int k = 0; k < n_in; ++k) acc += xr[k] * wr[k];
                y[(size_t)r * n_out + o] = acc + bias;
            }
        }
        free(wr);
    }
}

/* RMSNorm: y = x * g / sqrt(mean(x^2) + eps), row by row. */
static void rmsnorm(double *y, const double *x, const void *g, int wdtype,
                    int rows, int h, double eps)
{
    for (int r = 0; r < rows; ++r) {
        const double *xr = x + (size_t)r * h;
        double ss = 0.0;
        for (int k = 0; k < h; ++k) ss += xr[k] * xr[k];
        double inv = 1.0 / sqrt(ss / h + eps);
        for (int k = 0; k < h; ++k) y[(size_t)r * h + k] = xr[k] * inv * wget(g, wdtype, (size_t)k);
    }
}

/* Rotary embedding, rotate-half pairing (i, i + d/2), on one head vector at position pos. */
static void rope(double *v, int d, int pos, double theta)
{
    int half = d / 2;
    for (int i = 0; i < half; ++i) {
        double ang = (double)pos * pow(theta, -2.0 * i / d);
        double c = cos(ang), s = sin(ang);
        double a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

static double silu(double x) { return x / (1.0 + exp(-x)); }

static void embed_rows(double *x, const orc_cfg *c, const orc_weights *w, const int32_t *ids, int rows)
{
    for (int r = 0; r < rows; ++r)
        for (int k = 0; k < c->hidden; ++k)
            x[(size_t)r * c->hidden + k] = wget(w->embed, c->wdtype, (size_t)ids[r] * c->hidden + k);
}

/* q,k,v projections of normed rows, then RoPE on q and k at the rows' positions. */
static void qkv_rope(double *q, double *k, double *v, const double *xn, const orc_cfg *c,
                     const orc_weights *w, int l, int rows, const int32_t *pos)
{
    int h = c->hidden, d = c->head_dim, qd = c->n_q_heads * d, kd = c->n_kv_heads * d;
    int bias = c->has_qkv_bias;
    dense(q, xn, w->wq[l], bias ? w->bq[l] : NULL, c->wdtype, rows, h, qd);
    dense(k, xn, w->wk[l], bias ? w->bk[l] : NULL, c->wdtype, rows, h, kd);
    dense(v, xn, w->wv[l], bias ? w->bv[l] : NULL, c->wdtype, rows, h, kd);
    for (int r = 0; r < rows; ++r) {
        for (int hq = 0; hq < c->n_q_heads; ++hq) rope(q + (size_t)r * qd + hq * d, d, pos[r], c->rope_theta);
        for (int hk = 0; hk < c->n_kv_heads; ++hk) rope(k + (size_t)r * kd + hk * d, d, pos[r], c->rope_theta);
    }
    round_rows(c, q, (size_t)rows * qd);
    round_rows(c, k, (size_t)rows * kd);
    round_rows(c, v, (size_t)rows * kd);
}

/* x += att * Wo ; x += (silu(xn Wg) * (xn Wu)) Wd   (second half of a decoder layer) */
static void out_and_ffn(double *x, const double *att, const orc_cfg *c, const orc_weights *w, int l, int rows)
{
    int h = c->hidden, qd = c->n_q_heads * c->head_dim, F = c->ffn;
    double *t = malloc(sizeof(double) * (size_t)rows * h);
    double *xn = malloc(sizeof(double) * (size_t)rows * h);
    double *g = malloc(sizeof(double) * (size_t)rows * F);
    double *u = malloc(sizeof(double) * (size_t)rows * F);
    dense(t, att, w->wo[l], NULL, c->wdtype, rows, qd, h);
    for (size_t i = 0; i < (size_t)rows * h; ++i) x[i] += t[i];
    rmsnorm(xn, x, w->ffn_norm[l], c->wdtype, rows, h, c->rms_eps);
    round_rows(c, xn, (size_t)rows * h);
    dense(g, xn, w->w_gate[l], NULL, c->wdtype, rows, h, F);
    dense(u, xn, w->w_up[l], NULL, c->wdtype, rows, h, F);
    for (size_t i = 0; i < (size_t)rows * F; ++i) g[i] = silu(g[i]) * u[i];
    round_rows(c, g, (size_t)rows * F);
    dense(t, g, w->w_down[l], NULL, c->wdtype, rows, F, h);
    for (size_t i = 0; i < (size_t)rows * h; ++i) x[i] += t[i];
    free(t); free(xn); free(g); free(u);
}

/* Z = logit_scale * RMSNorm_final(x) W_lm^T for the given rows. */
static void lm_head(double *logits, const double *x, const orc_cfg *c, const orc_weights *w, int rows)
{
    int h = c->hidden, V = c->vocab;
    double *xn = malloc(sizeof(double) * (size_t)rows * h);
    rmsnorm(xn, x, w->final_norm, c->wdtype, rows, h, c->rms_eps);
    round_rows(c, xn, (size_t)rows * h);
    dense(logits, xn, w->lm_head, NULL, c->wdtype, rows, h, V);
    for (size_t i = 0; i < (size_t)rows * V; ++i) logits[i] *= c->logit_scale;
    free(xn);
}

/* ------------------------------------------------- confidence and gamma */

/* argmax with the lowest index winning exact ties */
int32_t orc_argmax(const double *z, int32_t V)
{
    int32_t best = 0;
    for (int32_t v = 1; v < V; ++v)
        if (z[v] > z[best]) best = v;
    return best;
}

/* Logit-value confidence: softmax(z)[argmax z] = 1 / sum_v exp(z_v - max z). */
double orc_conf_logit(const double *z, int32_t V)
{
    double m = z[orc_argmax(z, V)], s = 0.0;
    for (int32_t v = 0; v < V; ++v) s += exp(z[v] - m);
    return 1.0 / s;
}

/* Entropy-normalised confidence: 1 - H(softmax(z)) / log|V|. */
double orc_conf_entropy(const double *z, int32_t V)
{
    double m = z[orc_argmax(z, V)], s = 0.0;
    for (int32_t v = 0; v < V; ++v) s += exp(z[v] - m);
    double H = 0.0;
    for (int32_t v = 0; v < V; ++v) {
        double p = exp(z[v] - m) / s;
        if (p > 0.0) H -= p * log(p);
    }
    return 1.0 - H / log((double)V);
}

/*
 * Longest-prefix length.  rule 0: the paper's rule, the largest j whose
 * cumulative product of confidences is >= tau, never below 1.  rule 1: the
 * number of leading positions whose own confidence is >= tau, never below 1
 * (the phrasing "first position whose confidence falls below tau").
 */
int32_t orc_gamma(const float *conf, int32_t D, float tau, int32_t rule)
{
    int32_t best = 1;
    if (rule == 0) {
        float prod = 1.0f;
        for (int32_t j = 1; j <= D; ++j) {
            prod = prod * conf[j - 1];
            if (prod >= tau && j > best) best = j;
        }
    } else {
        int32_t j = 0;
        while (j < D && conf[j] >= tau) ++j;
        if (j > best) best = j;
    }
    return best;
}

/* ids, conf (as float) and gamma from D rows of logits. */
static void decide(const double *logits, const orc_cfg *c, int D, float tau, int rule, int conf_fn,
                   int32_t *ids, float *conf, int32_t *gamma)
{
    for (int k = 0; k < D; ++k) {
        const double *z = logits + (size_t)k * c->vocab;
        ids[k] = orc_argmax(z, c->vocab);
        conf[k] = (float)(conf_fn == 0 ? orc_conf_logit(z, c->vocab) : orc_conf_entropy(z, c->vocab));
    }
    *gamma = orc_gamma(conf, D, tau, rule);
}

/* ------------------------------------------------------ 1. brute force */

/*
 * Forward over T rows (ids, positions 0..T-1) under an explicit T x T 0/1 mask
 * (mask[u*T+v] = 1 iff row u may attend to row v).  Writes the final residual
 * stream x_out [T, hidden].
 */
static void forward_masked(double *x, const orc_cfg *c, const orc_weights *w,
                           const int32_t *ids, int T, const uint8_t *mask)
{
    int h = c->hidden, d = c->head_dim, Hq = c->n_q_heads, Hk = c->n_kv_heads;
    int qd = Hq * d, kd = Hk * d, G = Hq / Hk;
    double *xn = malloc(sizeof(double) * (size_t)T * h);
    double *q = malloc(sizeof(double) * (size_t)T * qd);
    double *k = malloc(sizeof(double) * (size_t)T * kd);
    double *v = malloc(sizeof(double) * (size_t)T * kd);
    double *att = malloc(sizeof(double) * (size_t)T * qd);
    int32_t *pos = malloc(sizeof(int32_t) * (size_t)T);
    for (int r = 0; r < T; ++r) pos[r] = r;
    embed_rows(x, c, w, ids, T);
    for (int l = 0; l < c->n_layers; ++l) {
        rmsnorm(xn, x, w->attn_norm[l], c->wdtype, T, h, c->rms_eps);
        round_rows(c, xn, (size_t)T * h);
        qkv_rope(q, k, v, xn, c, w, l, T, pos);
#pragma omp parallel for schedule(dynamic)
        for (int u = 0; u < T; ++u) {
            double *sc = malloc(sizeof(double) * (size_t)T);
            for (int hq = 0; hq < Hq; ++hq) {
                int hk = hq / G;
                const double *qu = q + (size_t)u * qd + hq * d;
                double m = -INFINITY;
                for (int t = 0; t < T; ++t) {
                    if (!mask[(size_t)u * T + t]) continue;
                    const double *kt = k + (size_t)t * kd + hk * d;
                    double s = 0.0;
                    for (int i = 0; i < d; ++i) s += qu[i] * kt[i];
                    sc[t] = s / sqrt((double)d);
                    if (sc[t] > m) m = sc[t];
                }
                double den = 0.0;
                for (int t = 0; t < T; ++t)
                    if (mask[(size_t)u * T + t]) den += exp(sc[t] - m);
                double *o = att + (size_t)u * qd + hq * d;
                for (int i = 0; i < d; ++i) o[i] = 0.0;
                for (int t = 0; t < T; ++t) {
                    if (!mask[(size_t)u * T + t]) continue;
                    double p = (c->bf16_points ? round_bf16(exp(sc[t] - m)) : exp(sc[t] - m)) / den;
                    const double *vt = v + (size_t)t * kd + hk * d;
                    for (int i = 0; i < d; ++i) o[i] += p * vt[i];
                }
            }
            free(sc);
        }
        round_rows(c, att, (size_t)T * qd);
        out_and_ffn(x, att, c, w, l, T);
    }
    free(xn); free(q); free(k); free(v); free(att); free(pos);
}

/*
 * Logits of rows [r0, r0+nr) of a forward over `ids` under an arbitrary mask.
 * Exposed so that tests can probe the mask's effect directly.
 */
int orc_forward_masked_logits(const orc_cfg *c, const orc_weights *w, const int32_t *ids, int32_t T,
                              const uint8_t *mask, int32_t r0, int32_t nr, double *logits)
{
    double *x = malloc(sizeof(double) * (size_t)T * c->hidden);
    forward_masked(x, c, w, ids, T, mask);
    lm_head(logits, x + (size_t)r0 * c->hidden, c, w, nr);
    free(x);
    return 0;
}

/*
 * The inference mask for known length n and block size D: T = n + D - 1, block start s = n - 1.
 * causal != 0 gives the ablation's variant: the block's rows attend causally too, i.e. the plain lower triangle.
 */
void orc_block_mask(uint8_t *mask, int32_t n, int32_t D, int32_t causal)
{
    int T = n + D - 1, s = n - 1;
    for (int u = 0; u < T; ++u)
        for (int v = 0; v < T; ++v)
            mask[(size_t)u * T + v] = (uint8_t)((v <= u) || (!causal && u >= s && v >= s));
}

/*
 * One decode step by full recomputation.  tokens[0..n) are the known tokens.
 * Outputs: logits [D,V] (may be NULL), ids[D], conf[D], *gamma.
 */
int orc_brute_step(const orc_cfg *c, const orc_weights *w, const int32_t *tokens, int32_t n, int32_t D,
                   float tau, int32_t rule, int32_t conf_fn,
                   double *logits_out, int32_t *ids, float *conf, int32_t *gamma)
{
    if (n < 1 || D < 1) return -1;
    int T = n + D - 1;
    int32_t *u = malloc(sizeof(int32_t) * (size_t)T);
    uint8_t *mask = malloc((size_t)T * T);
    for (int i = 0; i < n; ++i) u[i] = tokens[i];
    for (int i = n; i < T; ++i) u[i] = c->mask_token_id;
    orc_block_mask(mask, n, D, c->block_causal);
    double *logits = logits_out ? logits_out : malloc(sizeof(double) * (size_t)D * c->vocab);
    orc_forward_masked_logits(c, w, u, T, mask, n - 1, D, logits);
    decide(logits, c, D, tau, rule, conf_fn, ids, conf, gamma);
    if (!logits_out) free(logits);
    free(u); free(mask);
    return 0;
}

/* ---------------------------------------- 2. textbook next-token decoder */

/* Logits of the next token after tokens[0..n): plain causal decoder, no mask matrix. */
int orc_ntp_logits(const orc_cfg *c, const orc_weights *w, const int32_t *tokens, int32_t n, double *logits)
{
    int h = c->hidden, d = c->head_dim, Hq = c->n_q_heads, Hk = c->n_kv_heads;
    int qd = Hq * d, kd = Hk * d, G = Hq / Hk;
    double *x = malloc(sizeof(double) * (size_t)n * h), *xn = malloc(sizeof(double) * (size_t)n * h);
    double *q = malloc(sizeof(double) * (size_t)n * qd), *k = malloc(sizeof(double) * (size_t)n * kd);
    double *v = malloc(sizeof(double) * (size_t)n * kd), *att = malloc(sizeof(double) * (size_t)n * qd);
    double *sc = malloc(sizeof(double) * (size_t)n);
    int32_t *pos = malloc(sizeof(int32_t) * (size_t)n);
    for (int r = 0; r < n; ++r) pos[r] = r;
    embed_rows(x, c, w, tokens, n);
    for (int l = 0; l < c->n_layers; ++l) {
        rmsnorm(xn, x, w->attn_norm[l], c->wdtype, n, h, c->rms_eps);
        round_rows(c, xn, (size_t)n * h);
        qkv_rope(q, k, v, xn, c, w, l, n, pos);
        for (int u = 0; u < n; ++u)
            for (int hq = 0; hq < Hq; ++hq) {
                int hk = hq / G;
                double m = -INFINITY, den = 0.0;
                for (int t = 0; t <= u; ++t) {
                    double s = 0.0;
                    for (int i = 0; i < d; ++i) s += q[(size_t)u * qd + hq * d + i] * k[(size_t)t * kd + hk * d + i];
                    sc[t] = s / sqrt((double)d);
                    if (sc[t] > m) m = sc[t];
                }
                for (int t = 0; t <= u; ++t) den += exp(sc[t] - m);
                for (int i = 0; i < d; ++i) {
                    double o = 0.0;
                    for (int t = 0; t <= u; ++t)
                        o += (c->bf16_points ? round_bf16(exp(sc[t] - m)) : exp(sc[t] - m)) / den * v[(size_t)t * kd + hk * d + i];
                    att[(size_t)u * qd + hq * d + i] = o;
                }
            }
        round_rows(c, att, (size_t)n * qd);
        out_and_ffn(x, att, c, w, l, n);
    }
    lm_head(logits, x + (size_t)(n - 1) * h, c, w, 1);
    free(x); free(xn); free(q); free(k); free(v); free(att); free(sc); free(pos);
    return 0;
}

/* ------------------------------------------ 3. incremental (cached) route */

/*
 * One sequence.  tokens[0..n) are known; the cache holds K/V for positions
 * [0, c) and those entries are the K/V of the real token at that position
 * computed under causal attention.  Tokens [c, n) are "pending": accepted but
 * not cached yet.  A step feeds the pending tokens as causal rows (their K/V
 * go to the cache slots of their positions) followed by the D block rows
 * (x_last again at position s = n-1, then D-1 masks), whose K/V are used
 * inside the step and then discarded.
 */
typedef struct {
    orc_cfg cfg;
    const orc_weights *w;
    int32_t max_len, n, c;
    int32_t *tokens;
    double *K, *V;             /* [L][max_len][Hk*d] */
    int32_t step_valid;        /* a step has been computed since the last commit */
    int32_t last_D;
    int32_t *last_ids;
    int32_t last_gamma;
} orc_seq;

orc_seq *orc_seq_new(const orc_cfg *c, const orc_weights *w, int32_t max_len)
{
    orc_seq *s = calloc(1, sizeof(orc_seq));
    s->cfg = *c; s->w = w; s->max_len = max_len;
    size_t kv = (size_t)c->n_layers * max_len * c->n_kv_heads * c->head_dim;
    s->K = malloc(sizeof(double) * kv);
    s->V = malloc(sizeof(double) * kv);
    s->tokens = malloc(sizeof(int32_t) * (size_t)max_len);
    s->last_ids = malloc(sizeof(int32_t) * 64);
    return s;
}

void orc_seq_free(orc_seq *s)
{
    if (!s) return;
    free(s->K); free(s->V); free(s->tokens); free(s->last_ids); free(s);
}

int32_t orc_seq_len(const orc_seq *s) { return s->n; }
int32_t orc_seq_cached(const orc_seq *s) { return s->c; }
const int32_t *orc_seq_tokens(const orc_seq *s) { return s->tokens; }

/*
 * Rows = the (n - c) pending tokens, then n_block block rows.  Pending K/V are
 * written to the cache; logits of the block rows go to logits_out.
 */
static int seq_forward(orc_seq *s, int n_block, double *logits_out)
{
    const orc_cfg *c = &s->cfg;
    const orc_weights *w = s->w;
    int h = c->hidden, d = c->head_dim, Hq = c->n_q_heads, Hk = c->n_kv_heads;
    int qd = Hq * d, kd = Hk * d, G = Hq / Hk;
    int p = s->n - s->c, R = p + n_block, st = s->n - 1;
    if (n_block > 0 && st + n_block > s->max_len) return -2;
    if (R == 0) return 0;
    int32_t *ids = malloc(sizeof(int32_t) * (size_t)R), *pos = malloc(sizeof(int32_t) * (size_t)R);
    for (int r = 0; r < p; ++r) { ids[r] = s->tokens[s->c + r]; pos[r] = s->c + r; }
    for (int j = 0; j < n_block; ++j) {
        ids[p + j] = j == 0 ? s->tokens[s->n - 1] : c->mask_token_id;
        pos[p + j] = st + j;
    }
    double *x = malloc(sizeof(double) * (size_t)R * h), *xn = malloc(sizeof(double) * (size_t)R * h);
    double *q = malloc(sizeof(double) * (size_t)R * qd), *k = malloc(sizeof(double) * (size_t)R * kd);
    double *v = malloc(sizeof(double) * (size_t)R * kd), *att = malloc(sizeof(double) * (size_t)R * qd);
    embed_rows(x, c, w, ids, R);
    for (int l = 0; l < c->n_layers; ++l) {
        double *Kc = s->K + (size_t)l * s->max_len * kd, *Vc = s->V + (size_t)l * s->max_len * kd;
        rmsnorm(xn, x, w->attn_norm[l], c->wdtype, R, h, c->rms_eps);
        round_rows(c, xn, (size_t)R * h);
        qkv_rope(q, k, v, xn, c, w, l, R, pos);
        /* pending rows: their K/V are final; place them in the cache */
        for (int r = 0; r < p; ++r) {
            memcpy(Kc + (size_t)pos[r] * kd, k + (size_t)r * kd, sizeof(double) * kd);
            memcpy(Vc + (size_t)pos[r] * kd, v + (size_t)r * kd, sizeof(double) * kd);
        }
#pragma omp parallel for schedule(dynamic)
        for (int r = 0; r < R; ++r) {
            int is_block = r >= p;
            /* visible cache keys: causal row at position q sees [0, q]; a block row sees
               [0, s) (not the causal copy of x_last at s) and then the D block keys */
            int n_cache = is_block ? st : pos[r] + 1;
            /* block keys: all of the block, or (causal variant) the block rows up to this one */
            int n_keys = n_cache + (is_block ? (c->block_causal ? r - p + 1 : n_block) : 0);
            double *sc = malloc(sizeof(double) * (size_t)n_keys);
            for (int hq = 0; hq < Hq; ++hq) {
                int hk = hq / G;
                const double *qu = q + (size_t)r * qd + hq * d;
                double m = -INFINITY, den = 0.0;
                for (int t = 0; t < n_keys; ++t) {
                    const double *kt = t < n_cache ? Kc + (size_t)t * kd + hk * d
                                                   : k + (size_t)(p + t - n_cache) * kd + hk * d;
                    double a = 0.0;
                    for (int i = 0; i < d; ++i) a += qu[i] * kt[i];
                    sc[t] = a / sqrt((double)d);
                    if (sc[t] > m) m = sc[t];
                }
                for (int t = 0; t < n_keys; ++t) den += exp(sc[t] - m);
                double *o = att + (size_t)r * qd + hq * d;
                for (int i = 0; i < d; ++i) o[i] = 0.0;
                for (int t = 0; t < n_keys; ++t) {
                    const double *vt = t < n_cache ? Vc + (size_t)t * kd + hk * d
                                                   : v + (size_t)(p + t - n_cache) * kd + hk * d;
                    double pr = (c->bf16_points ? round_bf16(exp(sc[t] - m)) : exp(sc[t] - m)) / den;
                    for (int i = 0; i < d; ++i) o[i] += pr * vt[i];
                }
            }
            free(sc);
        }
        round_rows(c, att, (size_t)R * qd);
        out_and_ffn(x, att, c, w, l, R);
    }
    if (n_block > 0 && logits_out) lm_head(logits_out, x + (size_t)p * h, c, w, n_block);
    free(ids); free(pos); free(x); free(xn); free(q); free(k); free(v); free(att);
    return 0;
}

/* Causal forward over a prompt; afterwards c = n = len. */
int orc_seq_prefill(orc_seq *s, const int32_t *ids, int32_t len)
{
    if (len < 1 || len > s->max_len) return -1;
    memcpy(s->tokens, ids, sizeof(int32_t) * (size_t)len);
    s->n = len; s->c = 0; s->step_valid = 0;
    int rc = seq_forward(s, 0, NULL);
    s->c = s->n;
    return rc;
}

/* One block-decode step.  Does not change n or c; may be repeated. */
int orc_seq_step(orc_seq *s, int32_t D, float tau, int32_t rule, int32_t conf_fn,
                 double *logits_out, int32_t *ids, float *conf, int32_t *gamma)
{
    if (D < 1 || D > 64 || s->n < 1) return -1;
    double *logits = logits_out ? logits_out : malloc(sizeof(double) * (size_t)D * s->cfg.vocab);
    int rc = seq_forward(s, D, logits);
    if (rc == 0) {
        decide(logits, &s->cfg, D, tau, rule, conf_fn, ids, conf, gamma);
        memcpy(s->last_ids, ids, sizeof(int32_t) * (size_t)D);
        s->last_gamma = *gamma; s->last_D = D; s->step_valid = 1;
    }
    if (!logits_out) free(logits);
    return rc;
}

/*
 * Publish the step: the pending K/V become cache (c = n) and `count` tokens are
 * appended as the next step's pending tokens.  ids == NULL commits the step's
 * own first gamma tokens.
 */
int orc_seq_commit(orc_seq *s, const int32_t *ids, int32_t count)
{
    if (!s->step_valid) return -3;
    if (!ids) { ids = s->last_ids; count = s->last_gamma; }
    if (count < 1 || count > s->last_D || s->n + count > s->max_len) return -1;
    s->c = s->n;
    memcpy(s->tokens + s->n, ids, sizeof(int32_t) * (size_t)count);
    s->n += count;
    s->step_valid = 0;
    return 0;
}

/* ------------------------------- self-speculative verification (Sec. 3.4, Eq. 10) */

/*
 * gamma_verify from the speculative tokens yhat[0..D) and the verification
 * predictions ytilde[0..D).  rule 1 is the equation as printed: the largest j
 * with yhat^j == ytilde^j, or 1.  rule 0 is the reading used by default: the
 * longest prefix on which every position agrees (ytilde^j is computed with
 * yhat^1..yhat^{j-1} as context, so it says nothing once one of them is wrong),
 * or 1.
 */
int32_t orc_gamma_verify(const int32_t *yhat, const int32_t *ytilde, int32_t D, int32_t rule)
{
    int32_t best = 1;
    if (rule == 1) {
        for (int32_t j = 1; j <= D; ++j)
            if (yhat[j - 1] == ytilde[j - 1] && j > best) best = j;
    } else {
        int32_t j = 0;
        while (j < D && yhat[j] == ytilde[j]) ++j;
        if (j > best) best = j;
    }
    return best;
}

/* A deep copy of the sequence with room for max_len positions. */
static orc_seq *seq_clone(const orc_seq *s, int32_t max_len)
{
    orc_seq *t = orc_seq_new(&s->cfg, s->w, max_len);
    size_t kd = (size_t)s->cfg.n_kv_heads * s->cfg.head_dim;
    t->n = s->n; t->c = s->c;
    memcpy(t->tokens, s->tokens, sizeof(int32_t) * (size_t)s->n);
    for (int l = 0; l < s->cfg.n_layers; ++l) {
        memcpy(t->K + (size_t)l * max_len * kd, s->K + (size_t)l * s->max_len * kd, sizeof(double) * (size_t)s->n * kd);
        memcpy(t->V + (size_t)l * max_len * kd, s->V + (size_t)l * s->max_len * kd, sizeof(double) * (size_t)s->n * kd);
    }
    return t;
}

/*
 * Second pass of a self-speculative step, after orc_seq_step produced the D
 * speculative tokens yhat.  Verification input j (j = 1..D) is the sequence
 * extended by yhat^1..yhat^{j-1} with the mask tokens following it, i.e. exactly
 * the input of an ordinary block-decode step on that longer sequence; ytilde^j is
 * the token that step predicts first.  Input 1 is the first pass itself, so
 * ytilde^1 = yhat^1.  Each input is run on its own copy of the sequence.
 * logits_out (optional) [D][V]: row j-1 = the logits ytilde^j was taken from (row 0
 * is not written).  On success the step's gamma becomes gamma_verify, which is
 * what a commit without arguments then publishes.
 */
int orc_seq_verify(orc_seq *s, int32_t rule, double *logits_out, int32_t *ytilde, int32_t *gamma)
{
    if (!s->step_valid) return -3;
    const int D = s->last_D, V = s->cfg.vocab;
    ytilde[0] = s->last_ids[0];
    double *z = malloc(sizeof(double) * (size_t)D * V);
    int32_t *ids = malloc(sizeof(int32_t) * (size_t)D);
    float *conf = malloc(sizeof(float) * (size_t)D);
    int rc = 0;
    for (int j = 2; j <= D && rc == 0; ++j) {
        orc_seq *t = seq_clone(s, s->n + 2 * D);
        t->step_valid = 1; t->last_D = D;
        rc = orc_seq_commit(t, s->last_ids, j - 1);
        int32_t g;
        if (rc == 0) rc = orc_seq_step(t, D, 1.0f, 0, 0, z, ids, conf, &g);
        if (rc == 0) {
            ytilde[j - 1] = ids[0];
            if (logits_out) memcpy(logits_out + (size_t)(j - 1) * V, z, sizeof(double) * (size_t)V);
        }
        orc_seq_free(t);
    }
    if (rc == 0) {
        *gamma = orc_gamma_verify(s->last_ids, ytilde, D, rule);
        s->last_gamma = *gamma;
    }
    free(z); free(ids); free(conf);
    return rc;
}

/* Read back a cached K or V vector (layer, position, kv head) for tests. */
int orc_seq_read_kv(const orc_seq *s, int32_t layer, int32_t pos, int32_t kv_head, double *k_out, double *v_out)
{
    int d = s->cfg.head_dim, kd = s->cfg.n_kv_heads * d;
    if (pos < 0 || pos >= s->c) return -1;
    size_t off = ((size_t)layer * s->max_len + pos) * kd + (size_t)kv_head * d;
    memcpy(k_out, s->K + off, sizeof(double) * d);
    memcpy(v_out, s->V + off, sizeof(double) * d);
    return 0;
}

/* ------------------------------------------------- single-output probes */

/*
 * Outputs that can be computed one at a time, for checks at sizes where a whole
 * forward is out of reach.  Each takes its inputs as plain double arrays.
 */

/* One logit: logit_scale * <xhat, W_lm[v]> where xhat is an already normalised row. */
double orc_probe_logit(const orc_cfg *c, const orc_weights *w, const double *xhat, int32_t v)
{
    double acc = 0.0;
    for (int k = 0; k < c->hidden; ++k) acc += xhat[k] * wget(w->lm_head, c->wdtype, (size_t)v * c->hidden + k);
    return acc * c->logit_scale;
}

/* All logits of one row: logit_scale * W_lm xhat. */
void orc_probe_logits_row(const orc_cfg *c, const orc_weights *w, const double *xhat, double *out)
{
    dense(out, xhat, w->lm_head, NULL, c->wdtype, 1, c->hidden, c->vocab);
    for (int v = 0; v < c->vocab; ++v) out[v] *= c->logit_scale;
}

/* One output feature of a linear layer: <x, W[o]> (+ b[o]). */
double orc_probe_linear(const void *W, const void *b, int32_t wdtype, const double *x, int32_t n_in, int32_t o)
{
    double acc = 0.0;
    for (int k = 0; k < n_in; ++k) acc += x[k] * wget(W, wdtype, (size_t)o * n_in + k);
    return acc + (b ? wget(b, wdtype, (size_t)o) : 0.0);
}

/* One attention output vector: softmax(q K^T / sqrt(d)) V over n_keys given keys/values [n_keys, d]. */
void orc_probe_attend(const double *q, const double *K, const double *V, int32_t n_keys, int32_t d, double *out)
{
    double *sc = malloc(sizeof(double) * (size_t)n_keys), m = -INFINITY, den = 0.0;
    for (int t = 0; t < n_keys; ++t) {
        double a = 0.0;
        for (int i = 0; i < d; ++i) a += q[i] * K[(size_t)t * d + i];
        sc[t] = a / sqrt((double)d);
        if (sc[t] > m) m = sc[t];
    }
    for (int t = 0; t < n_keys; ++t) den += exp(sc[t] - m);
    for (int i = 0; i < d; ++i) out[i] = 0.0;
    for (int t = 0; t < n_keys; ++t)
        for (int i = 0; i < d; ++i) out[i] += exp(sc[t] - m) / den * V[(size_t)t * d + i];
    free(sc);
}

void orc_probe_rmsnorm(const double *x, const void *g, int32_t wdtype, int32_t h, double eps, double *y)
{
    rmsnorm(y, x, g, wdtype, 1, h, eps);
}

void orc_probe_rope(double *v, int32_t d, int32_t pos, double theta) { rope(v, d, pos, theta); }
double orc_probe_silu(double x) { return silu(x); }
double orc_probe_round_bf16(double x) { return round_bf16(x); }
