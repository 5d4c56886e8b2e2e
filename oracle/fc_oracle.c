/*
 * FreeCache cached denoising layer-step: CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  It shares no code with the HIP path, is never
 * called by it, and must not be used as a fallback for it.
 *
 * What it computes (paper, section 3.2.1 "FreeCache", paragraphs
 * "Initialization and Partitioning", "Windowed Re-computation" and
 * "Progressive Caching"; cost rows of Table 1):
 *   1. the fused Q/K/V projection of the rows of the active window only
 *      (Table 1, row "W_Q, W_K, W_V projections", with the row count L
 *      replaced by the window size A),
 *   2. rotary position embedding of q and k (the paper is silent on the
 *      position encoding; Dream/LLaDA-style half-split RoPE is this build's
 *      reading),
 *   3. the overwrite of exactly those rows of a persistent K/V cache
 *      ("KV projections are recomputed only for tokens within this window";
 *      everything outside is frozen),
 *   4. bidirectional softmax attention of the window's queries over the first
 *      kv_len cached rows (Table 1, rows "QK^T" and "Attention Score x Value",
 *      L x L replaced by A x L), grouped-query aware, with no mask.
 *
 * The second half of the file widens the step to the whole transformer layer
 * on the window rows (Table 1, rows "Output projection (W_out)", "FFN W_1" and
 * "FFN W_2", again with L replaced by A): RMS normalisation, the attention path
 * above, the output projection with its residual, and a gated feed-forward
 * network with its residual.  The paper names the modules but not their inner
 * form; pre-normalisation with RMSNorm and a SiLU-gated W_1 (the form of the
 * Dream and LLaDA checkpoints the paper evaluates) is this build's reading.
 *
 * All sums run in double, in ascending index order, with no blocking, fusion
 * or reordering.  Values are rounded only where the storage format demands it:
 * q, k, v when they are stored, the attention output, and every activation
 * tensor that the layer hands from one module to the next.
 *
 * Array layouts (row-major, all "storage" arrays hold floats whose values are
 * exactly representable in the storage dtype):
 *   X      [B][A][d]             W  [N][d], N = (Hq + 2 Hkv) Dh, rows ordered
 *   bias   [N] or NULL               q heads | k heads | v heads
 *   pos    [B][A] absolute position, or -1 for a padded (skipped) row
 *   Q      [B][Hq][A][Dh]
 *   Knew, Vnew [B][A][Hkv][Dh]
 *   Kc, Vc [B][Hkv][Smax][Dh]
 *   O      [B][A][Hq*Dh]
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { FCO_F32 = 0, FCO_BF16 = 1 };

typedef struct {
    int32_t batch;       /* B */
    int32_t hidden;      /* d */
    int32_t n_q_heads;   /* Hq */
    int32_t n_kv_heads;  /* Hkv, divides Hq */
    int32_t head_dim;    /* Dh, even */
    int32_t max_seq;     /* Smax: rows per (batch, kv head) in the cache */
    int32_t dtype;       /* FCO_F32 or FCO_BF16: the storage format */
    double rope_base;
    double softmax_scale; /* <= 0 means 1/sqrt(Dh) */
} fco_config;

/* Round a double to the storage format, round-to-nearest-even, directly from
 * double (no intermediate float rounding for bf16).  bf16 = 1 sign, 8 exponent,
 * 7 stored significand bits: 8 significant bits, minimum normal 2^-126. */
double fco_round_to_storage(double x, int32_t dtype)
{
    if (dtype == FCO_F32) return (double)(float)x;
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);          /* |x| = m * 2^e, m in [0.5, 1) */
    int q = e - 8;               /* exponent of the last kept bit */
    if (q < -133) q = -133;      /* bf16 subnormal spacing 2^-133 */
    double r = ldexp(rint(ldexp(x, -q)), q); /* rint: ties to even */
    const double bf16_max = (2.0 - ldexp(1.0, -7)) * ldexp(1.0, 127);
    if (fabs(r) > bf16_max) return x > 0 ? INFINITY : -INFINITY;
    return r;
}

/* Element-wise fco_round_to_storage over an array. */
void fco_round_array(const double *in, double *out, int64_t n, int32_t dtype)
{
    for (int64_t i = 0; i < n; ++i) out[i] = fco_round_to_storage(in[i], dtype);
}

static int cfg_ok(const fco_config *c)
{
    return c && c->batch > 0 && c->hidden > 0 && c->n_q_heads > 0 && c->n_kv_heads > 0 &&
           c->n_q_heads % c->n_kv_heads == 0 && c->head_dim > 0 && c->head_dim % 2 == 0 &&
           c->max_seq > 0 && (c->dtype == FCO_F32 || c->dtype == FCO_BF16);
}

/* Steps 1-2: project the window rows, rotate q and k, round to storage.
 * pre (optional, [B][A][N] doubles) receives the rotated, not yet rounded
 * values in the order q heads | k heads | v heads. */
int fco_project_rope(const fco_config *c, int32_t A, const float *X, const float *W,
                     const float *bias, const int32_t *pos, float *Q, float *Knew,
                     float *Vnew, double *pre)
{
    if (!cfg_ok(c) || A < 1 || !X || !W || !pos || !Q || !Knew || !Vnew) return 1;
    const int B = c->batch, d = c->hidden, Hq = c->n_q_heads, Hkv = c->n_kv_heads;
    const int Dh = c->head_dim, half = Dh / 2;
    const int N = (Hq + 2 * Hkv) * Dh;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int a = 0; a < A; ++a) {
            double *y = (double *)malloc(sizeof(double) * (size_t)N);
            const float *x = X + ((size_t)b * A + a) * d;
            const int32_t p = pos[(size_t)b * A + a];
            for (int n = 0; n < N; ++n) {
                const float *w = W + (size_t)n * d;
                double acc = 0.0;
                for (int k = 0; k < d; ++k) acc += (double)x[k] * (double)w[k];
                if (bias) acc += (double)bias[n];
                y[n] = acc;
            }
            /* rotary embedding on the Hq + Hkv heads that hold q and k */
            if (p >= 0) {
                for (int h = 0; h < Hq + Hkv; ++h) {
                    double *v = y + (size_t)h * Dh;
                    for (int i = 0; i < half; ++i) {
                        const double theta = pow(c->rope_base, -2.0 * (double)i / (double)Dh);
                        const double ang = (double)p * theta;
                        const double cs = cos(ang), sn = sin(ang);
                        const double x0 = v[i], x1 = v[i + half];
                        v[i] = x0 * cs - x1 * sn;
                        v[i + half] = x1 * cs + x0 * sn;
                    }
                }
            }
            for (int n = 0; n < N; ++n) {
                double val = (p >= 0) ? y[n] : 0.0;
                if (pre) pre[((size_t)b * A + a) * N + n] = val;
                float r = (float)fco_round_to_storage(val, c->dtype);
                int h = n / Dh, i = n % Dh;
                if (h < Hq)
                    Q[(((size_t)b * Hq + h) * A + a) * Dh + i] = r;
                else if (h < Hq + Hkv)
                    Knew[(((size_t)b * A + a) * Hkv + (h - Hq)) * Dh + i] = r;
                else
                    Vnew[(((size_t)b * A + a) * Hkv + (h - Hq - Hkv)) * Dh + i] = r;
            }
            free(y);
        }
    }
    return 0;
}

/* Step 3: overwrite the cache rows of the window; nothing else is touched.
 * Returns 2 if a position falls outside [0, Smax). */
int fco_scatter(const fco_config *c, int32_t A, const float *Knew, const float *Vnew,
                const int32_t *pos, float *Kc, float *Vc)
{
    if (!cfg_ok(c) || A < 1 || !Knew || !Vnew || !pos || !Kc || !Vc) return 1;
    const int B = c->batch, Hkv = c->n_kv_heads, Dh = c->head_dim, Smax = c->max_seq;
    for (int b = 0; b < B; ++b)
        for (int a = 0; a < A; ++a)
            if (pos[(size_t)b * A + a] >= Smax) return 2;
    for (int b = 0; b < B; ++b) {
        for (int a = 0; a < A; ++a) {
            const int32_t p = pos[(size_t)b * A + a];
            if (p < 0) continue;
            for (int j = 0; j < Hkv; ++j) {
                const size_t src = (((size_t)b * A + a) * Hkv + j) * Dh;
                const size_t dst = (((size_t)b * Hkv + j) * Smax + p) * Dh;
                memcpy(Kc + dst, Knew + src, sizeof(float) * (size_t)Dh);
                memcpy(Vc + dst, Vnew + src, sizeof(float) * (size_t)Dh);
            }
        }
    }
    return 0;
}

/* Step 4: O[b,a,h] = softmax(scale * q . Kc^T) Vc over rows [0, kv_len) of kv
 * head floor(h / g).  No mask.  probs (optional, [B][Hq][A][kv_len] doubles)
 * receives the normalised attention weights.  Rows with pos = -1 give zeros. */
int fco_attend(const fco_config *c, int32_t A, const float *Q, const float *Kc,
               const float *Vc, const int32_t *pos, int32_t kv_len, float *O, double *probs)
{
    if (!cfg_ok(c) || A < 1 || !Q || !Kc || !Vc || !O) return 1;
    if (kv_len < 1 || kv_len > c->max_seq) return 2;
    const int B = c->batch, Hq = c->n_q_heads, Hkv = c->n_kv_heads, Dh = c->head_dim;
    const int Smax = c->max_seq, g = Hq / Hkv;
    const double scale = c->softmax_scale > 0 ? c->softmax_scale : 1.0 / sqrt((double)Dh);
#pragma omp parallel for collapse(3) schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < Hq; ++h) {
            for (int a = 0; a < A; ++a) {
                float *o = O + ((size_t)b * A + a) * ((size_t)Hq * Dh) + (size_t)h * Dh;
                double *pr = probs ? probs + (((size_t)b * Hq + h) * A + a) * (size_t)kv_len : NULL;
                if (pos && pos[(size_t)b * A + a] < 0) {
                    for (int i = 0; i < Dh; ++i) o[i] = 0.0f;
                    if (pr) for (int t = 0; t < kv_len; ++t) pr[t] = 0.0;
                    continue;
                }
                const int j = h / g;
                const float *q = Q + (((size_t)b * Hq + h) * A + a) * Dh;
                const float *K = Kc + ((size_t)b * Hkv + j) * (size_t)Smax * Dh;
                const float *V = Vc + ((size_t)b * Hkv + j) * (size_t)Smax * Dh;
                double *s = (double *)malloc(sizeof(double) * (size_t)kv_len);
                double *acc = (double *)calloc((size_t)Dh, sizeof(double));
                double m = -INFINITY;
                for (int t = 0; t < kv_len; ++t) {
                    double dot = 0.0;
                    for (int i = 0; i < Dh; ++i) dot += (double)q[i] * (double)K[(size_t)t * Dh + i];
                    s[t] = scale * dot;
                    if (s[t] > m) m = s[t];
                }
                double l = 0.0;
                for (int t = 0; t < kv_len; ++t) {
                    s[t] = exp(s[t] - m);
                    l += s[t];
                }
                for (int t = 0; t < kv_len; ++t)
                    for (int i = 0; i < Dh; ++i) acc[i] += s[t] * (double)V[(size_t)t * Dh + i];
                for (int i = 0; i < Dh; ++i) o[i] = (float)fco_round_to_storage(acc[i] / l, c->dtype);
                if (pr) for (int t = 0; t < kv_len; ++t) pr[t] = s[t] / l;
                free(s);
                free(acc);
            }
        }
    }
    return 0;
}

/* One cached layer-step: every row of the window is projected and stored
 * before any attention is computed, because attention is bidirectional and
 * each window query reads each fresh key. */
int fco_layer_step(const fco_config *c, int32_t A, const float *X, const float *W,
                   const float *bias, const int32_t *pos, int32_t kv_len, float *Kc,
                   float *Vc, float *Q, float *O)
{
    if (!cfg_ok(c) || A < 1) return 1;
    const size_t nkv = (size_t)c->batch * A * c->n_kv_heads * c->head_dim;
    float *Knew = (float *)malloc(sizeof(float) * nkv);
    float *Vnew = (float *)malloc(sizeof(float) * nkv);
    int rc = fco_project_rope(c, A, X, W, bias, pos, Q, Knew, Vnew, NULL);
    if (!rc) {
        for (int i = 0; i < c->batch * A && !rc; ++i)
            if (pos[i] >= kv_len) rc = 2;
    }
    if (!rc) rc = fco_scatter(c, A, Knew, Vnew, pos, Kc, Vc);
    if (!rc) rc = fco_attend(c, A, Q, Kc, Vc, pos, kv_len, O, NULL);
    free(Knew);
    free(Vnew);
    return rc;
}

/*
 * Window schedule (section 3.2.1).  The generation region [P, P+G) is cut into
 * N = ceil(G / Bk) blocks; cached step s works on block i = floor(s /
 * steps_per_block).
 *   mode 0 (block window): the window is block i alone.
 *   mode 1 (reducing window, the paper's literal statement): the window is
 *          block i and every later block, so it shrinks as blocks complete.
 * refresh_after is 1 when refresh_every > 0 and (s + 1) is a multiple of it:
 * the caller then re-projects the generation region before the next step.
 * Returns 1 for invalid arguments, 2 when s is past the last block.
 */
int fco_window(int32_t step, int32_t P, int32_t G, int32_t Bk, int32_t steps_per_block,
               int32_t refresh_every, int32_t mode, int32_t *win_start, int32_t *rows,
               int32_t *refresh_after)
{
    if (step < 0 || P < 0 || G < 1 || Bk < 1 || steps_per_block < 1 || refresh_every < 0 ||
        (mode != 0 && mode != 1) || !win_start || !rows || !refresh_after)
        return 1;
    const int32_t N = (G + Bk - 1) / Bk;
    const int32_t i = step / steps_per_block;
    if (i >= N) return 2;
    *win_start = P + i * Bk;
    if (mode == 1) {
        *rows = G - i * Bk;
    } else {
        int32_t left = G - i * Bk;
        *rows = left < Bk ? left : Bk;
    }
    *refresh_after = (refresh_every > 0 && (step + 1) % refresh_every == 0) ? 1 : 0;
    return 0;
}

/* -------------------------------------------------------------------------
 * The rest of the layer on the window rows (Table 1: W_out, FFN W_1, FFN W_2).
 */

/* RMS normalisation of each row: out[r][k] = x[r][k] / sqrt(mean_k x[r][k]^2 + eps) * w[k],
 * rounded to the storage format. */
int fco_rmsnorm(const float *X, const float *w, double eps, int64_t rows, int32_t d,
                int32_t dtype, float *out)
{
    if (!X || !w || !out || rows < 1 || d < 1 || !(eps >= 0.0)) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const float *x = X + (size_t)r * d;
        double ss = 0.0;
        for (int k = 0; k < d; ++k) ss += (double)x[k] * (double)x[k];
        const double inv = 1.0 / sqrt(ss / (double)d + eps);
        for (int k = 0; k < d; ++k)
            out[(size_t)r * d + k] = (float)fco_round_to_storage((double)x[k] * inv * (double)w[k], dtype);
    }
    return 0;
}

/* out[m][n] = res[m][n] + sum_k X[m][k] W[n][k], one rounding to storage.  res may be NULL.
 * This is the output projection W_out and the second FFN matrix W_2, each with the residual
 * connection of a pre-normalised layer folded in. */
int fco_linear_residual(const float *X, const float *W, const float *res, int64_t M, int32_t K,
                        int32_t N, int32_t dtype, float *out)
{
    if (!X || !W || !out || M < 1 || K < 1 || N < 1) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *x = X + (size_t)m * K;
        for (int n = 0; n < N; ++n) {
            const float *w = W + (size_t)n * K;
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += (double)x[k] * (double)w[k];
            if (res) acc += (double)res[(size_t)m * N + n];
            out[(size_t)m * N + n] = (float)fco_round_to_storage(acc, dtype);
        }
    }
    return 0;
}

/* First FFN matrix in its gated form: with g = X Wg^T and u = X Wu^T (both kept in double),
 * out[m][f] = silu(g[m][f]) * u[m][f], silu(t) = t / (1 + exp(-t)); one rounding to storage. */
int fco_ffn_gate_up(const float *X, const float *Wg, const float *Wu, int64_t M, int32_t K,
                    int32_t F, int32_t dtype, float *out)
{
    if (!X || !Wg || !Wu || !out || M < 1 || K < 1 || F < 1) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *x = X + (size_t)m * K;
        for (int f = 0; f < F; ++f) {
            const float *wg = Wg + (size_t)f * K, *wu = Wu + (size_t)f * K;
            double g = 0.0, u = 0.0;
            for (int k = 0; k < K; ++k) g += (double)x[k] * (double)wg[k];
            for (int k = 0; k < K; ++k) u += (double)x[k] * (double)wu[k];
            const double act = g / (1.0 + exp(-g)) * u;
            out[(size_t)m * F + f] = (float)fco_round_to_storage(act, dtype);
        }
    }
    return 0;
}

/* Weights of one pre-normalised transformer layer. */
typedef struct {
    const float *norm1;  /* [d] */
    const float *w_qkv;  /* [N][d] */
    const float *b_qkv;  /* [N] or NULL */
    const float *w_out;  /* [d][Hq*Dh] */
    const float *norm2;  /* [d] */
    const float *w_gate; /* [d_ff][d] */
    const float *w_up;   /* [d_ff][d] */
    const float *w_down; /* [d][d_ff] */
    int32_t d_ff;
    double eps;
} fco_layer_weights;

/* One cached step of the whole layer on the window rows X [B][A][d]:
 *   h1 = rmsnorm(X; norm1)
 *   (Q, cache rows, O) = the attention path of fco_layer_step on h1
 *   X2 = X + O W_out^T
 *   h2 = rmsnorm(X2; norm2)
 *   Y  = X2 + (silu(h2 Wg^T) * (h2 Wu^T)) W_down^T
 * Every named tensor is rounded to storage.  X2 (optional, [B][A][d]) receives the
 * intermediate residual stream.  A padded row (pos < 0) has O = 0 and is otherwise treated like
 * any other row. */
int fco_full_layer_step(const fco_config *c, int32_t A, const float *X, const fco_layer_weights *w,
                        const int32_t *pos, int32_t kv_len, float *Kc, float *Vc, float *Y,
                        float *X2)
{
    if (!cfg_ok(c) || A < 1 || !X || !w || !pos || !Y || w->d_ff < 1) return 1;
    const int64_t M = (int64_t)c->batch * A;
    const int d = c->hidden, E = c->n_q_heads * c->head_dim, F = w->d_ff;
    float *h = (float *)malloc(sizeof(float) * (size_t)M * d);
    float *q = (float *)malloc(sizeof(float) * (size_t)M * E);
    float *o = (float *)malloc(sizeof(float) * (size_t)M * E);
    float *x2 = (float *)malloc(sizeof(float) * (size_t)M * d);
    float *act = (float *)malloc(sizeof(float) * (size_t)M * F);
    int rc = fco_rmsnorm(X, w->norm1, w->eps, M, d, c->dtype, h);
    if (!rc) rc = fco_layer_step(c, A, h, w->w_qkv, w->b_qkv, pos, kv_len, Kc, Vc, q, o);
    if (!rc) rc = fco_linear_residual(o, w->w_out, X, M, E, d, c->dtype, x2);
    if (!rc) rc = fco_rmsnorm(x2, w->norm2, w->eps, M, d, c->dtype, h);
    if (!rc) rc = fco_ffn_gate_up(h, w->w_gate, w->w_up, M, d, F, c->dtype, act);
    if (!rc) rc = fco_linear_residual(act, w->w_down, x2, M, F, d, c->dtype, Y);
    if (!rc && X2) memcpy(X2, x2, sizeof(float) * (size_t)M * d);
    free(h);
    free(q);
    free(o);
    free(x2);
    free(act);
    return rc;
}

/* -------------------------------------------------------------------------
 * Unmasking step of a diffusion language model on the window rows (paper, section 3.1, the three
 * equations that define M_t, z_t and the arg-max fill of the selected positions U_t; section 3.2.1
 * for the window the rows come from).
 */

/* Vocabulary projection of M rows and, per row, the arg-max token and its softmax probability:
 *   z[m][v] = sum_k X[m][k] Wv[v][k]          (double, never rounded)
 *   tok[m]  = the smallest v with z[m][v] = max_v z[m][v]
 *   conf[m] = softmax(z[m])[tok[m]] = 1 / sum_v exp(z[m][v] - z[m][tok[m]])
 * logits (optional, [M][V] doubles) receives z. */
int fco_lm_head_argmax(const float *X, const float *Wv, int64_t M, int32_t K, int32_t V,
                       int32_t *tok, double *conf, double *logits)
{
    if (!X || !Wv || !tok || !conf || M < 1 || K < 1 || V < 1) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *x = X + (size_t)m * K;
        double *z = (double *)malloc(sizeof(double) * (size_t)V);
        int best = 0;
        for (int v = 0; v < V; ++v) {
            const float *w = Wv + (size_t)v * K;
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += (double)x[k] * (double)w[k];
            z[v] = acc;
            if (acc > z[best]) best = v;
        }
        double sum = 0.0;
        for (int v = 0; v < V; ++v) sum += exp(z[v] - z[best]);
        tok[m] = best;
        conf[m] = 1.0 / sum;
        if (logits) memcpy(logits + (size_t)m * V, z, sizeof(double) * (size_t)V);
        free(z);
    }
    return 0;
}

/* Confidence-ranked unmasking of one step.  For every sequence b the candidates are the window
 * rows a with pos[b][a] >= 0 whose token is still the mask (tokens[b][pos[b][a]] == mask_id: the
 * set M_t restricted to the window).  The n_unmask candidates with the largest confidence (ties:
 * the smaller a first) form U_t and receive their arg-max token; all of them if fewer remain.
 * pos_next[b][.] lists the positions of the window rows that are still masked afterwards, in row
 * order, padded with -1; count_next[b] is their number.
 * tokens [B][L] is updated in place.  Returns 2 if a position is >= L. */
int fco_unmask_select(const int32_t *tok, const double *conf, const int32_t *pos, int32_t B, int32_t A,
                      int32_t n_unmask, int32_t mask_id, int32_t *tokens, int32_t L, int32_t *pos_next,
                      int32_t *count_next)
{
    if (!tok || !conf || !pos || !tokens || !pos_next || !count_next || B < 1 || A < 1 || L < 1 || n_unmask < 0)
        return 1;
    for (int64_t i = 0; i < (int64_t)B * A; ++i)
        if (pos[i] >= L) return 2;
    for (int b = 0; b < B; ++b) {
        const int32_t *p = pos + (size_t)b * A;
        int32_t *seq = tokens + (size_t)b * L;
        char *cand = (char *)calloc((size_t)A, 1);
        int n_cand = 0;
        for (int a = 0; a < A; ++a)
            if (p[a] >= 0 && seq[p[a]] == mask_id) {
                cand[a] = 1;
                ++n_cand;
            }
        int take = n_unmask < n_cand ? n_unmask : n_cand;
        while (take-- > 0) { /* repeated selection of the best remaining candidate */
            int best = -1;
            for (int a = 0; a < A; ++a)
                if (cand[a] && (best < 0 || conf[(size_t)b * A + a] > conf[(size_t)b * A + best])) best = a;
            cand[best] = 0;
            seq[p[best]] = tok[(size_t)b * A + best];
        }
        int n = 0;
        for (int a = 0; a < A; ++a)
            if (cand[a]) pos_next[(size_t)b * A + n++] = p[a];
        count_next[b] = n;
        for (; n < A; ++n) pos_next[(size_t)b * A + n] = -1;
        free(cand);
    }
    return 0;
}

/* Row gather: out[i][:] = table[idx[i]][:] for idx[i] in [0, R), zeros for a negative idx[i].  It is the
 * embedding lookup of the token ids of the window rows (x_t restricted to the window, section 3.1) and
 * the compaction of a block's rows.  Returns 2 if an index is >= R. */
int fco_gather_rows(const float *table, int64_t R, int32_t d, const int32_t *idx, int64_t n, float *out)
{
    if (!table || !idx || !out || R < 1 || d < 1 || n < 1) return 1;
    for (int64_t i = 0; i < n; ++i)
        if (idx[i] >= R) return 2;
    for (int64_t i = 0; i < n; ++i) {
        if (idx[i] < 0)
            memset(out + (size_t)i * d, 0, sizeof(float) * (size_t)d);
        else
            memcpy(out + (size_t)i * d, table + (size_t)idx[i] * d, sizeof(float) * (size_t)d);
    }
    return 0;
}

/* -------------------------------------------------------------------------
 * Guided Diffusion acceptance (paper, section 3.2.2 and Algorithm 1; Top-K match and the guidance
 * threshold tau from the appendix "Implementation Details").
 *
 * For every sequence b let i_1 < ... < i_m be the still masked window rows (pos >= 0 and
 * tokens[b][pos] == mask_id), in row order.  For row i_j:
 *   t_j   = argmax_v dlm[b][i_j][v]  (smallest v on ties),  zd_j = that largest logit,
 *   top_j = the topk token ids of ar[b][i_j][.] with the largest logits (ties: smaller id first),
 *           za_j = the largest AR logit,
 *   match_j = t_j in top_j  and  (tau <= 0 or zd_j > (float)(tau * za_j))   -- float32 product.
 * k = the largest prefix length with match_1 .. match_k all true.  The first max(k, 1) masked rows
 * are filled with their DLM tokens (if no prefix agrees only i_1 is filled); n_accept[b] is that number
 * (0 when nothing is masked).  pos_next / count_next list the rows that stay masked, as in
 * fco_unmask_select.  Returns 2 if a position is >= L.
 */
int fco_guided_accept(const float *dlm, const float *ar, const int32_t *pos, int32_t B, int32_t A, int32_t V,
                      int32_t topk, float tau, int32_t mask_id, int32_t *tokens, int32_t L, int32_t *n_accept,
                      int32_t *pos_next, int32_t *count_next)
{
    if (!dlm || !ar || !pos || !tokens || !n_accept || !pos_next || !count_next || B < 1 || A < 1 || V < 1 || L < 1 ||
        topk < 1 || topk > V)
        return 1;
    for (int64_t i = 0; i < (int64_t)B * A; ++i)
        if (pos[i] >= L) return 2;
    for (int b = 0; b < B; ++b) {
        const int32_t *p = pos + (size_t)b * A;
        int32_t *seq = tokens + (size_t)b * L;
        int *rows = (int *)malloc(sizeof(int) * (size_t)A), *tdlm = (int *)malloc(sizeof(int) * (size_t)A);
        char *used = (char *)malloc((size_t)V);
        int m = 0;
        for (int a = 0; a < A; ++a)
            if (p[a] >= 0 && seq[p[a]] == mask_id) rows[m++] = a;
        int k = 0, prefix_open = 1;
        for (int j = 0; j < m; ++j) {
            const float *zd = dlm + ((size_t)b * A + rows[j]) * V, *za = ar + ((size_t)b * A + rows[j]) * V;
            int t = 0;
            for (int v = 1; v < V; ++v)
                if (zd[v] > zd[t]) t = v;
            tdlm[j] = t;
            /* the topk largest AR logits by repeated selection */
            memset(used, 0, (size_t)V);
            int in_top = 0, best0 = -1;
            for (int r = 0; r < topk; ++r) {
                int best = -1;
                for (int v = 0; v < V; ++v)
                    if (!used[v] && (best < 0 || za[v] > za[best])) best = v;
                used[best] = 1;
                if (r == 0) best0 = best;
                if (best == t) in_top = 1;
            }
            const float thr = tau * za[best0]; /* float32 product */
            const int match = in_top && (!(tau > 0.0f) || zd[t] > thr);
            if (prefix_open && match)
                ++k;
            else
                prefix_open = 0;
        }
        const int n = m == 0 ? 0 : (k > 0 ? k : 1);
        for (int j = 0; j < n; ++j) seq[p[rows[j]]] = tdlm[j];
        n_accept[b] = n;
        int c = 0;
        for (int j = n; j < m; ++j) pos_next[(size_t)b * A + c++] = p[rows[j]];
        count_next[b] = c;
        for (; c < A; ++c) pos_next[(size_t)b * A + c] = -1;
        free(rows);
        free(tdlm);
        free(used);
    }
    return 0;
}

/* -------------------------------------------------------------------------
 * KV drift diagnostic (paper, section 3.2.1, the figure that motivates FreeCache: the similarity of a
 * token's K / V projection to its projection at the previous step).  For rows [start, start + rows)
 * of the cache and a snapshot of the same rows taken earlier (plain layout [B][Hkv][rows][Dh]):
 *   sim[b][j][r] = <now, prev> / (|now| |prev|)   (cosine similarity over the head dimension),
 * 0 when either vector is zero.  sim_k, sim_v: [B][Hkv][rows] doubles.
 */
int fco_kv_similarity(const fco_config *c, const float *Kc, const float *Vc, const float *k_prev,
                      const float *v_prev, int32_t start, int32_t rows, double *sim_k, double *sim_v)
{
    if (!cfg_ok(c) || !Kc || !Vc || !k_prev || !v_prev || !sim_k || !sim_v || rows < 1) return 1;
    if (start < 0 || start > c->max_seq - rows) return 2;
    const int B = c->batch, Hkv = c->n_kv_heads, Dh = c->head_dim, Smax = c->max_seq;
    for (int b = 0; b < B; ++b)
        for (int j = 0; j < Hkv; ++j)
            for (int r = 0; r < rows; ++r) {
                const size_t now = (((size_t)b * Hkv + j) * Smax + start + r) * Dh;
                const size_t old = (((size_t)b * Hkv + j) * rows + r) * Dh;
                for (int which = 0; which < 2; ++which) {
                    const float *x = (which ? Vc : Kc) + now, *y = (which ? v_prev : k_prev) + old;
                    double dot = 0.0, nx = 0.0, ny = 0.0;
                    for (int i = 0; i < Dh; ++i) {
                        dot += (double)x[i] * (double)y[i];
                        nx += (double)x[i] * (double)x[i];
                        ny += (double)y[i] * (double)y[i];
                    }
                    const double s = (nx > 0.0 && ny > 0.0) ? dot / (sqrt(nx) * sqrt(ny)) : 0.0;
                    (which ? sim_v : sim_k)[((size_t)b * Hkv + j) * rows + r] = s;
                }
            }
    return 0;
}
