/*
 * CPU oracle for selective Jacobi decoding of a block-autoregressive normalizing flow.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the tests, the smoke
 * check and the benchmark's CPU-baseline leg call.  The product (the HIP library) never links,
 * imports or executes anything from here, and nothing here includes anything of the product.
 *
 * What it computes, with the passage each part follows:
 *   - the flow's forward map of one block (Sec. 3.1, eq. 4): one parallel pass,
 *         y_1 = x_1,   y_l = (x_l - g(x_<l)) * exp(s(x_<l));
 *   - the strictly sequential inverse of one block (Sec. 3.1, eq. 5), token after token,
 *         x_1 = y_1,   x_l = y_l * exp(-s(x_<l)) + g(x_<l),
 *     both straight from the definition (a full conditioner pass per token) and with a key/value
 *     cache (Sec. 3.5), the two being compared in the tests;
 *   - the Jacobi iteration map F (App. B, Def. A.1) and Jacobi decoding (Sec. 3.3, Alg. 1):
 *     start from a guess, apply F to all tokens at once, stop when consecutive iterates are close;
 *   - the cascade of K blocks (Sec. 3.1, eq. 2) with a per-block choice of sequential or Jacobi
 *     inversion (Sec. 3.5), and a token reversal in alternate blocks (the permutation mentioned
 *     below eq. 4).
 *
 * Notation used here: T tokens (the paper's L), D token dimension, K blocks, N transformer layers
 * per block, W width, H heads.  mu = g_k and alpha = -s_k, so the inverse reads
 * x_l = y_l * exp(alpha_l) + mu_l and the forward reads y_l = (x_l - mu_l) * exp(-alpha_l).
 *
 * The paper leaves the conditioner network as "a causal transformer"; the one fixed here is:
 * token embedding x W_in + b_in + learned positions; N pre-LayerNorm layers of causal multi-head
 * attention (scale 1/sqrt(dh)) and a GELU (erf form) MLP, each added to the residual stream; a
 * final LayerNorm and a linear head giving [mu | alpha] per token.  LayerNorm uses the biased
 * variance and eps 1e-5.  The head's row l-1 parameterises token l (strictly preceding context);
 * token 1 has mu = alpha = 0.
 *
 * Stopping rule: per sample, delta = mean_{l,d} |x^t - x^(t-1)| (criterion 0) or the maximum
 * (criterion 1, the rule as printed in Alg. 1), stop when delta < tau, or after `cap` passes
 * (cap = T unless lowered: by Prop. 3.2 the T-th iterate is exact).  The iteration count is the
 * number of conditioner passes including the last one; the newest iterate is returned.
 *
 * Arithmetic type: REAL (float by default; the build also makes a double version).  Weights are
 * float32 values in the documented blob order and are widened on use.
 *
 * Parity pins (tests/test_oracle_*.py, all CPU): forward(inverse(z)) = z; Jacobi from any start
 * equals the sequential inverse after T passes and stays there; prefix exactness after each pass;
 * one token => one pass; strict causality by perturbation; identity flow when the head is zero;
 * a context-free chain with a closed form; LayerNorm / GELU / attention / the whole conditioner
 * against library routines; tau = 0, tau = inf; batch independence.  The numbers the paper prints
 * (iteration tables, timings, MSEs) depend on trained weights that are not available: parity
 * unpinned for those.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef REAL
#define REAL float
#endif
typedef REAL real;

typedef struct {
    int32_t n_blocks, n_layers, width, n_heads, mlp_ratio, seq_len, token_dim;
    uint32_t reverse_mask;
    int32_t mask_nearest; /* o of eq. 6: the attention of position t sees keys 0..t-o only (0: plain causal) */
} orc_config;

typedef struct {
    const float *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o, *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} layer_w;

#define ORC_MAX_LAYERS 64
typedef struct {
    const float *w_in, *b_in, *pos;
    layer_w layer[ORC_MAX_LAYERS];
    const float *lnf_g, *lnf_b, *w_head, *b_head;
} block_w;

static size_t block_floats(const orc_config *c) {
    size_t D = c->token_dim, W = c->width, T = c->seq_len, R = c->mlp_ratio, N = c->n_layers;
    size_t per_layer = 2 * W + W * 3 * W + 3 * W + W * W + W + 2 * W + W * R * W + R * W + R * W * W + W;
    return D * W + W + T * W + N * per_layer + 2 * W + W * 2 * D + 2 * D;
}

static void map_block(const orc_config *c, const float *blob, int j, block_w *b) {
    size_t D = c->token_dim, W = c->width, T = c->seq_len, R = c->mlp_ratio;
    const float *p = blob + (size_t)j * block_floats(c);
    b->w_in = p; p += D * W;
    b->b_in = p; p += W;
    b->pos = p; p += T * W;
    for (int l = 0; l < c->n_layers; ++l) {
        layer_w *lw = &b->layer[l];
        lw->ln1_g = p; p += W;
        lw->ln1_b = p; p += W;
        lw->w_qkv = p; p += W * 3 * W;
        lw->b_qkv = p; p += 3 * W;
        lw->w_o = p; p += W * W;
        lw->b_o = p; p += W;
        lw->ln2_g = p; p += W;
        lw->ln2_b = p; p += W;
        lw->w_fc1 = p; p += W * R * W;
        lw->b_fc1 = p; p += R * W;
        lw->w_fc2 = p; p += R * W * W;
        lw->b_fc2 = p; p += W;
    }
    b->lnf_g = p; p += W;
    b->lnf_b = p; p += W;
    b->w_head = p; p += W * 2 * D;
    b->b_head = p;
}

/* ---------------------------------------------------------------- primitives (one token row) */

/* y = (x - mean) / sqrt(var + 1e-5) * g + b, biased variance over the row */
static void layernorm_row(const real *x, const float *g, const float *b, int W, real *y) {
    real mean = 0;
    for (int i = 0; i < W; ++i) mean += x[i];
    mean /= (real)W;
    real var = 0;
    for (int i = 0; i < W; ++i) { real d = x[i] - mean; var += d * d; }
    var /= (real)W;
    real rstd = (real)1 / (real)sqrt((double)(var + (real)1e-5));
    for (int i = 0; i < W; ++i) y[i] = (x[i] - mean) * rstd * (real)g[i] + (real)b[i];
}

/* y[n] = bias[n] + sum_k a[k] * Wm[k][n],  Wm row-major [K][N].  The sum over k runs in index
 * order for every n; the compiler may only vectorise across n (no contraction, no reassociation:
 * the build passes -ffp-contract=off and no fast-math), so all clones give identical results. */
__attribute__((target_clones("default", "avx2")))
static void linear_row(const real *a, const float *Wm, const float *bias, int K, int N, real *y) {
    for (int n = 0; n < N; ++n) y[n] = (real)bias[n];
    for (int k = 0; k < K; ++k) {
        real ak = a[k];
        const float *w = Wm + (size_t)k * N;
        for (int n = 0; n < N; ++n) y[n] += ak * (real)w[n];
    }
}

static real gelu_erf(real v) {
    return (real)(0.5 * (double)v * (1.0 + erf((double)v * 0.70710678118654752440)));
}

/* Causal attention for one query row: head h of q attends keys/values of rows 0..t (inclusive).
 * Kc, Vc are [T][W] with head h in columns h*dh..; scores scratch holds t+1 reals.
 * A row that sees no key at all (t < 0, which only the masked variant of eq. 6 produces) gets a
 * zero attention output. */
static void attend_row(const real *q, const real *Kc, const real *Vc, int t, int W, int H, real *o, real *scores) {
    int dh = W / H;
    if (t < 0) { for (int i = 0; i < W; ++i) o[i] = 0; return; }
    real scale = (real)(1.0 / sqrt((double)dh));
    for (int h = 0; h < H; ++h) {
        const real *qh = q + h * dh;
        real mx = -INFINITY;
        for (int s = 0; s <= t; ++s) {
            const real *kh = Kc + (size_t)s * W + h * dh;
            real dot = 0;
            for (int d = 0; d < dh; ++d) dot += qh[d] * kh[d];
            scores[s] = dot * scale;
            if (scores[s] > mx) mx = scores[s];
        }
        real den = 0;
        for (int s = 0; s <= t; ++s) { scores[s] = (real)exp((double)(scores[s] - mx)); den += scores[s]; }
        real *oh = o + h * dh;
        for (int d = 0; d < dh; ++d) oh[d] = 0;
        for (int s = 0; s <= t; ++s) {
            real p = scores[s] / den;
            const real *vh = Vc + (size_t)s * W + h * dh;
            for (int d = 0; d < dh; ++d) oh[d] += p * vh[d];
        }
    }
}

/* ---------------------------------------------------------------- conditioner */

typedef struct {
    real *h;      /* [T][W] residual stream */
    real *a;      /* [T][W] LayerNorm output / attention output */
    real *qkv;    /* [T][3W] */
    real *kc;     /* [N][T][W] keys   */
    real *vc;     /* [N][T][W] values */
    real *q;      /* [T][W] */
    real *f;      /* [T][R*W] */
    real *t1;     /* [R*W] temp row */
    real *scores; /* [T] */
    real *p;      /* [T][2D] raw head output: row l = parameters computed from tokens <= l */
} cond_ws;

static int ws_alloc(const orc_config *c, cond_ws *w) {
    size_t T = c->seq_len, W = c->width, R = c->mlp_ratio, N = c->n_layers, D = c->token_dim;
    w->h = (real *)malloc(sizeof(real) * T * W);
    w->a = (real *)malloc(sizeof(real) * T * W);
    w->qkv = (real *)malloc(sizeof(real) * T * 3 * W);
    w->kc = (real *)malloc(sizeof(real) * N * T * W);
    w->vc = (real *)malloc(sizeof(real) * N * T * W);
    w->q = (real *)malloc(sizeof(real) * T * W);
    w->f = (real *)malloc(sizeof(real) * T * R * W);
    w->t1 = (real *)malloc(sizeof(real) * (R * W > 3 * W ? R * W : 3 * W));
    w->scores = (real *)malloc(sizeof(real) * T);
    w->p = (real *)malloc(sizeof(real) * T * 2 * D);
    return (w->h && w->a && w->qkv && w->kc && w->vc && w->q && w->f && w->t1 && w->scores && w->p) ? 0 : -1;
}

static void ws_free(cond_ws *w) {
    free(w->h); free(w->a); free(w->qkv); free(w->kc); free(w->vc); free(w->q); free(w->f); free(w->t1);
    free(w->scores); free(w->p);
}

/* Whole-sequence conditioner pass, layer by layer, on x [T][D] given in the block's processing
 * order.  Writes w->p [T][2D]: row l holds the head output at position l (it has seen tokens
 * 0..l), i.e. the parameters of token l+1. */
static void cond_full(const orc_config *c, const block_w *bw, const real *x, cond_ws *w) {
    int T = c->seq_len, W = c->width, D = c->token_dim, H = c->n_heads, RW = c->mlp_ratio * c->width;
    for (int t = 0; t < T; ++t) {
        real *ht = w->h + (size_t)t * W;
        linear_row(x + (size_t)t * D, bw->w_in, bw->b_in, D, W, ht);
        for (int i = 0; i < W; ++i) ht[i] += (real)bw->pos[(size_t)t * W + i];
    }
    for (int l = 0; l < c->n_layers; ++l) {
        const layer_w *lw = &bw->layer[l];
        real *Kc = w->kc + (size_t)l * T * W, *Vc = w->vc + (size_t)l * T * W;
        for (int t = 0; t < T; ++t) {
            layernorm_row(w->h + (size_t)t * W, lw->ln1_g, lw->ln1_b, W, w->a + (size_t)t * W);
            real *r = w->qkv + (size_t)t * 3 * W;
            linear_row(w->a + (size_t)t * W, lw->w_qkv, lw->b_qkv, W, 3 * W, r);
            memcpy(w->q + (size_t)t * W, r, sizeof(real) * W);
            memcpy(Kc + (size_t)t * W, r + W, sizeof(real) * W);
            memcpy(Vc + (size_t)t * W, r + 2 * W, sizeof(real) * W);
        }
        for (int t = 0; t < T; ++t)
            attend_row(w->q + (size_t)t * W, Kc, Vc, t - c->mask_nearest, W, H, w->a + (size_t)t * W, w->scores);
        for (int t = 0; t < T; ++t) {
            real *ht = w->h + (size_t)t * W;
            linear_row(w->a + (size_t)t * W, lw->w_o, lw->b_o, W, W, w->t1);
            for (int i = 0; i < W; ++i) ht[i] += w->t1[i];
        }
        for (int t = 0; t < T; ++t) {
            real *ft = w->f + (size_t)t * RW;
            layernorm_row(w->h + (size_t)t * W, lw->ln2_g, lw->ln2_b, W, w->a + (size_t)t * W);
            linear_row(w->a + (size_t)t * W, lw->w_fc1, lw->b_fc1, W, RW, ft);
            for (int i = 0; i < RW; ++i) ft[i] = gelu_erf(ft[i]);
        }
        for (int t = 0; t < T; ++t) {
            real *ht = w->h + (size_t)t * W;
            linear_row(w->f + (size_t)t * RW, lw->w_fc2, lw->b_fc2, RW, W, w->t1);
            for (int i = 0; i < W; ++i) ht[i] += w->t1[i];
        }
    }
    for (int t = 0; t < T; ++t) {
        layernorm_row(w->h + (size_t)t * W, bw->lnf_g, bw->lnf_b, W, w->a + (size_t)t * W);
        linear_row(w->a + (size_t)t * W, bw->w_head, bw->b_head, W, 2 * D, w->p + (size_t)t * 2 * D);
    }
}

/* One token through all layers with the key/value cache (Sec. 3.5): position t, token row xt [D].
 * Rows 0..t-1 of the caches must have been filled by earlier calls.  Writes w->p row t. */
static void cond_step(const orc_config *c, const block_w *bw, const real *xt, int t, cond_ws *w) {
    int T = c->seq_len, W = c->width, D = c->token_dim, H = c->n_heads, RW = c->mlp_ratio * c->width;
    real *h = w->h, *a = w->a, *r = w->qkv, *f = w->f;
    linear_row(xt, bw->w_in, bw->b_in, D, W, h);
    for (int i = 0; i < W; ++i) h[i] += (real)bw->pos[(size_t)t * W + i];
    for (int l = 0; l < c->n_layers; ++l) {
        const layer_w *lw = &bw->layer[l];
        real *Kc = w->kc + (size_t)l * T * W, *Vc = w->vc + (size_t)l * T * W;
        layernorm_row(h, lw->ln1_g, lw->ln1_b, W, a);
        linear_row(a, lw->w_qkv, lw->b_qkv, W, 3 * W, r);
        memcpy(Kc + (size_t)t * W, r + W, sizeof(real) * W);
        memcpy(Vc + (size_t)t * W, r + 2 * W, sizeof(real) * W);
        attend_row(r, Kc, Vc, t - c->mask_nearest, W, H, a, w->scores);
        linear_row(a, lw->w_o, lw->b_o, W, W, w->t1);
        for (int i = 0; i < W; ++i) h[i] += w->t1[i];
        layernorm_row(h, lw->ln2_g, lw->ln2_b, W, a);
        linear_row(a, lw->w_fc1, lw->b_fc1, W, RW, f);
        for (int i = 0; i < RW; ++i) f[i] = gelu_erf(f[i]);
        linear_row(f, lw->w_fc2, lw->b_fc2, RW, W, w->t1);
        for (int i = 0; i < W; ++i) h[i] += w->t1[i];
    }
    layernorm_row(h, bw->lnf_g, bw->lnf_b, W, a);
    linear_row(a, bw->w_head, bw->b_head, W, 2 * D, w->p + (size_t)t * 2 * D);
}

/* Shifted parameters for token l (processing order): token 0 gets (0, 0), token l >= 1 takes
 * head row l-1, whose first D entries are mu and last D entries alpha. */
static void params_of(const orc_config *c, const cond_ws *w, int l, int d, real *mu, real *alpha) {
    int D = c->token_dim;
    if (l == 0) { *mu = 0; *alpha = 0; return; }
    const real *row = w->p + (size_t)(l - 1) * 2 * D;
    *mu = row[d];
    *alpha = row[D + d];
}

static void flip_tokens(const orc_config *c, int reversed, const real *in, real *out) {
    int T = c->seq_len, D = c->token_dim;
    for (int t = 0; t < T; ++t) {
        int s = reversed ? T - 1 - t : t;
        memcpy(out + (size_t)t * D, in + (size_t)s * D, sizeof(real) * D);
    }
}

/* F of Def. A.1 in processing order: xn = F(xp) given the block input u. */
static void jacobi_map(const orc_config *c, const block_w *bw, const real *u, const real *xp, real *xn, cond_ws *w) {
    int T = c->seq_len, D = c->token_dim;
    cond_full(c, bw, xp, w);
    for (int l = 0; l < T; ++l)
        for (int d = 0; d < D; ++d) {
            real mu, al;
            params_of(c, w, l, d, &mu, &al);
            xn[(size_t)l * D + d] = u[(size_t)l * D + d] * (real)exp((double)al) + mu;
        }
}

static real iterate_distance(const orc_config *c, int criterion, const real *a, const real *b) {
    size_t n = (size_t)c->seq_len * c->token_dim;
    real acc = 0;
    for (size_t i = 0; i < n; ++i) {
        real d = (real)fabs((double)(a[i] - b[i]));
        if (criterion == 1) { if (d > acc || d != d) acc = d; }
        else acc += d;
    }
    return criterion == 1 ? acc : acc / (real)n;
}

/* ---------------------------------------------------------------- exported, one sample */

#define EXPORT __attribute__((visibility("default")))

EXPORT int orc_real_bytes(void) { return (int)sizeof(real); }
EXPORT int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
EXPORT size_t orc_block_floats(const orc_config *c) { return block_floats(c); }

/* Conditioner on one sample, processing order in and out: mu, alpha [T][D] already shifted. */
EXPORT int orc_cond(const orc_config *c, const float *blob, int j, const real *x, real *mu, real *alpha) {
    block_w bw; cond_ws w;
    if (c->n_layers > ORC_MAX_LAYERS || ws_alloc(c, &w)) return -1;
    map_block(c, blob, j, &bw);
    cond_full(c, &bw, x, &w);
    for (int l = 0; l < c->seq_len; ++l)
        for (int d = 0; d < c->token_dim; ++d)
            params_of(c, &w, l, d, &mu[(size_t)l * c->token_dim + d], &alpha[(size_t)l * c->token_dim + d]);
    ws_free(&w);
    return 0;
}

/* eq. 4 for block j: canonical order in (x), canonical order out (y).  If logdet is not NULL it
 * receives log |det dy/dx| of this block: the map is triangular in the processing order with
 * diagonal exp(-alpha), so the log-determinant is minus the sum of all alpha (the term that the
 * change-of-variables formula, eq. 1, adds per block; token 1 has alpha = 0). */
static int forward_block_impl(const orc_config *c, const float *blob, int j, const real *x, real *y, real *logdet) {
    int T = c->seq_len, D = c->token_dim, rev = (c->reverse_mask >> j) & 1;
    block_w bw; cond_ws w;
    if (c->n_layers > ORC_MAX_LAYERS || ws_alloc(c, &w)) return -1;
    map_block(c, blob, j, &bw);
    real *u = (real *)malloc(sizeof(real) * T * D), *v = (real *)malloc(sizeof(real) * T * D);
    flip_tokens(c, rev, x, u);
    cond_full(c, &bw, u, &w);
    double sum_alpha = 0.0;
    for (int l = 0; l < T; ++l)
        for (int d = 0; d < D; ++d) {
            real mu, al;
            params_of(c, &w, l, d, &mu, &al);
            v[(size_t)l * D + d] = (u[(size_t)l * D + d] - mu) * (real)exp((double)(-al));
            sum_alpha += (double)al;
        }
    if (logdet) *logdet = (real)(-sum_alpha);
    flip_tokens(c, rev, v, y);
    free(u); free(v); ws_free(&w);
    return 0;
}

EXPORT int orc_forward_block(const orc_config *c, const float *blob, int j, const real *x, real *y) {
    return forward_block_impl(c, blob, j, x, y, NULL);
}

EXPORT int orc_forward_block_logdet(const orc_config *c, const float *blob, int j, const real *x, real *y, real *logdet) {
    return forward_block_impl(c, blob, j, x, y, logdet);
}

/* eq. 5 by the definition: for every token a full conditioner pass over the sequence built so
 * far; the not yet generated tokens hold `fill` (they cannot matter). */
EXPORT int orc_sequential_inverse_block_naive(const orc_config *c, const float *blob, int j, const real *z, real *x,
                                              double fill) {
    int T = c->seq_len, D = c->token_dim, rev = (c->reverse_mask >> j) & 1;
    block_w bw; cond_ws w;
    if (c->n_layers > ORC_MAX_LAYERS || ws_alloc(c, &w)) return -1;
    map_block(c, blob, j, &bw);
    real *u = (real *)malloc(sizeof(real) * T * D), *v = (real *)malloc(sizeof(real) * T * D);
    flip_tokens(c, rev, z, u);
    for (size_t i = 0; i < (size_t)T * D; ++i) v[i] = (real)fill;
    for (int d = 0; d < D; ++d) v[d] = u[d];
    for (int l = 1; l < T; ++l) {
        cond_full(c, &bw, v, &w);
        for (int d = 0; d < D; ++d) {
            real mu, al;
            params_of(c, &w, l, d, &mu, &al);
            v[(size_t)l * D + d] = u[(size_t)l * D + d] * (real)exp((double)al) + mu;
        }
    }
    flip_tokens(c, rev, v, x);
    free(u); free(v); ws_free(&w);
    return 0;
}

static void sequential_inverse_cached(const orc_config *c, const block_w *bw, const real *u, real *v, cond_ws *w) {
    int T = c->seq_len, D = c->token_dim;
    for (int d = 0; d < D; ++d) v[d] = u[d];
    for (int l = 1; l < T; ++l) {
        cond_step(c, bw, v + (size_t)(l - 1) * D, l - 1, w);
        for (int d = 0; d < D; ++d) {
            real mu, al;
            params_of(c, w, l, d, &mu, &al);
            v[(size_t)l * D + d] = u[(size_t)l * D + d] * (real)exp((double)al) + mu;
        }
    }
}

/* eq. 5 with the key/value cache: T-1 single-token conditioner steps. */
EXPORT int orc_sequential_inverse_block(const orc_config *c, const float *blob, int j, const real *z, real *x) {
    int T = c->seq_len, D = c->token_dim, rev = (c->reverse_mask >> j) & 1;
    block_w bw; cond_ws w;
    if (c->n_layers > ORC_MAX_LAYERS || ws_alloc(c, &w)) return -1;
    map_block(c, blob, j, &bw);
    real *u = (real *)malloc(sizeof(real) * T * D), *v = (real *)malloc(sizeof(real) * T * D);
    flip_tokens(c, rev, z, u);
    sequential_inverse_cached(c, &bw, u, v, &w);
    flip_tokens(c, rev, v, x);
    free(u); free(v); ws_free(&w);
    return 0;
}

/* One application of F (Def. A.1), canonical order: x_new = F(x_prev) for block input z. */
EXPORT int orc_jacobi_map(const orc_config *c, const float *blob, int j, const real *z, const real *x_prev,
                          real *x_new) {
    int T = c->seq_len, D = c->token_dim, rev = (c->reverse_mask >> j) & 1;
    block_w bw; cond_ws w;
    if (c->n_layers > ORC_MAX_LAYERS || ws_alloc(c, &w)) return -1;
    map_block(c, blob, j, &bw);
    real *u = (real *)malloc(sizeof(real) * T * D), *a = (real *)malloc(sizeof(real) * T * D),
         *b = (real *)malloc(sizeof(real) * T * D);
    flip_tokens(c, rev, z, u);
    flip_tokens(c, rev, x_prev, a);
    jacobi_map(c, &bw, u, a, b, &w);
    flip_tokens(c, rev, b, x_new);
    free(u); free(a); free(b); ws_free(&w);
    return 0;
}

/* Alg. 1 on processing-order data.  x0 may be NULL (zeros).  trace (nullable) receives delta of
 * every pass, iterates (nullable) every iterate x^1..x^it ([cap][T*D], processing order). */
static int jacobi_decode(const orc_config *c, const block_w *bw, const real *u, const real *x0, double tau,
                         int criterion, int max_iters, real *v, real *trace, real *iterates, real *last_delta,
                         cond_ws *w) {
    size_t n = (size_t)c->seq_len * c->token_dim;
    int cap = (max_iters > 0 && max_iters < c->seq_len) ? max_iters : c->seq_len;
    real *prev = (real *)malloc(sizeof(real) * n);
    if (x0) memcpy(prev, x0, sizeof(real) * n); else memset(prev, 0, sizeof(real) * n);
    int it = 0;
    real delta = 0;
    for (;;) {
        it += 1;
        jacobi_map(c, bw, u, prev, v, w);
        delta = iterate_distance(c, criterion, v, prev);
        if (trace) trace[it - 1] = delta;
        if (iterates) memcpy(iterates + (size_t)(it - 1) * n, v, sizeof(real) * n);
        if ((double)delta < tau || it == cap) break;
        memcpy(prev, v, sizeof(real) * n);
    }
    if (last_delta) *last_delta = delta;
    free(prev);
    return it;
}

/* Alg. 1 for block j, canonical order in/out.  Returns the pass count (>= 1) or -1. */
EXPORT int orc_jacobi_inverse_block(const orc_config *c, const float *blob, int j, const real *z, const real *x0,
                                    double tau, int criterion, int max_iters, real *x, real *trace,
                                    real *iterates) {
    int T = c->seq_len, D = c->token_dim, rev = (c->reverse_mask >> j) & 1;
    size_t n = (size_t)T * D;
    block_w bw; cond_ws w;
    if (c->n_layers > ORC_MAX_LAYERS || ws_alloc(c, &w)) return -1;
    map_block(c, blob, j, &bw);
    real *u = (real *)malloc(sizeof(real) * n), *v = (real *)malloc(sizeof(real) * n), *g = NULL;
    flip_tokens(c, rev, z, u);
    if (x0) { g = (real *)malloc(sizeof(real) * n); flip_tokens(c, rev, x0, g); }
    int it = jacobi_decode(c, &bw, u, g, tau, criterion, max_iters, v, trace, iterates, NULL, &w);
    flip_tokens(c, rev, v, x);
    if (iterates && rev) { /* hand iterates back in canonical order as well */
        for (int i = 0; i < it; ++i) { flip_tokens(c, 1, iterates + (size_t)i * n, u); memcpy(iterates + (size_t)i * n, u, sizeof(real) * n); }
    }
    free(u); free(v); free(g); ws_free(&w);
    return it;
}

/* ---------------------------------------------------------------- exported, batch */

/* The cascade (eq. 2) in sampling order with a per-block mode: bit j of jacobi_mask set => block
 * j by Alg. 1, else by eq. 5 (key/value cached).  init: 0 zeros, 1 the block's input.  iters
 * [K][B] receives pass counts (T-1 for a sequential block), deltas [K][B] the last delta of each
 * Jacobi block (0 for sequential).  Samples are independent and run in parallel threads. */
EXPORT int orc_sample(const orc_config *c, const float *blob, const real *z, real *x, int batch, uint32_t jacobi_mask,
                      double tau, int criterion, int init, int max_iters, int32_t *iters, real *deltas) {
    int T = c->seq_len, D = c->token_dim, K = c->n_blocks;
    size_t n = (size_t)T * D;
    if (c->n_layers > ORC_MAX_LAYERS) return -1;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < batch; ++b) {
        block_w bw; cond_ws w;
        if (ws_alloc(c, &w)) { fail = 1; continue; }
        real *cur = (real *)malloc(sizeof(real) * n), *u = (real *)malloc(sizeof(real) * n),
             *v = (real *)malloc(sizeof(real) * n);
        memcpy(cur, z + (size_t)b * n, sizeof(real) * n);
        for (int j = 0; j < K; ++j) {
            int rev = (c->reverse_mask >> j) & 1;
            map_block(c, blob, j, &bw);
            flip_tokens(c, rev, cur, u);
            int it; real dl = 0;
            if ((jacobi_mask >> j) & 1u) {
                it = jacobi_decode(c, &bw, u, init == 1 ? u : NULL, tau, criterion, max_iters, v, NULL, NULL, &dl, &w);
            } else {
                sequential_inverse_cached(c, &bw, u, v, &w);
                it = T - 1;
            }
            flip_tokens(c, rev, v, cur);
            if (iters) iters[(size_t)j * batch + b] = it;
            if (deltas) deltas[(size_t)j * batch + b] = dl;
        }
        memcpy(x + (size_t)b * n, cur, sizeof(real) * n);
        free(cur); free(u); free(v); ws_free(&w);
    }
    return fail ? -1 : 0;
}

/* The forward map of the whole flow: blocks K-1 .. 0 of eq. 4, so that forward(sample(z)) = z. */
EXPORT int orc_forward(const orc_config *c, const float *blob, const real *x, real *z, int batch) {
    size_t n = (size_t)c->seq_len * c->token_dim;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < batch; ++b) {
        real *cur = (real *)malloc(sizeof(real) * n), *nxt = (real *)malloc(sizeof(real) * n);
        memcpy(cur, x + (size_t)b * n, sizeof(real) * n);
        for (int j = c->n_blocks - 1; j >= 0; --j) {
            if (orc_forward_block(c, blob, j, cur, nxt)) fail = 1;
            real *t = cur; cur = nxt; nxt = t;
        }
        memcpy(z + (size_t)b * n, cur, sizeof(real) * n);
        free(cur); free(nxt);
    }
    return fail ? -1 : 0;
}

/* The same with the log-determinant of the whole forward map per sample: the sum over blocks (eq. 2's
 * composition, so the Jacobians multiply). */
EXPORT int orc_forward_logdet(const orc_config *c, const float *blob, const real *x, real *z, real *logdet, int batch) {
    size_t n = (size_t)c->seq_len * c->token_dim;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < batch; ++b) {
        real *cur = (real *)malloc(sizeof(real) * n), *nxt = (real *)malloc(sizeof(real) * n);
        memcpy(cur, x + (size_t)b * n, sizeof(real) * n);
        double total = 0.0;
        for (int j = c->n_blocks - 1; j >= 0; --j) {
            real ld = 0;
            if (forward_block_impl(c, blob, j, cur, nxt, &ld)) fail = 1;
            total += (double)ld;
            real *t = cur; cur = nxt; nxt = t;
        }
        memcpy(z + (size_t)b * n, cur, sizeof(real) * n);
        logdet[b] = (real)total;
        free(cur); free(nxt);
    }
    return fail ? -1 : 0;
}

/* ---------------------------------------------------------------- exported primitives (for the pins) */

EXPORT void orc_layernorm(const real *x, const float *g, const float *b, int rows, int W, real *y) {
    for (int r = 0; r < rows; ++r) layernorm_row(x + (size_t)r * W, g, b, W, y + (size_t)r * W);
}
EXPORT void orc_linear(const real *a, const float *Wm, const float *bias, int rows, int K, int N, real *y) {
    for (int r = 0; r < rows; ++r) linear_row(a + (size_t)r * K, Wm, bias, K, N, y + (size_t)r * N);
}
EXPORT void orc_gelu(const real *x, int n, real *y) {
    for (int i = 0; i < n; ++i) y[i] = gelu_erf(x[i]);
}
/* q, k, v, o: [T][W]; row t attends rows 0..t */
EXPORT void orc_causal_attention(const real *q, const real *k, const real *v, int T, int W, int H, real *o) {
    real *scores = (real *)malloc(sizeof(real) * T);
    for (int t = 0; t < T; ++t) attend_row(q + (size_t)t * W, k, v, t, W, H, o + (size_t)t * W, scores);
    free(scores);
}
