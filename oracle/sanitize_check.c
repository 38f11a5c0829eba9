/*
 * Sanitizer driver for the CPU oracle.  TEST INFRASTRUCTURE ONLY (built and run by
 * tests/test_oracle_sanitized.py with -fsanitize=address,undefined on the host; never part of the product).
 *
 * It includes the oracle's source, so that every function runs instrumented, and drives every exported
 * entry point on small flows whose buffers are allocated at exactly their stated sizes: an index past a
 * weight tensor, an iterate or a workspace, a misaligned access or a signed overflow ends the run.
 * Besides "no finding" it checks the invariants the paper fixes, so that the instrumented build is known
 * to compute the same thing: forward(inverse(z)) = z (eq. 4 / eq. 5), Jacobi decoding equals the sequential
 * inverse after T passes (Prop. 3.2), one token is exact in one pass.  The weights are drawn by a
 * linear congruential generator: no arithmetic of the method lives here.
 */
#include "sjd_oracle.c"
#include <stdio.h>

static uint32_t lcg_state = 12345u;
static float lcg_uniform(void) {           /* in (-1, 1) */
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return ((float)(lcg_state >> 8) / 8388608.0f) - 1.0f;
}

static double max_abs_diff(const real *a, const real *b, size_t n) {
    double m = 0;
    for (size_t i = 0; i < n; ++i) { double d = fabs((double)a[i] - (double)b[i]); if (d > m) m = d; }
    return m;
}

#define CHECK(cond, ...) do { if (!(cond)) { fprintf(stderr, "sanitize_check: " __VA_ARGS__); fprintf(stderr, "\n"); return 1; } } while (0)

static int run_case(int K, int N, int W, int H, int T, int D, int B, int mask_nearest) {
    orc_config c = {K, N, W, H, 4, T, D, 0, mask_nearest};
    for (int j = 1; j < K; j += 2) c.reverse_mask |= 1u << j;
    size_t nb = orc_block_floats(&c) * (size_t)K, n = (size_t)T * D;
    float *blob = (float *)malloc(sizeof(float) * nb);
    for (size_t i = 0; i < nb; ++i) blob[i] = 0.15f * lcg_uniform();
    real *z = (real *)malloc(sizeof(real) * n * B), *x = (real *)malloc(sizeof(real) * n * B),
         *y = (real *)malloc(sizeof(real) * n * B), *t0 = (real *)malloc(sizeof(real) * n),
         *t1 = (real *)malloc(sizeof(real) * n), *ld = (real *)malloc(sizeof(real) * B),
         *dl = (real *)malloc(sizeof(real) * K * B), *trace = (real *)malloc(sizeof(real) * T),
         *its = (real *)malloc(sizeof(real) * n * T);
    int32_t *iters = (int32_t *)malloc(sizeof(int32_t) * K * B);
    for (size_t i = 0; i < n * B; ++i) z[i] = (real)(2.0f * lcg_uniform());
    const double tol = sizeof(real) == 8 ? 1e-10 : 2e-4;
    const uint32_t all = K >= 32 ? 0xFFFFFFFFu : ((1u << K) - 1u);

    /* cascade three ways; forward takes each result back (Jacobi at tau = 0 is exact, Prop. 3.2) */
    const uint32_t masks[3] = {0u, all & ~1u, all};
    for (int m = 0; m < 3; ++m)
        for (int init = 0; init < 2; ++init) {
            CHECK(orc_sample(&c, blob, z, x, B, masks[m], 0.0, m & 1, init, 0, iters, dl) == 0, "orc_sample failed");
            CHECK(orc_forward(&c, blob, x, y, B) == 0, "orc_forward failed");
            CHECK(max_abs_diff(y, z, n * B) <= tol, "forward(inverse(z)) != z (mask %u, init %d): %g", masks[m], init,
                  max_abs_diff(y, z, n * B));
            CHECK(orc_forward_logdet(&c, blob, x, y, ld, B) == 0, "orc_forward_logdet failed");
            CHECK(max_abs_diff(y, z, n * B) <= tol, "forward with log-determinant disagrees with forward");
        }
    /* an early stop and a lowered cap */
    CHECK(orc_sample(&c, blob, z, x, B, all & ~1u, 1e-3, 0, 0, 2, iters, dl) == 0, "orc_sample (capped) failed");
    for (int j = 1; j < K; ++j) for (int b = 0; b < B; ++b) CHECK(iters[j * B + b] <= (T < 2 ? T : 2), "cap ignored");

    /* block-level entry points on the first sample */
    for (int j = 0; j < K; ++j) {
        CHECK(orc_sequential_inverse_block(&c, blob, j, z, t0) == 0, "sequential failed");
        CHECK(orc_sequential_inverse_block_naive(&c, blob, j, z, t1, 7.5) == 0, "naive sequential failed");
        CHECK(max_abs_diff(t0, t1, n) <= tol, "cached and by-definition sequential inverses differ (block %d)", j);
        int it = orc_jacobi_inverse_block(&c, blob, j, z, z, 0.0, 1, 0, t1, trace, its);
        CHECK(it == T, "tau = 0 must run T passes, ran %d", it);
        CHECK(max_abs_diff(t0, t1, n) <= tol, "Jacobi after T passes != sequential inverse (block %d)", j);
        CHECK(max_abs_diff(its + (size_t)(T - 1) * n, t1, n) == 0.0, "last recorded iterate is not the result");
        CHECK(orc_jacobi_map(&c, blob, j, z, t0, t1) == 0, "jacobi_map failed");
        CHECK(max_abs_diff(t0, t1, n) <= tol, "the sequential inverse is not a fixed point of F (block %d)", j);
        CHECK(orc_forward_block(&c, blob, j, t0, t1) == 0, "forward_block failed");
        CHECK(max_abs_diff(t1, z, n) <= tol, "forward block does not invert the inverse (block %d)", j);
        CHECK(orc_forward_block_logdet(&c, blob, j, t0, t1, ld) == 0, "forward_block_logdet failed");
        CHECK(orc_cond(&c, blob, j, t0, t1, y) == 0, "cond failed");
        for (int d = 0; d < D; ++d) CHECK(t1[d] == 0 && y[d] == 0, "first processed token must have mu = alpha = 0");
    }
    /* exported primitives */
    {
        real *q = (real *)malloc(sizeof(real) * T * W), *o = (real *)malloc(sizeof(real) * T * W),
             *w2 = (real *)malloc(sizeof(real) * T * 2 * D);
        for (size_t i = 0; i < (size_t)T * W; ++i) q[i] = (real)lcg_uniform();
        block_w bw; map_block(&c, blob, 0, &bw);
        orc_layernorm(q, bw.lnf_g, bw.lnf_b, T, W, o);
        orc_linear(o, bw.w_head, bw.b_head, T, W, 2 * D, w2);
        orc_gelu(q, T * W, o);
        orc_causal_attention(q, q, q, T, W, H, o);
        free(q); free(o); free(w2);
    }
    free(blob); free(z); free(x); free(y); free(t0); free(t1); free(ld); free(dl); free(trace); free(its); free(iters);
    return 0;
}

int main(void) {
    /*             K  N  W   H  T  D  B  o */
    if (run_case(3, 2, 16, 2, 7, 3, 3, 0)) return 1;
    if (run_case(2, 1, 8, 1, 1, 2, 2, 0)) return 1;      /* one token */
    if (run_case(2, 1, 12, 3, 5, 1, 1, 2)) return 1;     /* masked-dependency probe, head size 4 */
    if (run_case(4, 1, 8, 2, 9, 2, 5, 0)) return 1;      /* more samples than threads on small hosts */
    printf("sanitize_check: ok\n");
    return 0;
}
