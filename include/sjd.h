/*
 * sjd.h - C boundary of the MI355X (gfx950) library for selective Jacobi decoding: the inverse
 * (sampling) pass of a block-autoregressive normalizing flow whose conditioner is a causal
 * transformer.
 *
 * Vocabulary.  T tokens per sample (the paper's L), D values per token, K flow blocks, N
 * transformer layers per block, W width, H heads, B batch.  Blocks are numbered in SAMPLING
 * order: block 0 is the first one applied to the latent (the paper's "first (K-th) layer",
 * Sec. 3.5).  For a block with input y (the paper's z_{k+1}) and output x (z_k), per token l:
 *     x_1 = y_1,    x_l = y_l * exp(alpha_l) + mu_l,    (mu, alpha)_l = conditioner(x_<l),
 * which is eq. 5 with mu = g_k and alpha = -s_k.  The conditioner sees tokens strictly before l.
 * Bit j of sjd_config.reverse_mask makes block j work on the reversed token order (the
 * permutation mentioned below eq. 4); data crossing this boundary is always in canonical order.
 *
 * Memory.  Every pointer named *_dev is DEVICE memory owned by the caller (contiguous float32
 * [batch, T, D]); pointers named *_host are HOST memory owned by the caller.  The library neither
 * frees nor keeps them.  z_dev and x_dev must not overlap.  The handle owns the weights, the
 * key/value cache and all workspaces, sized at creation for max_batch.
 *
 * Streams.  `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  All work
 * is enqueued on it.  Calls that run Jacobi decoding read one integer per pass back to the host
 * (the number of samples still iterating) and therefore synchronise that stream; all calls
 * return with their outputs complete.  One handle must not be used from two threads at once.
 *
 * Errors.  Every int-returning call gives SJD_OK (0) or a negative code; nothing throws or aborts
 * across this boundary.  sjd_last_error() returns a thread-local description of the last failure.
 *
 * This library has no CPU path: every step runs in HIP kernels, and creation fails with SJD_EHIP
 * when no gfx950 device is usable.
 */
#ifndef SJD_H
#define SJD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SJD_OK 0
#define SJD_EINVAL (-1)     /* null pointer, bad shape, batch > max_batch, NaN tau, bad block index ... */
#define SJD_ENOMEM (-2)     /* host or device allocation failed */
#define SJD_EHIP (-3)       /* a HIP call failed; see sjd_last_error() */
#define SJD_ENONFINITE (-4) /* a sample's iterate difference was NaN/Inf when its loop ended; outputs are written */
#define SJD_ESTATE (-5)     /* weights not loaded yet */

#define SJD_MAX_BLOCKS 32

#define SJD_DTYPE_F32 0  /* everything float32 (correctness configuration) */
#define SJD_DTYPE_BF16 1 /* bf16 weights, matrix operands, stored activations and KV cache; float32 state
                            (x, mu, alpha), residual stream, LayerNorm statistics, softmax, accumulators, delta */
#define SJD_DTYPE_F16 2  /* as SJD_DTYPE_BF16 but every 16-bit operand is IEEE half: three more mantissa bits
                            for the same matrix-core rate.  bf16-valued weights convert exactly (values below
                            2^-14 in magnitude to within 2^-25). */

#if defined(__GNUC__)
#define SJD_API __attribute__((visibility("default")))
#else
#define SJD_API
#endif

typedef struct sjd_flow sjd_flow; /* opaque */

typedef struct {
    int32_t n_blocks;   /* K, 1..SJD_MAX_BLOCKS */
    int32_t n_layers;   /* N >= 1 */
    int32_t width;      /* W, a multiple of n_heads and of 4; the 16-bit modes need W % 64 == 0 */
    int32_t n_heads;    /* H */
    int32_t mlp_ratio;  /* hidden = mlp_ratio * W */
    int32_t seq_len;    /* T >= 1 */
    int32_t token_dim;  /* D >= 1 */
    int32_t max_batch;  /* largest batch any call will pass */
    int32_t dtype;      /* SJD_DTYPE_* */
    uint32_t reverse_mask;
} sjd_config;

/* Options of Jacobi decoding (Sec. 3.3, Alg. 1). */
typedef struct {
    float tau;              /* stop a sample when its delta < tau (strict).  tau = 0 runs to the cap. */
    int32_t criterion;      /* 0: delta = mean over (l, d) of |x^t - x^(t-1)|;  1: the maximum (Alg. 1 as printed) */
    int32_t init;           /* 0: x^0 = 0 (Alg. 1);  1: x^0 = the block's input;  2: x^0 = what x_dev holds on entry,
                               e.g. the caller's own N(0, I) draw (the initialisation study of Sec. 4.3) */
    int32_t max_iters;      /* 0 or >= T: the cap is T (Prop. 3.2: the T-th iterate is exact); else a lower cap */
    int32_t drop_converged; /* 1: converged samples leave the batch the conditioner runs on;  0: they stay
                               (and are ignored).  Results and counts are the same either way. */
    float refine_below;     /* 16-bit flows only; 0: off.  A sample whose delta has fallen below this level runs its
                               remaining passes of the block in float32 arithmetic (float32 weights and activations).
                               The rounding of 16-bit operands keeps delta from falling much below 1e-4 (IEEE half) or
                               1e-3 (bf16): with tau under that floor, set this a few times above it (1e-3 for half)
                               and the pass counts follow exact arithmetic again.  Per sample, so a sample's result
                               still does not depend on the batch.  The first use allocates float32 workspaces for
                               about 8192 rows in the handle. */
} sjd_jacobi_opts;

typedef struct {
    int32_t block_iters[SJD_MAX_BLOCKS];     /* conditioner passes launched (max over samples); T-1 for a sequential block */
    float mean_sample_iters[SJD_MAX_BLOCKS]; /* mean over samples of each sample's own pass count */
    float block_ms[SJD_MAX_BLOCKS];          /* device time of the block, from events on the stream */
} sjd_stats;

/* Timing of kernel families inside the library (for roofline reports).  Off by default. */
/* One family per kernel (template instantiation) that a profiler would list, so that a family's average launch
 * time can be compared with a kernel trace directly. */
#define SJD_PROF_GEMM 0        /* whole-sequence passes: the fused q/k/v projection (bias epilogue, 16-bit out) */
#define SJD_PROF_ATTENTION 1   /* whole-sequence causal attention */
#define SJD_PROF_EPILOGUE 2    /* fused affine update / difference reduction / convergence; step advance of the sequential inverse */
#define SJD_PROF_DECODE_GEMM 3 /* single-token steps: LayerNorm + q/k/v projection */
#define SJD_PROF_DECODE_ATTN 4 /* KV-cached single-token attention */
#define SJD_PROF_OTHER 5       /* embedding, LayerNorm, ... */
#define SJD_PROF_DECODE_FUSED 6 /* the sequential inverse of a whole block as one persistent kernel */
#define SJD_PROF_GEMM_RESID 7  /* whole-sequence passes: attention-output and MLP-output projections (one kernel:
                                  float32 residual epilogue; they differ in k) */
#define SJD_PROF_GEMM_FC1 8    /* whole-sequence passes: MLP input projection (GELU epilogue) */
#define SJD_PROF_DECODE_RESID 9 /* single-token steps: attention-output and MLP-output projections */
#define SJD_PROF_GEMM_HEAD 10  /* whole-sequence passes: the [mu | alpha] head */
#define SJD_PROF_DECODE_FC1 11 /* single-token steps: LayerNorm + MLP input projection + GELU */
#define SJD_PROF_DECODE_HEAD 12 /* single-token steps: final LayerNorm + head */
#define SJD_PROF_FAMILIES 13
typedef struct {
    double ms[SJD_PROF_FAMILIES];       /* summed device time per family since the last reset */
    int64_t launches[SJD_PROF_FAMILIES];
    double flops[SJD_PROF_FAMILIES];    /* algorithmic flops of those launches (2*M*N*K, causal attention counted on the lower triangle) */
    double bytes[SJD_PROF_FAMILIES];    /* algorithmic bytes: operands read once + results written once */
} sjd_profile;

/* Creates a flow for `cfg` on the current HIP device and allocates every buffer it will need.
 * *out receives the handle.  SJD_EINVAL for shapes outside the limits stated at sjd_config. */
SJD_API int sjd_flow_create(const sjd_config *cfg, sjd_flow **out);

/* "Load flow weights": copies the functions s_k, g_k of every block (Alg. 1, Input) to the device.
 * host_blob is HOST memory: K blocks in sampling order, each a run of little-endian float32
 * tensors, matrices row-major [in, out]:
 *     w_in [D,W]  b_in [W]  pos [T,W]
 *     N x { ln1_g [W] ln1_b [W]  w_qkv [W,3W] b_qkv [3W]  w_o [W,W] b_o [W]
 *           ln2_g [W] ln2_b [W]  w_fc1 [W,R*W] b_fc1 [R*W]  w_fc2 [R*W,W] b_fc2 [W] }
 *     lnf_g [W] lnf_b [W]  w_head [W,2D] b_head [2D]          (head columns: [mu | alpha])
 * q, k, v are the three W-wide column groups of w_qkv; head h owns columns h*dh..(h+1)*dh of each.
 * nbytes must equal the size that layout implies, else SJD_EINVAL.  In the 16-bit modes matrices
 * are rounded to that type (nearest even) on load.  The blob is not referenced after the call returns. */
SJD_API int sjd_flow_load_weights(sjd_flow *flow, const void *host_blob, size_t nbytes);

/* Jacobi decoding of block `block` (Sec. 3.3, Alg. 1; iteration map of App. B, Def. A.1):
 * x^0 per opts->init, then x^t = F(x^(t-1)) for all tokens at once, each sample stopping by its own
 * delta (see sjd_jacobi_opts) or at the cap.  z_dev: the block's input; x_dev: receives each
 * sample's newest iterate.  iters_per_sample_host (nullable, [batch]): passes each sample took,
 * counting the last one.  block_iters_host (nullable): passes launched.  SJD_ENONFINITE if a
 * sample ended with a non-finite delta. */
SJD_API int sjd_jacobi_inverse_block(sjd_flow *flow, int block, const float *z_dev, float *x_dev, int batch,
                             const sjd_jacobi_opts *opts, int32_t *iters_per_sample_host,
                             int32_t *block_iters_host, void *hip_stream);

/* Jacobi decoding of one block with a per-pass record (the convergence curves of Sec. 4.3 and
 * App. B: how fast the iterates approach the sequential solution).  Works like
 * sjd_jacobi_inverse_block and additionally fills, for pass p = 0 .. passes-1 and sample b,
 *   delta_trace_host[p * batch + b] = that sample's delta after pass p+1 (criterion of opts),
 *   err_trace_host  [p * batch + b] = || x^(p+1) - x_ref ||_2 over the sample's T*D values
 * (HOST arrays of at least cap * batch floats, cap = the pass cap of opts; err_trace_host may be
 * NULL; x_ref_dev is DEVICE memory [batch, T, D], typically the sequential inverse, and may be NULL
 * when no error trace is wanted).  A sample that has stopped keeps its last iterate, so its
 * entries repeat from then on. */
SJD_API int sjd_jacobi_trace_block(sjd_flow *flow, int block, const float *z_dev, float *x_dev, const float *x_ref_dev,
                                   int batch, const sjd_jacobi_opts *opts, float *delta_trace_host,
                                   float *err_trace_host, int32_t *iters_per_sample_host, int32_t *block_iters_host,
                                   void *hip_stream);

/* Forward (data -> latent) map of block `block`, eq. 4: one whole-sequence conditioner pass on
 * x_dev, then y = (x - mu) * exp(-alpha) for every token (the first processed token is copied).
 * logdet_dev (nullable, DEVICE, [batch] float32) receives log |det dy/dx| = -sum alpha of each
 * sample, the block's term in the change-of-variables formula (eq. 1); with accumulate != 0 it is
 * added to what logdet_dev holds.  x_dev and y_dev may not overlap. */
SJD_API int sjd_forward_block(sjd_flow *flow, int block, const float *x_dev, float *y_dev, float *logdet_dev,
                              int accumulate, int batch, void *hip_stream);

/* The whole forward map z_K = f^-1(x): blocks K-1 .. 0 of eq. 4 (the inverse of sjd_sample's cascade,
 * eq. 2), K conditioner passes in all.  logdet_dev (nullable, DEVICE, [batch]) receives the sum of
 * the blocks' log-determinants. */
SJD_API int sjd_forward(sjd_flow *flow, const float *x_dev, float *z_dev, float *logdet_dev, int batch,
                        void *hip_stream);

/* Sequential inverse of block `block` (Sec. 3.1, eq. 5) with a key/value cache (Sec. 3.5):
 * T-1 single-token conditioner steps. */
SJD_API int sjd_sequential_inverse_block(sjd_flow *flow, int block, const float *z_dev, float *x_dev, int batch,
                                 void *hip_stream);

/* The whole cascade x = f_0(...f_{K-1}(z_K)) (Sec. 3.1, eq. 2) with a per-block mode (Sec. 3.5):
 * bit j of jacobi_mask set => block j by Jacobi decoding, clear => sequentially.  ~1u is the
 * selective strategy, 0 the sequential baseline, ~0u Jacobi everywhere.  stats_host (nullable) and
 * iters_host (nullable, [K][batch] passes per block and sample) are filled on return.
 * opts->init = 2 is refused here (there is no caller-held first iterate inside the cascade). */
SJD_API int sjd_sample(sjd_flow *flow, const float *z_dev, float *x_dev, int batch, uint32_t jacobi_mask,
               const sjd_jacobi_opts *opts, sjd_stats *stats_host, int32_t *iters_host, void *hip_stream);

/* One whole-sequence conditioner pass of block `block` on x_dev [batch, T, D] (canonical order):
 * mu_dev, alpha_dev [batch, T, D] receive the parameters of every token computed from the tokens
 * before it (zeros for the first processed token).  This is s_k, g_k of eq. 5 evaluated for all l
 * at once, i.e. the inside of F (Def. A.1); exported so that it can be checked on its own. */
SJD_API int sjd_conditioner(sjd_flow *flow, int block, const float *x_dev, float *mu_dev, float *alpha_dev, int batch,
                    void *hip_stream);

/* One dense projection of the conditioner on its own, C = epi(A * W + bias), in a 16-bit mode: the
 * building block of every whole-sequence pass (the s_k, g_k networks of eq. 5 are stacks of these),
 * exported so that each matrix-core kernel can be checked against the oracle on small shapes.
 * All pointers are DEVICE memory.  a_dev: [M, K] 16-bit row-major.  wt_dev: the weight TRANSPOSED,
 * [N rounded up to a multiple of 256, K] 16-bit, K contiguous, padding rows zero.  bias_dev [N] float32.
 * epilogue 0: c_dev [M, N] 16-bit = A W + bias;  1: c_dev = GELU(A W + bias) (erf form);
 * 2: resid_out_dev [M, N] float32 += A W + bias (c_dev unused).  K must be a multiple of 64.
 * kernel: 0 chosen by shape, 1..3 a specific tile kernel, 4 the persistent eight-wave kernel (K a multiple of 128
 * and N a multiple of 256; other shapes fall back to 0).  dtype: SJD_DTYPE_BF16 or SJD_DTYPE_F16. */
SJD_API int sjd_op_linear_h16(int dtype, int kernel, const void *a_dev, const void *wt_dev, const float *bias_dev,
                              float *resid_out_dev, void *c_dev, int M, int N, int K, int epilogue, void *hip_stream);

/* The same building block on the activation-stationary kernels that 16-bit flows of width 512 use for
 * their whole-sequence passes (N a multiple of 256), exported for the same reason.
 * epilogue 0 / 1 (K = 512): a_dev is the float32 residual stream [M, 512]; the op computes
 * c_dev [M, N] 16-bit = epi(LayerNorm(a; ln_g_dev, ln_b_dev [512] float32, eps 1e-5) W + bias) - LayerNorm
 * is part of the launch.  epilogue 2 (K a multiple of 512): a_dev is [M, K] 16-bit, resid_out_dev [M, N]
 * float32 += A W + bias (ln pointers unused); K = 512 runs the panel kernel (N <= 512), K > 512 the kernel
 * that streams the left operand through LDS.  wt_dev as for sjd_op_linear_h16 ([N, K] transposed 16-bit);
 * the op makes a temporary device copy of it in the kernels' fragment order (it allocates and frees
 * 2 N K bytes).  All pointers are DEVICE memory.  SJD_EINVAL for shapes outside the kernels' range. */
SJD_API int sjd_op_panel_linear_h16(int dtype, const void *a_dev, const float *ln_g_dev, const float *ln_b_dev,
                                    const void *wt_dev, const float *bias_dev, float *resid_out_dev, void *c_dev, int M,
                                    int N, int K, int epilogue, void *hip_stream);

/* sjd_op_panel_linear_h16 for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same results (bit for bit);
 * the temporary fragment-order copy of the weight lives in a device array of the library (4 MiB, present on
 * every GPU the library runs on until the process ends) instead of a per-call allocation, so the weight is
 * limited to 2 N K <= 4 MiB (SJD_EINVAL beyond, e.g. N = 1024 with K = 4096).  The call allocates and frees
 * nothing.  Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU race and must
 * be serialised by the caller; calls in sequence need no clearing in between (each rewrites all it reads). */
SJD_API int sjd_op_panel_linear_h16_noalloc(int dtype, const void *a_dev, const float *ln_g_dev, const float *ln_b_dev,
                                            const void *wt_dev, const float *bias_dev, float *resid_out_dev, void *c_dev,
                                            int M, int N, int K, int epilogue, void *hip_stream);

/* Whole-sequence causal multi-head attention of the conditioner on its own (the attention inside s_k, g_k of
 * eq. 5, evaluated for all positions at once as in the map F of Def. A.1), head size 64, in the mode `dtype`
 * (the 16-bit modes, or SJD_DTYPE_F32 for the float32 kernel that refined passes and float32 flows use);
 * exported so that the matrix-core attention kernels can be checked against the oracle at any token count.
 * qkv_dev: DEVICE, [n_samples * T, 3 * H * 64] row-major in that type, columns [q | k | v], head h owning
 * columns 64 h .. 64 h + 63 of each group.  o_dev: DEVICE, [n_samples * T, H * 64] in that type, position t
 * attending positions 0..t with scale 1/8.  No T x T buffer is formed.  SJD_EINVAL for non-positive sizes or
 * T > 4096. */
SJD_API int sjd_op_attention_h16(int dtype, const void *qkv_dev, void *o_dev, int n_samples, int T, int H,
                                 void *hip_stream);

/* Which kernels the whole-sequence passes of a 16-bit flow use for their projections: 0 automatic (the
 * activation-stationary kernels for width 512 from 2048 rows on, the tile kernels otherwise), 1 tile
 * kernels with separate LayerNorm launches everywhere, 2 activation-stationary kernels for every row count
 * (SJD_EINVAL unless the flow is 16-bit with width 512).  The two give the same bits. */
SJD_API int sjd_flow_set_projection_path(sjd_flow *flow, int path);

/* The masked-dependency probe of Sec. 3.2, eq. 6: with o > 0 every attention of the conditioner ignores
 * the o nearest preceding positions (position p sees keys 0..p-o; a position that sees no key gets a
 * zero attention output), in every call of this flow (sequential, Jacobi, conditioner, forward).
 * o = 0 (the default) is the model itself.  A diagnostic: it runs on the row-wise attention kernel and
 * plain per-step launches, not on the tuned paths.  0 <= o <= T, else SJD_EINVAL. */
SJD_API int sjd_flow_set_mask_nearest(sjd_flow *flow, int o);

/* How sjd_sequential_inverse_block (and the sequential blocks of sjd_sample) run in the 16-bit modes:
 * 0 automatic (the persistent kernel where it applies, else per-step launches), 1 per-step launches
 * replayed as a graph, 2 the persistent kernel (SJD_EINVAL at the call if the configuration is outside
 * what it covers: head size 64, W in {256, 512, 768, 1024}, MLP ratio 4, batch <= 256), 3 the persistent
 * kernel started with an ordinary launch instead of a cooperative one (for tools that cannot follow
 * cooperative launches; needs an otherwise idle device, and reports SJD_EHIP instead of waiting
 * forever if its workgroups do not all become resident).  All compute eq. 5 with the
 * key/value cache of Sec. 3.5; they differ in how the T-1 dependent steps are scheduled on the GPU. */
SJD_API int sjd_flow_set_sequential_path(sjd_flow *flow, int path);

/* Number of workgroups of the persistent sequential kernel: 0 (the default) = one per CU of the device,
 * else a multiple of 32 in 32..CUs (SJD_EINVAL otherwise).  For callers that run the sequential block of
 * one batch beside other work, on a stream restricted to that many CUs by a CU mask: the kernel needs
 * all its workgroups resident at once, one per CU, and finds its XCD groups by itself.  The mask must
 * enable the same number of CUs in every shader engine of every XCD (on this part: mask bits
 * 0 .. n_cus-1), or a workgroup may never be placed and the call ends with SJD_EHIP after its bounded
 * wait.  Use path 3 (ordinary launch) there.  Results do not depend on the count. */
SJD_API int sjd_flow_set_sequential_cus(sjd_flow *flow, int n_cus);

/* Kernel-family timing: when enabled, every launch of the selected families (bit f of
 * family_mask = SJD_PROF_* f) is bracketed by events on the caller's stream.  Costs a little time per launch.
 * What an empty event pair measures on the device (a few microseconds, calibrated on first use) is taken off
 * every span, so that the many small launches of single-token steps are not overstated. */
SJD_API int sjd_profile_enable(sjd_flow *flow, uint32_t family_mask);
SJD_API int sjd_profile_read(sjd_flow *flow, sjd_profile *out_host, int reset);

/* Device bytes held by the handle (weights + cache + workspaces). */
SJD_API size_t sjd_flow_device_bytes(const sjd_flow *flow);

SJD_API const char *sjd_last_error(void);
SJD_API void sjd_flow_destroy(sjd_flow *flow);

#ifdef __cplusplus
}
#endif
#endif /* SJD_H */
