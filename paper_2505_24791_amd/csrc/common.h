// Shared declarations of the HIP library: element types, launchers of every kernel family.
// gfx950 only (64-wide wavefronts, MFMA, 160 KB LDS per CU).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sjd {

typedef __bf16 bf16;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16;
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16>(bf16 v) { return (float)v; }
template <> __device__ __forceinline__ float to_f32<f16>(f16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ f16 from_f32<f16>(float v) { return (f16)v; }
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }

// The two 16-bit operand types of the MFMA kernels: vectors of 4 / 8 elements and the
// 32x32x16 matrix instruction with float32 accumulation.
template <typename HT> struct Half16;
template <> struct Half16<bf16> {
    typedef bf16x4 v4;
    typedef bf16x8 v8;
    static __device__ __forceinline__ f32x16 mfma(v8 a, v8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    // c + the sum of the eight values of p, in float32 (two values per instruction)
    static __device__ __forceinline__ float add_all(v8 p, float c) {
        typedef __bf16 v2 __attribute__((ext_vector_type(2)));
        const v2 one = {(__bf16)1.f, (__bf16)1.f};
        c = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(p, p, 0, 1), one, c, false);
        c = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(p, p, 2, 3), one, c, false);
        c = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(p, p, 4, 5), one, c, false);
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(p, p, 6, 7), one, c, false);
    }
};
template <> struct Half16<f16> {
    typedef f16x4 v4;
    typedef f16x8 v8;
    static __device__ __forceinline__ f32x16 mfma(v8 a, v8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float add_all(v8 p, float c) {
        typedef _Float16 v2 __attribute__((ext_vector_type(2)));
        const v2 one = {(_Float16)1.f, (_Float16)1.f};
        c = __builtin_amdgcn_fdot2(__builtin_shufflevector(p, p, 0, 1), one, c, false);
        c = __builtin_amdgcn_fdot2(__builtin_shufflevector(p, p, 2, 3), one, c, false);
        c = __builtin_amdgcn_fdot2(__builtin_shufflevector(p, p, 4, 5), one, c, false);
        return __builtin_amdgcn_fdot2(__builtin_shufflevector(p, p, 6, 7), one, c, false);
    }
};

typedef float f32x4v __attribute__((ext_vector_type(4)));

template <typename HT> struct Mfma16;
template <> struct Mfma16<bf16> {
    static __device__ __forceinline__ f32x4v run(bf16x8 a, bf16x8 b, f32x4v c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mfma16<f16> {
    static __device__ __forceinline__ f32x4v run(f16x8 a, f16x8 b, f32x4v c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
};

// Fragment-major layout of a [rows, K] operand of the 16x16x32 MFMA: the 64 x 8 elements one wave
// feeds to one instruction (lane = 16*(k%32/8) + row%16 holds 8 consecutive k) are contiguous,
// fragment (row/16, k/32) after fragment.  KS = K/32.  Returns the element index of (row, k).
__device__ __forceinline__ size_t frag_off(int row, int k, int KS) {
    return ((((size_t)(row >> 4) * KS + (k >> 5)) * 64 + (((k & 31) >> 3) << 4) + (row & 15)) << 3) + (k & 7);
}

__device__ __forceinline__ float gelu_erf(float v) { return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f)); }

// A float32 value that is about to be rounded to 16 bits, made opaque to the compiler.  Otherwise it
// folds the fma that produces the value into the conversion (v_fma_mix: one rounding instead of
// two) for some elements of an unrolled loop and not for others, and two kernels that compute the
// same thing differ in the last bit of a few results per hundred thousand.
__device__ __forceinline__ float keep_f32(float v) {
    asm("" : "+v"(v));
    return v;
}

// GELU (erf form) for results that are stored in 16 bits: erf by the rational-times-exponential
// formula 7.1.26 of Abramowitz & Stegun (absolute error below 1.5e-7, far inside the 2^-11
// relative rounding of the stored value) at a quarter of the instructions of erff.
__device__ __forceinline__ float gelu_erf_h16(float v) {
    // x = |v| / sqrt 2;  t = 1 / (1 + p x);  erf x = 1 - (a1 t + ... + a5 t^5) exp(-x^2)
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752440f, fabsf(v), 1.0f));   // v_rcp_f32 (1 ulp); a correctly rounded 1/x costs ten instructions
    float p = fmaf(1.061405429f, t, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    p *= t;
    const float ex = __builtin_amdgcn_exp2f((v * v) * (-0.5f * 1.44269504088896340736f));   // exp(-v^2 / 2) = 2^(-v^2 log2(e) / 2)
    const float e = fmaf(-p, ex, 1.0f);                  // erf(|v| / sqrt 2)
    const float h = 0.5f * v;
    return keep_f32(fmaf(fabsf(h), e, h));               // 0.5 v (1 + sign(v) erf(|v| / sqrt 2))
}

// Row -> (sample, token) mapping shared by the embedding and the epilogues.  A whole-sequence pass
// runs on `rows_per_sample = T` rows per active sample; a single-token step on one row per sample.
struct RowMap {
    const int32_t *active;  // [n_rows / rows_per_sample] sample indices, or nullptr for the identity
    int32_t rows_per_sample;
    int32_t t0;             // processing-order position of a sample's first row
    int32_t T;              // tokens per sample
    int32_t reversed;       // 1: processing position p is canonical token T-1-p
};

// Epilogue selector of the dense projections.
enum Epi : int {
    EPI_BIAS = 0,          // out = acc + bias
    EPI_BIAS_GELU = 1,     // out = gelu(acc + bias)
    EPI_BIAS_RESIDUAL = 2, // out(float) = resid(float) + acc + bias, in place allowed
};

// ---- launchers (all asynchronous on `s`) ---------------------------------------------------

// h[m, :] = x[b, tok, :] * w_in + b_in + pos[p, :]
void launch_embed(const float *x, const float *w_in, const float *b_in, const float *pos, float *h, int n_rows,
                  int D, int W, RowMap map, hipStream_t s);

// y = LayerNorm(x) * g + b over rows of width W (biased variance, eps 1e-5); OutT float, bf16 or f16
template <typename OutT>
void launch_layernorm(const float *x, const float *g, const float *b, OutT *y, int n_rows, int W, hipStream_t s);

// float32 projection: C[M,N] = epi(A[M,K] * B[K,N] + bias)
void launch_gemm_f32(const float *A, const float *B, const float *bias, const float *resid, float *C, int M, int N,
                     int K, Epi epi, hipStream_t s);

// 16-bit MFMA projection (HT = bf16 or f16): C[M,N] = epi(A[M,K] * Bt[N,K]^T + bias); Bt holds the
// weight transposed, K contiguous, with at least round_up(N, 256) rows (zero filled).  K % 64 == 0.
// OutT = HT (EPI_BIAS, EPI_BIAS_GELU) or float (EPI_BIAS, EPI_BIAS_RESIDUAL).
// kernel: 0 = chosen by shape; 1 = 256x128x32 staged through registers; 2 = 256x256x64 LDS-direct;
// 3 = 128x128x64; 4 = the persistent eight-wave kernel of gemm_p8.hip where it applies (else as 0)
// (the explicit choices exist so that each kernel can be checked on small shapes).
template <typename HT, typename OutT>
void launch_gemm_h16(const HT *A, const HT *Bt, const float *bias, const float *resid, OutT *C, int M, int N, int K,
                     Epi epi, hipStream_t s, int kernel = 0);

// Persistent eight-wave projection (gemm_p8.hip): the same contract as launch_gemm_h16 (resid, when given, is C
// itself: the float32 stream is updated in place) for K % 128 == 0 and N % 256 == 0; bit-identical to the tile kernels.
bool gemm_p8_applicable(int M, int N, int K);
template <typename HT, typename OutT>
void launch_gemm_p8(const HT *A, const HT *Bt, const float *bias, OutT *C, int M, int N, int K, Epi epi, hipStream_t s);

// Activation-stationary projections for K = 512 (gemm_panel.hip).  Wf: the weight in the fragment order of
// the 32x32x16 instruction (launch_weights_to_panel_frag from the transposed [N, 512] copy; N % 256 == 0).
//   launch_ln_gemm_panel:    C[M,N] (16-bit) = epi(LayerNorm(H[M,512]; g, b) * W + bias), epi = EPI_BIAS or EPI_BIAS_GELU
//   launch_gemm_panel_resid: H[M,N] (float32) += A[M,512] * W + bias
// Bit-identical to launch_layernorm + launch_gemm_h16.  gemm_panel_applicable: the shape is covered
// (out_bytes: element size of the output).
bool gemm_panel_applicable(int M, int N, int K, int out_bytes);
template <typename HT> void launch_weights_to_panel_frag(const HT *wt, HT *dst, int N, hipStream_t s);
template <typename HT>
void launch_ln_gemm_panel(const float *H, const float *g, const float *b, const HT *Wf, const float *bias, HT *C, int M,
                          int N, Epi epi, hipStream_t s);
template <typename HT>
void launch_gemm_panel_resid(const HT *A, const HT *Wf, const float *bias, float *H, int M, int N, hipStream_t s);

// Residual projection for long k (gemm_stream.hip): H[M,N] (float32) += A[M,K] * W + bias with the left operand
// streamed through LDS in chunks of 256 k and the weights in the fragment order of the 32x32x16 instruction
// (launch_weights_to_frag32 from the transposed [N, K] copy).  K % 512 == 0, N % 256 == 0; bit-identical to
// launch_gemm_h16.
bool gemm_stream_applicable(int M, int N, int K);
template <typename HT> void launch_weights_to_frag32(const HT *wt, HT *dst, int N, int K, hipStream_t s);
template <typename HT>
void launch_gemm_stream_resid(const HT *A, const HT *Wf, const float *bias, float *H, int M, int N, int K, hipStream_t s);

// Causal attention, one wave per (sample, head, query row); works for any shape and both types.
// q rows: q + (sample*q_rows_per_sample + r) * q_stride; row r (processing position t0 + r) attends
// keys 0..t0+r-mask_o found at k + sample_index*kv_sample_stride + key*kv_stride (+ head*dh); same for v.
// kv_index: nullptr => sample i uses cache slot i, else slot kv_index[i].
template <typename QT, typename KVT>
void launch_attention_rows(const QT *q, int64_t q_stride, const KVT *k, const KVT *v, int64_t kv_stride,
                           int64_t kv_sample_stride, QT *o, int64_t o_stride, int n_samples, int q_rows_per_sample,
                           int t0, int H, int dh, int mask_o, hipStream_t s);

// Single-token step: writes this step's k, v (from the fused qkv row) into the cache at position t,
// then attends keys 0..t.  qkv [B, 3W], cache [B, T, W] each for k and v, o [B, W].
template <typename AT>
void launch_decode_attention(const AT *qkv, AT *kcache, AT *vcache, AT *o, int B, int T, int t, int H, int dh,
                             int mask_o, hipStream_t s);

// Flash-style causal attention on 16-bit qkv [n_samples*T, 3W] (head size 64), o [n_samples*T, W].
template <typename HT>
void launch_flash_attention_h16(const HT *qkv, HT *o, int n_samples, int T, int H, hipStream_t s);
// the same in float32 (float32 matrix instruction), head size 64
void launch_flash_attention_f32(const float *qkv, float *o, int n_samples, int T, int H, hipStream_t s);

// Skinny 16-bit projection for single-token steps (M <= 256 rows, K % 32 == 0); same contract as
// launch_gemm_h16.
// frag: operands in the fragment-major layout of the 16x16x32 MFMA (A [M <= 64, K], Wt, and C unless
// it is a float output without residual).  Otherwise everything is row-major.
template <typename HT, typename OutT>
void launch_skinny_gemm(const HT *A, const HT *Wt, const float *bias, const float *resid, OutT *C, int M, int N, int K,
                        Epi epi, bool frag, hipStream_t s);

// The same with LayerNorm of the float32 rows Hs [M, K] fused in front (gain g, shift be); returns
// false (nothing launched) when the shape is outside what the fused kernel covers (K in
// {256, 512, 768, 1024}).  Fragment-major operands only (Hs, Wt, and a 16-bit C).
template <typename HT, typename OutT>
bool launch_skinny_ln_gemm(const float *Hs, const float *g, const float *be, const HT *Wt, const float *bias, OutT *C,
                           int M, int N, int K, Epi epi, hipStream_t s);

// Single-token attention for head size 64 with the position read from device memory (*t_dev):
// appends this step's k, v to the cache [B, T, W] and attends keys 0..t.
template <typename HT>
void launch_decode_attention_h16(const HT *qkv, HT *kcache, HT *vcache, HT *o, const int32_t *t_dev, int B, int T, int H,
                                 bool frag, hipStream_t s);

// Step boundary of the sequential inverse: x_{t+1} from the head row of position t (eq. 5), its
// embedding into h, and t <- t+1 (device counter).  first != 0: x_0 = z_0, embedding of position 0, t <- 0.
void launch_decode_advance(const float *p, const float *z, float *x, const float *w_in, const float *b_in,
                           const float *pos, float *h, int32_t *t_dev, uint32_t *ticket, int B, int T, int D, int W,
                           int reversed, int first, bool frag, hipStream_t s);

// Jacobi epilogue.  p [n_rows, 2D] head output (row r of a sample parameterises position r+1).
// For every listed sample that is still active: x <- z*exp(alpha)+mu in place, delta, pass count,
// convergence flag.  Then the last workgroup rebuilds the active list.  shared_params != 0: p holds the head output
// of ONE sample, [T, 2D], which parameterises every listed sample (see run_jacobi: the pass from x^0 = 0).
struct JacobiState {
    float *delta;          // [B] last delta of each sample
    int32_t *iters;        // [B] passes taken
    int32_t *done;         // [B] 1 once converged or capped
    int32_t *nonfinite;    // [1] set when a sample finishes with a non-finite delta
    int32_t *active_in;    // [B] samples this pass ran on (n_listed entries)
    int32_t *active_out;   // [B] compacted list of samples still running
    int32_t *n_active_out; // [2] samples still running; how many of them are marked fine (they end the list)
    uint32_t *ticket;      // [1] workgroup counter, zero before the launch, zero again after
    int32_t *fine;         // [B] 1 once a sample's delta has fallen below the refinement level (it stays 1)
};
// The update of Alg. 1 for the n samples listed in st.active_in (head output p: row block i belongs to entry i;
// with shared_params one sample's parameters serve all): x <- z * exp(alpha) + mu, delta, pass count, done flag;
// a sample whose delta falls below refine_below is marked fine.
void launch_jacobi_update(const float *p, const float *z, float *x, JacobiState st, int n, int T, int D, int reversed,
                          float tau, int criterion, int cap, int shared_params, float refine_below, hipStream_t s);
// Rebuilds the list of samples that still iterate: first those not marked fine, then the fine ones, each part in
// increasing order; st.n_active_out receives both counts.  keep_all: finished samples stay listed (first part).
void launch_jacobi_compact(JacobiState st, int n_listed, int keep_all, hipStream_t s);

// x^0 and state initialisation for a Jacobi block: x = 0 or z; iters = 0; done = 0; active = 0..B-1
void launch_jacobi_init(const float *z, float *x, JacobiState st, int B, int T, int D, int init, hipStream_t s);

// Sequential step epilogue: position t+1 of every sample from head row p[b, :]:
// x[b, tok(t+1), :] = z[b, tok(t+1), :] * exp(alpha) + mu.  With t = -1 copies position 0 (x_1 = y_1).
void launch_decode_epilogue(const float *p, const float *z, float *x, int B, int T, int D, int t, int reversed,
                            hipStream_t s);

// mu/alpha extraction for sjd_conditioner: shifted parameters in canonical order.
// Arguments of the persistent sequential-inverse kernel (decode_persistent.hip).  All pointers are device memory.
struct SeqLayer {
    const float *ln1_g, *ln1_b, *b_qkv, *b_o, *ln2_g, *ln2_b, *b_fc1, *b_fc2;
    const void *f_qkv, *f_o, *f_fc1, *f_fc2;  // fragment-major 16-bit weights
};
constexpr int kSeqMaxLayers = 32;
struct SeqArgs {
    SeqLayer layers[kSeqMaxLayers];  // in the kernel-argument segment: read with scalar loads, no pointer chasing
    int n_layers, ratio;
    const float *lnf_g, *lnf_b, *b_head;
    const void *f_head;
    const float *w_in, *b_in, *pos;
    const float *z;
    float *x;
    float *hs;             // float32 residual stream, fragment-major, 8 groups x 16*MB rows
    void *qkv, *o, *ff;    // 16-bit activations, fragment-major, same rows
    float *p;              // head output, row-major [rows, 2D]
    void *kcache, *vcache; // [layer][max_batch][T][W] 16-bit
    size_t kv_layer_stride;  // elements between layers
    int B, T, D, reversed;
    int *sync;             // [0..7] members per XCD, [8] arrivals, [9] status, [64*(g+1)] barrier counter of XCD g
    int spin_max;
};
size_t seq_persistent_lds_bytes(int MB, int T, int D);
// One workgroup of 512 threads per CU (grid = number of CUs), as a cooperative launch or a plain one.  W = 256 S.
hipError_t launch_seq_persistent(bool is_bf16, const SeqArgs &args, int MB, int S, int grid, bool cooperative,
                                 hipStream_t s);

void launch_jacobi_trace(const float *x, const float *x_ref, JacobiState st, float *delta_out, float *err_out, int B,
                         int T, int D, hipStream_t s);
void launch_forward_epilogue(const float *p, const float *x, float *y, float *logdet, int B, int T, int D, int reversed,
                             int accumulate, hipStream_t s);
void launch_split_params(const float *p, float *mu, float *alpha, int B, int T, int D, int reversed, hipStream_t s);

// Weight preparation on the device: dst[n, k] (16-bit, row length ldb, zero padded) = src[k, n] (float [K, N]).
template <typename HT>
void launch_transpose_to_h16(const float *src, HT *dst, int K, int N, int ldb, int n_rows_padded, hipStream_t s);

// Weight preparation for the skinny kernels: fragment-major 16-bit copy of src [K, N] (see decode.hip).
template <typename HT>
void launch_weights_to_frag(const float *src, HT *dst, int K, int N, int n_rows_padded, hipStream_t s);

}  // namespace sjd
