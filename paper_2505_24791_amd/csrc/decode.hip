// Kernels of the single-token steps of the sequential inverse (eq. 5 with the key/value cache of
// Sec. 3.5) in the 16-bit modes.  A step handles one position of every sample: M = B rows only,
// so every projection is a skinny product bound by streaming its weights, and the whole step is
// bound by launch latency and by reading the cached keys/values.  The step index lives in device
// memory (advanced by the step's last kernel), so one captured graph of the step can be replayed
// for every position.
#include "common.h"

namespace sjd {

// ------------------------------------------------------------------------------------------------
// Skinny projection C[M, N] = epi(A[M, K] * Wt[N, K]^T + bias), M <= 256.
// 16x16x32 MFMA; both operands go straight from global memory (L2) to registers, 16 bytes per
// lane, with all k-steps of a wave in flight at once where they fit (a step of this size is bound
// by latency and instruction issue, not by bandwidth).  A workgroup owns 16*NB columns.
//   SPLITK: the four waves share the same MB row blocks (M <= 16*MB) and each takes a quarter of
//           K; the partial sums meet in LDS, are added in wave order (deterministic), and the
//           16x16 output blocks are shared out among the waves for the epilogue.
//   else  : wave w owns row blocks w*MB .. w*MB+MB-1 (M <= 64*MB) over the whole K.
// Fragment-major layout of a [rows, K] operand: the 64 x 8 elements one wave feeds to a 16x16x32
// MFMA (lane = 16*(k%32/8) + row%16 holds 8 consecutive k) are stored contiguously, fragment
// (row/16, k/32) after fragment.  A wave then loads an operand fragment as one contiguous run
// (1 KB of 16-bit data), instead of sixteen 64-byte pieces of sixteen rows.

template <typename HT, int MB, int NB, int UU, int STEP>
__device__ __forceinline__ void skinny_group(const HT *const (&ap)[MB], const HT *const (&bp)[NB], int s,
                                             f32x4v (&acc)[MB][NB]) {
    typedef typename Half16<HT>::v8 v8;
    v8 fa[UU][MB], fb[UU][NB];
#pragma unroll
    for (int u = 0; u < UU; ++u) {
#pragma unroll
        for (int j = 0; j < NB; ++j) fb[u][j] = *reinterpret_cast<const v8 *>(bp[j] + (size_t)(s + u) * STEP);
#pragma unroll
        for (int i = 0; i < MB; ++i) fa[u][i] = *reinterpret_cast<const v8 *>(ap[i] + (size_t)(s + u) * STEP);
    }
#pragma unroll
    for (int u = 0; u < UU; ++u)
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j) acc[i][j] = Mfma16<HT>::run(fa[u][i], fb[u][j], acc[i][j]);
}

// NW = waves per workgroup.  SPLITK: all NW waves share the MB row blocks and split K NW ways.
// FRAG: A, Wt and a 16-bit or residual C are in fragment-major layout (SPLITK only); a float C
// without residual (the head output) stays row-major.
template <typename HT, int MB, int NB, int NW, bool SPLITK, bool FRAG, int EPI, typename OutT>
__global__ __launch_bounds__(64 * NW) void skinny_gemm_kernel(const HT *__restrict__ A, const HT *__restrict__ Wt,
                                                             const float *__restrict__ bias, const float *resid,
                                                             OutT *C, int M, int N, int K) {
    constexpr int U = (MB + NB) <= 5 ? 8 : 4;  // k-steps in flight per wave
    constexpr int NBLK = MB * NB;
    __shared__ f32x4v red[SPLITK ? NW * NBLK * 64 : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, kg = lane >> 4;
    const int n0 = blockIdx.x * 16 * NB;
    const int mb0 = SPLITK ? (int)blockIdx.y * MB : wave * MB;  // SPLITK: blockIdx.y selects a group of 16*MB rows
    const int steps = K / 32;
    const int s_begin = SPLITK ? (wave * steps) / NW : 0;
    const int s_end = SPLITK ? ((wave + 1) * steps) / NW : steps;
    constexpr int STEP = FRAG ? 512 : 32;                       // elements between consecutive k-steps
    constexpr bool OUT_FRAG = FRAG && !(sizeof(OutT) == 4 && EPI == EPI_BIAS);
    const int KSN = N / 32;                                     // k-steps of C when it is the next operand

    f32x4v acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = f32x4v{0.f, 0.f, 0.f, 0.f};

    const HT *ap[MB];
    const HT *bp[NB];
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        if (FRAG) {
            ap[i] = A + ((size_t)(mb0 + i) * steps * 64 + lane) * 8;
        } else {
            int row = (mb0 + i) * 16 + r;
            row = row < M ? row : M - 1;
            ap[i] = A + (size_t)row * K + kg * 8;
        }
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        if (FRAG) bp[j] = Wt + ((size_t)(blockIdx.x * NB + j) * steps * 64 + lane) * 8;
        else bp[j] = Wt + (size_t)(n0 + j * 16 + r) * K + kg * 8;
    }

    // The epilogue's operands are fetched up front so that they are not a second dependent round
    // trip.  In SPLITK mode output block q = i*NB + j is finished by wave q % NW.
    float bv[NBLK];
    float rv[(EPI == EPI_BIAS_RESIDUAL) ? NBLK * 4 : 1];
#pragma unroll
    for (int q = 0; q < NBLK; ++q) {
        const int i = q / NB, j = q % NB;
        const int col = n0 + j * 16 + r;
        const bool mine = !SPLITK || (q % NW) == wave;
        bv[q] = (mine && col < N) ? bias[col] : 0.f;
        if (EPI == EPI_BIAS_RESIDUAL) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = (mb0 + i) * 16 + 4 * kg + v;
                const size_t ro = OUT_FRAG ? frag_off(row, col, KSN) : (size_t)row * N + col;
                rv[q * 4 + v] = (mine && row < M && col < N) ? resid[ro] : 0.f;
            }
        }
    }

    int s = s_begin;
    for (; s + U <= s_end; s += U) skinny_group<HT, MB, NB, U, STEP>(ap, bp, s, acc);
    if (U >= 8 && s + 4 <= s_end) { skinny_group<HT, MB, NB, 4, STEP>(ap, bp, s, acc); s += 4; }
    if (s + 2 <= s_end) { skinny_group<HT, MB, NB, 2, STEP>(ap, bp, s, acc); s += 2; }
    if (s < s_end) skinny_group<HT, MB, NB, 1, STEP>(ap, bp, s, acc);

    if (SPLITK) {
#pragma unroll
        for (int q = 0; q < NBLK; ++q) red[(wave * NBLK + q) * 64 + lane] = acc[q / NB][q % NB];
        __syncthreads();
    }
    // 16x16 accumulator: register v of lane (r, kg) is row 4*kg + v, column r
#pragma unroll
    for (int q = 0; q < NBLK; ++q) {
        const int i = q / NB, j = q % NB;
        if (SPLITK && (q % NW) != wave) continue;
        f32x4v t = acc[i][j];
        if (SPLITK) {
            t = red[q * 64 + lane];
#pragma unroll
            for (int w = 1; w < NW; ++w) t += red[(w * NBLK + q) * 64 + lane];
        }
        const int col = n0 + j * 16 + r;
        if (col >= N) continue;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = (mb0 + i) * 16 + 4 * kg + v;
            if (row >= M) continue;
            float val = t[v] + bv[q];
            if (EPI == EPI_BIAS_GELU) val = gelu_erf_h16(val);
            if (EPI == EPI_BIAS_RESIDUAL) val += rv[q * 4 + v];
            const size_t co = OUT_FRAG ? frag_off(row, col, KSN) : (size_t)row * N + col;
            C[co] = from_f32<OutT>(val);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// LayerNorm fused into a skinny projection: C = epi(LayerNorm(Hs) * Wt^T + bias) for M <= 16*MB rows
// and K = 32*S*NW.  The NW waves split K; a wave keeps its float32 slice of every row in
// registers, the row statistics (mean, then centred sum of squares: two passes, as in the
// stand-alone LayerNorm) meet in LDS, and the normalised slice feeds the MFMA directly, so the
// normalised activation never goes to memory.  Hs (float32), Wt and a 16-bit C are fragment-major;
// a float C (the head output) is row-major.
template <typename HT, int MB, int NW, int S, int EPI, typename OutT>
__global__ __launch_bounds__(64 * NW) void skinny_ln_gemm_kernel(const float *__restrict__ Hs,
                                                                const float *__restrict__ g,
                                                                const float *__restrict__ be,
                                                                const HT *__restrict__ Wt,
                                                                const float *__restrict__ bias, OutT *__restrict__ C,
                                                                int M, int N) {
    typedef typename Half16<HT>::v8 v8;
    constexpr int K = 32 * S * NW;
    __shared__ f32x4v red[NW * MB * 64];
    __shared__ float stat[NW][MB * 16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, kg = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int mb0 = blockIdx.y * MB;        // blockIdx.y selects a group of 16*MB rows
    const int k0 = wave * 32 * S + kg * 8;  // this lane's first k; step s adds 32*s
    constexpr int KS = K / 32;
    constexpr bool OUT_FRAG = sizeof(OutT) == 2;
    const int KSN = N / 32;

    v8 fb[S];
#pragma unroll
    for (int s = 0; s < S; ++s)
        fb[s] = *reinterpret_cast<const v8 *>(Wt + (((size_t)blockIdx.x * KS + wave * S + s) * 64 + lane) * 8);
    f32x4 xr[MB][S][2];
#pragma unroll
    for (int i = 0; i < MB; ++i) {
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const float *hp = Hs + (((size_t)(mb0 + i) * KS + wave * S + s) * 64 + lane) * 8;
            xr[i][s][0] = *reinterpret_cast<const f32x4 *>(hp);
            xr[i][s][1] = *reinterpret_cast<const f32x4 *>(hp + 4);
        }
    }
    f32x4 gr[S][2], br[S][2];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        gr[s][0] = *reinterpret_cast<const f32x4 *>(g + k0 + 32 * s);
        gr[s][1] = *reinterpret_cast<const f32x4 *>(g + k0 + 32 * s + 4);
        br[s][0] = *reinterpret_cast<const f32x4 *>(be + k0 + 32 * s);
        br[s][1] = *reinterpret_cast<const f32x4 *>(be + k0 + 32 * s + 4);
    }
    const int col = n0 + r;
    const float bv = (wave < MB && col < N) ? bias[col] : 0.f;

    // pass 1: row means
    float mean[MB], rstd[MB];
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        float sum = 0.f;
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e) sum += xr[i][s][0][e] + xr[i][s][1][e];
        sum += __shfl_xor(sum, 16, 64);
        sum += __shfl_xor(sum, 32, 64);
        if (kg == 0) stat[wave][i * 16 + r] = sum;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        float t = stat[0][i * 16 + r];
#pragma unroll
        for (int w = 1; w < NW; ++w) t += stat[w][i * 16 + r];
        mean[i] = t * (1.0f / (float)K);
    }
    __syncthreads();
    // pass 2: centred sums of squares
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        float m2 = 0.f;
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
                for (int e = 0; e < 4; ++e) { const float d = xr[i][s][h2][e] - mean[i]; m2 = fmaf(d, d, m2); }
        m2 += __shfl_xor(m2, 16, 64);
        m2 += __shfl_xor(m2, 32, 64);
        if (kg == 0) stat[wave][i * 16 + r] = m2;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        float t = stat[0][i * 16 + r];
#pragma unroll
        for (int w = 1; w < NW; ++w) t += stat[w][i * 16 + r];
        rstd[i] = 1.0f / sqrtf(t * (1.0f / (float)K) + 1e-5f);
    }

    f32x4v acc[MB];
#pragma unroll
    for (int i = 0; i < MB; ++i) acc[i] = f32x4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            v8 fa;
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    fa[4 * h2 + e] = from_f32<HT>((xr[i][s][h2][e] - mean[i]) * rstd[i] * gr[s][h2][e] + br[s][h2][e]);
            acc[i] = Mfma16<HT>::run(fa, fb[s], acc[i]);
        }

#pragma unroll
    for (int i = 0; i < MB; ++i) red[(wave * MB + i) * 64 + lane] = acc[i];
    __syncthreads();
    // row block i is summed (wave order) and finished by wave i
    if (wave < MB && col < N) {
        const int i = wave;
        f32x4v t = red[i * 64 + lane];
#pragma unroll
        for (int w = 1; w < NW; ++w) t += red[(w * MB + i) * 64 + lane];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = (mb0 + i) * 16 + 4 * kg + v;
            if (row >= M) continue;
            float val = t[v] + bv;
            if (EPI == EPI_BIAS_GELU) val = gelu_erf_h16(val);
            const size_t co = OUT_FRAG ? frag_off(row, col, KSN) : (size_t)row * N + col;
            C[co] = from_f32<OutT>(val);
        }
    }
}

template <typename HT, int MB, int NW, int S, int EPI, typename OutT>
static void launch_ln_cfg(const float *Hs, const float *g, const float *be, const HT *Wt, const float *bias, OutT *C,
                          int M, int N, hipStream_t s) {
    hipLaunchKernelGGL((skinny_ln_gemm_kernel<HT, MB, NW, S, EPI, OutT>), dim3((N + 15) / 16, (M + 16 * MB - 1) / (16 * MB)),
                       dim3(64 * NW), 0, s, Hs, g, be, Wt, bias, C, M, N);
}

template <typename HT, int EPI, typename OutT>
static bool launch_ln_epi(const float *Hs, const float *g, const float *be, const HT *Wt, const float *bias, OutT *C,
                          int M, int N, int K, hipStream_t s) {
    const int mb = M <= 32 ? 2 : 4;
#define SJD_LN_CASE(MBv, NWv, Sv)                                                          \
    if (mb == MBv && K == 32 * NWv * Sv) {                                                 \
        launch_ln_cfg<HT, MBv, NWv, Sv, EPI, OutT>(Hs, g, be, Wt, bias, C, M, N, s);       \
        return true;                                                                       \
    }
    // measured on configuration 2: with four row blocks eight waves beat sixteen (fewer LDS reads
    // for the row statistics), so the wave count is kept at eight there
    SJD_LN_CASE(2, 16, 1) SJD_LN_CASE(2, 8, 3) SJD_LN_CASE(2, 16, 2) SJD_LN_CASE(2, 8, 1)
    SJD_LN_CASE(4, 8, 2) SJD_LN_CASE(4, 8, 3) SJD_LN_CASE(4, 8, 4) SJD_LN_CASE(4, 8, 1)
#undef SJD_LN_CASE
    return false;
}

template <typename HT, typename OutT>
bool launch_skinny_ln_gemm(const float *Hs, const float *g, const float *be, const HT *Wt, const float *bias, OutT *C,
                           int M, int N, int K, Epi epi, hipStream_t s) {
    if (M <= 0 || N <= 0) return true;
    if constexpr (sizeof(OutT) == 4) {
        return launch_ln_epi<HT, EPI_BIAS, float>(Hs, g, be, Wt, bias, C, M, N, K, s);
    } else {
        if (epi == EPI_BIAS_GELU) return launch_ln_epi<HT, EPI_BIAS_GELU, HT>(Hs, g, be, Wt, bias, C, M, N, K, s);
        return launch_ln_epi<HT, EPI_BIAS, HT>(Hs, g, be, Wt, bias, C, M, N, K, s);
    }
}
template bool launch_skinny_ln_gemm<bf16, bf16>(const float *, const float *, const float *, const bf16 *,
                                                const float *, bf16 *, int, int, int, Epi, hipStream_t);
template bool launch_skinny_ln_gemm<bf16, float>(const float *, const float *, const float *, const bf16 *,
                                                 const float *, float *, int, int, int, Epi, hipStream_t);
template bool launch_skinny_ln_gemm<f16, f16>(const float *, const float *, const float *, const f16 *, const float *,
                                              f16 *, int, int, int, Epi, hipStream_t);
template bool launch_skinny_ln_gemm<f16, float>(const float *, const float *, const float *, const f16 *, const float *,
                                                float *, int, int, int, Epi, hipStream_t);

template <typename HT, int MB, int NB, int NW, bool SPLITK, bool FRAG, int EPI, typename OutT>
static void launch_skinny_cfg(const HT *A, const HT *Wt, const float *bias, const float *resid, OutT *C, int M, int N,
                              int K, hipStream_t s) {
    const int grid = (N + 16 * NB - 1) / (16 * NB);
    const int groups = SPLITK ? (M + 16 * MB - 1) / (16 * MB) : 1;
    hipLaunchKernelGGL((skinny_gemm_kernel<HT, MB, NB, NW, SPLITK, FRAG, EPI, OutT>), dim3(grid, groups), dim3(64 * NW), 0,
                       s, A, Wt, bias, resid, C, M, N, K);
}

template <typename HT, int EPI, typename OutT>
static void launch_skinny_epi(const HT *A, const HT *Wt, const float *bias, const float *resid, OutT *C, int M, int N,
                              int K, bool frag, hipStream_t s) {
    // Fragment-major operands: a workgroup owns one 16-column block and a group of up to 64 rows, K
    // split over 8 waves (16 for at most 32 rows): every wave has a handful of loads and matrix
    // instructions, which is what a launch of this size needs.  Row-major operands: waves split the
    // rows and a workgroup owns 32 columns.
    if (frag) {
        // A long k with few columns (the MLP output at width 1024: 64 column blocks, each workgroup reading all of
        // the [M, 4096] activation) leaves three quarters of the CUs idle, and the activation is most of what a
        // workgroup reads: there, 16 rows per workgroup and two workgroups per column block (both on the same XCD:
        // the weight slice comes from memory once).  Same bits: a row's sum does not depend on the rows beside it.
        if (M > 16 && M <= 32 && K >= 2048 && N <= 1024)
            launch_skinny_cfg<HT, 1, 1, 16, true, true, EPI, OutT>(A, Wt, bias, resid, C, M, N, K, s);
        else if (M <= 32) launch_skinny_cfg<HT, 2, 1, 16, true, true, EPI, OutT>(A, Wt, bias, resid, C, M, N, K, s);
        else launch_skinny_cfg<HT, 4, 1, 8, true, true, EPI, OutT>(A, Wt, bias, resid, C, M, N, K, s);
    } else if (M <= 128) {
        launch_skinny_cfg<HT, 2, 2, 4, false, false, EPI, OutT>(A, Wt, bias, resid, C, M, N, K, s);
    } else {
        launch_skinny_cfg<HT, 4, 2, 4, false, false, EPI, OutT>(A, Wt, bias, resid, C, M, N, K, s);
    }
}

template <typename HT, typename OutT>
void launch_skinny_gemm(const HT *A, const HT *Wt, const float *bias, const float *resid, OutT *C, int M, int N, int K,
                        Epi epi, bool frag, hipStream_t s) {
    if (M <= 0 || N <= 0) return;
    if constexpr (sizeof(OutT) == 4) {
        if (epi == EPI_BIAS_RESIDUAL)
            launch_skinny_epi<HT, EPI_BIAS_RESIDUAL, float>(A, Wt, bias, resid, C, M, N, K, frag, s);
        else launch_skinny_epi<HT, EPI_BIAS, float>(A, Wt, bias, resid, C, M, N, K, frag, s);
    } else {
        if (epi == EPI_BIAS_GELU) launch_skinny_epi<HT, EPI_BIAS_GELU, HT>(A, Wt, bias, resid, C, M, N, K, frag, s);
        else launch_skinny_epi<HT, EPI_BIAS, HT>(A, Wt, bias, resid, C, M, N, K, frag, s);
    }
}
template void launch_skinny_gemm<bf16, bf16>(const bf16 *, const bf16 *, const float *, const float *, bf16 *, int, int,
                                             int, Epi, bool, hipStream_t);
template void launch_skinny_gemm<bf16, float>(const bf16 *, const bf16 *, const float *, const float *, float *, int,
                                              int, int, Epi, bool, hipStream_t);
template void launch_skinny_gemm<f16, f16>(const f16 *, const f16 *, const float *, const float *, f16 *, int, int, int,
                                           Epi, bool, hipStream_t);
template void launch_skinny_gemm<f16, float>(const f16 *, const f16 *, const float *, const float *, float *, int, int,
                                             int, Epi, bool, hipStream_t);

// ------------------------------------------------------------------------------------------------
// Single-token attention against the cache, head size 64.  One workgroup per (sample, head); its
// 256 threads are 32 key groups x 8 sixteen-byte chunks of the head.  Position t = *t_dev: this
// step's k, v are appended to the cache and used from the fresh row; keys 0..t-1 come from the cache.
// frag != 0: qkv [B, 3W] and o [B, W] are fragment-major (see frag_off), else row-major.
template <typename HT>
__global__ __launch_bounds__(256) void decode_attention_h16_kernel(const HT *__restrict__ qkv, HT *kcache, HT *vcache,
                                                                   HT *__restrict__ o, const int32_t *__restrict__ t_dev,
                                                                   int T, int H, int frag) {
    typedef typename Half16<HT>::v8 v8;
    extern __shared__ float sc[];  // [T] scores, then [4][64] partial outputs + [8] scalars
    __shared__ float wmax[4], wsum[4];
    __shared__ float opart[4][64];
    const int t = *t_dev;
    const int W = H * 64;
    const int h = blockIdx.x % H, b = blockIdx.x / H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int dc = tid & 7, sg = tid >> 3;
    // 8-element chunk c (0..7) of this head's q / k / v in the fused row of sample b
    const int KS3 = 3 * W / 32;
    auto chunk = [&](int part, int c) -> const HT * {
        const int k = part * W + h * 64 + c * 8;
        return frag ? qkv + frag_off(b, k, KS3) : qkv + (size_t)b * 3 * W + k;
    };
    const HT *kfresh = chunk(1, dc), *vfresh = chunk(2, dc);   // this thread's chunk of the fresh k, v
    HT *kc = kcache + (size_t)b * T * W + h * 64;
    HT *vc = vcache + (size_t)b * T * W + h * 64;
    if (tid < 8) __builtin_nontemporal_store(*reinterpret_cast<const v8 *>(chunk(1, tid)), reinterpret_cast<v8 *>(kc + (size_t)t * W + tid * 8));
    else if (tid < 16)
        __builtin_nontemporal_store(*reinterpret_cast<const v8 *>(chunk(2, tid - 8)), reinterpret_cast<v8 *>(vc + (size_t)t * W + (tid - 8) * 8));
    float qf[8];
    {
        const v8 q8 = *reinterpret_cast<const v8 *>(chunk(0, dc));
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[e] = (float)q8[e] * 0.125f;  // 1/sqrt(64)
    }
    const int n = t + 1;
    // Keys and values are walked four rows per thread at a time with all four loads issued before the first
    // is used: with one load in flight per thread a workgroup has 4 KB on its way, and the step is spent
    // waiting for memory latency thirty times over; rows past the end re-read the fresh row and are ignored.
    // Each thread still accumulates its rows in index order.
    constexpr int U = 4;   // eight rows in flight were slower (measured at 1024 tokens, 32 samples)
    float mx = -INFINITY;
    // A row of the cache is read once per step and the whole cache is far larger than any cache level: read it
    // as streaming data, so that it does not push the block's weights - which every step reads again - out of
    // the memory-side cache (measured at 1024 tokens, width 1024: the projections of a step got 12 % faster).
    auto ldc = [&](const HT *ptr) -> v8 { return __builtin_nontemporal_load(reinterpret_cast<const v8 *>(ptr)); };
    for (int s0 = sg; s0 < n; s0 += 32 * U) {
        v8 k8[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = s0 + 32 * u;
            k8[u] = ldc(s < t ? kc + (size_t)s * W + dc * 8 : kfresh);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = s0 + 32 * u;
            if (s < n) {                       // the eight lanes of a key group agree on s
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) d = fmaf(qf[e], (float)k8[u][e], d);
                d += __shfl_xor(d, 1, 64);
                d += __shfl_xor(d, 2, 64);
                d += __shfl_xor(d, 4, 64);
                if (dc == 0) sc[s] = d;
                mx = fmaxf(mx, d);
            }
        }
    }
    // the first values are requested before the maximum is known
    v8 vq[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int s = sg + 32 * u;
        vq[u] = ldc(s < t ? vc + (size_t)s * W + dc * 8 : vfresh);
    }
    mx = wave_max(mx);
    if (lane == 0) wmax[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    float psum = 0.f;
    for (int s0 = sg; s0 < n; s0 += 32 * U) {
        v8 vn[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {          // the next four rows, while these four are used
            const int s = s0 + 32 * (U + u);
            vn[u] = ldc(s < t ? vc + (size_t)s * W + dc * 8 : vfresh);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = s0 + 32 * u;
            if (s < n) {
                const float p = expf(sc[s] - mx);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] = fmaf(p, (float)vq[u][e], acc[e]);
                psum += p;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) vq[u] = vn[u];
    }
    // combine the 8 key groups of this wave (lanes differing in bits 3..5), then the 4 waves
#pragma unroll
    for (int off = 8; off < 64; off <<= 1) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], off, 64);
        psum += __shfl_xor(psum, off, 64);
    }
    if (lane < 8) {
#pragma unroll
        for (int e = 0; e < 8; ++e) opart[wave][lane * 8 + e] = acc[e];
        if (lane == 0) wsum[wave] = psum;
    }
    __syncthreads();
    if (tid < 8) {
        const float den = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
        v8 ov;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int d = tid * 8 + e;
            ov[e] = from_f32<HT>((((opart[0][d] + opart[1][d]) + opart[2][d]) + opart[3][d]) / den);
        }
        const int k = h * 64 + tid * 8;
        HT *dst = frag ? o + frag_off(b, k, W / 32) : o + (size_t)b * W + k;
        *reinterpret_cast<v8 *>(dst) = ov;
    }
}

template <typename HT>
void launch_decode_attention_h16(const HT *qkv, HT *kcache, HT *vcache, HT *o, const int32_t *t_dev, int B, int T, int H,
                                 bool frag, hipStream_t s) {
    if (B <= 0) return;
    hipLaunchKernelGGL(decode_attention_h16_kernel<HT>, dim3(B * H), dim3(256), (size_t)T * sizeof(float), s, qkv, kcache,
                       vcache, o, t_dev, T, H, frag ? 1 : 0);
}
template void launch_decode_attention_h16<bf16>(const bf16 *, bf16 *, bf16 *, bf16 *, const int32_t *, int, int, int,
                                                bool, hipStream_t);
template void launch_decode_attention_h16<f16>(const f16 *, f16 *, f16 *, f16 *, const int32_t *, int, int, int, bool,
                                               hipStream_t);

// ------------------------------------------------------------------------------------------------
// End of a step fused with the start of the next: from the head row of position t compute
// position l = t+1 of every sample, x_l = z_l * exp(alpha) + mu (eq. 5), then embed it,
// h[b, :] = x_l * w_in + b_in + pos[l, :].  With first != 0: l = 0, x_0 = z_0 and t is set to 0.
// The workgroup that finishes last advances the step counter.
__global__ __launch_bounds__(1024) void decode_advance_kernel(const float *__restrict__ p, const float *__restrict__ z,
                                                              float *__restrict__ x, const float *__restrict__ w_in,
                                                              const float *__restrict__ b_in,
                                                              const float *__restrict__ pos, float *__restrict__ h,
                                                              int32_t *t_dev, uint32_t *ticket, int T, int D, int W,
                                                              int reversed, int first, int frag) {
    extern __shared__ float xs[];
    const int b = blockIdx.x;
    const int nt = blockDim.x;
    const int t = first ? -1 : *t_dev;
    const int l = t + 1;
    if (l < T) {
        const int tok = reversed ? T - 1 - l : l;
        for (int d = threadIdx.x; d < D; d += nt) {
            const size_t idx = ((size_t)b * T + tok) * D + d;
            float xn = z[idx];
            if (l > 0) xn = fmaf(xn, expf(p[(size_t)b * 2 * D + D + d]), p[(size_t)b * 2 * D + d]);
            x[idx] = xn;
            xs[d] = xn;
        }
        __syncthreads();
        for (int w = threadIdx.x; w < W; w += nt) {
            float acc = b_in[w];
            const float pw = pos[(size_t)l * W + w];
            // sixteen rows of the embedding matrix are requested before the first is used (one dependent round
            // trip per row otherwise); the sum still runs over d in index order
            int d = 0;
            for (; d + 16 <= D; d += 16) {
                float wv[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) wv[u] = w_in[(size_t)(d + u) * W + w];
#pragma unroll
                for (int u = 0; u < 16; ++u) acc = fmaf(xs[d + u], wv[u], acc);
            }
            for (; d < D; ++d) acc = fmaf(xs[d], w_in[(size_t)d * W + w], acc);
            const size_t ho = frag ? frag_off(b, w, W / 32) : (size_t)b * W + w;
            h[ho] = acc + pw;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        // every workgroup has read *t_dev before it draws its ticket
        const uint32_t k = atomicAdd(ticket, 1u);
        if (k == gridDim.x - 1) {
            *ticket = 0u;
            *t_dev = l;
        }
    }
}

void launch_decode_advance(const float *p, const float *z, float *x, const float *w_in, const float *b_in,
                           const float *pos, float *h, int32_t *t_dev, uint32_t *ticket, int B, int T, int D, int W,
                           int reversed, int first, bool frag, hipStream_t s) {
    if (B <= 0) return;
    // one thread per column of the embedding where the width allows: a thread's columns are walked one after
    // the other, each costing its own round trips to L2
    const int threads = W >= 1024 ? 1024 : (W >= 512 ? 512 : 256);
    hipLaunchKernelGGL(decode_advance_kernel, dim3(B), dim3(threads), D * sizeof(float), s, p, z, x, w_in, b_in, pos, h,
                       t_dev, ticket, T, D, W, reversed, first, frag ? 1 : 0);
}

}  // namespace sjd
