// 16-bit (bf16 or f16 operands) MFMA projection with float32 accumulation: C[M,N] = epi(A[M,K] * Bt[N,K]^T + bias).
//
// Both operands are K-contiguous (the weights are stored transposed at load time), which is the
// shape v_mfma_f32_32x32x16_{bf16,f16} wants: every lane feeds 8 consecutive k of one row.  A workgroup
// of four waves (2 x 2) owns a BM x BN tile; a wave owns (BM/2) x (BN/2) as 32x32 MFMA blocks.
// K is walked in index order in steps of 64 through LDS (rows padded by 16 bytes against bank
// conflicts), the next step's global loads being in flight while the current one is multiplied.
// No split-K and no atomics: an output row depends only on its own row of A, so results are
// independent of which other rows share the tile or the batch.
#include "common.h"

namespace sjd {

constexpr int G_BK = 64;
constexpr int G_PAD = 8;
constexpr int G_LDS_STRIDE = G_BK + G_PAD;  // in bf16 elements

template <typename HT, int BM, int BN, typename OutT, int EPI>
__global__ __launch_bounds__(256) void gemm_h16_kernel(const HT *__restrict__ A, const HT *__restrict__ Bt,
                                                        const float *__restrict__ bias, const float *resid, OutT *C,
                                                        int M, int N, int K, int tiles_n) {
    constexpr int MI = BM / 64, NI = BN / 64;    // 32x32 blocks per wave in each direction
    constexpr int A_CHUNKS = BM * 8 / 256;        // 16-byte chunks per thread per k-step
    constexpr int B_CHUNKS = BN * 8 / 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    typedef typename Half16<HT>::v8 v8;
    HT *As = reinterpret_cast<HT *>(smem_raw);
    HT *Bs = As + BM * G_LDS_STRIDE;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int tile = blockIdx.x;
    const int tm = tile / tiles_n, tn = tile - tm * tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // global -> register staging: chunk c covers row c/8, k offset 8*(c%8)
    v8 ra[A_CHUNKS], rb[B_CHUNKS];
    const HT *a_ptr[A_CHUNKS];
    const HT *b_ptr[B_CHUNKS];
#pragma unroll
    for (int r = 0; r < A_CHUNKS; ++r) {
        const int c = tid + r * 256;
        int row = m0 + (c >> 3);
        row = row < M ? row : M - 1;  // rows past the end are read from the last row and never stored
        a_ptr[r] = A + (size_t)row * K + (c & 7) * 8;
    }
#pragma unroll
    for (int r = 0; r < B_CHUNKS; ++r) {
        const int c = tid + r * 256;
        b_ptr[r] = Bt + (size_t)(n0 + (c >> 3)) * K + (c & 7) * 8;  // Bt rows are padded up to the tile
    }
#pragma unroll
    for (int r = 0; r < A_CHUNKS; ++r) ra[r] = *reinterpret_cast<const v8 *>(a_ptr[r]);
#pragma unroll
    for (int r = 0; r < B_CHUNKS; ++r) rb[r] = *reinterpret_cast<const v8 *>(b_ptr[r]);

    const int KT = K / G_BK;
    for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r) {
            const int c = tid + r * 256;
            *reinterpret_cast<v8 *>(&As[(c >> 3) * G_LDS_STRIDE + (c & 7) * 8]) = ra[r];
        }
#pragma unroll
        for (int r = 0; r < B_CHUNKS; ++r) {
            const int c = tid + r * 256;
            *reinterpret_cast<v8 *>(&Bs[(c >> 3) * G_LDS_STRIDE + (c & 7) * 8]) = rb[r];
        }
        __syncthreads();
        if (kt + 1 < KT) {
#pragma unroll
            for (int r = 0; r < A_CHUNKS; ++r) ra[r] = *reinterpret_cast<const v8 *>(a_ptr[r] + (size_t)(kt + 1) * G_BK);
#pragma unroll
            for (int r = 0; r < B_CHUNKS; ++r) rb[r] = *reinterpret_cast<const v8 *>(b_ptr[r] + (size_t)(kt + 1) * G_BK);
        }
#pragma unroll
        for (int ks = 0; ks < G_BK / 16; ++ks) {
            v8 fa[MI], fb[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i)
                fa[i] = *reinterpret_cast<const v8 *>(&As[(wm0 + 32 * i + l32) * G_LDS_STRIDE + ks * 16 + 8 * g]);
#pragma unroll
            for (int j = 0; j < NI; ++j)
                fb[j] = *reinterpret_cast<const v8 *>(&Bs[(wn0 + 32 * j + l32) * G_LDS_STRIDE + ks * 16 + 8 * g]);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = Half16<HT>::mfma(fa[i], fb[j], acc[i][j]);
        }
        __syncthreads();
    }

    // accumulator layout of the 32x32 block: register v of lane (l32, g) is row 8*(v/4) + 4*g + v%4, column l32
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int col = n0 + wn0 + 32 * j + l32;
        if (col >= N) continue;
        const float bv = bias[col];
#pragma unroll
        for (int i = 0; i < MI; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm0 + 32 * i + 8 * (v >> 2) + 4 * g + (v & 3);
                if (row >= M) continue;
                float val = acc[i][j][v] + bv;
                if (EPI == EPI_BIAS_GELU) val = gelu_erf(val);
                if (EPI == EPI_BIAS_RESIDUAL) val += resid[(size_t)row * N + col];
                C[(size_t)row * N + col] = from_f32<OutT>(val);
            }
        }
    }
}

template <typename HT, int BM, int BN, typename OutT, int EPI>
static void launch_tile(const HT *A, const HT *Bt, const float *bias, const float *resid, OutT *C, int M, int N,
                        int K, hipStream_t s) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const size_t smem = (size_t)(BM + BN) * G_LDS_STRIDE * sizeof(HT);
    auto kern = gemm_h16_kernel<HT, BM, BN, OutT, EPI>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), smem, s, A, Bt, bias, resid, C, M, N, K, tiles_n);
}

template <typename HT, typename OutT, int EPI>
static void pick_tile(const HT *A, const HT *Bt, const float *bias, const float *resid, OutT *C, int M, int N,
                      int K, hipStream_t s) {
    launch_tile<HT, 128, 128, OutT, EPI>(A, Bt, bias, resid, C, M, N, K, s);
}

template <typename HT, typename OutT>
void launch_gemm_h16(const HT *A, const HT *Bt, const float *bias, const float *resid, OutT *C, int M, int N, int K,
                     Epi epi, hipStream_t s) {
    if (M <= 0 || N <= 0) return;
    if constexpr (sizeof(OutT) == 4) {
        if (epi == EPI_BIAS_RESIDUAL) pick_tile<HT, float, EPI_BIAS_RESIDUAL>(A, Bt, bias, resid, C, M, N, K, s);
        else pick_tile<HT, float, EPI_BIAS>(A, Bt, bias, resid, C, M, N, K, s);
    } else {
        if (epi == EPI_BIAS_GELU) pick_tile<HT, HT, EPI_BIAS_GELU>(A, Bt, bias, resid, C, M, N, K, s);
        else pick_tile<HT, HT, EPI_BIAS>(A, Bt, bias, resid, C, M, N, K, s);
    }
}
template void launch_gemm_h16<bf16, bf16>(const bf16 *, const bf16 *, const float *, const float *, bf16 *, int, int,
                                          int, Epi, hipStream_t);
template void launch_gemm_h16<bf16, float>(const bf16 *, const bf16 *, const float *, const float *, float *, int, int,
                                           int, Epi, hipStream_t);
template void launch_gemm_h16<f16, f16>(const f16 *, const f16 *, const float *, const float *, f16 *, int, int, int,
                                        Epi, hipStream_t);
template void launch_gemm_h16<f16, float>(const f16 *, const f16 *, const float *, const float *, float *, int, int,
                                          int, Epi, hipStream_t);

}  // namespace sjd
