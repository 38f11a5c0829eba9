// float32 projection for the all-float32 correctness configuration: C = epi(A * B + bias).
// 64x64 output tile per workgroup, 4x4 outputs per thread, K walked in index order so that every
// output is one running fused-multiply-add chain over k (no split-K, no atomics): a row's result
// does not depend on the other rows of its tile.
#include "common.h"

namespace sjd {

constexpr int F32_BM = 64, F32_BN = 64, F32_BK = 16;

template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ A, const float *__restrict__ B,
                                                       const float *__restrict__ bias, const float *resid, float *C,
                                                       int M, int N, int K) {
    __shared__ float As[F32_BK][F32_BM + 4];
    __shared__ float Bs[F32_BK][F32_BN + 4];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * F32_BM, n0 = blockIdx.x * F32_BN;
    const int tx = tid & 15, ty = tid >> 4;  // thread owns rows ty*4.., cols tx*4..
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < K; k0 += F32_BK) {
        // A tile: 64 rows x 16 k = 1024 elements, 4 per thread; stored k-major
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int e = tid + r * 256;
            const int row = e >> 4, kk = e & 15;
            const int gm = m0 + row, gk = k0 + kk;
            As[kk][row] = (gm < M && gk < K) ? A[(size_t)gm * K + gk] : 0.f;
        }
        // B tile: 16 k x 64 cols
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int e = tid + r * 256;
            const int kk = e >> 6, col = e & 63;
            const int gk = k0 + kk, gn = n0 + col;
            Bs[kk][col] = (gk < K && gn < N) ? B[(size_t)gk * N + gn] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < F32_BK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tx * 4 + j;
            if (gn >= N) continue;
            float v = acc[i][j] + bias[gn];
            if (EPI == EPI_BIAS_GELU) v = gelu_erf(v);
            if (EPI == EPI_BIAS_RESIDUAL) v += resid[(size_t)gm * N + gn];
            C[(size_t)gm * N + gn] = v;
        }
    }
}

void launch_gemm_f32(const float *A, const float *B, const float *bias, const float *resid, float *C, int M, int N,
                     int K, Epi epi, hipStream_t s) {
    if (M <= 0 || N <= 0) return;
    dim3 grid((N + F32_BN - 1) / F32_BN, (M + F32_BM - 1) / F32_BM);
    switch (epi) {
        case EPI_BIAS:
            hipLaunchKernelGGL(gemm_f32_kernel<EPI_BIAS>, grid, dim3(256), 0, s, A, B, bias, resid, C, M, N, K);
            break;
        case EPI_BIAS_GELU:
            hipLaunchKernelGGL(gemm_f32_kernel<EPI_BIAS_GELU>, grid, dim3(256), 0, s, A, B, bias, resid, C, M, N, K);
            break;
        case EPI_BIAS_RESIDUAL:
            hipLaunchKernelGGL(gemm_f32_kernel<EPI_BIAS_RESIDUAL>, grid, dim3(256), 0, s, A, B, bias, resid, C, M, N, K);
            break;
    }
}

}  // namespace sjd
