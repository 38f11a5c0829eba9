// float32 projections (float32 flows, and the refined passes of 16-bit flows): C = epi(A * B + bias).
// Two kernels; the second, on the float32 matrix instruction, takes the shapes it covers.
// The first: 64x64 output tile per workgroup, 4x4 outputs per thread, K walked in index order so that every
// output is one running fused-multiply-add chain over k (no split-K, no atomics): a row's result
// does not depend on the other rows of its tile.
#include "common.h"
#include <cstdint>

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

// ------------------------------------------------------------------------------------------------
// The same product on the float32 matrix instruction (32x32x2), for K % 16 == 0 and N % 4 == 0.
// 128x128 output tile per workgroup, four waves of 64x64; k-tiles of 16 in two LDS buffers (one barrier
// per k-tile), the next k-tile's values on their way into registers meanwhile.  A lane feeds one value per
// operand and instruction; step s of lane half g stands for k = 8 g + s of the k-tile, so a lane's eight
// values of A are two 16-byte LDS reads.  Every output is still a fixed-order sum over k that depends on its
// own row of A only (no split-K): a row's result does not depend on the rows around it.
// LDS: A [128 rows][16 k], 16-byte chunk c of row r in slot c ^ fm_swz(r) (the 16 lanes of one pass of a
// 16-byte read are rows {0-7, 16-23} or {8-15, 24-31}: 4 (r % 4) + slot is distinct over them);
// B [16 k][128 columns], column j of row k at j ^ 32 (k / 8), so the two halves of a wave use different banks.
constexpr int FM_BM = 128, FM_BN = 128, FM_BK = 16;
__device__ __forceinline__ int fm_swz(int r) { return ((r >> 2) & 1) | (((r >> 4) & 1) << 1); }

template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_mfma_kernel(const float *__restrict__ A, const float *__restrict__ B,
                                                            const float *__restrict__ bias, const float *resid,
                                                            float *C, int M, int N, int K) {
    __shared__ __attribute__((aligned(16))) float As[2][FM_BM * FM_BK];
    __shared__ __attribute__((aligned(16))) float Bs[2][FM_BK * FM_BN];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * FM_BM, n0 = blockIdx.x * FM_BN;
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // staging: A tile = 128 rows x 4 chunks, B tile = 16 rows x 32 chunks; two chunks of each per thread
    f32x4 ra[2], rb[2];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int c = tid + r * 256;
            const int row = c >> 2, ch = c & 3;
            const int gm = m0 + row;
            ra[r] = gm < M ? *reinterpret_cast<const f32x4 *>(A + (size_t)gm * K + k0 + ch * 4) : f32x4{0.f, 0.f, 0.f, 0.f};
            const int kk = c >> 5, cc = c & 31;
            const int gn = n0 + cc * 4;
            rb[r] = gn < N ? *reinterpret_cast<const f32x4 *>(B + (size_t)(k0 + kk) * N + gn) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int c = tid + r * 256;
            const int row = c >> 2, ch = c & 3;
            *reinterpret_cast<f32x4 *>(&As[buf][row * FM_BK + ((ch ^ fm_swz(row)) << 2)]) = ra[r];
            const int kk = c >> 5, cc = c & 31;
            *reinterpret_cast<f32x4 *>(&Bs[buf][kk * FM_BN + ((cc * 4) ^ ((kk >> 3) << 5))]) = rb[r];
        }
    };
    const int KT = K / FM_BK;
    fetch(0);
    stage(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) fetch((kt + 1) * FM_BK);
        float af[2][8];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = 64 * wm + 32 * i + l32;
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                const f32x4 t = *reinterpret_cast<const f32x4 *>(&As[buf][row * FM_BK + (((2 * g + h2) ^ fm_swz(row)) << 2)]);
#pragma unroll
                for (int e = 0; e < 4; ++e) af[i][4 * h2 + e] = t[e];
            }
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            float bf[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) bf[j] = Bs[buf][(8 * g + s) * FM_BN + ((64 * wn + 32 * j + l32) ^ (g << 5))];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][s], bf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) stage(buf ^ 1);   // the other buffer was last read before the previous barrier
        __syncthreads();
    }
    // accumulator register v of block (i, j): row 32 i + 8 (v / 4) + 4 g + v % 4, column 32 j + l32
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int gn = n0 + 64 * wn + 32 * j + l32;
        if (gn >= N) continue;
        const float bv = bias[gn];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int gm = m0 + 64 * wm + 32 * i + 8 * (v >> 2) + 4 * g + (v & 3);
                if (gm >= M) continue;
                float val = acc[i][j][v] + bv;
                if (EPI == EPI_BIAS_GELU) val = gelu_erf(val);
                if (EPI == EPI_BIAS_RESIDUAL) val += resid[(size_t)gm * N + gn];
                C[(size_t)gm * N + gn] = val;
            }
    }
}

void launch_gemm_f32(const float *A, const float *B, const float *bias, const float *resid, float *C, int M, int N,
                     int K, Epi epi, hipStream_t s) {
    if (M <= 0 || N <= 0) return;
    // the choice depends on the matrix shape only, never on the number of rows: a row gives the same bits
    // whatever batch it is computed in
    const bool aligned = ((uintptr_t)A % 16 == 0) && ((uintptr_t)B % 16 == 0);   // 16-byte loads of both operands
    if (K % FM_BK == 0 && N % 4 == 0 && K >= FM_BK && aligned) {
        dim3 grid((N + FM_BN - 1) / FM_BN, (M + FM_BM - 1) / FM_BM);
        switch (epi) {
            case EPI_BIAS:
                hipLaunchKernelGGL(gemm_f32_mfma_kernel<EPI_BIAS>, grid, dim3(256), 0, s, A, B, bias, resid, C, M, N, K);
                break;
            case EPI_BIAS_GELU:
                hipLaunchKernelGGL(gemm_f32_mfma_kernel<EPI_BIAS_GELU>, grid, dim3(256), 0, s, A, B, bias, resid, C, M, N, K);
                break;
            case EPI_BIAS_RESIDUAL:
                hipLaunchKernelGGL(gemm_f32_mfma_kernel<EPI_BIAS_RESIDUAL>, grid, dim3(256), 0, s, A, B, bias, resid, C, M, N, K);
                break;
        }
        return;
    }
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
