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

constexpr int G_PAD = 8;  // LDS row padding in elements (16 bytes): keeps 16-byte fragment reads conflict-free

// Workgroups are numbered so that the ones resident on one XCD at a time (ids congruent mod 8 go
// to the same XCD and so share an L2) work on neighbouring tiles: each XCD gets a contiguous run of
// tiles in n-fastest order, i.e. a few row panels of A against all of the (small) weight matrix.
__device__ __forceinline__ int xcd_tile(int wg, int n_tiles) {
    const int per = (n_tiles + 7) >> 3;
    const int t = (wg & 7) * per + (wg >> 3);
    return t;
}

template <typename HT, int BM, int BN, int BK, int WGS_PER_CU, typename OutT, int EPI>
__global__ __launch_bounds__(256, WGS_PER_CU) void gemm_h16_kernel(const HT *__restrict__ A, const HT *__restrict__ Bt,
                                                       const float *__restrict__ bias, const float *resid, OutT *C,
                                                       int M, int N, int K, int tiles_n, int n_tiles) {
    typedef typename Half16<HT>::v8 v8;
    constexpr int MI = BM / 64, NI = BN / 64;    // 32x32 blocks per wave in each direction
    constexpr int CPR = BK / 8;                   // 16-byte chunks per tile row
    constexpr int A_CHUNKS = BM * CPR / 256;      // chunks per thread per k-step
    constexpr int B_CHUNKS = BN * CPR / 256;
    constexpr int G_LDS_STRIDE = BK + G_PAD;
    constexpr int G_BK = BK;
    constexpr int STAGE = (BM + BN) * G_LDS_STRIDE;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    HT *smem = reinterpret_cast<HT *>(smem_raw);

    const int tile = xcd_tile(blockIdx.x, n_tiles);
    if (tile >= n_tiles) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
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

    // global -> register staging: chunk c covers row c/CPR, k offset 8*(c%CPR)
    v8 ra[A_CHUNKS], rb[B_CHUNKS];
    const HT *a_ptr[A_CHUNKS];
    const HT *b_ptr[B_CHUNKS];
#pragma unroll
    for (int r = 0; r < A_CHUNKS; ++r) {
        const int c = tid + r * 256;
        int row = m0 + c / CPR;
        row = row < M ? row : M - 1;  // rows past the end are read from the last row and never stored
        a_ptr[r] = A + (size_t)row * K + (c % CPR) * 8;
    }
#pragma unroll
    for (int r = 0; r < B_CHUNKS; ++r) {
        const int c = tid + r * 256;
        b_ptr[r] = Bt + (size_t)(n0 + c / CPR) * K + (c % CPR) * 8;  // Bt rows are padded up to the tile
    }
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r) ra[r] = *reinterpret_cast<const v8 *>(a_ptr[r] + (size_t)kt * G_BK);
#pragma unroll
        for (int r = 0; r < B_CHUNKS; ++r) rb[r] = *reinterpret_cast<const v8 *>(b_ptr[r] + (size_t)kt * G_BK);
    };
    auto store_tile = [&](int stage) {
        HT *As = smem + stage * STAGE, *Bs = As + BM * G_LDS_STRIDE;
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r) {
            const int c = tid + r * 256;
            *reinterpret_cast<v8 *>(&As[(c / CPR) * G_LDS_STRIDE + (c % CPR) * 8]) = ra[r];
        }
#pragma unroll
        for (int r = 0; r < B_CHUNKS; ++r) {
            const int c = tid + r * 256;
            *reinterpret_cast<v8 *>(&Bs[(c / CPR) * G_LDS_STRIDE + (c % CPR) * 8]) = rb[r];
        }
    };

    // two LDS stages: while stage kt&1 is multiplied, tile kt+1 is written to the other stage and
    // tile kt+2 is on its way from global memory
    const int KT = K / G_BK;
    load_tile(0);
    store_tile(0);
    if (KT > 1) load_tile(1);
    __syncthreads();
    constexpr int KSUB = G_BK / 16;
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < KT) store_tile(cur ^ 1);
        if (kt + 2 < KT) load_tile(kt + 2);
        const HT *As = smem + cur * STAGE, *Bs = As + BM * G_LDS_STRIDE;
        // operand fragments are double-buffered in registers: the reads of sub-step ks+1 are issued
        // before the matrix instructions of sub-step ks and interleaved with them
        v8 fa[2][MI], fb[2][NI];
        auto read_frags = [&](int ks, int buf) {
#pragma unroll
            for (int i = 0; i < MI; ++i)
                fa[buf][i] = *reinterpret_cast<const v8 *>(&As[(wm0 + 32 * i + l32) * G_LDS_STRIDE + ks * 16 + 8 * g]);
#pragma unroll
            for (int j = 0; j < NI; ++j)
                fb[buf][j] = *reinterpret_cast<const v8 *>(&Bs[(wn0 + 32 * j + l32) * G_LDS_STRIDE + ks * 16 + 8 * g]);
        };
        read_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) {
            const int b = ks & 1;
            if (ks + 1 < KSUB) read_frags(ks + 1, b ^ 1);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) acc[i][j] = Half16<HT>::mfma(fa[b][i], fb[b][j], acc[i][j]);
            if (ks + 1 < KSUB) {
                // one LDS read, then its share of the matrix instructions
#pragma unroll
                for (int q = 0; q < MI + NI; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, (MI * NI) / (MI + NI), 0);
                }
            }
        }
        __syncthreads();
    }

    // Epilogue through LDS.  In the accumulators a lane owns one column and sixteen rows of each
    // 32x32 block (register v of lane (l32, g) is row 8*(v/4) + 4*g + v%4, column l32), which would
    // mean one 4-byte access per element.  Each wave therefore parks 32 rows of its sub-tile at a
    // time in its own slice of the (now idle) staging memory and takes them back row-wise, four
    // consecutive columns per lane, so that bias, GELU, the float32 residual read-modify-write and
    // the store all move 8 or 16 bytes per lane in runs of whole rows.
    constexpr int WN = BN / 2;                 // columns of a wave's sub-tile
    constexpr int EP = WN + 4;                 // LDS row pitch in floats
    constexpr int LPR = WN / 4;                // lanes per row when reading back
    constexpr int RPI = 64 / LPR;              // rows per read instruction
    float *ep = reinterpret_cast<float *>(smem_raw) + wave * 32 * EP;
    const int rl = lane / LPR, cl = (lane % LPR) * 4;
    const int colg = n0 + wn0 + cl;            // first of this lane's four columns
    f32x4 bv4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int e = 0; e < 4; ++e) bv4[e] = (colg + e < N) ? bias[colg + e] : 0.f;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) ep[(8 * (v >> 2) + 4 * g + (v & 3)) * EP + 32 * j + l32] = acc[i][j][v];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int rr = 0; rr < 32; rr += RPI) {
            const int rloc = rr + rl;
            const int row = m0 + wm0 + 32 * i + rloc;
            f32x4 val = *reinterpret_cast<const f32x4 *>(&ep[rloc * EP + cl]);
            if (row < M && colg < N) {
                val += bv4;
                if (EPI == EPI_BIAS_GELU) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) val[e] = gelu_erf_h16(val[e]);
                }
                OutT *dst = C + (size_t)row * N + colg;
                if (colg + 3 < N && (N & 3) == 0) {
                    if constexpr (sizeof(OutT) == 4) {
                        if (EPI == EPI_BIAS_RESIDUAL) val += *reinterpret_cast<const f32x4 *>(resid + (size_t)row * N + colg);
                        *reinterpret_cast<f32x4 *>(dst) = val;
                    } else {
                        typename Half16<HT>::v4 o4;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o4[e] = from_f32<HT>(val[e]);
                        *reinterpret_cast<typename Half16<HT>::v4 *>(dst) = o4;
                    }
                } else {  // ragged right edge, or rows not 16-byte aligned
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (colg + e < N) {
                            float t = val[e];
                            if (EPI == EPI_BIAS_RESIDUAL) t += resid[(size_t)row * N + colg + e];
                            dst[e] = from_f32<OutT>(t);
                        }
                }
            }
        }
    }
}

template <typename HT, int BM, int BN, int BK, int WGS_PER_CU, typename OutT, int EPI>
static void launch_tile(const HT *A, const HT *Bt, const float *bias, const float *resid, OutT *C, int M, int N,
                        int K, hipStream_t s) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int n_tiles = tiles_m * tiles_n;
    const int grid = ((n_tiles + 7) / 8) * 8;
    size_t smem = (size_t)2 * (BM + BN) * (BK + G_PAD) * sizeof(HT);
    const size_t ep = (size_t)4 * 32 * (BN / 2 + 4) * sizeof(float);  // epilogue parking space
    if (smem < ep) smem = ep;
    auto kern = gemm_h16_kernel<HT, BM, BN, BK, WGS_PER_CU, OutT, EPI>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), smem, s, A, Bt, bias, resid, C, M, N, K, tiles_n, n_tiles);
}

// Tile choice.  256x128x32 with two workgroups per CU: one workgroup's epilogue and barrier stalls
// hide behind the other's matrix instructions (measured 5-40 % faster than 256x256x64 with one
// workgroup per CU on every projection of the workloads).  128x128 covers small problems.  Weight
// matrices are padded to 256 rows, so tiles never read past a matrix.
template <typename HT, typename OutT, int EPI>
static void pick_tile(const HT *A, const HT *Bt, const float *bias, const float *resid, OutT *C, int M, int N, int K,
                      hipStream_t s) {
    const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
    if (N >= 128 && M >= 256 && t128 >= 512) launch_tile<HT, 256, 128, 32, 2, OutT, EPI>(A, Bt, bias, resid, C, M, N, K, s);
    else launch_tile<HT, 128, 128, 64, 1, OutT, EPI>(A, Bt, bias, resid, C, M, N, K, s);
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
