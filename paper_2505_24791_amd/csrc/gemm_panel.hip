// Activation-stationary projections for K = 512 (the width of the headline workload):
//   C[M,N] = epi(LayerNorm(H)[M,512] * W + bias)   (QKV and MLP-input projections), or
//   H[M,N] += A[M,512] * W + bias                   (attention-output projection).
//
// The tile kernels of gemm_h16.hip spend half of a tile's time outside their k-loop at K = 512 and
// read both operands from LDS (with 64x64 per wave the LDS reads alone are as long as the matrix
// instructions).  Here a workgroup of four waves keeps a 128-row panel of the left operand, all of K,
// in LDS (128 KB) for its whole life and walks over groups of 256 output columns; a wave owns
// 128 x 64 of a group and streams its weight fragments straight from L2 into registers, eight
// k-steps ahead (the weights are stored in fragment order, so such a load is 1 KB contiguous).
// The main loop has no barrier and reads LDS for one operand only (4 fragment reads per 8 matrix
// instructions).  The panel is built once per workgroup - LayerNorm included, which takes the
// separate LayerNorm launch and its 16-bit round trip through HBM out of the pass.  k is walked in
// index order with the same 32x32x16 instruction as the tile kernels, and LayerNorm uses the
// arithmetic of layernorm_vec_kernel, so results are bit-identical to LayerNorm + tile kernel.
#include "common.h"
#include <atomic>

namespace sjd {

namespace {

constexpr int PK = 512, PKS = PK / 16;        // k and k-steps
constexpr int P_PD = 8;                       // weight prefetch depth in k-steps
constexpr int P_PANEL_BYTES = 128 * PK * 2;
constexpr int P_EP = 68;                      // pitch of the epilogue parking rows in floats
constexpr int P_LDS = P_PANEL_BYTES + 4 * 16 * P_EP * 4;

typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

// Panel row r keeps its 16-byte chunk c in slot c ^ swz(r).  A 16-byte LDS read of a wave is served in
// four passes of 16 lanes (rows {0-7, 16-23} or {8-15, 24-31} of a 32-row fragment, one chunk), 64
// banks wide; rows are 1 KB apart, so the bank group of a read is its slot modulo 16: bits 0-2 and 4
// of the row make the sixteen rows of a pass distinct.
__device__ __forceinline__ int panel_swz(int row) { return (row & 7) | (((row >> 4) & 1) << 3); }

template <typename HT, int EPI, bool LN, int NIT>
__global__ __launch_bounds__(256, 1) void gemm_panel_kernel(const void *__restrict__ A_in, const float *__restrict__ ln_g,
                                                            const float *__restrict__ ln_b, const HT *__restrict__ Wf,
                                                            const float *__restrict__ bias, void *C_out, int M, int N,
                                                            int n_split, int n_panels) {
    typedef typename Half16<HT>::v8 v8;
    typedef typename Half16<HT>::v4 v4;
    constexpr bool OUT_F32 = EPI == EPI_BIAS_RESIDUAL;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    // workgroup ids congruent mod 8 share an XCD: the workgroups of one panel sit on one XCD, so the
    // second one finds the panel's rows in that L2
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int panel = (idx / n_split) * 8 + xcd, part = idx % n_split;
    if (panel >= n_panels) return;
    const int m0 = panel * 128;
    const int cols_part = N / n_split;
    // stores (and residual loads) past row M-1 fall outside the buffer and are dropped (return zero)
    const rsrc_t c_rs = __builtin_amdgcn_make_buffer_rsrc(C_out, 0, M * N * (OUT_F32 ? 4 : 2), 0x00020000);
    // this wave's two 32-column blocks of group it: nb = (part * cols_part + it * 256 + wave * 64) / 32 + j
    auto b_ptr = [&](int it, int j, int ks) -> const v8 * {
        const int nb = (part * cols_part + it * 256 + wave * 64) / 32 + j;
        return reinterpret_cast<const v8 *>(Wf + (((size_t)nb * PKS + ks) * 64 + lane) * 8);
    };
    v8 bq[P_PD][2];
#pragma unroll
    for (int p = 0; p < P_PD; ++p)
#pragma unroll
        for (int j = 0; j < 2; ++j) bq[p][j] = *b_ptr(0, j, p);
    __builtin_amdgcn_sched_barrier(0);

    // ---- the panel: wave w builds rows w, w + 4, ...; a row is one instruction wide
    if constexpr (LN) {
        const float *H = reinterpret_cast<const float *>(A_in);
        f32x4 g4[2], b4[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            g4[k] = reinterpret_cast<const f32x4 *>(ln_g)[k * 64 + lane];
            b4[k] = reinterpret_cast<const f32x4 *>(ln_b)[k * 64 + lane];
        }
        // Eight rows at a time, the next eight on their way from HBM meanwhile.  The sums of eight rows
        // are reduced together: at the levels of lane bits 5, 4 and 3 a lane passes on the half of the rows
        // it does not keep, so that lane l ends up with the total of row l / 8 - the same tree of additions
        // per row as wave_sum (bits 5, 4, .., 0), in 10 exchanges instead of 48.
        auto load8 = [&](int bt, f32x4 (&v)[8][2]) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = wave + 4 * (bt + u);
                const int rc = m0 + r < M ? m0 + r : M - 1;      // rows past the end: any valid row, never stored
                const f32x4 *xr = reinterpret_cast<const f32x4 *>(H + (size_t)rc * PK);
#pragma unroll
                for (int k = 0; k < 2; ++k) v[u][k] = xr[k * 64 + lane];
            }
        };
        const bool hi5 = lane & 32, hi4 = lane & 16, hi3 = lane & 8;
        auto reduce8 = [&](const float (&s)[8], float (&tot)[8]) {
            float a[4], b[2];
#pragma unroll
            for (int j = 0; j < 4; ++j) a[j] = (hi5 ? s[j + 4] : s[j]) + __shfl_xor(hi5 ? s[j] : s[j + 4], 32, 64);
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j] = (hi4 ? a[j + 2] : a[j]) + __shfl_xor(hi4 ? a[j] : a[j + 2], 16, 64);
            float c = (hi3 ? b[1] : b[0]) + __shfl_xor(hi3 ? b[0] : b[1], 8, 64);
            c += __shfl_xor(c, 4, 64);
            c += __shfl_xor(c, 2, 64);
            c += __shfl_xor(c, 1, 64);
#pragma unroll
            for (int u = 0; u < 8; ++u) tot[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, c), u * 8));
        };
        auto rows8 = [&](int bt, const f32x4 (&v)[8][2]) {
            float s[8], q[8], mean[8], tot[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                s[u] = 0.f;
#pragma unroll
                for (int k = 0; k < 2; ++k) s[u] += (v[u][k][0] + v[u][k][1]) + (v[u][k][2] + v[u][k][3]);
            }
            reduce8(s, tot);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                mean[u] = tot[u] / (float)PK;
                q[u] = 0.f;
#pragma unroll
                for (int k = 0; k < 2; ++k)
#pragma unroll
                    for (int e = 0; e < 4; ++e) { const float d = v[u][k][e] - mean[u]; q[u] = fmaf(d, d, q[u]); }
            }
            reduce8(q, tot);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = wave + 4 * (bt + u);
                const float rstd = 1.0f / sqrtf(tot[u] / (float)PK + 1e-5f);
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    v4 h4;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        h4[e] = from_f32<HT>(keep_f32((v[u][k][e] - mean[u]) * rstd * g4[k][e] + b4[k][e]));
                    const int chunk = k * 32 + (lane >> 1);      // columns 4 (64 k + lane) .. + 3
                    *reinterpret_cast<v4 *>(lds + r * 1024 + ((chunk ^ panel_swz(r)) << 4) + (lane & 1) * 8) = h4;
                }
            }
        };
        f32x4 va[8][2], vb[8][2];
        load8(0, va);
        load8(8, vb);
        __builtin_amdgcn_sched_barrier(0);   // the loads stay where they are written: a batch ahead of their use
        rows8(0, va);
        __builtin_amdgcn_sched_barrier(0);
        load8(16, va);
        __builtin_amdgcn_sched_barrier(0);
        rows8(8, vb);
        __builtin_amdgcn_sched_barrier(0);
        load8(24, vb);
        __builtin_amdgcn_sched_barrier(0);
        rows8(16, va);
        rows8(24, vb);
    } else {
        const HT *A = reinterpret_cast<const HT *>(A_in);
        for (int bt = 0; bt < 32; bt += 8) {
            v8 t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = wave + 4 * (bt + u);
                const int rc = m0 + r < M ? m0 + r : M - 1;
                t[u] = *reinterpret_cast<const v8 *>(A + (size_t)rc * PK + lane * 8);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = wave + 4 * (bt + u);
                *reinterpret_cast<v8 *>(lds + r * 1024 + ((lane ^ panel_swz(r)) << 4)) = t[u];
            }
        }
    }
    __syncthreads();

    float *ep = reinterpret_cast<float *>(lds + P_PANEL_BYTES) + wave * 16 * P_EP;
    const int sw = panel_swz(l32);
    const unsigned char *a_base = lds + l32 * 1024;
    const int rl = lane >> 4, cl = (lane & 15) * 4;

#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        f32x16 acc[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        v8 fa[2][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) fa[0][i] = *reinterpret_cast<const v8 *>(a_base + i * 32 * 1024 + ((g ^ sw) << 4));
        __builtin_amdgcn_sched_barrier(0);
        // Every matrix instruction is a slot: the panel fragments of the next k-step are read in the
        // first four slots, a weight fragment is requested again (P_PD k-steps ahead, running on into
        // the next column group) as soon as its last use has been issued.  The fences keep the
        // compiler from moving the loads next to their uses.
#pragma unroll
        for (int ks = 0; ks < PKS; ++ks) {
            const int b = ks & 1, slot = ks % P_PD;
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                const int i = m & 3, j = m >> 2;
                if (m < 4 && ks + 1 < PKS)
                    fa[b ^ 1][m] = *reinterpret_cast<const v8 *>(a_base + m * 32 * 1024 + (((2 * (ks + 1) + g) ^ sw) << 4));
                if (m == 4) {
                    if (ks + P_PD < PKS) bq[slot][0] = *b_ptr(it, 0, ks + P_PD);
                    else if (it + 1 < NIT) bq[slot][0] = *b_ptr(it + 1, 0, ks + P_PD - PKS);
                }
                acc[i][j] = Half16<HT>::mfma(fa[b][i], bq[slot][j], acc[i][j]);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (ks + P_PD < PKS) bq[slot][1] = *b_ptr(it, 1, ks + P_PD);
            else if (it + 1 < NIT) bq[slot][1] = *b_ptr(it + 1, 1, ks + P_PD - PKS);
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- epilogue.  In the accumulators a lane owns one column and sixteen rows of a 32x32 block
        // (register v: row 8 (v / 4) + 4 g + v % 4).  Sixteen rows x 64 columns at a time go through the
        // wave's parking slice and come back row-wise, four columns per lane, so that bias, GELU, the
        // residual and the store move 8 or 16 bytes per lane in whole 128/256-byte rows.  No branches
        // (rows past M are dropped by the buffer bounds): the slice is rewritten while the previous
        // rows are converted and stored - a wave's LDS operations execute in order.
        const int col0 = part * cols_part + it * 256 + wave * 64;
        const f32x4 bv4 = *reinterpret_cast<const f32x4 *>(bias + col0 + cl);
        f32x4 val[2][4], res[2][4];
#pragma unroll
        for (int n = 0; n <= 8; ++n) {
            if (n < 8) {
                const int i = n >> 1, hh = n & 1;
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int vv = 0; vv < 8; ++vv)
                        ep[(8 * (vv >> 2) + 4 * g + (vv & 3)) * P_EP + 32 * j + l32] = acc[i][j][8 * hh + vv];
                asm volatile("" ::: "memory");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int q = 0; q < 4; ++q) val[n & 1][q] = *reinterpret_cast<const f32x4 *>(&ep[(4 * q + rl) * P_EP + cl]);
                if constexpr (OUT_F32) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int row = m0 + 32 * i + 16 * hh + 4 * q + rl;
                        res[n & 1][q] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(c_rs, (row * N + col0 + cl) * 4, 0, 0));
                    }
                }
                asm volatile("" ::: "memory");
                __builtin_amdgcn_wave_barrier();
            }
            if (n > 0) {
                const int i = (n - 1) >> 1, hh = (n - 1) & 1;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int row = m0 + 32 * i + 16 * hh + 4 * q + rl;
                    f32x4 o = val[(n - 1) & 1][q] + bv4;
                    if constexpr (EPI == EPI_BIAS_GELU) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = gelu_erf_h16(o[e]);
                    }
                    if constexpr (OUT_F32) {
                        o += res[(n - 1) & 1][q];
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(i32x4, o), c_rs, (row * N + col0 + cl) * 4, 0, 0);
                    } else {
                        v4 o4;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o4[e] = from_f32<HT>(o[e]);
                        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(i32x2, o4), c_rs, (row * N + col0 + cl) * 2, 0, 0);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// wt [N (padded), 512] row-major -> fragment order: fragment (nb, ks) = 64 lanes x 16 bytes, lane (l32, g)
// holds wt[32 nb + l32][16 ks + 8 g .. + 8] - the second operand of the 32x32x16 instruction
template <typename HT>
__global__ __launch_bounds__(256) void weights_to_panel_frag_kernel(const HT *__restrict__ wt, HT *__restrict__ dst, int N) {
    typedef typename Half16<HT>::v8 v8;
    const size_t i = blockIdx.x * 256ull + threadIdx.x;   // one 16-byte piece
    if (i >= (size_t)N * PK / 8) return;
    const int lane = (int)(i & 63);
    const size_t f = i >> 6;
    const int ks = (int)(f % PKS), nb = (int)(f / PKS), l32 = lane & 31, g = lane >> 5;
    *reinterpret_cast<v8 *>(dst + i * 8) = *reinterpret_cast<const v8 *>(wt + (size_t)(32 * nb + l32) * PK + 16 * ks + 8 * g);
}

// Column groups per workgroup: whole rounds of workgroups on the device's CUs, a panel build
// (about one group's time with LayerNorm, half without) per workgroup.
int pick_groups(int n_panels, int groups, bool ln, int max_nit) {
    int best = 1;
    double best_cost = 1e30;
    for (int nit = 1; nit <= max_nit; ++nit) {
        if (groups % nit) continue;
        const long wgs = (long)n_panels * (groups / nit);
        const double cost = (double)((wgs + 255) / 256) * ((ln ? 1.0 : 0.5) + nit);
        if (cost <= best_cost) { best_cost = cost; best = nit; }
    }
    return best;
}

template <typename HT, int EPI, bool LN, int NIT>
void launch_nit(const void *A, const float *g, const float *b, const HT *Wf, const float *bias, void *C, int M, int N,
                hipStream_t s) {
    const int n_panels = (M + 127) / 128, n_split = N / 256 / NIT;
    auto kern = gemm_panel_kernel<HT, EPI, LN, NIT>;
    static std::atomic<bool> attr_set{false};   // callers may come from several host threads
    if (!attr_set.load(std::memory_order_acquire)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        attr_set.store(true, std::memory_order_release);
    }
    const int grid = ((n_panels + 7) / 8) * n_split * 8;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), P_LDS, s, A, g, b, Wf, bias, C, M, N, n_split, n_panels);
}

}  // namespace

bool gemm_panel_applicable(int M, int N, int K, int out_bytes) {
    return K == PK && M >= 1 && N >= 256 && N % 256 == 0 && ((long long)M + 128) * N * out_bytes < (1ll << 31);
}

template <typename HT>
void launch_weights_to_panel_frag(const HT *wt, HT *dst, int N, hipStream_t s) {
    const size_t pieces = (size_t)N * PK / 8;
    hipLaunchKernelGGL(weights_to_panel_frag_kernel<HT>, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, s, wt, dst, N);
}
template void launch_weights_to_panel_frag<bf16>(const bf16 *, bf16 *, int, hipStream_t);
template void launch_weights_to_panel_frag<f16>(const f16 *, f16 *, int, hipStream_t);

template <typename HT>
void launch_ln_gemm_panel(const float *H, const float *g, const float *b, const HT *Wf, const float *bias, HT *C, int M,
                          int N, Epi epi, hipStream_t s) {
    if (M <= 0) return;
    const int nit = pick_groups((M + 127) / 128, N / 256, true, 4);
#define SJD_PANEL_CASE(E, n) case n: launch_nit<HT, E, true, n>(H, g, b, Wf, bias, C, M, N, s); break;
    if (epi == EPI_BIAS_GELU) {
        switch (nit) { SJD_PANEL_CASE(EPI_BIAS_GELU, 1) SJD_PANEL_CASE(EPI_BIAS_GELU, 2) SJD_PANEL_CASE(EPI_BIAS_GELU, 3) SJD_PANEL_CASE(EPI_BIAS_GELU, 4) }
    } else {
        switch (nit) { SJD_PANEL_CASE(EPI_BIAS, 1) SJD_PANEL_CASE(EPI_BIAS, 2) SJD_PANEL_CASE(EPI_BIAS, 3) SJD_PANEL_CASE(EPI_BIAS, 4) }
    }
#undef SJD_PANEL_CASE
}
template void launch_ln_gemm_panel<bf16>(const float *, const float *, const float *, const bf16 *, const float *, bf16 *, int, int, Epi, hipStream_t);
template void launch_ln_gemm_panel<f16>(const float *, const float *, const float *, const f16 *, const float *, f16 *, int, int, Epi, hipStream_t);

template <typename HT>
void launch_gemm_panel_resid(const HT *A, const HT *Wf, const float *bias, float *H, int M, int N, hipStream_t s) {
    if (M <= 0) return;
    const int nit = pick_groups((M + 127) / 128, N / 256, false, 2);
    if (nit == 2) launch_nit<HT, EPI_BIAS_RESIDUAL, false, 2>(A, nullptr, nullptr, Wf, bias, H, M, N, s);
    else launch_nit<HT, EPI_BIAS_RESIDUAL, false, 1>(A, nullptr, nullptr, Wf, bias, H, M, N, s);
}
template void launch_gemm_panel_resid<bf16>(const bf16 *, const bf16 *, const float *, float *, int, int, hipStream_t);
template void launch_gemm_panel_resid<f16>(const f16 *, const f16 *, const float *, float *, int, int, hipStream_t);

}  // namespace sjd
