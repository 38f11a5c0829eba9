// 16-bit (bf16 or f16 operands) MFMA projection with float32 accumulation: C[M,N] = epi(A[M,K] * Bt[N,K]^T + bias).
//
// Both operands are K-contiguous (the weights are stored transposed at load time), which is the
// shape v_mfma_f32_32x32x16_{bf16,f16} wants: every lane feeds 8 consecutive k of one row.  A workgroup
// of four waves (2 x 2) owns a BM x BN tile; a wave owns (BM/2) x (BN/2) as 32x32 MFMA blocks.
// K is walked in index order through LDS.  Two main loops: one stages tiles through registers into
// two padded LDS buffers; the other fills four LDS stages with LDS-direct loads (see below).
// No split-K and no atomics: an output row depends only on its own row of A, so results are
// independent of which other rows share the tile or the batch.
#include "common.h"
#include <atomic>

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

// Epilogue through LDS.  In the accumulators a lane owns one column and sixteen rows of each
// 32x32 block (register v of lane (l32, g) is row 8*(v/4) + 4*g + v%4, column l32), which would
// mean one 4-byte access per element.  Each wave therefore parks 32 rows of its sub-tile at a
// time in its own slice of the (now idle) staging memory and takes them back row-wise, four
// consecutive columns per lane, so that bias, GELU, the float32 residual read-modify-write and
// the store all move 8 or 16 bytes per lane in runs of whole rows.  (row0, col0): first row and
// column of the wave's sub-tile.  The caller has synchronised the workgroup after its last use of LDS.
template <typename HT, int MI, int NI, int BN, typename OutT, int EPI>
__device__ __forceinline__ void tile_epilogue(f32x16 (&acc)[MI][NI], unsigned char *smem_raw,
                                              const float *__restrict__ bias, const float *resid, OutT *C, int M, int N,
                                              int row0, int col0, int lane, int wave) {
    const int l32 = lane & 31, g = lane >> 5;
    constexpr int WN = BN / 2;                 // columns of a wave's sub-tile
    constexpr int EP = WN + 4;                 // LDS row pitch in floats
    constexpr int LPR = WN / 4;                // lanes per row when reading back
    constexpr int RPI = 64 / LPR;              // rows per read instruction
    float *ep = reinterpret_cast<float *>(smem_raw) + wave * 32 * EP;
    const int rl = lane / LPR, cl = (lane % LPR) * 4;
    const int colg = col0 + cl;                // first of this lane's four columns
    f32x4 bv4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int e = 0; e < 4; ++e) bv4[e] = (colg + e < N) ? bias[colg + e] : 0.f;
    constexpr int NQ = 32 / RPI;               // read-back instructions per 32 rows
    const bool vec_ok = colg + 3 < N && (N & 3) == 0;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) ep[(8 * (v >> 2) + 4 * g + (v & 3)) * EP + 32 * j + l32] = acc[i][j][v];
        // a wave's LDS operations complete in order: the reads below see these writes without a wait;
        // the compiler only has to keep the order
        asm volatile("" ::: "memory");
        __builtin_amdgcn_wave_barrier();
        // All reads (LDS, then the residual) are issued before the first store: a wait for a load while
        // stores are in flight waits for the stores as well (one counter, no order between the two kinds),
        // which, once per row group, used to be most of the epilogue's time.
        f32x4 val[NQ], res[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) val[q] = *reinterpret_cast<const f32x4 *>(&ep[(q * RPI + rl) * EP + cl]);
        if (EPI == EPI_BIAS_RESIDUAL && sizeof(OutT) == 4 && vec_ok) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int row = row0 + 32 * i + q * RPI + rl;
                const int rc = row < M ? row : M - 1;        // rows past the end: any valid row, value not used
                res[q] = *reinterpret_cast<const f32x4 *>(resid + (size_t)rc * N + colg);
            }
        }
        // Uses in straight-line code: the waits for the loads above are placed here, once.  Left to the
        // conditional blocks below, every block waits again "for the bias" (it cannot know that an
        // earlier, skipped block already did) and with that for the stores issued so far.
        asm volatile("" : "+v"(bv4));
        if (EPI == EPI_BIAS_RESIDUAL && sizeof(OutT) == 4 && vec_ok) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) asm volatile("" : "+v"(res[q]));
        }
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int row = row0 + 32 * i + q * RPI + rl;
            if (row < M && colg < N) {
                f32x4 v4 = val[q] + bv4;
                if (EPI == EPI_BIAS_GELU) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v4[e] = gelu_erf_h16(v4[e]);
                }
                OutT *dst = C + (size_t)row * N + colg;
                if (vec_ok) {
                    if constexpr (sizeof(OutT) == 4) {
                        if (EPI == EPI_BIAS_RESIDUAL) v4 += res[q];
                        *reinterpret_cast<f32x4 *>(dst) = v4;
                    } else {
                        typename Half16<HT>::v4 o4;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o4[e] = from_f32<HT>(v4[e]);
                        *reinterpret_cast<typename Half16<HT>::v4 *>(dst) = o4;
                    }
                } else {  // ragged right edge, or rows not 16-byte aligned
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (colg + e < N) {
                            float t = v4[e];
                            if (EPI == EPI_BIAS_RESIDUAL) t += resid[(size_t)row * N + colg + e];
                            dst[e] = from_f32<OutT>(t);
                        }
                }
            }
        }
    }
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

    // global -> register staging: chunk c covers row c/CPR, k offset 8*(c%CPR).  Two register sets, so
    // that two k-tiles can be on their way while a third is multiplied: at K = 512 a k-tile is 0.25 us
    // of matrix work against 1 us of load latency.
    struct Regs { v8 a[A_CHUNKS], b[B_CHUNKS]; };
    Regs S0, S1;
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
    auto load_tile = [&](int kt, Regs &q) {
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r) q.a[r] = *reinterpret_cast<const v8 *>(a_ptr[r] + (size_t)kt * G_BK);
#pragma unroll
        for (int r = 0; r < B_CHUNKS; ++r) q.b[r] = *reinterpret_cast<const v8 *>(b_ptr[r] + (size_t)kt * G_BK);
    };
    auto store_tile = [&](int stage, const Regs &q) {
        HT *As = smem + stage * STAGE, *Bs = As + BM * G_LDS_STRIDE;
#pragma unroll
        for (int r = 0; r < A_CHUNKS; ++r) {
            const int c = tid + r * 256;
            *reinterpret_cast<v8 *>(&As[(c / CPR) * G_LDS_STRIDE + (c % CPR) * 8]) = q.a[r];
        }
#pragma unroll
        for (int r = 0; r < B_CHUNKS; ++r) {
            const int c = tid + r * 256;
            *reinterpret_cast<v8 *>(&Bs[(c / CPR) * G_LDS_STRIDE + (c % CPR) * 8]) = q.b[r];
        }
    };
    constexpr int KSUB = G_BK / 16;
    auto multiply = [&](int stage) {
        const HT *As = smem + stage * STAGE, *Bs = As + BM * G_LDS_STRIDE;
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) {
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
                for (int j = 0; j < NI; ++j) acc[i][j] = Half16<HT>::mfma(fa[i], fb[j], acc[i][j]);
        }
    };

    const int KT = K / G_BK;
    if (KT >= 4 && (KT & 1) == 0) {
        // Two LDS stages and two register sets; tile t travels in set t & 1.  In iteration kt, tile kt+1
        // goes from its set to stage (kt+1)&1, the set is refilled with tile kt+3, stage kt&1 is
        // multiplied.  The steady state and the last three iterations are written out without
        // conditions: a wait for the older set's loads then leaves the newer set's in flight (with
        // conditions around the loads the compiler has to wait for everything at every join).
        load_tile(0, S0);
        __builtin_amdgcn_sched_barrier(0);   // keep the issue order of the sets: the waits count loads
        load_tile(1, S1);
        __builtin_amdgcn_sched_barrier(0);
        store_tile(0, S0);
        load_tile(2, S0);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        int kt = 0;
        for (; kt + 5 < KT; kt += 2) {
            store_tile(1, S1); load_tile(kt + 3, S1); multiply(0); __syncthreads();
            store_tile(0, S0); load_tile(kt + 4, S0); multiply(1); __syncthreads();
        }
        // kt == KT - 4 (even)
        store_tile(1, S1); load_tile(kt + 3, S1); multiply(0); __syncthreads();
        store_tile(0, S0); multiply(1); __syncthreads();
        store_tile(1, S1); multiply(0); __syncthreads();
        multiply(1);
        __syncthreads();
    } else {
        // any other k-tile count: one register set, conditions in the loop
        load_tile(0, S0);
        store_tile(0, S0);
        if (KT > 1) load_tile(1, S0);
        __syncthreads();
        for (int kt = 0; kt < KT; ++kt) {
            const int cur = kt & 1;
            if (kt + 1 < KT) store_tile(cur ^ 1, S0);
            if (kt + 2 < KT) load_tile(kt + 2, S0);
            multiply(cur);
            __syncthreads();
        }
    }

    tile_epilogue<HT, MI, NI, BN, OutT, EPI>(acc, smem_raw, bias, resid, C, M, N, m0 + wm0, n0 + wn0, lane, wave);
}

// ------------------------------------------------------------------------------------------------
// 256x256 tile, k-tiles of 64, two LDS stages filled by LDS-direct global loads
// (global_load_lds_dwordx4: no staging registers, no LDS write instructions).  A 1 KB load of a
// wave covers 8 rows x 128 bytes - whole cache lines, which matters: at this tile size the kernel
// moves (256+256)*2 bytes per 2*256*256 flops from L2, and half-used lines double that - and lands
// in LDS in lane order (lane 8r + c holds a 16-byte chunk of row r).  Which chunk a lane fetches is
// swizzled so that the 16-byte fragment reads of the 32x32x16 MFMA (lane l32 + 32 g wants row l32,
// chunk 2 ks + g) fall on all LDS banks in every pass of the read (see the kernel).  The compiler does not see the
// dependence between an LDS-direct load and a later LDS read, so the waits are written out: a
// wave waits for its own loads of tile kt+1 before the barrier that publishes that tile.  Every
// matrix instruction is a slot, with the LDS reads and global loads pinned between the slots.
#define SJD_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define SJD_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

template <typename HT, typename OutT, int EPI>
__global__ __launch_bounds__(256, 1) void gemm_h16_dma_kernel(const HT *__restrict__ A, const HT *__restrict__ Bt,
                                                              const float *__restrict__ bias, const float *resid,
                                                              OutT *C, int M, int N, int K, int tiles_n, int n_tiles) {
    typedef typename Half16<HT>::v8 v8;
    constexpr int BM = 256, BN = 256, BK = 64;
    constexpr int MI = 4, NI = 4, KSUB = BK / 16;
    constexpr int OPB = 32 * 1024;            // bytes of one operand in one stage: 32 blocks of 8 rows x 128 B
    constexpr int STB = 2 * OPB;              // bytes per stage
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

    const int tile = xcd_tile(blockIdx.x, n_tiles);
    if (tile >= n_tiles) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps LDS bases in scalar registers
    const int l32 = lane & 31, g = lane >> 5;
    const int tm = tile / tiles_n, tn = tile - tm * tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int wm = wave >> 1, wn = wave & 1;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // This wave loads, per k-tile, the 8-row blocks 8 wave + i (i = 0..7) of A and of B.
    // Row r of a 32-row fragment group keeps chunk c in slot c ^ swz(r), swz(r) = bits 1, 2 and 4 of r.
    // A 16-byte LDS read of a wave is served in four passes of 16 lanes (lanes that agree in bits 3 and
    // 5), 64 banks wide: the 16 rows of a pass ({0-7, 16-23} or {8-15, 24-31} of the group, one chunk)
    // must fall on 16 different 16-byte bank groups, (8 (r & 1) + slot) mod 16 - which this does.
    const int lr = lane >> 3;                              // row within the 8-row block
    const int lc0 = (lane & 7) ^ ((lr >> 1) & 3);          // chunk fetched, blocks with bit 4 of the row clear
    uint32_t a_eoff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int row = m0 + (wave * 8 + i) * 8 + lr;
        row = row < M ? row : M - 1;                       // rows past the end: re-read the last row, never stored
        a_eoff[i] = (uint32_t)row * (uint32_t)K + (uint32_t)((lc0 ^ (((i >> 1) & 1) << 2)) * 8);
    }
    const uint32_t b_row = (uint32_t)(n0 + wave * 64 + lr) * (uint32_t)K;
    const uint32_t b_eoff[2] = {b_row + (uint32_t)(lc0 * 8), b_row + (uint32_t)((lc0 ^ 4) * 8)};
    const size_t b_istep = (size_t)8 * K;                   // Bt rows are padded to the tile: no clamp
    const int KT = K / BK;
    auto issue_load = [&](int kt_, int q) {                 // block q (0..15) of this wave's sixteen
        const int ktc = kt_ < KT ? kt_ : KT - 1;            // past the end: reload the last tile into the dead stage
        unsigned char *st = smem_raw + (kt_ & 1) * STB;
        if (q < 8) {
            __builtin_amdgcn_global_load_lds(SJD_GPTR(A + (size_t)ktc * BK + a_eoff[q]), SJD_LPTR(st + (wave * 8 + q) * 1024),
                                             16, 0, 0);
        } else {
            const int i = q - 8;
            __builtin_amdgcn_global_load_lds(SJD_GPTR(Bt + (size_t)ktc * BK + i * b_istep + b_eoff[(i >> 1) & 1]),
                                             SJD_LPTR(st + OPB + (wave * 8 + i) * 1024), 16, 0, 0);
        }
    };
    v8 fa[2][MI], fb[2][NI];
    // fragment (32 rows of row block r of the wave's sub-tile, k-step ks): row l32 is row l32 & 7 of
    // 8-row block 4 r + (l32 >> 3); its chunk 2 ks + g sits in slot (2 ks + g) ^ swz(l32)
    const int swz = ((l32 >> 1) & 3) | (((l32 >> 4) & 1) << 2);
    const int frag_base = l32 * 128;
    int frag_k[KSUB];
#pragma unroll
    for (int ks = 0; ks < KSUB; ++ks) frag_k[ks] = frag_base + (((2 * ks + g) ^ swz) << 4);
    auto read_one = [&](int stage, int ks, int buf, int r) {
        const unsigned char *st = smem_raw + stage * STB + frag_k[ks];
        if (r < MI) fa[buf][r] = *reinterpret_cast<const v8 *>(st + (wm * 16 + 4 * r) * 1024);
        else fb[buf][r - MI] = *reinterpret_cast<const v8 *>(st + OPB + (wn * 16 + 4 * (r - MI)) * 1024);
    };

#pragma unroll
    for (int q = 0; q < 16; ++q) issue_load(0, q);
    __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0): tile 0 has landed
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int r = 0; r < 8; ++r) read_one(0, 0, 0, r);

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) {
            const int b = ks & 1;
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                if (ks + 1 < KSUB) {
                    // fragments of the next k-step, issued in the first half of this one
                    if (m < 8) read_one(cur, ks + 1, b ^ 1, m);
                } else {
                    if (m == 8) {
                        // own loads of tile kt+1 complete, own LDS reads done; then everyone's
                        __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
                        __builtin_amdgcn_s_barrier();
                    }
                    if (m >= 8) read_one(cur ^ 1, 0, b ^ 1, m - 8);   // first k-step of the next tile
                }
                // the sixteen loads of tile kt+1 go out in the first two k-steps, one per two slots:
                // the stage they fill was released by the barrier of the previous k-tile
                if (ks < 2 && (m & 1) == 1) issue_load(kt + 1, ks * 8 + (m >> 1));
                acc[m / NI][m % NI] = Half16<HT>::mfma(fa[b][m / NI], fb[b][m % NI], acc[m / NI][m % NI]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0);  // every outstanding LDS-direct load has landed before LDS is reused
    __syncthreads();
    tile_epilogue<HT, MI, NI, BN, OutT, EPI>(acc, smem_raw, bias, resid, C, M, N, m0 + wm * 128, n0 + wn * 128, lane, wave);
}

template <typename HT, typename OutT, int EPI>
static void launch_dma(const HT *A, const HT *Bt, const float *bias, const float *resid, OutT *C, int M, int N, int K,
                       hipStream_t s) {
    const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
    const int n_tiles = tiles_m * tiles_n;
    const int grid = ((n_tiles + 7) / 8) * 8;
    const size_t smem = 4 * 32 * 1024;
    auto kern = gemm_h16_dma_kernel<HT, OutT, EPI>;
    static std::atomic<bool> attr_set{false};   // callers may come from several host threads
    if (!attr_set.load(std::memory_order_acquire)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), smem, s, A, Bt, bias, resid, C, M, N, K, tiles_n, n_tiles);
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
    static std::atomic<bool> attr_set{false};   // callers may come from several host threads
    if (!attr_set.load(std::memory_order_acquire)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), smem, s, A, Bt, bias, resid, C, M, N, K, tiles_n, n_tiles);
}

// Kernel choice, from measurements on the workloads' shapes (TFLOP/s, M = 32768):
//   256x128x32 staged through registers, two workgroups per CU: one workgroup's epilogue and barrier
//     stalls hide behind the other's matrix instructions - best when the epilogue is a large share
//     (GELU: 648 vs 606; float32 residual with K = 1024: 610 vs 578) and for K <= 768;
//   256x256x32 LDS-direct, one workgroup per CU: best main loop (K = 4096: 1025 vs 820) - used when
//     the k-loop dominates.
//   128x128x64 covers small problems.  Weight matrices are padded to 256 rows, so tiles never read
//   past a matrix.
template <typename HT, typename OutT, int EPI>
static void pick_tile(const HT *A, const HT *Bt, const float *bias, const float *resid, OutT *C, int M, int N, int K,
                      int kernel, hipStream_t s) {
    if (kernel == 1) return launch_tile<HT, 256, 128, 32, 2, OutT, EPI>(A, Bt, bias, resid, C, M, N, K, s);
    if (kernel == 2 && (long long)M * K < (1ll << 32) && (long long)(N + 256) * K < (1ll << 32))
        return launch_dma<HT, OutT, EPI>(A, Bt, bias, resid, C, M, N, K, s);
    if (kernel == 3) return launch_tile<HT, 128, 128, 64, 1, OutT, EPI>(A, Bt, bias, resid, C, M, N, K, s);
    // the persistent kernel updates the residual stream in place: resid, when used, must be C
    const bool p8_ok = gemm_p8_applicable(M, N, K) && (EPI != EPI_BIAS_RESIDUAL || (const void *)resid == (const void *)C);
    if (kernel == 4 && p8_ok) return launch_gemm_p8<HT, OutT>(A, Bt, bias, C, M, N, K, (Epi)EPI, s);
    const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
    const long t256 = (long)((M + 255) / 256) * ((N + 255) / 256);
    // the persistent kernel from one 256x256 tile per CU on (measured on the workloads' shapes: +15..30 % at
    // K <= 1024, even at K = 4096; with fewer tiles the finer grain of the kernels below wins)
    if (p8_ok && t256 >= 256) return launch_gemm_p8<HT, OutT>(A, Bt, bias, C, M, N, K, (Epi)EPI, s);
    const bool deep = K >= 3072 || (EPI == EPI_BIAS && K >= 768 && N >= 768);
    // the LDS-direct kernel forms element offsets of A in 32 bits
    const bool dma_ok = (long long)M * K < (1ll << 32) && (long long)(N + 256) * K < (1ll << 32);
    if (deep && dma_ok && M >= 256 && N >= 256 && t256 >= 256) launch_dma<HT, OutT, EPI>(A, Bt, bias, resid, C, M, N, K, s);
    // measured: below ~3500 tiles of 128x128 the smaller tile wins (finer tail, shorter prologue per tile)
    else if (N >= 128 && M >= 256 && t128 >= 3584) launch_tile<HT, 256, 128, 32, 2, OutT, EPI>(A, Bt, bias, resid, C, M, N, K, s);
    else launch_tile<HT, 128, 128, 64, 1, OutT, EPI>(A, Bt, bias, resid, C, M, N, K, s);
}

template <typename HT, typename OutT>
void launch_gemm_h16(const HT *A, const HT *Bt, const float *bias, const float *resid, OutT *C, int M, int N, int K,
                     Epi epi, hipStream_t s, int kernel) {
    if (M <= 0 || N <= 0) return;
    if constexpr (sizeof(OutT) == 4) {
        if (epi == EPI_BIAS_RESIDUAL) pick_tile<HT, float, EPI_BIAS_RESIDUAL>(A, Bt, bias, resid, C, M, N, K, kernel, s);
        else pick_tile<HT, float, EPI_BIAS>(A, Bt, bias, resid, C, M, N, K, kernel, s);
    } else {
        if (epi == EPI_BIAS_GELU) pick_tile<HT, HT, EPI_BIAS_GELU>(A, Bt, bias, resid, C, M, N, K, kernel, s);
        else pick_tile<HT, HT, EPI_BIAS>(A, Bt, bias, resid, C, M, N, K, kernel, s);
    }
}
template void launch_gemm_h16<bf16, bf16>(const bf16 *, const bf16 *, const float *, const float *, bf16 *, int, int,
                                          int, Epi, hipStream_t, int);
template void launch_gemm_h16<bf16, float>(const bf16 *, const bf16 *, const float *, const float *, float *, int, int,
                                           int, Epi, hipStream_t, int);
template void launch_gemm_h16<f16, f16>(const f16 *, const f16 *, const float *, const float *, f16 *, int, int, int,
                                        Epi, hipStream_t, int);
template void launch_gemm_h16<f16, float>(const f16 *, const f16 *, const float *, const float *, float *, int, int,
                                          int, Epi, hipStream_t, int);

}  // namespace sjd
