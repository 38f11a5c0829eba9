// Persistent 16-bit MFMA projection, eight waves per workgroup: C[M,N] = epi(A[M,K] * Bt[N,K]^T + bias).
//
// The tile kernels of gemm_h16.hip run one tile per workgroup: every tile pays its first loads and the
// drain of its epilogue's stores in full, because the next workgroup cannot start on the CU before this
// one has gone (128 KB of LDS each).  Here one workgroup per CU stays resident and walks over its tiles:
//   * 256 x 256 output tile; k-tiles of 32 in four 32 KB LDS stages filled by LDS-direct loads
//     (no staging registers), requested three k-tiles ahead;
//   * eight waves, two per SIMD, each owning 128 x 64 of the tile (128 accumulator registers);
//   * the request stream runs on across tiles: the first three k-tiles of the NEXT tile are requested during
//     the last ones of this tile and the first has landed before the epilogue starts, so a tile begins with
//     operands already in LDS;
//   * the epilogue parks accumulators in LDS of its own (32 KB beyond the stages), so the stages keep
//     filling meanwhile, and its stores drain while the next tile multiplies.
// k is walked in index order with the 32x32x16 instruction, an output row depends on its own row of A
// only: results are bit-identical to the tile kernels and independent of the batch.
// Covers K % 128 == 0 and N % 256 == 0 (every projection of the workloads but the head).
// What bounds it (timing probes on M = 32768, N = 1024, K = 4096; 1.05 PFLOP/s as is): the same loop
// without its global loads runs at 1.49 PFLOP/s, with loads that land in registers instead of LDS at 1.13,
// without its LDS fragment reads (loads kept) at 1.00, without the barrier at 1.05; k-tiles of 64 in two
// stages, one wave per SIMD, or padded row strides change nothing.  It is the operand traffic from L2
// (64 KB per CU per 8.4 MFLOP, about 8 TB/s in all) that costs the difference, not latency, LDS or the barrier.
#include "common.h"
#include <atomic>

namespace sjd {

namespace {

constexpr int Q_BM = 256, Q_BN = 256;
constexpr int Q_CB = 4;                     // column tiles per column block of the tile order
constexpr int D_BK = 32, D_KSUB = D_BK / 16, D_NS = 4;   // k-tile, k-steps per k-tile, LDS stages
constexpr int D_OPB = 16 * 1024;            // bytes of one operand in one stage: 256 rows x 64 B
constexpr int D_STB = 2 * D_OPB;            // bytes per stage
constexpr int D_PARK = D_NS * D_STB;        // offset of the epilogue parking space: 8 waves x 16 rows x 64 floats
constexpr int D_LDS = D_PARK + 8 * 4096;    // 160 KB
constexpr int kOutside = 0x7FFFFFF0;        // a lane offset past any buffer range this kernel declares

typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

#define SJD_Q_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define SJD_Q_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

template <typename HT, typename OutT, int EPI>
__global__ __launch_bounds__(512) void gemm_h16_p8_kernel(const HT *__restrict__ A, const HT *__restrict__ Bt,
                                                             const float *__restrict__ bias, OutT *C, int M, int N,
                                                             int K, int tiles_m, int tiles_n, int col_block) {
    typedef typename Half16<HT>::v8 v8;
    typedef typename Half16<HT>::v4 v4;
    constexpr bool OUT_F32 = sizeof(OutT) == 4;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    // Workgroup ids congruent mod 8 share an XCD (and its L2).  Each XCD owns a contiguous range of row panels
    // and walks it column block by column block (Q_CB column tiles wide), row by row inside a block; its
    // workgroups take the tiles of that order round-robin.  So at any time the 32 workgroups of an XCD work on
    // about eight row panels against the same few column tiles of the weight, and the next round keeps those
    // column tiles: the weight rows of a column block (2 MB at k = 1024) stay in the 4 MB L2 while the row
    // panels stream past them, instead of the whole weight being fetched again for every pair of row panels
    // (measured on the MLP input projection, M = 32768, N = 4096, K = 1024: 637 MB per launch went through the
    // L2-miss counters in plain row-major tile order, for 75 MB of operands; blocks of 4 column tiles are
    // 5-10 % faster than row-major order on the q/k/v and MLP input shapes, blocks of 2 are slower, 6 the same).
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, n_slots = gridDim.x >> 3;
    const int rp0 = (int)((long long)xcd * tiles_m / 8), nrp = (int)((long long)(xcd + 1) * tiles_m / 8) - rp0;
    const int n_mine = nrp * tiles_n;
    auto tile_of = [&](int li) {
        if (li >= n_mine) return -1;
        const int cb = li / (nrp * col_block);
        const int left = tiles_n - cb * col_block, cbw = left < col_block ? left : col_block;
        const int lo = li - cb * nrp * col_block;
        const int r = lo / cbw;
        return (rp0 + r) * tiles_n + cb * col_block + (lo - r * cbw);
    };
    int li = slot;
    int tile = tile_of(li);
    if (tile < 0) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS bases stay in scalar registers
    const int l32 = lane & 31, g = lane >> 5;
    const int wm = wave >> 2, wn = wave & 3;                     // this wave's 128 x 64 part of the tile
    const int KT = K / D_BK;

    // Loads.  A stage holds a k-tile of 32: rows of 64 bytes (four 16-byte chunks), A then B, 16 KB each.  Per
    // k-tile a wave brings the 16-row blocks 2 wave + i (i = 0, 1) of A and of B, 1 KB each: lane 4 r + c delivers
    // the chunk that belongs in slot c of row r.  Row r of a 32-row fragment group keeps chunk c in slot
    // c ^ swz(r), swz(r) = bits 2 and 4 of r: a 16-byte LDS read of a wave is served in four passes of 16 lanes
    // (rows {0-7, 16-23} or {8-15, 24-31} of the group, one chunk) over 64 banks; with rows 64 bytes apart the
    // bank group of a read is 4 (r mod 4) + slot, which this makes distinct over the sixteen rows of a pass.
    // Addresses are a wave-uniform 64-bit base (the tile's first row, advanced by the k-tile) plus a
    // per-lane 32-bit byte offset inside the tile: few registers, and no 32-bit overflow however large M is.
    const int lr = lane >> 2;                                    // row within the 16-row block
    const int lc0 = (lane & 3) ^ ((lr >> 2) & 1);                // chunk fetched for blocks with bit 4 of the row clear
    const uint32_t row_bytes = (uint32_t)K * 2u;
    struct Src { uint32_t a_off[2]; const char *a_base, *b_base; };
    auto make_src = [&](int t) {
        Src s;
        const int tm = t / tiles_n, tn = t - tm * tiles_n;
        const int last = M - 1 - tm * Q_BM;                      // last valid row of this tile (tile-relative, >= 0)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int row = (wave * 2 + i) * 16 + lr;
            row = row < last ? row : last;                       // rows past the end: re-read the last row, never stored
            s.a_off[i] = (uint32_t)row * row_bytes + (uint32_t)((lc0 ^ (i << 1)) * 16);
        }
        s.a_base = reinterpret_cast<const char *>(A + (size_t)tm * Q_BM * K);
        s.b_base = reinterpret_cast<const char *>(Bt + (size_t)tn * Q_BN * K);   // Bt rows are padded to the tile
        return s;
    };
    uint32_t b_off[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
        b_off[i] = (uint32_t)((wave * 2 + i) * 16 + lr) * row_bytes + (uint32_t)((lc0 ^ (i << 1)) * 16);
    // An LDS-direct load: 64 lanes x 16 bytes from (wave-uniform base) + (per-lane 32-bit offset) to 1 KB of LDS
    // at the wave-uniform byte address lds_addr (through M0).  Written out so that the address stays split
    // into a scalar base and a 32-bit lane offset (two registers per lane per load otherwise).  M0 is set
    // inside the statement and nothing else in this kernel reads it (no other LDS-direct access, no
    // indexed register moves), so nothing of the compiler's is lost.
    auto dma = [&](const char *base, uint32_t off, uint32_t lds_addr) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(lds_addr), "v"(off), "s"(base) : "memory");
    };
    const uint32_t lds0 = (uint32_t)(uintptr_t)SJD_Q_LPTR(lds);
    auto issue_load = [&](const Src &s, int kt, int stage, int q) {   // q = 0..3: this wave's four blocks
        const uint32_t st = lds0 + (uint32_t)(stage * D_STB);
        if (q < 2) dma(s.a_base + (size_t)kt * (D_BK * 2), s.a_off[q], st + (uint32_t)((wave * 2 + q) * 1024));
        else dma(s.b_base + (size_t)kt * (D_BK * 2), b_off[q - 2], st + (uint32_t)(D_OPB + (wave * 2 + q - 2) * 1024));
    };

    // Fragments: row l32 of a 32-row group, chunk 2 ks + g, found in slot (2 ks + g) ^ swz(l32); rows are 64 B
    // apart.  A fragments are refreshed in place right after their last use in a k-step, B fragments
    // (used by all four row groups) alternate between two sets.
    const int swz = ((l32 >> 2) & 1) | (((l32 >> 4) & 1) << 1);
    int fk[D_KSUB];
#pragma unroll
    for (int ks = 0; ks < D_KSUB; ++ks) fk[ks] = l32 * 64 + (((2 * ks + g) ^ swz) << 4);
    const int a_lds = wm * (128 * 64), b_lds = D_OPB + wn * (64 * 64);
    v8 fa[4], fb[2][2];
    auto read_a = [&](int stage, int ks, int i) {
        fa[i] = *reinterpret_cast<const v8 *>(lds + (stage * D_STB + a_lds + 32 * i * 64) + fk[ks]);
    };
    auto read_b = [&](int stage, int ks, int buf, int j) {
        fb[buf][j] = *reinterpret_cast<const v8 *>(lds + (stage * D_STB + b_lds + 32 * j * 64) + fk[ks]);
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // One k-tile: 16 matrix instructions of this wave, each a slot with its LDS reads and loads pinned.
    // `next` / `next_kt`: the k-tile requested during this one - three k-tiles ahead, into the stage that the
    // previous k-tile used (released by the barrier that ended it).  After the second slot of the last k-step:
    // wait until this wave's loads of the NEXT k-tile have landed (the eight younger ones, of the two k-tiles
    // after it, may stay in flight: loads complete in order) and its LDS reads are done, then the barrier;
    // the rest of the k-step reads the next k-tile's first fragments.
    auto ktile = [&](int stage, const Src &next, int next_kt) {
#pragma unroll
        for (int ks = 0; ks < D_KSUB; ++ks) {
            const int b = ks & 1;
            const bool last = ks + 1 == D_KSUB;
            const int rs = last ? (stage + 1) % D_NS : stage, rk = last ? 0 : ks + 1;   // where the next k-step's fragments are
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                const int i = m >> 1, j = m & 1;
                if (ks == 0 && j == 1) issue_load(next, next_kt, (stage + 3) % D_NS, i);
                if (!last && m == 0) { read_b(rs, rk, b ^ 1, 0); read_b(rs, rk, b ^ 1, 1); }
                acc[i][j] = Half16<HT>::mfma(fa[i], fb[b][j], acc[i][j]);
                __builtin_amdgcn_sched_barrier(0);
                if (last && m == 1) {
                    __builtin_amdgcn_s_waitcnt(0x0078);   // vmcnt(8) lgkmcnt(0)
                    __builtin_amdgcn_s_barrier();
                    read_b(rs, rk, b ^ 1, 0);
                    read_b(rs, rk, b ^ 1, 1);
                }
                if (j == 1) read_a(rs, rk, i);           // row group i is done for this k-step: fetch the next one's
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    Src cur = make_src(tile);
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
        for (int q = 0; q < 4; ++q) issue_load(cur, t, t, q);
    __builtin_amdgcn_s_waitcnt(0x0F78);       // vmcnt(8): the first k-tile has landed
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int i = 0; i < 4; ++i) read_a(0, 0, i);
    read_b(0, 0, 0, 0);
    read_b(0, 0, 0, 1);

    float *ep = reinterpret_cast<float *>(lds + D_PARK) + wave * 1024;
    const int rl = lane >> 4, cl = (lane & 15) * 4;

    while (true) {
        const int tm = tile / tiles_n, tn = tile - tm * tiles_n;
        li += n_slots;
        const int tile_next = tile_of(li);
        // no next tile: request this tile's first k-tile again (in bounds, never used)
        const Src nxt = make_src(tile_next >= 0 ? tile_next : tile);

        // four k-tiles per trip (stages 0..3); in the last trip the requests run over into the next tile's first
        // three k-tiles - by selecting the source, not by branching: one straight-line loop body
        for (int kt = 0; kt < KT; kt += 4) {
            ktile(0, cur, kt + 3);
            const bool wrap = kt + 4 >= KT;
            Src sel;
#pragma unroll
            for (int i = 0; i < 2; ++i) sel.a_off[i] = wrap ? nxt.a_off[i] : cur.a_off[i];
            sel.a_base = wrap ? nxt.a_base : cur.a_base;
            sel.b_base = wrap ? nxt.b_base : cur.b_base;
            const int k0 = wrap ? 0 : kt + 4;
            ktile(1, sel, k0);
            ktile(2, sel, k0 + 1);
            ktile(3, sel, k0 + 2);
        }
        // here: stage 0 holds the next tile's first k-tile (two more are on their way), fa / fb[0] its first fragments

        // ---- epilogue.  In the accumulators a lane owns one column and sixteen rows of a 32x32 block
        // (register v: row 8 (v / 4) + 4 g + v % 4).  Sixteen rows x 64 columns at a time go through the
        // wave's parking slice and come back row-wise, four columns per lane, so that bias, GELU, the
        // residual and the stores move 8 or 16 bytes per lane in whole rows.  The slice has no padding:
        // rows with g = 1 keep their two 32-column halves swapped, which puts the 64 lanes of a write on
        // 64 different banks.  No branches: rows past M fall outside the buffer descriptor and are dropped.
        {
            const int row0 = tm * Q_BM + wm * 128, col0 = tn * Q_BN + wn * 64;
            int rows_left = M - row0;
            rows_left = rows_left < 0 ? 0 : (rows_left > 128 ? 128 : rows_left);
            OutT *cbase = C + (size_t)row0 * N + col0;
            const int n_bytes = rows_left > 0 ? ((rows_left - 1) * N + 64) * (int)sizeof(OutT) : 0;
            const rsrc_t c_rs = __builtin_amdgcn_make_buffer_rsrc(cbase, 0, n_bytes, 0x00020000);
            // The lane part of every address is one register, made opaque per tile: left alone, the compiler
            // moves the 32 row offsets of a tile out of the tile loop and keeps them in registers it does not have.
            // The row-group part of an address is wave-uniform and travels as the scalar offset of the access.
            int lane_off = (rl * N + cl) * (int)sizeof(OutT);
            asm volatile("" : "+v"(lane_off));
            const int row_step = N * (int)sizeof(OutT);
            const f32x4 bv4 = *reinterpret_cast<const f32x4 *>(bias + col0 + cl);
#pragma unroll
            for (int n = 0; n < 8; ++n) {
                const int i = n >> 1, hh = n & 1;
                f32x4 val[4], res[4];
                if constexpr (EPI == EPI_BIAS_RESIDUAL) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int r0 = 32 * i + 16 * hh + 4 * q;
                        res[q] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(c_rs, r0 + rl < rows_left ? lane_off : kOutside, r0 * row_step, 0));
                    }
                }
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int vv = 0; vv < 8; ++vv)
                        ep[(8 * (vv >> 2) + 4 * g + (vv & 3)) * 64 + 32 * (j ^ g) + l32] = acc[i][j][8 * hh + vv];
                asm volatile("" ::: "memory");       // a wave's LDS operations execute in order: no wait, only the order
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    val[q] = *reinterpret_cast<const f32x4 *>(&ep[(4 * q + rl) * 64 + (cl ^ (32 * (q & 1)))]);
                asm volatile("" ::: "memory");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int r0 = 32 * i + 16 * hh + 4 * q;
                    const int s_off = r0 * row_step;
                    const int v_off = r0 + rl < rows_left ? lane_off : kOutside;   // rows past M: an offset no buffer holds
                    f32x4 o = val[q] + bv4;
                    if constexpr (EPI == EPI_BIAS_GELU) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = gelu_erf_h16(o[e]);
                    }
                    if constexpr (OUT_F32) {
                        if constexpr (EPI == EPI_BIAS_RESIDUAL) o += res[q];
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(i32x4, o), c_rs, v_off, s_off, 0);
                    } else {
                        v4 o4;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o4[e] = from_f32<HT>(o[e]);
                        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(i32x2, o4), c_rs, v_off, s_off, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (tile_next < 0) break;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        tile = tile_next;
        cur = nxt;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);       // the loads of the unused last requests have landed before the LDS goes away
}

int p8_cus() {
    static std::atomic<int> cus{0};
    int c = cus.load(std::memory_order_acquire);
    if (c == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        c = (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) ? prop.multiProcessorCount : 256;
        if (c < 8) c = 8;
        cus.store(c, std::memory_order_release);
    }
    return c;
}

}  // namespace

bool gemm_p8_applicable(int M, int N, int K) {
    return M >= 1 && N >= 256 && N % 256 == 0 && K >= 128 && K % 128 == 0 && (long long)N * 4 * 128 < (1ll << 31) &&
           (long long)((M + 255) / 256) * (N / 256) < (1ll << 30);
}

template <typename HT, typename OutT, int EPI>
static void launch_p8_one(const HT *A, const HT *Bt, const float *bias, OutT *C, int M, int N, int K, hipStream_t s) {
    const int tiles_m = (M + Q_BM - 1) / Q_BM, tiles_n = N / Q_BN;
    const int per_xcd = ((tiles_m + 7) / 8) * tiles_n;      // tiles of the XCD with the most row panels
    const int slots = per_xcd < p8_cus() / 8 ? per_xcd : p8_cus() / 8;
    auto kern = gemm_h16_p8_kernel<HT, OutT, EPI>;
    static std::atomic<bool> attr_set{false};   // callers may come from several host threads
    if (!attr_set.load(std::memory_order_acquire)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, D_LDS);
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3(8 * slots), dim3(512), D_LDS, s, A, Bt, bias, C, M, N, K, tiles_m, tiles_n, Q_CB);
}

template <typename HT, typename OutT>
void launch_gemm_p8(const HT *A, const HT *Bt, const float *bias, OutT *C, int M, int N, int K, Epi epi, hipStream_t s) {
    if constexpr (sizeof(OutT) == 4) {
        if (epi == EPI_BIAS_RESIDUAL) launch_p8_one<HT, float, EPI_BIAS_RESIDUAL>(A, Bt, bias, C, M, N, K, s);
        else launch_p8_one<HT, float, EPI_BIAS>(A, Bt, bias, C, M, N, K, s);
    } else {
        if (epi == EPI_BIAS_GELU) launch_p8_one<HT, HT, EPI_BIAS_GELU>(A, Bt, bias, C, M, N, K, s);
        else launch_p8_one<HT, HT, EPI_BIAS>(A, Bt, bias, C, M, N, K, s);
    }
}
template void launch_gemm_p8<bf16, bf16>(const bf16 *, const bf16 *, const float *, bf16 *, int, int, int, Epi, hipStream_t);
template void launch_gemm_p8<bf16, float>(const bf16 *, const bf16 *, const float *, float *, int, int, int, Epi, hipStream_t);
template void launch_gemm_p8<f16, f16>(const f16 *, const f16 *, const float *, f16 *, int, int, int, Epi, hipStream_t);
template void launch_gemm_p8<f16, float>(const f16 *, const f16 *, const float *, float *, int, int, int, Epi, hipStream_t);

}  // namespace sjd
