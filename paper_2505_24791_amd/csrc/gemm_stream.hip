// Residual projection for long k (the MLP-output projection): H[M,N] += A[M,K] * W + bias, K a multiple of
// 512, N a multiple of 256, 16-bit operands, float32 residual stream.
//
// Same division of labour as the panel kernels (gemm_panel.hip) - the left operand through LDS, the
// weights straight from L2 into registers in fragment order, eight k-steps ahead, four waves of
// 128 x 64 per workgroup - but the left operand does not fit LDS for K > 512, so it streams through
// two 64 KB buffers in chunks of 256 k: while chunk c is multiplied the waves fetch chunk c + 1 with
// LDS-direct loads (no staging registers, no LDS write instructions), two per k-step in the first
// half of the chunk.  One barrier per chunk, i.e. per 128 matrix instructions of a wave.  k is
// walked in index order with the 32x32x16 instruction: results are bit-identical to the tile kernels.
//
// Waits.  With LDS-direct loads in flight the compiler no longer counts how many younger loads may stay
// outstanding when a register load is needed - it waits for all of them (vmcnt(0)), which would undo the
// weight look-ahead twice per chunk.  The weight loads are therefore written as inline assembly (which
// the compiler does not track) and every wait of the main loop is written out from the fixed issue
// order of a wave's memory instructions: per k-step [piece, piece (k-steps 0-7 of a chunk)], weight
// fragment 0 (slot 4), weight fragment 1 (after slot 7).  Loads return in order, so "at most n younger
// ones outstanding" means the one needed has arrived.
#include "common.h"
#include <atomic>

namespace sjd {

namespace {

constexpr int S_CK = 256, S_CKS = S_CK / 16;  // k per chunk and k-steps per chunk
constexpr int S_PD = 8;                       // weight prefetch depth in k-steps
constexpr int S_BUF = 128 * S_CK * 2;         // one buffer: 128 rows x 512 bytes
constexpr int S_EP = 68;                      // pitch of the epilogue parking rows in floats
constexpr int S_LDS = 2 * S_BUF + 4 * 16 * S_EP * 4;

typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef int i32x4 __attribute__((ext_vector_type(4)));

#define SJD_S_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define SJD_S_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

// Row r of a buffer keeps its 16-byte chunk c (of 32) in slot c ^ swz(r).  A 16-byte LDS read of a wave
// is served in four passes of 16 lanes (rows {0-7, 16-23} or {8-15, 24-31} of a 32-row fragment, one
// chunk), 64 banks wide; rows are 512 bytes apart, so the bank group of a read is its slot modulo 16.
__device__ __forceinline__ int stream_swz(int row) { return (row & 7) | (((row >> 4) & 1) << 3); }

// 16-byte global load the compiler does not track (see "Waits" above)
template <typename V8, typename HT>
__device__ __forceinline__ void load_untracked(V8 &dst, const HT *p) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(p) : "memory");
}
// Waits.  A wait is a statement that owns the registers it is for: they are in/out operands of the
// s_waitcnt, so whatever consumes them afterwards depends on the wait, and from the (untracked) load that
// writes them to this statement they are live values that the allocator may not hand to anything else.
// n (14..31, or 0) folds to a constant once the loops around the call are unrolled.
template <typename V8>
__device__ __forceinline__ void wait_vm_for(V8 &frag, int n) {
    switch (n) {
#define SJD_S_W(k) case k: asm volatile("s_waitcnt vmcnt(" #k ")" : "+v"(frag)); break;
        SJD_S_W(14) SJD_S_W(15) SJD_S_W(16) SJD_S_W(17) SJD_S_W(18) SJD_S_W(19) SJD_S_W(20) SJD_S_W(21) SJD_S_W(22)
        SJD_S_W(23) SJD_S_W(24) SJD_S_W(25) SJD_S_W(26) SJD_S_W(27) SJD_S_W(28) SJD_S_W(29) SJD_S_W(30) SJD_S_W(31)
#undef SJD_S_W
    default: asm volatile("s_waitcnt vmcnt(0)" : "+v"(frag)); break;
    }
}
// every load has landed; all sixteen ring registers pass through the statement
template <typename V8>
__device__ __forceinline__ void wait_all_for(V8 (&bq)[S_PD][2]) {
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)"
                 : "+v"(bq[0][0]), "+v"(bq[0][1]), "+v"(bq[1][0]), "+v"(bq[1][1]), "+v"(bq[2][0]), "+v"(bq[2][1]),
                   "+v"(bq[3][0]), "+v"(bq[3][1]), "+v"(bq[4][0]), "+v"(bq[4][1]), "+v"(bq[5][0]), "+v"(bq[5][1]),
                   "+v"(bq[6][0]), "+v"(bq[6][1]), "+v"(bq[7][0]), "+v"(bq[7][1]));
}
static_assert(S_PD == 8, "wait_all_for names eight ring slots");
// k-steps among the seven before k-step ks of a chunk (running over from the previous chunk) that requested pieces
constexpr int pieces_window(int ks) {
    int f = 0;
    for (int d = 1; d <= 7; ++d) f += ((ks - d + S_CKS) % S_CKS) < 8 ? 1 : 0;
    return f;
}

template <typename HT>
__global__ __launch_bounds__(256, 1) void gemm_stream_resid_kernel(const HT *__restrict__ A, const HT *__restrict__ Wf,
                                                                   const float *__restrict__ bias, float *H, int M, int N,
                                                                   int K, int n_groups, int n_panels) {
    typedef typename Half16<HT>::v8 v8;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    // workgroup ids congruent mod 8 share an XCD: the workgroups of one row panel (one per column group)
    // sit on one XCD and run at the same time, so the panel's rows come from HBM once
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int panel = (idx / n_groups) * 8 + xcd, grp = idx % n_groups;
    if (panel >= n_panels) return;
    const int m0 = panel * 128;
    const int KS = K / 16, NC = K / S_CK;             // k-steps in all, chunks (even)
    const rsrc_t c_rs = __builtin_amdgcn_make_buffer_rsrc(H, 0, M * N * 4, 0x00020000);   // rows past M: dropped / zero

    // weights: this wave's two 32-column blocks; fragment (nb, ks) at ((nb KS + ks) 64 + lane) 16 bytes
    const HT *wbase[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) wbase[j] = Wf + ((size_t)((grp * 256 + wave * 64) / 32 + j) * KS * 64 + lane) * 8;
    v8 bq[S_PD][2];
#pragma unroll
    for (int p = 0; p < S_PD; ++p)
#pragma unroll
        for (int j = 0; j < 2; ++j) load_untracked(bq[p][j], wbase[j] + (size_t)p * 512);

    // left operand: this wave fetches rows 32 wave .. + 31 of every chunk, two rows (64 slots) per load;
    // lane l of load q brings the chunk that belongs in slot l % 32 of row 32 wave + 2 q + l / 32
    uint32_t a_off[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int r = 32 * wave + 2 * q + (lane >> 5);
        const int rc = m0 + r < M ? m0 + r : M - 1;   // rows past the end: any valid row, never stored
        a_off[q] = (uint32_t)rc * (uint32_t)K + (uint32_t)(((lane & 31) ^ stream_swz(r)) * 8);
    }
    auto fetch = [&](int chunk, int buf, int q) {
        __builtin_amdgcn_global_load_lds(SJD_S_GPTR(A + (size_t)chunk * S_CK + a_off[q]),
                                         SJD_S_LPTR(lds + buf * S_BUF + (32 * wave + 2 * q) * 512), 16, 0, 0);
    };
#pragma unroll
    for (int q = 0; q < 16; ++q) fetch(0, 0, q);
    wait_all_for(bq);                         // chunk 0 and the first weight fragments have landed
    __builtin_amdgcn_s_barrier();

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int sw = stream_swz(l32);
    const unsigned char *a_base = lds + l32 * 512;
    v8 fa[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[0][i] = *reinterpret_cast<const v8 *>(a_base + i * 32 * 512 + ((g ^ sw) << 4));

    // One chunk = 16 k-steps = 128 matrix instructions of this wave, each a slot with its loads pinned:
    // slots 0-3 read the panel fragments of the next k-step; k-steps 0-7 request two pieces of the next
    // chunk each (into the other buffer, released by the barrier that ended the previous chunk); a
    // weight fragment is requested again, eight k-steps ahead, as soon as its last use has been issued.
    // In front of the last k-step, whose fragment reads already belong to the next chunk: wait for this
    // wave's own pieces (sixteen weight loads issued since stay in flight), then the barrier.
    auto chunk_body = [&](int c, int buf) {
        // past the end of k: refetch the last chunk and the last eight weight fragments (in bounds, unused) -
        // selects, not branches: at a join the compiler would wait for every load in flight
        const int last = c + 1 < NC ? 0 : 1;
        const int cn = c + 1 - last;
        const HT *wahead[2];                                       // the fragments of k-steps 16 .. 23 from this chunk's start
#pragma unroll
        for (int j = 0; j < 2; ++j) wahead[j] = wbase[j] + (size_t)((c + 1) * S_CKS - 8 * last) * 512;
        const HT *wcur[2] = {wbase[0] + (size_t)c * S_CKS * 512, wbase[1] + (size_t)c * S_CKS * 512};
#pragma unroll
        for (int ks = 0; ks < S_CKS; ++ks) {
            const int b = ks & 1, slot = ks % S_PD;
            if (ks == S_CKS - 1) {
                __builtin_amdgcn_s_waitcnt(0x4070);   // vmcnt(16) lgkmcnt(0)
                __builtin_amdgcn_s_barrier();
            }
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                const int i = m & 3, j = m >> 2;
                if (m < 4) {
                    const unsigned char *src = ks + 1 < S_CKS ? a_base + buf * S_BUF + (((2 * (ks + 1) + g) ^ sw) << 4)
                                                              : a_base + (buf ^ 1) * S_BUF + ((g ^ sw) << 4);
                    fa[b ^ 1][m] = *reinterpret_cast<const v8 *>(src + m * 32 * 512);
                }
                // fragment 0 of this k-step was requested in slot 4 eight k-steps ago: since then fragment 1 of
                // that k-step, two fragments in each of seven k-steps and the pieces of that window
                if (m == 0) wait_vm_for(bq[slot][0], 15 + 2 * pieces_window(ks));
                if (ks < 8 && m < 2) fetch(cn, buf ^ 1, 2 * ks + m);
                if (m == 4) {
                    // fragment 1: requested after slot 7 eight k-steps ago; since then seven k-steps and this one's pieces
                    wait_vm_for(bq[slot][1], 14 + 2 * pieces_window(ks) + (ks < 8 ? 2 : 0));
                    __builtin_amdgcn_sched_barrier(0);
                    load_untracked(bq[slot][0], ks + S_PD < S_CKS ? wcur[0] + (size_t)(ks + S_PD) * 512
                                                                  : wahead[0] + (size_t)(ks + S_PD - S_CKS) * 512);
                }
                acc[i][j] = Half16<HT>::mfma(fa[b][i], bq[slot][j], acc[i][j]);
                __builtin_amdgcn_sched_barrier(0);
            }
            load_untracked(bq[slot][1], ks + S_PD < S_CKS ? wcur[1] + (size_t)(ks + S_PD) * 512
                                                          : wahead[1] + (size_t)(ks + S_PD - S_CKS) * 512);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    for (int c = 0; c < NC; c += 2) {
        chunk_body(c, 0);
        chunk_body(c + 1, 1);
    }
    // Every load has landed: the LDS-direct ones, and the last sixteen weight fragments, which nobody uses.
    // Their registers are operands of this wait, so they stay allocated up to here: nothing else can be
    // given a register that a load is still going to write.
    wait_all_for(bq);
    __builtin_amdgcn_s_barrier();

    // ---- epilogue.  In the accumulators a lane owns one column and sixteen rows of a 32x32 block
    // (register v: row 8 (v / 4) + 4 g + v % 4).  Sixteen rows x 64 columns at a time go through the
    // wave's parking slice and come back row-wise, four columns per lane, so that the residual is read
    // and written 16 bytes per lane in whole 256-byte rows.  No branches (rows past M are dropped by the
    // buffer bounds); the slice is rewritten while the previous rows are added and stored.
    float *ep = reinterpret_cast<float *>(lds + 2 * S_BUF) + wave * 16 * S_EP;
    const int rl = lane >> 4, cl = (lane & 15) * 4;
    const int col0 = grp * 256 + wave * 64;
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
                    ep[(8 * (vv >> 2) + 4 * g + (vv & 3)) * S_EP + 32 * j + l32] = acc[i][j][8 * hh + vv];
            asm volatile("" ::: "memory");       // a wave's LDS operations execute in order: no wait, only the order
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                val[n & 1][q] = *reinterpret_cast<const f32x4 *>(&ep[(4 * q + rl) * S_EP + cl]);
                const int row = m0 + 16 * n + 4 * q + rl;
                res[n & 1][q] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(c_rs, (row * N + col0 + cl) * 4, 0, 0));
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
        }
        if (n > 0) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row = m0 + 16 * (n - 1) + 4 * q + rl;
                f32x4 o = val[(n - 1) & 1][q] + bv4;
                o += res[(n - 1) & 1][q];
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(i32x4, o), c_rs, (row * N + col0 + cl) * 4, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// wt [N (padded), K] row-major -> fragment order: fragment (nb, ks) = 64 lanes x 16 bytes, lane (l32, g)
// holds wt[32 nb + l32][16 ks + 8 g .. + 8] - the second operand of the 32x32x16 instruction
template <typename HT>
__global__ __launch_bounds__(256) void weights_to_frag32_kernel(const HT *__restrict__ wt, HT *__restrict__ dst, int N, int K) {
    typedef typename Half16<HT>::v8 v8;
    const size_t i = blockIdx.x * 256ull + threadIdx.x;   // one 16-byte piece
    if (i >= (size_t)N * K / 8) return;
    const int lane = (int)(i & 63), KS = K / 16;
    const size_t f = i >> 6;
    const int ks = (int)(f % KS), nb = (int)(f / KS), l32 = lane & 31, g = lane >> 5;
    *reinterpret_cast<v8 *>(dst + i * 8) = *reinterpret_cast<const v8 *>(wt + (size_t)(32 * nb + l32) * K + 16 * ks + 8 * g);
}

}  // namespace

bool gemm_stream_applicable(int M, int N, int K) {
    return K >= 512 && K % 512 == 0 && M >= 1 && N >= 256 && N % 256 == 0 && ((long long)M + 128) * N * 4 < (1ll << 31) &&
           (long long)M * K < (1ll << 31);
}

template <typename HT>
void launch_weights_to_frag32(const HT *wt, HT *dst, int N, int K, hipStream_t s) {
    const size_t pieces = (size_t)N * K / 8;
    hipLaunchKernelGGL(weights_to_frag32_kernel<HT>, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, s, wt, dst, N, K);
}
template void launch_weights_to_frag32<bf16>(const bf16 *, bf16 *, int, int, hipStream_t);
template void launch_weights_to_frag32<f16>(const f16 *, f16 *, int, int, hipStream_t);

template <typename HT>
void launch_gemm_stream_resid(const HT *A, const HT *Wf, const float *bias, float *H, int M, int N, int K, hipStream_t s) {
    if (M <= 0) return;
    const int n_panels = (M + 127) / 128, n_groups = N / 256;
    auto kern = gemm_stream_resid_kernel<HT>;
    static std::atomic<bool> attr_set{false};   // callers may come from several host threads
    if (!attr_set.load(std::memory_order_acquire)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, S_LDS);
        attr_set.store(true, std::memory_order_release);
    }
    const int grid = ((n_panels + 7) / 8) * n_groups * 8;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), S_LDS, s, A, Wf, bias, H, M, N, K, n_groups, n_panels);
}
template void launch_gemm_stream_resid<bf16>(const bf16 *, const bf16 *, const float *, float *, int, int, int, hipStream_t);
template void launch_gemm_stream_resid<f16>(const f16 *, const f16 *, const float *, float *, int, int, int, hipStream_t);

}  // namespace sjd
