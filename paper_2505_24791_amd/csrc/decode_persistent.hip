// Sequential inverse of one block (eq. 5 with the key/value cache of Sec. 3.5) as ONE persistent
// kernel, for the 16-bit modes with head size 64.
//
// A step of the sequential inverse is a chain of ~5 N dependent skinny projections on a handful
// of rows; launched one by one every link costs a kernel boundary (about 2 us) plus a cold start.
// Here the chain runs inside one cooperative launch of one workgroup per CU.  The workgroups
// that share an XCD (they share its L2) form a group; each group takes an equal share of the
// samples and carries them through the whole block on its own, so groups never talk to each other
// and the only synchronisation is a barrier among the ~32 workgroups of a group.  Inside a group
// every projection is split by output columns over the members; what one member writes
// (activations, a few KB per stage) the others read back through the shared L2:
//   * the writer's stores are write-through; it waits for their acknowledgement (vmcnt) before it
//     arrives at the barrier with a relaxed device-scope atomic add on the group's counter;
//   * readers poll that counter with relaxed loads, then read the activations with loads that
//     carry the sc1 scope bit, which never hit in the CU's own vector cache;
//   * no L2 write-back or invalidate is needed, because writer and reader use the same L2.  (A
//     barrier with release/acquire fences at device scope costs ~7 us for 32 members here, this
//     one ~1 us.)
// Weights are read-only and come through the normal cached path.  Every spin is bounded: if a
// barrier does not complete within the spin limit the workgroup records an error and leaves, the
// others of its group follow at their next barrier, and the host reports the failure.
//
// The arithmetic per row is that of the step kernels in decode.hip: LayerNorm statistics in two
// passes over a row held in registers, 16x16x32 MFMA with K split over the 8 waves of a
// workgroup and partial sums added in wave order, float32 residual stream.  A row's result does
// not depend on which group or member computes it.
#include "common.h"

namespace sjd {

namespace {

constexpr int P_NW = 8;  // waves per workgroup
constexpr int P_THREADS = 64 * P_NW;
constexpr int P_CB = 4;  // 16-column blocks per round of a LayerNorm-fused projection
constexpr int P_EB = 2;  // embedding column blocks of a member whose w_in slice is kept in LDS

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void *p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}
// 16-byte / 4-byte loads with the sc1 scope bit: served by L2, never by this CU's vector cache
__device__ __forceinline__ i32x4 ld16_l2(rsrc_t rs, uint32_t byte_off) {
    return __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)byte_off, 0, 16));
}
// the same for rows of the key/value cache, with the streaming hint on top: a row is read once per step and
// the cache is far larger than any cache level, so it should not displace the weights, which every step reads again
__device__ __forceinline__ i32x4 ld16_l2_stream(rsrc_t rs, uint32_t byte_off) {
    return __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)byte_off, 0, 16 | 2));
}
__device__ __forceinline__ float ld4_l2(rsrc_t rs, uint32_t byte_off) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)byte_off, 0, 16));
}

struct Ctx {
    int tid, lane, wave, r, kg;
    int slot, n;        // this workgroup's index in its group, members of the group
    int rb0;            // first 16-row block of the group in the workspaces
    int row0, nrows;    // first sample of the group, samples of the group
    int epoch;
    int *cnt, *status;
    int spin_max;
#ifdef SJD_SEQ_TIMELINE
    int *tl; int *tl_k; bool tl_on; long long tl_t0;   // tl_k: counter in LDS
#endif
};

// Development aid, compiled in only with -DSJD_SEQ_TIMELINE: member 0 of group 0 records the 100 MHz
// clock at stage boundaries (and a few points inside stages) of one step into the tail of the
// synchronisation words.
#ifdef SJD_SEQ_TIMELINE
#define SJD_TLC(cc_) do { if ((cc_).tl_on && (cc_).tid == 0) { const int k_ = (*(cc_).tl_k)++; if (k_ < 300) (cc_).tl[k_] = (int)(wall_clock64() - (cc_).tl_t0); } } while (0)
#else
#define SJD_TLC(c) do { } while (0)
#endif

// A copy of the per-thread indices that the optimiser cannot see through: addresses derived from it
// are recomputed where they are used instead of being hoisted out of the step loop and kept in
// registers for the whole kernel (which costs far more than the few integer instructions).
__device__ __forceinline__ Ctx local_ctx(const Ctx &c) {
    Ctx d = c;
    asm volatile("" : "+v"(d.lane), "+v"(d.tid), "+v"(d.r), "+v"(d.kg));
    d.wave = __builtin_amdgcn_readfirstlane(d.wave);
    d.slot = __builtin_amdgcn_readfirstlane(d.slot);
    d.rb0 = __builtin_amdgcn_readfirstlane(d.rb0);
    asm volatile("" : "+s"(d.wave), "+s"(d.slot), "+s"(d.rb0));
    return d;
}

// Barrier among the workgroups of one group (see the header).  Returns false after a time-out.
__device__ __forceinline__ bool group_barrier(Ctx &c, volatile int *sh_ok) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's stores have been acknowledged by L2
    __syncthreads();
    ++c.epoch;
    if (c.tid == 0) {
        __hip_atomic_fetch_add(c.cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int target = c.epoch * c.n;
        int it = 0, ok = 1;
        while (__hip_atomic_load(c.cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (++it > c.spin_max) { ok = 0; break; }
            __builtin_amdgcn_s_sleep(1);
        }
        if (!ok) __hip_atomic_store(c.status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *sh_ok = ok;
    }
    __syncthreads();
    return *sh_ok != 0;
}

// Weight fragments of a stage, fetched ahead of the barrier that precedes the stage (weights do
// not depend on what the other members are still computing).
template <typename HT, int S> struct LnPre { typename Half16<HT>::v8 f[P_CB][S]; };
template <typename HT, int S, int KMUL> struct ResPre { typename Half16<HT>::v8 f[KMUL * S]; };
struct NoPrefetch { __device__ __forceinline__ void operator()() const {} };

// first-round weights of a LayerNorm-fused projection: column blocks slot, slot+n, ... (clamped, so
// that the loads are unconditional; blocks past the end are never used)
template <typename HT, int S>
__device__ __forceinline__ void ln_prefetch(const Ctx &c, const HT *__restrict__ Wt, int N, int cb0, LnPre<HT, S> &w) {
    typedef typename Half16<HT>::v8 v8;
    constexpr int KS = 8 * S;
    const int nbt = (N + 15) >> 4;
#pragma unroll
    for (int cc = 0; cc < P_CB; ++cc) {
        int cb = cb0 + cc * c.n;
        cb = cb < nbt ? cb : nbt - 1;
#pragma unroll
        for (int s = 0; s < S; ++s)
            w.f[cc][s] = *reinterpret_cast<const v8 *>(Wt + (((size_t)cb * KS + c.wave * S + s) * 64 + c.lane) * 8);
    }
}

// C[:, cols of this member] = epi(LayerNorm(Hs) * Wt^T + bias) for the group's 16*MB workspace rows,
// K = W = 256 S.  Hs float32 fragment-major (read through L2), Wt fragment-major, C fragment-major
// when 16-bit, row-major [row, N] when float.  Column block cb belongs to member cb % n.
// pre: the weights of the first round; pf(): issues the next stage's weight loads (called once the
// activation loads of this stage are under way).  LOCAL: C holds the group's rows only (row 0 = the
// group's first row), e.g. a buffer in LDS.
template <typename HT, int MB, int S, int EPI, typename OutT, class PF, bool LOCAL = false>
__device__ __forceinline__ void ln_gemm_stage(const Ctx &c_in, rsrc_t hs_rs, const float *__restrict__ g,
                                              const float *__restrict__ be, const HT *__restrict__ Wt,
                                              const float *__restrict__ bias, OutT *C, int N, f32x4v *red,
                                              float *stat, LnPre<HT, S> &pre, PF pf) {
    typedef typename Half16<HT>::v8 v8;
    constexpr int W = 256 * S;
    const Ctx c = local_ctx(c_in);
    const int k0 = c.wave * 32 * S + c.kg * 8;
    f32x4 xr[MB][S][2];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const uint32_t off = (uint32_t)((((c.rb0 + i) * (8 * S) + c.wave * S + s) * 64 + c.lane) * 8) * 4u;
            xr[i][s][0] = __builtin_bit_cast(f32x4, ld16_l2(hs_rs, off));
            xr[i][s][1] = __builtin_bit_cast(f32x4, ld16_l2(hs_rs, off + 16u));
        }
    f32x4 gr[S][2], br[S][2];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        gr[s][0] = *reinterpret_cast<const f32x4 *>(g + k0 + 32 * s);
        gr[s][1] = *reinterpret_cast<const f32x4 *>(g + k0 + 32 * s + 4);
        br[s][0] = *reinterpret_cast<const f32x4 *>(be + k0 + 32 * s);
        br[s][1] = *reinterpret_cast<const f32x4 *>(be + k0 + 32 * s + 4);
    }
    // bias of the output blocks this wave will finish in the first round (q = wave, wave + 8, ...)
    const int nbt = (N + 15) >> 4;
    constexpr int NQ = (P_CB * MB + P_NW - 1) / P_NW;
    float bv0[NQ];
#pragma unroll
    for (int qi = 0; qi < NQ; ++qi) {
        const int q = c.wave + qi * P_NW;
        const int col = (c.slot + (q / MB) * c.n) * 16 + c.r;
        bv0[qi] = (q < P_CB * MB && col < N) ? bias[col] : 0.f;
    }
    pf();
    // row statistics: mean, then centred sum of squares; partial sums of the 8 waves meet in LDS
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
        if (c.kg == 0) stat[c.wave * (MB * 16) + i * 16 + c.r] = sum;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        float t = stat[i * 16 + c.r];
#pragma unroll
        for (int w = 1; w < P_NW; ++w) t += stat[w * (MB * 16) + i * 16 + c.r];
        mean[i] = t * (1.0f / (float)W);
    }
    __syncthreads();
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
        if (c.kg == 0) stat[c.wave * (MB * 16) + i * 16 + c.r] = m2;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        float t = stat[i * 16 + c.r];
#pragma unroll
        for (int w = 1; w < P_NW; ++w) t += stat[w * (MB * 16) + i * 16 + c.r];
        rstd[i] = 1.0f / sqrtf(t * (1.0f / (float)W) + 1e-5f);
    }
    SJD_TLC(c);   // statistics done (activations have arrived)
    v8 fa[MB][S];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    fa[i][s][4 * h2 + e] =
                        from_f32<HT>((xr[i][s][h2][e] - mean[i]) * rstd[i] * gr[s][h2][e] + br[s][h2][e]);

    // One round: the member's next (up to) P_CB column blocks.  The first round is straight-line code
    // (its weights and biases were requested earlier), so that the waits in front of its matrix
    // instructions cover exactly the loads they need and not the prefetches issued behind them.
    auto round = [&](int cb0, bool first) {
        f32x4v acc[P_CB][MB];
#pragma unroll
        for (int cc = 0; cc < P_CB; ++cc)
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                acc[cc][i] = f32x4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < S; ++s) acc[cc][i] = Mfma16<HT>::run(fa[i][s], pre.f[cc][s], acc[cc][i]);
                red[(c.wave * (P_CB * MB) + cc * MB + i) * 64 + c.lane] = acc[cc][i];
            }
        __syncthreads();
        SJD_TLC(c);   // partial sums in LDS
        // output block q = (cc, i) is summed in wave order and finished by wave q % 8
#pragma unroll
        for (int qi = 0; qi < NQ; ++qi) {
            const int q = c.wave + qi * P_NW;
            if (q >= P_CB * MB) break;
            const int cc = q / MB, i = q % MB;
            const int cb = cb0 + cc * c.n;
            const int col = cb * 16 + c.r;
            if (cb < nbt && col < N) {
                f32x4v t = red[q * 64 + c.lane];
#pragma unroll
                for (int w = 1; w < P_NW; ++w) t += red[(w * (P_CB * MB) + q) * 64 + c.lane];
                const float bv = first ? bv0[qi] : bias[col];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = ((LOCAL ? 0 : c.rb0) + i) * 16 + 4 * c.kg + v;   // LOCAL: C is the workgroup's own buffer
                    float val = t[v] + bv;
                    if (EPI == EPI_BIAS_GELU) val = gelu_erf_h16(val);
                    if constexpr (sizeof(OutT) == 2) C[frag_off(row, col, N >> 5)] = from_f32<OutT>(val);
                    else C[(size_t)row * N + col] = val;
                }
            }
        }
        __syncthreads();
    };
    round(c.slot, true);
    for (int cb0 = c.slot + P_CB * c.n; cb0 < nbt; cb0 += P_CB * c.n) {
        ln_prefetch<HT, S>(c, Wt, N, cb0, pre);
        round(cb0, false);
    }
}

// weights of one column block of a residual projection: the KMUL*S k-steps of this wave
template <typename HT, int S, int KMUL>
__device__ __forceinline__ void res_prefetch(const Ctx &c, const HT *__restrict__ Wt, int cb, ResPre<HT, S, KMUL> &w) {
    typedef typename Half16<HT>::v8 v8;
    constexpr int nbt = 16 * S, KSA = 8 * S * KMUL, KSW = S * KMUL;
    cb = cb < nbt ? cb : nbt - 1;
#pragma unroll
    for (int u = 0; u < KSW; ++u)
        w.f[u] = *reinterpret_cast<const v8 *>(Wt + (((size_t)cb * KSA + c.wave * KSW + u) * 64 + c.lane) * 8);
}

// Hs[:, cols of this member] += A * Wt^T + bias for the group's rows; N = W = 256 S, K = KMUL * W.
// A 16-bit fragment-major (read through L2), Hs float32 fragment-major (read through L2, written).
template <typename HT, int MB, int S, int KMUL, class PF>
__device__ __forceinline__ void gemm_resid_stage(const Ctx &c_in, rsrc_t a_rs, const HT *__restrict__ Wt,
                                                 const float *__restrict__ bias, rsrc_t hs_rs, float *hs,
                                                 f32x4v *red, ResPre<HT, S, KMUL> &pre, PF pf) {
    typedef typename Half16<HT>::v8 v8;
    constexpr int W = 256 * S, KSN = W / 32, nbt = W / 16, KSA = 8 * S * KMUL, KSW = S * KMUL;
    const Ctx c = local_ctx(c_in);
    v8 fa[MB][KSW];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int u = 0; u < KSW; ++u) {
            const uint32_t off = (uint32_t)((((c.rb0 + i) * KSA + c.wave * KSW + u) * 64 + c.lane) * 8) * 2u;
            fa[i][u] = __builtin_bit_cast(v8, ld16_l2(a_rs, off));
        }
    // every wave fetches residual values and bias of the block (only waves < MB use them: no branch
    // between the loads and the matrix instructions; rows past the workspace read as zero)
    float rv[4], bv;
    uint32_t eo[4];
    auto fetch_resid = [&](int cb) {
        const int cbc = cb < nbt ? cb : nbt - 1;
        const int col = cbc * 16 + c.r;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            eo[v] = (uint32_t)frag_off((c.rb0 + c.wave) * 16 + 4 * c.kg + v, col, KSN);
            rv[v] = ld4_l2(hs_rs, eo[v] * 4u);
        }
        bv = bias[col];
    };
    auto block = [&](int cb) {
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            f32x4v acc = f32x4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < KSW; ++u) acc = Mfma16<HT>::run(fa[i][u], pre.f[u], acc);
            red[(c.wave * MB + i) * 64 + c.lane] = acc;
        }
        SJD_TLC(c);   // operands have arrived, products done
        __syncthreads();
        SJD_TLC(c);
        if (c.wave < MB && cb < nbt) {
            f32x4v t = red[c.wave * 64 + c.lane];
#pragma unroll
            for (int w = 1; w < P_NW; ++w) t += red[(w * MB + c.wave) * 64 + c.lane];
#pragma unroll
            for (int v = 0; v < 4; ++v) hs[eo[v]] = (t[v] + bv) + rv[v];
        }
        __syncthreads();
    };
    fetch_resid(c.slot);
    pf();
    block(c.slot);                                          // straight-line first block (see ln_gemm_stage)
    for (int cb = c.slot + c.n; cb < nbt; cb += c.n) {
        res_prefetch<HT, S, KMUL>(c, Wt, cb, pre);
        fetch_resid(cb);
        block(cb);
    }
}

// Single-token attention of the group's (sample, head) pairs against the cache at position t:
// pair (row, h) belongs to member (row * H + h) % n.  A pair is handled by four waves (32 key
// groups x 8 sixteen-byte chunks of the head), two pairs at a time per workgroup; the partition
// of the keys and the order of the partial sums are the same for every batch size.  This step's k
// and v are appended to the cache.  Cached rows do not depend on the current step, so the first
// P_AU rows of every thread (keys and values) are requested before the barrier that precedes
// the stage (att_prefetch) and only q and the fresh row are waited for afterwards.
constexpr int P_NSUB = 2;
constexpr int P_AU = 8;  // cache rows per thread and batch
template <typename HT> struct AttPre { typename Half16<HT>::v8 k[P_AU], v[P_AU]; };

template <typename HT, int S>
__device__ __forceinline__ void att_fetch(const Ctx &c, rsrc_t kc_rs, rsrc_t vc_rs, int k0, int j0, int t, int T,
                                          AttPre<HT> &w) {
    typedef typename Half16<HT>::v8 v8;
    constexpr int W = 256 * S, H = W / 64;
    const int sub = c.tid >> 8, stid = c.tid & 255, dc = stid & 7, sg = stid >> 3;
    const int npairs = c.nrows * H;
    int pi = c.slot + (k0 + sub) * c.n;
    pi = pi < npairs ? pi : 0;
    const int row = pi / H, h = pi - row * H;
    const size_t cbase = ((size_t)(c.row0 + row) * T) * W + h * 64;
#pragma unroll
    for (int u = 0; u < P_AU; ++u) {
        const int s = sg + 32 * (j0 + u);
        const int sr = s < t ? s : 0;                      // rows at or past t: any cached row, value not used
        const uint32_t off = (uint32_t)(cbase + (size_t)sr * W + dc * 8) * 2u;
        w.k[u] = __builtin_bit_cast(v8, ld16_l2_stream(kc_rs, off));
        w.v[u] = __builtin_bit_cast(v8, ld16_l2_stream(vc_rs, off));
    }
}

template <typename HT, int S>
__device__ __forceinline__ void attention_stage(const Ctx &c_in, rsrc_t qkv_rs, HT *kc, HT *vc, rsrc_t kc_rs, rsrc_t vc_rs,
                                                HT *o, int t, int T, float *sc_all, float *opart, float *wred) {
    typedef typename Half16<HT>::v8 v8;
    constexpr int W = 256 * S, H = W / 64, KS3 = 3 * W / 32;
    const Ctx c = local_ctx(c_in);
    const int sub = c.tid >> 8, stid = c.tid & 255;
    const int dc = stid & 7, sg = stid >> 3;               // chunk of the head, key group (0..31)
    float *sc = sc_all + (size_t)sub * T;
    const int npairs = c.nrows * H;
    const int mine = npairs > c.slot ? (npairs - c.slot + c.n - 1) / c.n : 0;   // pairs of this member
    const int nk = t + 1;
    const int nbatch = (nk + 32 * P_AU - 1) / (32 * P_AU);  // batches of P_AU rows per thread
    for (int k0 = 0; k0 < mine; k0 += P_NSUB) {
        const int pi = c.slot + (k0 + sub) * c.n;
        const bool valid = (k0 + sub) < mine;
        const int row = valid ? pi / H : 0, h = valid ? pi - row * H : 0;
        const int b = c.row0 + row, wsrow = c.rb0 * 16 + row;
        auto chunk = [&](int part, int ci) -> v8 {
            return __builtin_bit_cast(v8, ld16_l2(qkv_rs, (uint32_t)frag_off(wsrow, part * W + h * 64 + ci * 8, KS3) * 2u));
        };
        const v8 kfresh = chunk(1, dc), vfresh = chunk(2, dc), q8 = chunk(0, dc);
        const size_t cbase = ((size_t)b * T) * W + h * 64;
        if (valid && stid < 16) {   // threads 0..7 hold the fresh k chunks, 8..15 the fresh v chunks (dc = stid & 7)
            HT *dst = (stid < 8 ? kc : vc) + cbase + (size_t)t * W + dc * 8;
            *reinterpret_cast<v8 *>(dst) = stid < 8 ? kfresh : vfresh;
        }
        float qf[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[e] = (float)q8[e] * 0.125f;  // 1/sqrt(64)
        AttPre<HT> pre;
        att_fetch<HT, S>(c, kc_rs, vc_rs, k0, 0, t, T, pre);   // first batch of cached keys and values, in one go
        // scores of batch 0 (values stay in registers), further batches fetch keys only
        float mx = -INFINITY;
        float d0[P_AU];
#pragma unroll
        for (int u = 0; u < P_AU; ++u) {
            const int s = sg + 32 * u;
            const v8 k8 = s < t ? pre.k[u] : kfresh;
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) d = fmaf(qf[e], (float)k8[e], d);
            d += __shfl_xor(d, 1, 64);
            d += __shfl_xor(d, 2, 64);
            d += __shfl_xor(d, 4, 64);
            d0[u] = d;
            if (s < nk) mx = fmaxf(mx, d);
        }
        for (int jb = 1; jb < nbatch; ++jb) {
            v8 kk[P_AU];
#pragma unroll
            for (int u = 0; u < P_AU; ++u) {
                const int s = sg + 32 * (jb * P_AU + u);
                const int sr = s < t ? s : 0;
                kk[u] = __builtin_bit_cast(v8, ld16_l2_stream(kc_rs, (uint32_t)(cbase + (size_t)sr * W + dc * 8) * 2u));
            }
#pragma unroll
            for (int u = 0; u < P_AU; ++u) {
                const int s = sg + 32 * (jb * P_AU + u);
                const v8 k8 = s < t ? kk[u] : kfresh;
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) d = fmaf(qf[e], (float)k8[e], d);
                d += __shfl_xor(d, 1, 64);
                d += __shfl_xor(d, 2, 64);
                d += __shfl_xor(d, 4, 64);
                if (s < nk) {
                    if (dc == 0) sc[s] = d;
                    mx = fmaxf(mx, d);
                }
            }
        }
        mx = wave_max(mx);
        SJD_TLC(c);   // scores done (q, fresh row and cached keys have arrived)
        if (c.lane == 0) wred[c.wave] = mx;
        __syncthreads();
        SJD_TLC(c);
        mx = fmaxf(fmaxf(wred[4 * sub], wred[4 * sub + 1]), fmaxf(wred[4 * sub + 2], wred[4 * sub + 3]));
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        float psum = 0.f;
#pragma unroll
        for (int u = 0; u < P_AU; ++u) {
            const int s = sg + 32 * u;
            if (s < nk) {
                const float p = expf(d0[u] - mx);
                const v8 v8v = s < t ? pre.v[u] : vfresh;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] = fmaf(p, (float)v8v[e], acc[e]);
                psum += p;
            }
        }
        for (int jb = 1; jb < nbatch; ++jb) {
            v8 vv[P_AU];
#pragma unroll
            for (int u = 0; u < P_AU; ++u) {
                const int s = sg + 32 * (jb * P_AU + u);
                const int sr = s < t ? s : 0;
                vv[u] = __builtin_bit_cast(v8, ld16_l2_stream(vc_rs, (uint32_t)(cbase + (size_t)sr * W + dc * 8) * 2u));
            }
#pragma unroll
            for (int u = 0; u < P_AU; ++u) {
                const int s = sg + 32 * (jb * P_AU + u);
                if (s < nk) {
                    const float p = expf(sc[s] - mx);
                    const v8 v8v = s < t ? vv[u] : vfresh;
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[e] = fmaf(p, (float)v8v[e], acc[e]);
                    psum += p;
                }
            }
        }
        // the 8 key groups of a wave (lanes differing in bits 3..5), then the pair's four waves in order
#pragma unroll
        for (int off = 8; off < 64; off <<= 1) {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], off, 64);
            psum += __shfl_xor(psum, off, 64);
        }
        SJD_TLC(c);   // weighted values summed within the wave
        if (c.lane < 8) {
#pragma unroll
            for (int e = 0; e < 8; ++e) opart[c.wave * 64 + c.lane * 8 + e] = acc[e];
            if (c.lane == 0) wred[P_NW + c.wave] = psum;
        }
        __syncthreads();
        if (valid && stid < 8) {
            const int w0 = 4 * sub;
            const float den = ((wred[P_NW + w0] + wred[P_NW + w0 + 1]) + wred[P_NW + w0 + 2]) + wred[P_NW + w0 + 3];
            v8 ov;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int d = stid * 8 + e;
                ov[e] = from_f32<HT>((((opart[w0 * 64 + d] + opart[(w0 + 1) * 64 + d]) + opart[(w0 + 2) * 64 + d]) +
                                      opart[(w0 + 3) * 64 + d]) / den);
            }
            *reinterpret_cast<v8 *>(o + frag_off(wsrow, h * 64 + stid * 8, W / 32)) = ov;
        }
        __syncthreads();  // sc, opart and wred are reused by the next round
    }
}

template <typename HT, int MB, int S>
__global__ __launch_bounds__(P_THREADS) void seq_persistent_kernel(SeqArgs a) {
    constexpr int W = 256 * S, RW_ROWS = 16 * MB;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    __shared__ int sh[8];
    f32x4v *red = reinterpret_cast<f32x4v *>(lds_raw);                       // [8][P_CB*MB][64]
    float *stat = reinterpret_cast<float *>(lds_raw + (size_t)P_NW * P_CB * MB * 64 * 16);  // [8][MB*16]
    float *xs = stat + P_NW * MB * 16;                                        // [16*MB][D]
    float *opart = xs + RW_ROWS * a.D;                                        // [8][64]
    float *wred = opart + P_NW * 64;                                          // [16]
    float *sc = wred + 16;                                                    // [2][T]
    float *wemb = sc + 2 * a.T;                                               // [P_EB][D + 1][16]: w_in slice, then b_in
    float *pl = wemb + (size_t)P_EB * (a.D + 1) * 16;                         // [16*MB][2D]: this step's [mu | alpha] of the group's rows

    Ctx c;
    c.tid = threadIdx.x; c.lane = c.tid & 63; c.wave = c.tid >> 6; c.r = c.lane & 15; c.kg = c.lane >> 4;
    c.epoch = 0; c.status = a.sync + 9; c.spin_max = a.spin_max;

    // ---- groups: the workgroups of one XCD, found from the hardware's XCC id
    if (c.tid == 0) {
        const int xcc = __builtin_amdgcn_s_getreg(20 | (3 << 11)) & 7;  // HW_REG_XCC_ID, bits 3:0
        const int slot = atomicAdd(&a.sync[xcc], 1);
        // the arrival is a release and the poll an acquire (device scope, once per launch): a member that sees
        // every arrival also sees every member count, so all members of a group compute the same group size
        __hip_atomic_fetch_add(&a.sync[8], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        int it = 0, ok = 1;
        while (__hip_atomic_load(&a.sync[8], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < (int)gridDim.x) {
            if (++it > a.spin_max) { ok = 0; break; }
            __builtin_amdgcn_s_sleep(2);
        }
        int n = 0, groups = 0, gidx = 0;
        for (int g = 0; g < 8; ++g) {
            const int m = __hip_atomic_load(&a.sync[g], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
            if (m > 0) { if (g < xcc) ++gidx; ++groups; }
            if (g == xcc) n = m;
        }
        if (!ok) __hip_atomic_store(c.status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sh[0] = ok; sh[1] = slot; sh[2] = n; sh[3] = groups; sh[4] = gidx; sh[5] = xcc;
    }
    __syncthreads();
    if (!sh[0]) return;
    c.slot = sh[1]; c.n = sh[2];
    const int groups = sh[3], gidx = sh[4];
    c.cnt = a.sync + 64 * (sh[5] + 1);
    const int per = (a.B + groups - 1) / groups;  // samples per group
    if (per > RW_ROWS) {                           // fewer groups than the host planned for
        if (c.tid == 0) __hip_atomic_store(c.status, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    c.row0 = gidx * per;
    c.nrows = a.B - c.row0 < per ? a.B - c.row0 : per;
    c.rb0 = gidx * MB;
    if (c.nrows <= 0) return;                      // groups are independent: an idle one just leaves

    const int T = a.T, D = a.D;
    HT *qkv = reinterpret_cast<HT *>(a.qkv), *o = reinterpret_cast<HT *>(a.o), *ff = reinterpret_cast<HT *>(a.ff);
    const uint32_t ws_rows = 8u * RW_ROWS;
    const rsrc_t qkv_rs = make_rsrc(qkv, ws_rows * 3u * W * 2u);
    const rsrc_t o_rs = make_rsrc(o, ws_rows * W * 2u);
    const rsrc_t ff_rs = make_rsrc(ff, ws_rows * (uint32_t)a.ratio * W * 2u);
    volatile int *sh_ok = &sh[6];
    // this member's slices of the embedding matrix and bias stay in LDS for the whole block
    for (int bi = 0, cb = c.slot; bi < P_EB && cb < W / 16; ++bi, cb += c.n)
        for (int e = c.tid; e < (D + 1) * 16; e += P_THREADS) {
            const int d = e >> 4, cl = e & 15;
            wemb[(size_t)bi * (D + 1) * 16 + e] = d < D ? a.w_in[(size_t)d * W + cb * 16 + cl] : a.b_in[cb * 16 + cl];
        }
    // latent values of position 0 (each thread keeps the ones it will turn into x)
    constexpr int ZPT = (RW_ROWS * 64 + P_THREADS - 1) / P_THREADS;   // token sizes up to 64
    float zreg[ZPT];
#pragma unroll
    for (int q = 0; q < ZPT; ++q) {
        const int e = c.tid + q * P_THREADS;
        zreg[q] = 0.f;
        if (e < RW_ROWS * D) {
            const int row = e / D, d = e - row * D;
            if (row < c.nrows) zreg[q] = a.z[((size_t)(c.row0 + row) * T + (a.reversed ? T - 1 : 0)) * D + d];
        }
    }
    __syncthreads();
    Ctx ch = c;      // the head projection: every member takes every column block
    ch.slot = 0; ch.n = 1;

    for (int l = 0; l < T; ++l) {
#ifdef SJD_SEQ_TIMELINE
        Ctx &cm = const_cast<Ctx &>(c);
        cm.tl_on = gidx == 0 && c.slot == 0 && l == T / 2;
        cm.tl = a.sync + 640; cm.tl_t0 = wall_clock64(); cm.tl_k = &sh[7]; if (c.tid == 0) sh[7] = 0;
#endif
        // ---- x_l of the group's samples (eq. 5; x_0 = z_0), kept in LDS for the embedding; the latent
        // values were requested one step ahead
        const int tok = a.reversed ? T - 1 - l : l;
        const int tok_next = a.reversed ? T - 2 - l : l + 1;
        // The residual stream lives in two copies that alternate with the step: the embedding of step l+1
        // is written while slower members may still read the stream of step l for their head projection.
        float *hs = a.hs + (size_t)(l & 1) * ws_rows * W;
        const rsrc_t hs_rs = make_rsrc(hs, ws_rows * W * 4u);
#pragma unroll
        for (int q = 0; q < ZPT; ++q) {
            const int e = c.tid + q * P_THREADS;
            if (e < RW_ROWS * D) {
                const int row = e / D, d = e - row * D;
                float xn = 0.f;
                if (row < c.nrows) {
                    const size_t idx = ((size_t)(c.row0 + row) * T + tok) * D + d;
                    xn = zreg[q];
                    if (l > 0) xn = fmaf(xn, expf(pl[row * 2 * D + D + d]), pl[row * 2 * D + d]);
                    if (c.slot == 0) a.x[idx] = xn;
                    if (l + 1 < T) zreg[q] = a.z[((size_t)(c.row0 + row) * T + tok_next) * D + d];
                }
                xs[e] = xn;
            }
        }
        if (l == T - 1) break;
        __syncthreads();
        // ---- embedding of this member's column blocks: hs = x_l * w_in + b_in + pos[l]
        {
            int bi = 0;
            for (int cb = c.slot; cb < W / 16; cb += c.n, ++bi) {
                for (int e = c.tid; e < RW_ROWS * 16; e += P_THREADS) {
                    const int row = e >> 4, cl = e & 15, col = cb * 16 + cl;
                    float acc = a.pos[(size_t)l * W + col];
                    if (bi < P_EB) {
                        const float *we = wemb + (size_t)bi * (D + 1) * 16;
                        acc += we[D * 16 + cl];
                        for (int d = 0; d < D; ++d) acc = fmaf(xs[row * D + d], we[d * 16 + cl], acc);
                    } else {
                        acc += a.b_in[col];
                        for (int d = 0; d < D; ++d) acc = fmaf(xs[row * D + d], a.w_in[(size_t)d * W + col], acc);
                    }
                    hs[frag_off(c.rb0 * 16 + row, col, W / 32)] = acc;
                }
            }
        }
        // Weights of a stage are requested one stage ahead where the registers allow it (W <= 512),
        // else at the start of the stage itself.
        constexpr bool AHEAD = S <= 2;
        LnPre<HT, S> wln;
        ResPre<HT, S, 1> wo;
        ResPre<HT, S, 4> wf2;
        if (AHEAD) ln_prefetch<HT, S>(c, (const HT *)a.layers[0].f_qkv, 3 * W, c.slot, wln);
        SJD_TLC(c);
        if (!group_barrier(c, sh_ok)) return;
        SJD_TLC(c);

        for (int ly = 0; ly < a.n_layers; ++ly) {
            const SeqLayer &lw = a.layers[ly];
            HT *kc = reinterpret_cast<HT *>(a.kcache) + (size_t)ly * a.kv_layer_stride;
            HT *vc = reinterpret_cast<HT *>(a.vcache) + (size_t)ly * a.kv_layer_stride;
            const rsrc_t kc_rs = make_rsrc(kc, (uint32_t)(a.kv_layer_stride * 2u));
            const rsrc_t vc_rs = make_rsrc(vc, (uint32_t)(a.kv_layer_stride * 2u));
            if (!AHEAD) ln_prefetch<HT, S>(c, (const HT *)lw.f_qkv, 3 * W, c.slot, wln);
            ln_gemm_stage<HT, MB, S, EPI_BIAS, HT>(c, hs_rs, lw.ln1_g, lw.ln1_b, (const HT *)lw.f_qkv, lw.b_qkv, qkv,
                                                  3 * W, red, stat, wln, NoPrefetch());
            SJD_TLC(c);
            if (!group_barrier(c, sh_ok)) return;
            SJD_TLC(c);
            if (AHEAD) res_prefetch<HT, S, 1>(c, (const HT *)lw.f_o, c.slot, wo);
            attention_stage<HT, S>(c, qkv_rs, kc, vc, kc_rs, vc_rs, o, l, T, sc, opart, wred);
            SJD_TLC(c);
            if (!group_barrier(c, sh_ok)) return;
            SJD_TLC(c);
            if (!AHEAD) res_prefetch<HT, S, 1>(c, (const HT *)lw.f_o, c.slot, wo);
            gemm_resid_stage<HT, MB, S, 1>(c, o_rs, (const HT *)lw.f_o, lw.b_o, hs_rs, hs, red, wo, [&]() {
                if (AHEAD) ln_prefetch<HT, S>(c, (const HT *)lw.f_fc1, 4 * W, c.slot, wln);
            });
            SJD_TLC(c);
            if (!group_barrier(c, sh_ok)) return;
            SJD_TLC(c);
            if (!AHEAD) ln_prefetch<HT, S>(c, (const HT *)lw.f_fc1, 4 * W, c.slot, wln);
            ln_gemm_stage<HT, MB, S, EPI_BIAS_GELU, HT>(c, hs_rs, lw.ln2_g, lw.ln2_b, (const HT *)lw.f_fc1, lw.b_fc1, ff,
                                                       4 * W, red, stat, wln, [&]() {
                if (AHEAD) res_prefetch<HT, S, 4>(c, (const HT *)lw.f_fc2, c.slot, wf2);
            });
            SJD_TLC(c);
            if (!group_barrier(c, sh_ok)) return;
            SJD_TLC(c);
            const bool last = ly + 1 == a.n_layers;
            const HT *next_w = (const HT *)(last ? a.f_head : a.layers[last ? ly : ly + 1].f_qkv);
            const int next_n = last ? 2 * D : 3 * W;
            if (!AHEAD) res_prefetch<HT, S, 4>(c, (const HT *)lw.f_fc2, c.slot, wf2);
            gemm_resid_stage<HT, MB, S, 4>(c, ff_rs, (const HT *)lw.f_fc2, lw.b_fc2, hs_rs, hs, red, wf2, [&]() {
                if (AHEAD) { if (last) ln_prefetch<HT, S>(ch, next_w, next_n, 0, wln); else ln_prefetch<HT, S>(c, next_w, next_n, c.slot, wln); }
            });
            SJD_TLC(c);
            if (!group_barrier(c, sh_ok)) return;
            SJD_TLC(c);
        }
        // ---- head: every member computes all of [mu | alpha] for the group's rows (a few column blocks)
        // into its own LDS, so that x_l and the next embedding follow without another group barrier
        if (!AHEAD) ln_prefetch<HT, S>(ch, (const HT *)a.f_head, 2 * D, 0, wln);
        ln_gemm_stage<HT, MB, S, EPI_BIAS, float, NoPrefetch, true>(ch, hs_rs, a.lnf_g, a.lnf_b, (const HT *)a.f_head, a.b_head,
                                                                   pl, 2 * D, red, stat, wln, NoPrefetch());
        SJD_TLC(c);
        SJD_TLC(c);
    }
}

}  // namespace

size_t seq_persistent_lds_bytes(int MB, int T, int D) {
    size_t need = (size_t)P_NW * P_CB * MB * 64 * 16 + (size_t)P_NW * MB * 16 * 4 + (size_t)16 * MB * D * 4 +
                  (size_t)P_NW * 64 * 4 + 16 * 4 + (size_t)2 * T * 4 + (size_t)P_EB * (D + 1) * 16 * 4 + (size_t)16 * MB * 2 * D * 4;
    const size_t one_per_cu = 84 * 1024;  // more than half of a CU's LDS: exactly one workgroup per CU
    if (need < one_per_cu) need = one_per_cu;
    return (need + 255) & ~(size_t)255;
}

template <typename HT>
static const void *pick_kernel(int MB, int S) {
#define SJD_PK(MBv, Sv) if (MB == MBv && S == Sv) return reinterpret_cast<const void *>(&seq_persistent_kernel<HT, MBv, Sv>);
    SJD_PK(1, 1) SJD_PK(1, 2) SJD_PK(1, 3) SJD_PK(1, 4) SJD_PK(2, 1) SJD_PK(2, 2) SJD_PK(2, 3) SJD_PK(2, 4)
#undef SJD_PK
    return nullptr;
}

hipError_t launch_seq_persistent(bool is_bf16, const SeqArgs &args, int MB, int S, int grid, bool cooperative,
                                 hipStream_t s) {
    const void *kern = is_bf16 ? pick_kernel<bf16>(MB, S) : pick_kernel<f16>(MB, S);
    if (!kern) return hipErrorInvalidValue;
    const size_t lds = seq_persistent_lds_bytes(MB, args.T, args.D);
    hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    SeqArgs a = args;
    void *params[] = {&a};
    if (cooperative) return hipLaunchCooperativeKernel(kern, dim3(grid), dim3(P_THREADS), params, (unsigned)lds, s);
    // plain launch: co-residency of the workgroups is then not guaranteed by the runtime; it holds when
    // the device is otherwise idle (one workgroup per CU), and every wait in the kernel is bounded
    return hipLaunchKernel(kern, dim3(grid), dim3(P_THREADS), params, lds, s);
}

}  // namespace sjd
