// Causal multi-head attention.
//
//  * attention_rows_kernel: one wave per (sample, head, query row), any head size and sequence
//    length, float32, bf16 or f16 storage, float32 arithmetic.  It serves the float32 configuration's
//    whole-sequence passes and, with a key/value cache, every single-token step of the sequential
//    inverse (Sec. 3.5), where it is bound by reading the cached prefix from HBM.
//  * flash_attention_h16_kernel: whole-sequence causal attention for head size 64 on 16-bit data with
//    MFMA; K and V tiles are staged in LDS, scores never leave registers (online softmax in float32), so
//    there is no T x T buffer.
//  * flash_attention_f32_kernel: the same in float32 on the float32 matrix instruction (float32 flows and
//    the refined passes of 16-bit flows).
#include "common.h"

namespace sjd {

// ------------------------------------------------------------------------------------------------
// Row-wise kernel.  Keys 0..n_cached-1 come from the cache; if `fresh` is set the query's own
// position (key n_cached) comes from the row just computed, and that row's k, v are also written
// into the cache at position n_cached.  mask_o > 0: the masked-dependency probe of eq. 6, the query
// at position p sees keys 0..p-mask_o only; a row that sees no key gets a zero output.
template <typename QT, typename KVT>
__global__ __launch_bounds__(256) void attention_rows_kernel(const QT *__restrict__ q, int64_t q_stride,
                                                             const KVT *k, const KVT *v, int64_t kv_stride,
                                                             int64_t kv_sample_stride, const QT *__restrict__ kfresh,
                                                             const QT *__restrict__ vfresh, KVT *kstore, KVT *vstore,
                                                             QT *__restrict__ o, int64_t o_stride, int n_work,
                                                             int q_rows_per_sample, int t0, int H, int dh,
                                                             int max_keys, int mask_o) {
    extern __shared__ float smem[];
    const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int w = blockIdx.x * 4 + wv;
    if (w >= n_work) return;
    float *qs = smem + (size_t)wv * (dh + max_keys);
    float *sc = qs + dh;
    const int r = w % q_rows_per_sample;
    const int h = (w / q_rows_per_sample) % H;
    const int i = w / (q_rows_per_sample * H);
    const int64_t qrow = (int64_t)i * q_rows_per_sample + r;
    const int own = t0 + r;                                   // the query's position
    const int n_keys = own + 1 - mask_o > 0 ? own + 1 - mask_o : 0;
    const int fresh_at = kfresh ? own : own + 1;              // cache rows below this index are valid
    const int n_cached = n_keys < fresh_at ? n_keys : fresh_at;
    const QT *qp = q + qrow * q_stride + h * dh;
    for (int d = lane; d < dh; d += 64) qs[d] = to_f32<QT>(qp[d]);
    const KVT *kb = k + (int64_t)i * kv_sample_stride + h * dh;
    const KVT *vb = v + (int64_t)i * kv_sample_stride + h * dh;
    const QT *kf = kfresh ? kfresh + qrow * q_stride + h * dh : nullptr;
    const QT *vf = vfresh ? vfresh + qrow * q_stride + h * dh : nullptr;
    if (kf) {
        KVT *ks = kstore + (int64_t)i * kv_sample_stride + (int64_t)own * kv_stride + h * dh;
        KVT *vs = vstore + (int64_t)i * kv_sample_stride + (int64_t)own * kv_stride + h * dh;
        for (int d = lane; d < dh; d += 64) {
            ks[d] = from_f32<KVT>(to_f32<QT>(kf[d]));
            vs[d] = from_f32<KVT>(to_f32<QT>(vf[d]));
        }
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's LDS writes of q are visible to its lanes
    const float scale = 1.0f / sqrtf((float)dh);
    float mx = -INFINITY;
    for (int s = lane; s < n_keys; s += 64) {
        float dot = 0.f;
        if (s < n_cached) {
            const KVT *kr = kb + (int64_t)s * kv_stride;
            for (int d = 0; d < dh; ++d) dot = fmaf(qs[d], to_f32<KVT>(kr[d]), dot);
        } else {
            for (int d = 0; d < dh; ++d) dot = fmaf(qs[d], to_f32<QT>(kf[d]), dot);
        }
        dot *= scale;
        sc[s] = dot;
        mx = fmaxf(mx, dot);
    }
    mx = wave_max(mx);
    float den = 0.f;
    for (int s = lane; s < n_keys; s += 64) {
        const float e = expf(sc[s] - mx);
        sc[s] = e;
        den += e;
    }
    den = wave_sum(den);
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);
    const float inv = n_keys > 0 ? 1.0f / den : 0.f;
    for (int d = lane; d < dh; d += 64) {
        float acc = 0.f;
        for (int s = 0; s < n_cached; ++s) acc = fmaf(sc[s], to_f32<KVT>(vb[(int64_t)s * kv_stride + d]), acc);
        if (n_cached < n_keys) acc = fmaf(sc[n_cached], to_f32<QT>(vf[d]), acc);
        o[qrow * o_stride + h * dh + d] = from_f32<QT>(acc * inv);
    }
}

template <typename QT, typename KVT>
void launch_attention_rows(const QT *q, int64_t q_stride, const KVT *k, const KVT *v, int64_t kv_stride,
                           int64_t kv_sample_stride, QT *o, int64_t o_stride, int n_samples, int q_rows_per_sample,
                           int t0, int H, int dh, int mask_o, hipStream_t s) {
    const int n_work = n_samples * H * q_rows_per_sample;
    if (n_work <= 0) return;
    const int max_keys = t0 + q_rows_per_sample;
    const size_t smem = 4 * (size_t)(dh + max_keys) * sizeof(float);
    hipLaunchKernelGGL((attention_rows_kernel<QT, KVT>), dim3((n_work + 3) / 4), dim3(256), smem, s, q, q_stride, k, v,
                       kv_stride, kv_sample_stride, (const QT *)nullptr, (const QT *)nullptr, (KVT *)nullptr,
                       (KVT *)nullptr, o, o_stride, n_work, q_rows_per_sample, t0, H, dh, max_keys, mask_o);
}
template void launch_attention_rows<float, float>(const float *, int64_t, const float *, const float *, int64_t,
                                                  int64_t, float *, int64_t, int, int, int, int, int, int, hipStream_t);
template void launch_attention_rows<bf16, bf16>(const bf16 *, int64_t, const bf16 *, const bf16 *, int64_t, int64_t,
                                                bf16 *, int64_t, int, int, int, int, int, int, hipStream_t);
template void launch_attention_rows<f16, f16>(const f16 *, int64_t, const f16 *, const f16 *, int64_t, int64_t, f16 *,
                                              int64_t, int, int, int, int, int, int, hipStream_t);

template <typename AT>
void launch_decode_attention(const AT *qkv, AT *kcache, AT *vcache, AT *o, int B, int T, int t, int H, int dh,
                             int mask_o, hipStream_t s) {
    const int n_work = B * H;
    if (n_work <= 0) return;
    const int W = H * dh;
    const int max_keys = t + 1;
    const size_t smem = 4 * (size_t)(dh + max_keys) * sizeof(float);
    hipLaunchKernelGGL((attention_rows_kernel<AT, AT>), dim3((n_work + 3) / 4), dim3(256), smem, s, qkv,
                       (int64_t)3 * W, (const AT *)kcache, (const AT *)vcache, (int64_t)W, (int64_t)T * W,
                       qkv + W, qkv + 2 * W, kcache, vcache, o, (int64_t)W, n_work, 1, t, H, dh, max_keys, mask_o);
}
template void launch_decode_attention<float>(const float *, float *, float *, float *, int, int, int, int, int, int,
                                             hipStream_t);
template void launch_decode_attention<bf16>(const bf16 *, bf16 *, bf16 *, bf16 *, int, int, int, int, int, int,
                                            hipStream_t);
template void launch_decode_attention<f16>(const f16 *, f16 *, f16 *, f16 *, int, int, int, int, int, int, hipStream_t);

// ------------------------------------------------------------------------------------------------
// Flash-style kernel, head size 64.  A workgroup (4 waves) owns 128 query rows of one
// (sample, head); a wave owns 32 of them.  The score block is computed transposed,
// S^T = K Q^T, so that a lane holds one query column: row statistics of the online softmax are
// lane-local plus one cross-half exchange, and the probabilities are already laid out as the
// B operand of the second product O^T = V^T P^T (16 keys per instruction).
// K/V tiles of 64 keys are double-buffered in LDS (one barrier per tile; the next tile's rows are on their
// way into registers while the current one is used) and consumed in two steps of 32 keys, each a complete
// step of the online softmax; the accumulator is rescaled only when some row's running maximum moved.
// 121 registers: four workgroups per CU.
//
// The two 32-lane halves of a wave exchange a value in one instruction (v_permlane32_swap with both operands
// the same register): every lane gets the value of its position in the lower half and in the upper half.
__device__ __forceinline__ void wave_halves(float x, float &lower, float &upper) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    lower = __uint_as_float(r[0]);
    upper = __uint_as_float(r[1]);
}
constexpr int FA_BQ = 128, FA_BK = 64, FA_DH = 64;
// LDS tiles are swizzled instead of padded.  K [key][d]: the 16-byte chunk c of row `key` sits in slot
// c ^ (bits 1, 2 and 4 of key): a 16-byte read of a wave is served in four passes of 16 lanes (lanes
// that agree in bits 3 and 5) over 64 banks, and the 16 rows of a pass - {0-7, 16-23} or {8-15, 24-31}
// of a 32-key block - then fall on 16 different 16-byte bank groups (8 (key & 1) + slot).
constexpr int FA_KS = FA_DH;       // K tile row stride (elements)
__device__ __forceinline__ int fa_kswz(int key) { return ((key >> 1) & 3) | (((key >> 4) & 1) << 2); }
// V stays row-major in LDS (16-byte stores, no transposition on the way in) and the V^T fragments of the second
// product come out of the transposing 64-bit LDS read of gfx950, which works on groups of 16 lanes: output lane
// j of a group receives element (j % 4) of source lanes (j / 4) + 4 t, t = 0..3.  With source lane s pointing at
// row (s / 4), columns 4 (s % 4) .. + 3 of a 4 x 16 block of V (4 keys, 16 values of d), output lane j holds the
// four keys of column j: the k-contiguous piece of the A operand of O^T += V^T P^T for d = that column.
// V [key][d]: the 16-byte chunk c of row `key` sits in slot c ^ (4 (key / 2 % 2)): the four rows that a 16-lane
// group reads (128 bytes apart: rows of equal parity start on the same bank) then use disjoint bank groups
// (the LDS bank-conflict counter reads zero on this kernel).
typedef short i16x4 __attribute__((ext_vector_type(4)));

template <typename HT>
__global__ __launch_bounds__(256, 4) void flash_attention_h16_kernel(const HT *__restrict__ qkv, HT *__restrict__ o,
                                                                     int T, int H, int n_pairs, float scale_log2) {
    typedef typename Half16<HT>::v8 v8;
    typedef typename Half16<HT>::v4 v4;
    __shared__ __attribute__((aligned(16))) HT Ks[2][FA_BK * FA_KS];
    __shared__ __attribute__((aligned(16))) HT Vs[2][FA_BK * FA_DH];
    const int W = H * FA_DH;
    const int n_qt = (T + FA_BQ - 1) / FA_BQ;
    // Workgroups go to the eight XCDs round robin by their linear index, and each XCD has an L2 of its own:
    // the query tiles of one (sample, head) take consecutive slots of ONE XCD, so its keys and values come
    // from memory once and the other tiles find them in that L2.
    const int slot = (int)blockIdx.x >> 3;
    const int pair = (slot / n_qt) * 8 + ((int)blockIdx.x & 7);
    if (pair >= n_pairs) return;                // the grid is padded to a multiple of eight pairs
    const int qt = n_qt - 1 - slot % n_qt;      // heavy tiles first
    const int h = pair % H, i = pair / H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const HT *base = qkv + (size_t)i * T * 3 * W;
    const int q0 = qt * FA_BQ + wave * 32;
    const int qrow = q0 + l32;
    const int qrow_c = qrow < T ? qrow : T - 1;

    v8 qf[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
        qf[c] = *reinterpret_cast<const v8 *>(base + (size_t)qrow_c * 3 * W + h * FA_DH + 16 * c + 8 * g);

    f32x16 oacc[2];
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    // Q has to have arrived before the loop: otherwise the compiler, which cannot tell a first iteration from a
    // later one, waits for Q inside the loop by waiting for every younger load - the K/V loads of the next tile
    // that were issued a moment before - and the prefetch is lost.
    asm volatile("" :: "v"(qf[0]), "v"(qf[1]), "v"(qf[2]), "v"(qf[3]));

    // this lane's part of a transposing read: source row (4 g + j16 / 4) of the 8-key group, the 8-byte piece
    // (j16 % 4) of the 32 bytes that hold d = 32 db + 16 hh .. + 15, chunk slot swizzled by the row
    const int j16 = lane & 15, hh = (lane >> 4) & 1;
    int voff[2];                                 // element offsets inside a V tile, for db = 0, 1
#pragma unroll
    for (int db = 0; db < 2; ++db) {
        const int chunk = 4 * db + 2 * hh + ((j16 & 3) >> 1);
        const int slot_v = chunk ^ (((j16 >> 3) & 1) << 2);
        voff[db] = (4 * g + (j16 >> 2)) * FA_DH + slot_v * 8 + (j16 & 1) * 4;
    }

    const int last_row = min(qt * FA_BQ + FA_BQ - 1, T - 1);
    const int n_kt = last_row / FA_BK + 1;
    v8 kreg[2], vreg[2];
    // a thread's two 16-byte pieces of a tile: a wave-uniform tile base plus an offset that does not change from
    // tile to tile; only a last tile that reaches past the sequence clamps its rows (wave-uniform branch)
    uint32_t koff[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int c = tid + r * 256;
        koff[r] = (uint32_t)(((c >> 3) * 3 * W + h * FA_DH + (c & 7) * 8 + W) * (int)sizeof(HT));
    }
    auto fetch_tile = [&](int kt_) {
        if ((kt_ + 1) * FA_BK <= T) {
            const char *tb = reinterpret_cast<const char *>(base + (size_t)kt_ * FA_BK * 3 * W);
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                kreg[r] = *reinterpret_cast<const v8 *>(tb + koff[r]);
                vreg[r] = *reinterpret_cast<const v8 *>(tb + koff[r] + (size_t)W * sizeof(HT));
            }
        } else {
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int c = tid + r * 256;
                const int key = c >> 3, dc = c & 7;
                int krow = kt_ * FA_BK + key;
                krow = krow < T ? krow : T - 1;
                const HT *src = base + (size_t)krow * 3 * W + h * FA_DH + dc * 8;
                kreg[r] = *reinterpret_cast<const v8 *>(src + W);
                vreg[r] = *reinterpret_cast<const v8 *>(src + 2 * W);
            }
        }
    };
    auto stage_tile = [&](int buf) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int c = tid + r * 256;
            const int key = c >> 3, dc = c & 7;
            *reinterpret_cast<v8 *>(&Ks[buf][key * FA_KS + ((dc ^ fa_kswz(key)) << 3)]) = kreg[r];
            *reinterpret_cast<v8 *>(&Vs[buf][key * FA_DH + ((dc ^ (((key >> 1) & 1) << 2)) << 3)]) = vreg[r];
        }
    };
    fetch_tile(0);
    stage_tile(0);
    __syncthreads();
    for (int kt = 0; kt < n_kt; ++kt) {
        const int key0 = kt * FA_BK, buf = kt & 1;
        if (kt + 1 < n_kt) fetch_tile(kt + 1);
        const HT *Kt = Ks[buf], *Vt = Vs[buf];
        // the tile in two steps of 32 keys, each a complete step of the online softmax (16 accumulator registers
        // of scores instead of 32); a 32-key block that lies entirely above this wave's rows is skipped
        // (wave-uniform test)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const int kb0 = key0 + 32 * kb;
            if (kb0 > q0 + 31) continue;
            f32x16 sacc;
#pragma unroll
            for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const v8 kf = *reinterpret_cast<const v8 *>(&Kt[(32 * kb + l32) * FA_KS + (((2 * c + g) ^ fa_kswz(l32)) << 3)]);
                sacc = Half16<HT>::mfma(kf, qf[c], sacc);
            }
            // register v is key kb0 + 8 (v/4) + 4 g + v%4, query qrow; only blocks that reach the diagonal need
            // the causal mask; scores stay unscaled, the softmax scale (times log2 e) enters through one fused
            // multiply-add in front of the exponential
            float mx = -INFINITY;
            if (kb0 + 31 > q0) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = kb0 + 8 * (v >> 2) + 4 * g + (v & 3);
                    const float sv = key <= qrow ? sacc[v] : -INFINITY;
                    sacc[v] = sv;
                    mx = fmaxf(mx, sv);
                }
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[v]);
            }
            { float lo, hi; wave_halves(mx, lo, hi); mx = fmaxf(lo, hi) * scale_log2; }   // scale > 0: the maximum commutes with it
            const float m_new = fmaxf(m_run, mx);
            // rows past the end of the sequence may see no visible key; keep them finite
            const float m_use = m_new == -INFINITY ? 0.f : m_new;
            // a row whose maximum did not move has the factor exp2(0) = 1: when that holds for every row of the
            // wave the rescaling is skipped, with the same bits
            if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {
                const float corr = __builtin_amdgcn_exp2f(m_run - m_use);
                l_run *= corr;
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[db][v] *= corr;
                m_run = m_new;
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) sacc[v] = __builtin_amdgcn_exp2f(fmaf(sacc[v], scale_log2, -m_use));
            // the row sum is taken over the probabilities as they enter the second product (rounded to 16 bits),
            // two per instruction, in float32
            float psum = 0.f;

            // O^T += V^T P^T, 16 keys per instruction.  Slot e = 4 a + b of lane half g stands for key
            // kb0 + 16 c2 + 8 a + 4 g + b in both operands.
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2) {
                v8 pf;
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[e] = from_f32<HT>(sacc[8 * c2 + e]);
                psum = Half16<HT>::add_all(pf, psum);
#pragma unroll
                for (int db = 0; db < 2; ++db) {
                    union { i16x4 r; v4 h; } lo, hi;
                    const HT *vp = Vt + (32 * kb + 16 * c2) * FA_DH + voff[db];
                    lo.r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(vp));
                    hi.r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(vp + 8 * FA_DH));
                    v8 vf;
#pragma unroll
                    for (int e = 0; e < 4; ++e) { vf[e] = lo.h[e]; vf[4 + e] = hi.h[e]; }
                    oacc[db] = Half16<HT>::mfma(vf, pf, oacc[db]);
                }
            }
            { float lo, hi; wave_halves(psum, lo, hi); l_run += lo + hi; }
        }
        if (kt + 1 < n_kt) stage_tile(buf ^ 1);   // last read before the previous barrier
        __syncthreads();
    }
    if (qrow < T) {
        const float inv = 1.0f / l_run;
        HT *orow = o + ((size_t)i * T + qrow) * W + h * FA_DH;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                v4 ov;
#pragma unroll
                for (int b = 0; b < 4; ++b) ov[b] = from_f32<HT>(oacc[db][4 * a + b] * inv);
                *reinterpret_cast<v4 *>(orow + 32 * db + 8 * a + 4 * g) = ov;
            }
    }
}

template <typename HT>
void launch_flash_attention_h16(const HT *qkv, HT *o, int n_samples, int T, int H, hipStream_t s) {
    if (n_samples <= 0) return;
    const int n_qt = (T + FA_BQ - 1) / FA_BQ;
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)FA_DH);
    const int n_pairs = n_samples * H;
    const unsigned grid = (unsigned)((n_pairs + 7) / 8) * 8u * (unsigned)n_qt;
    hipLaunchKernelGGL(flash_attention_h16_kernel<HT>, dim3(grid), dim3(256), 0, s, qkv, o, T, H, n_pairs, scale_log2);
}
template void launch_flash_attention_h16<bf16>(const bf16 *, bf16 *, int, int, int, hipStream_t);
template void launch_flash_attention_h16<f16>(const f16 *, f16 *, int, int, int, hipStream_t);

// ------------------------------------------------------------------------------------------------
// The same scheme in float32 (head size 64) on the 32x32x2 float32 matrix instruction: a lane feeds ONE
// value per operand and instruction (lane half g = index g of the contracted pair).  The order in which the
// contracted index is walked is free as long as both operands agree, which removes every transposition:
//   S^T = K Q^T : step s of half g stands for d = 32 g + s, so a lane's 32 values of Q are one contiguous half
//                 row (registers), and its values of K four at a time a 16-byte LDS read;
//   O^T += V^T P^T : step s of half g stands for key 8 (s / 4) + 4 g + s % 4 of the 32-key block, which is
//                 exactly the key whose probability sits in accumulator register s of that lane half; V is
//                 read row-major, 32 consecutive d per half wave.
// LDS: K [64 keys][64 d], 16-byte chunk c of row `key` in slot c ^ fb_kswz(key) (the 16 lanes of one pass of a
// 16-byte read - lanes that agree in bits 3 and 5 - are rows {0-7, 16-23} or {8-15, 24-31} of a 32-key block
// and land on 16 different slots); V [64 keys][64 d], column col of row `key` at col ^ 32 (key / 4 % 2), so the two
// halves of a wave (keys 4 apart) read different halves of the banks.
constexpr int FB_BQ = 128, FB_BK = 64, FB_DH = 64;
__device__ __forceinline__ int fb_kswz(int key) { return (key & 7) | (((key >> 4) & 1) << 3); }

__global__ __launch_bounds__(256, 2) void flash_attention_f32_kernel(const float *__restrict__ qkv, float *__restrict__ o,
                                                                  int T, int H, int n_pairs, float scale_log2) {
    __shared__ __attribute__((aligned(16))) float Ks[FB_BK * FB_DH];
    __shared__ __attribute__((aligned(16))) float Vs[FB_BK * FB_DH];
    const int W = H * FB_DH;
    const int n_qt = (T + FB_BQ - 1) / FB_BQ;
    // the query tiles of one (sample, head) take consecutive slots of one XCD (see the 16-bit kernel)
    const int slot = (int)blockIdx.x >> 3;
    const int pair = (slot / n_qt) * 8 + ((int)blockIdx.x & 7);
    if (pair >= n_pairs) return;
    const int qt = n_qt - 1 - slot % n_qt;
    const int h = pair % H, i = pair / H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const float *base = qkv + (size_t)i * T * 3 * W;
    const int q0 = qt * FB_BQ + wave * 32;
    const int qrow = q0 + l32;
    const int qrow_c = qrow < T ? qrow : T - 1;

    float qf[32];                                  // Q[qrow][32 g + s]
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const f32x4 t = *reinterpret_cast<const f32x4 *>(base + (size_t)qrow_c * 3 * W + h * FB_DH + 32 * g + 4 * j);
#pragma unroll
        for (int e = 0; e < 4; ++e) qf[4 * j + e] = t[e];
    }
    f32x16 oacc[2];
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    // Q in registers before the loop (see the 16-bit kernel: the loop would otherwise wait for its own prefetch)
#pragma unroll
    for (int j = 0; j < 32; j += 4) asm volatile("" :: "v"(qf[j]), "v"(qf[j + 1]), "v"(qf[j + 2]), "v"(qf[j + 3]));

    const int last_row = min(qt * FB_BQ + FB_BQ - 1, T - 1);
    const int n_kt = last_row / FB_BK + 1;
    f32x4 kreg[4], vreg[4];
    auto fetch_tile = [&](int kt_) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int c = tid + r * 256;
            const int key = c >> 4, ch = c & 15;
            int krow = kt_ * FB_BK + key;
            krow = krow < T ? krow : T - 1;
            const float *src = base + (size_t)krow * 3 * W + h * FB_DH + ch * 4;
            kreg[r] = *reinterpret_cast<const f32x4 *>(src + W);
            vreg[r] = *reinterpret_cast<const f32x4 *>(src + 2 * W);
        }
    };
    fetch_tile(0);
    for (int kt = 0; kt < n_kt; ++kt) {
        const int key0 = kt * FB_BK;
        __syncthreads();  // previous tile fully consumed
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int c = tid + r * 256;
            const int key = c >> 4, ch = c & 15;
            *reinterpret_cast<f32x4 *>(&Ks[key * FB_DH + ((ch ^ fb_kswz(key)) << 2)]) = kreg[r];
            *reinterpret_cast<f32x4 *>(&Vs[key * FB_DH + ((ch ^ (((key >> 2) & 1) << 3)) << 2)]) = vreg[r];
        }
        __syncthreads();
        if (kt + 1 < n_kt) fetch_tile(kt + 1);
        if (key0 > q0 + 31) continue;  // tile lies entirely above this wave's rows (wave-uniform)

        f32x16 sacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) sacc[kb][v] = 0.f;
            const int key = 32 * kb + l32;
#pragma unroll
            for (int s4 = 0; s4 < 8; ++s4) {
                const f32x4 kf = *reinterpret_cast<const f32x4 *>(&Ks[key * FB_DH + (((8 * g + s4) ^ fb_kswz(key)) << 2)]);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf[e], qf[4 * s4 + e], sacc[kb], 0, 0, 0);
            }
        }
        // register v of block kb is key key0 + 32 kb + 8 (v/4) + 4 g + v%4, query qrow
        const bool diag = key0 + FB_BK - 1 > q0;
        float mx = -INFINITY;
        if (diag) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = key0 + 32 * kb + 8 * (v >> 2) + 4 * g + (v & 3);
                    const float sv = key <= qrow ? sacc[kb][v] : -INFINITY;
                    sacc[kb][v] = sv;
                    mx = fmaxf(mx, sv);
                }
        } else {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[kb][v]);
        }
        { float lo, hi; wave_halves(mx, lo, hi); mx = fmaxf(lo, hi) * scale_log2; }
        const float m_new = fmaxf(m_run, mx);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;   // rows past the end of the sequence stay finite
        const float corr = exp2f(m_run - m_use);
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float pv = exp2f(fmaf(sacc[kb][v], scale_log2, -m_use));
                sacc[kb][v] = pv;
                psum += pv;
            }
        { float lo, hi; wave_halves(psum, lo, hi); psum = lo + hi; }
        l_run = l_run * corr + psum;
        m_run = m_new;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[db][v] *= corr;

#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                const int key = 32 * kb + 8 * (s >> 2) + 4 * g + (s & 3);
#pragma unroll
                for (int db = 0; db < 2; ++db) {
                    const float vf = Vs[key * FB_DH + ((32 * db + l32) ^ (g << 5))];
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x2f32(vf, sacc[kb][s], oacc[db], 0, 0, 0);
                }
            }
    }
    // O^T block db: register v is d = 32 db + 8 (v/4) + 4 g + v%4, query qrow
    if (qrow < T) {
        const float inv = 1.0f / l_run;
        float *orow = o + ((size_t)i * T + qrow) * W + h * FB_DH;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 ov;
#pragma unroll
                for (int b = 0; b < 4; ++b) ov[b] = oacc[db][4 * a + b] * inv;
                *reinterpret_cast<f32x4 *>(orow + 32 * db + 8 * a + 4 * g) = ov;
            }
    }
}

void launch_flash_attention_f32(const float *qkv, float *o, int n_samples, int T, int H, hipStream_t s) {
    if (n_samples <= 0) return;
    const int n_qt = (T + FB_BQ - 1) / FB_BQ;
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)FB_DH);
    const int n_pairs = n_samples * H;
    const unsigned grid = (unsigned)((n_pairs + 7) / 8) * 8u * (unsigned)n_qt;
    hipLaunchKernelGGL(flash_attention_f32_kernel, dim3(grid), dim3(256), 0, s, qkv, o, T, H, n_pairs, scale_log2);
}


}  // namespace sjd
