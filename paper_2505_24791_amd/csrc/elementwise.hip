// Memory-bound kernels around the projections: token embedding, LayerNorm, the fused Jacobi
// epilogue (affine update + difference reduction + convergence, Alg. 1), the sequential-step
// epilogue (eq. 5 for one token), active-list compaction, and weight preparation.
#include "common.h"

namespace sjd {

// ------------------------------------------------------------------------------------------------
// Embedding: h[m, :] = x[b, tok, :] * w_in + b_in + pos[p, :]   (p = processing position of row m)
// A workgroup handles EMB_ROWS rows; a work item is four adjacent columns of eight of them: the
// four columns of w_in stay in registers across the rows (D is small, tens; W up to a few thousand),
// so w_in is read from L2 once per EMB_ROWS rows, and h is written 16 bytes per lane.  W % 4 == 0.
constexpr int EMB_ROWS = 16;
__global__ __launch_bounds__(256) void embed_kernel(const float *__restrict__ x, const float *__restrict__ w_in,
                                                    const float *__restrict__ b_in, const float *__restrict__ pos,
                                                    float *__restrict__ h, int n_rows, int D, int W, RowMap map) {
    extern __shared__ float xs[];   // [EMB_ROWS][D]
    __shared__ int prow[EMB_ROWS];
    const int m0 = blockIdx.x * EMB_ROWS;
    const int rows = n_rows - m0 < EMB_ROWS ? n_rows - m0 : EMB_ROWS;
    for (int e = threadIdx.x; e < EMB_ROWS * D; e += 256) {
        const int r = e / D, d = e - r * D;
        float v = 0.f;
        if (r < rows) {
            const int m = m0 + r;
            const int i = m / map.rows_per_sample;
            const int p = map.t0 + m % map.rows_per_sample;
            const int b = map.active ? map.active[i] : i;
            const int tok = map.reversed ? map.T - 1 - p : p;
            v = x[((size_t)b * map.T + tok) * D + d];
            if (d == 0) prow[r] = p;
        }
        xs[e] = v;
    }
    __syncthreads();
    const int ncg = W >> 2;
    for (int it = threadIdx.x; it < 2 * ncg; it += 256) {
        const int rh = it / ncg, w = (it - rh * ncg) * 4, r0 = rh * (EMB_ROWS / 2);
        const f32x4 bias = *reinterpret_cast<const f32x4 *>(b_in + w);
        f32x4 acc[EMB_ROWS / 2];
#pragma unroll
        for (int r = 0; r < EMB_ROWS / 2; ++r) acc[r] = bias;
        for (int d = 0; d < D; ++d) {
            const f32x4 wv = *reinterpret_cast<const f32x4 *>(w_in + (size_t)d * W + w);
#pragma unroll
            for (int r = 0; r < EMB_ROWS / 2; ++r) {
                const float xv = xs[(r0 + r) * D + d];
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[r][e] = fmaf(xv, wv[e], acc[r][e]);
            }
        }
#pragma unroll
        for (int r = 0; r < EMB_ROWS / 2; ++r)
            if (r0 + r < rows) {
                const f32x4 pv = *reinterpret_cast<const f32x4 *>(pos + (size_t)prow[r0 + r] * W + w);
                f32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = acc[r][e] + pv[e];
                *reinterpret_cast<f32x4 *>(h + (size_t)(m0 + r0 + r) * W + w) = o;
            }
    }
}

void launch_embed(const float *x, const float *w_in, const float *b_in, const float *pos, float *h, int n_rows, int D,
                  int W, RowMap map, hipStream_t s) {
    if (n_rows <= 0) return;
    hipLaunchKernelGGL(embed_kernel, dim3((n_rows + EMB_ROWS - 1) / EMB_ROWS), dim3(256), EMB_ROWS * D * sizeof(float), s, x,
                       w_in, b_in, pos, h, n_rows, D, W, map);
}

// ------------------------------------------------------------------------------------------------
// LayerNorm: one wave per row, two-pass statistics in float32 (mean, then centred variance).
template <typename OutT>
__global__ __launch_bounds__(256) void layernorm_kernel(const float *__restrict__ x, const float *__restrict__ g,
                                                        const float *__restrict__ b, OutT *__restrict__ y, int n_rows,
                                                        int W) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= n_rows) return;
    const float *xr = x + (size_t)row * W;
    float s = 0.f;
    for (int i = lane; i < W; i += 64) s += xr[i];
    const float mean = wave_sum(s) / (float)W;
    float v = 0.f;
    for (int i = lane; i < W; i += 64) { float d = xr[i] - mean; v = fmaf(d, d, v); }
    const float rstd = 1.0f / sqrtf(wave_sum(v) / (float)W + 1e-5f);
    OutT *yr = y + (size_t)row * W;
    for (int i = lane; i < W; i += 64) yr[i] = from_f32<OutT>(keep_f32((xr[i] - mean) * rstd * g[i] + b[i]));
}

// The same for widths that are multiples of 256: the row is read once, 16 bytes per lane and load,
// and stays in registers for both statistics passes and the output (W = 256 V).
template <typename OutT, int V>
__global__ __launch_bounds__(256) void layernorm_vec_kernel(const float *__restrict__ x, const float *__restrict__ g,
                                                            const float *__restrict__ b, OutT *__restrict__ y,
                                                            int n_rows) {
    constexpr int W = 256 * V;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= n_rows) return;
    const f32x4 *xr = reinterpret_cast<const f32x4 *>(x + (size_t)row * W);
    f32x4 v[V];
#pragma unroll
    for (int k = 0; k < V; ++k) v[k] = xr[k * 64 + lane];
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < V; ++k) s += (v[k][0] + v[k][1]) + (v[k][2] + v[k][3]);
    const float mean = wave_sum(s) / (float)W;
    float q = 0.f;
#pragma unroll
    for (int k = 0; k < V; ++k)
#pragma unroll
        for (int e = 0; e < 4; ++e) { const float d = v[k][e] - mean; q = fmaf(d, d, q); }
    const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)W + 1e-5f);
    OutT *yr = y + (size_t)row * W;
#pragma unroll
    for (int k = 0; k < V; ++k) {
        const f32x4 g4 = reinterpret_cast<const f32x4 *>(g)[k * 64 + lane];
        const f32x4 b4 = reinterpret_cast<const f32x4 *>(b)[k * 64 + lane];
        f32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = keep_f32((v[k][e] - mean) * rstd * g4[e] + b4[e]);
        if constexpr (sizeof(OutT) == 4) {
            reinterpret_cast<f32x4 *>(yr)[k * 64 + lane] = o;
        } else {
            typename Half16<OutT>::v4 h4;
#pragma unroll
            for (int e = 0; e < 4; ++e) h4[e] = from_f32<OutT>(o[e]);
            reinterpret_cast<typename Half16<OutT>::v4 *>(yr)[k * 64 + lane] = h4;
        }
    }
}

template <typename OutT>
void launch_layernorm(const float *x, const float *g, const float *b, OutT *y, int n_rows, int W, hipStream_t s) {
    if (n_rows <= 0) return;
    const dim3 grid((n_rows + 3) / 4), block(256);
    switch (W) {
    case 256: hipLaunchKernelGGL((layernorm_vec_kernel<OutT, 1>), grid, block, 0, s, x, g, b, y, n_rows); break;
    case 512: hipLaunchKernelGGL((layernorm_vec_kernel<OutT, 2>), grid, block, 0, s, x, g, b, y, n_rows); break;
    case 768: hipLaunchKernelGGL((layernorm_vec_kernel<OutT, 3>), grid, block, 0, s, x, g, b, y, n_rows); break;
    case 1024: hipLaunchKernelGGL((layernorm_vec_kernel<OutT, 4>), grid, block, 0, s, x, g, b, y, n_rows); break;
    default: hipLaunchKernelGGL(layernorm_kernel<OutT>, grid, block, 0, s, x, g, b, y, n_rows, W); break;
    }
}
template void launch_layernorm<float>(const float *, const float *, const float *, float *, int, int, hipStream_t);
template void launch_layernorm<bf16>(const float *, const float *, const float *, bf16 *, int, int, hipStream_t);
template void launch_layernorm<f16>(const float *, const float *, const float *, f16 *, int, int, hipStream_t);

// ------------------------------------------------------------------------------------------------
// Jacobi epilogue (Alg. 1, the update line and the stopping test; F of Def. A.1).
// One workgroup per listed sample.  The difference norm is reduced in a fixed order (lane
// partials -> wave shuffles -> waves in index order), so a sample's delta does not depend on
// which other samples are in flight.

__device__ __forceinline__ float nan_max(float a, float d) { return (d > a || d != d) ? d : a; }

__global__ __launch_bounds__(256) void jacobi_epilogue_kernel(const float *__restrict__ p, const float *__restrict__ z,
                                                              float *__restrict__ x, JacobiState st, int T, int D,
                                                              int reversed, float tau, int criterion, int cap,
                                                              int shared_params, float refine_below) {
    __shared__ float part[4];
    const int i = blockIdx.x;
    const int b = st.active_in[i];
    if (st.done[b]) return;  // only reachable when converged samples are kept in the batch
    const int n = T * D;
    // shared_params: p holds one sample's parameters, valid for every sample (the pass from the all-zero iterate)
    const float *pr = p + (shared_params ? 0 : (size_t)i * T * 2 * D);
    float acc = 0.f;
    // Eight elements of a thread at a time, all their loads issued before the first is used: one element per trip
    // is four dependent round trips to memory per element, 192 times over for a sample of 1024 x 48 values.  The
    // thread still accumulates its elements in index order (same bits as one at a time).
    constexpr int U = 8;
    for (int e0 = threadIdx.x; e0 < n; e0 += 256 * U) {
        float zv[U], xo[U], mu[U], al[U];
        size_t idx[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + 256 * u;
            const int ec = e < n ? e : threadIdx.x;          // past the end: re-read this thread's first element, unused
            const int l = ec / D, d = ec - l * D;
            const int tok = reversed ? T - 1 - l : l;
            idx[u] = ((size_t)b * T + tok) * D + d;
            zv[u] = z[idx[u]];
            xo[u] = x[idx[u]];
            const int lp = l > 0 ? l - 1 : 0;
            mu[u] = pr[(size_t)lp * 2 * D + d];
            al[u] = pr[(size_t)lp * 2 * D + D + d];
            if (l == 0) { mu[u] = 0.f; al[u] = 0.f; }        // the first processed token is copied
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + 256 * u;
            if (e < n) {
                const bool first = e < D;                    // l == 0
                const float xn = first ? zv[u] : fmaf(zv[u], expf(al[u]), mu[u]);
                const float diff = fabsf(xn - xo[u]);
                x[idx[u]] = xn;
                acc = criterion == 1 ? nan_max(acc, diff) : acc + diff;
            }
        }
    }
    if (criterion == 1) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc = nan_max(acc, __shfl_xor(acc, o, 64));
    } else {
        acc = wave_sum(acc);
    }
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float delta;
        if (criterion == 1) delta = nan_max(nan_max(nan_max(part[0], part[1]), part[2]), part[3]);
        else delta = (((part[0] + part[1]) + part[2]) + part[3]) / (float)n;
        const int it = st.iters[b] + 1;
        st.iters[b] = it;
        st.delta[b] = delta;
        if (delta < tau || it >= cap) {
            st.done[b] = 1;
            if (!(fabsf(delta) <= 3.0e38f)) *st.nonfinite = 1;
        }
        if (delta < refine_below) st.fine[b] = 1;
    }
}

// Rebuilds the list of samples that still iterate and counts them: first the samples that are not marked
// fine, then the fine ones (their passes run in float32), each part in increasing order of the sample index.
// With keep_all the list is left complete (finished samples go with the first part) and only the counts of
// unfinished samples are produced.
__global__ __launch_bounds__(256) void compact_active_kernel(JacobiState st, int n_listed, int keep_all) {
    __shared__ int wave_keep[4], wave_live[4];
    __shared__ int base_keep, base_live, base_fine;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (threadIdx.x == 0) { base_keep = 0; base_live = 0; base_fine = 0; }
    __syncthreads();
    for (int part = 0; part < 2; ++part) {
        for (int start = 0; start < n_listed; start += 256) {
            const int i = start + threadIdx.x;
            int b = -1, live = 0;
            if (i < n_listed) {
                b = st.active_in[i];
                const int alive = st.done[b] ? 0 : 1;
                const int fine = alive && st.fine[b];
                live = alive && fine == part;
            }
            const int keep = live || (part == 0 && keep_all && i < n_listed && st.done[b]);
            const unsigned long long mk = __ballot(keep), ml = __ballot(live);
            const int before = __popcll(mk & ((1ull << lane) - 1ull));
            if (lane == 0) { wave_keep[wv] = __popcll(mk); wave_live[wv] = __popcll(ml); }
            __syncthreads();
            int off = base_keep;
            for (int w = 0; w < wv; ++w) off += wave_keep[w];
            if (keep) st.active_out[off + before] = b;
            __syncthreads();
            if (threadIdx.x == 0) {
                const int lv = wave_live[0] + wave_live[1] + wave_live[2] + wave_live[3];
                base_keep += wave_keep[0] + wave_keep[1] + wave_keep[2] + wave_keep[3];
                base_live += lv;
                if (part == 1) base_fine += lv;
            }
            __syncthreads();
        }
    }
    if (threadIdx.x == 0) { st.n_active_out[0] = base_live; st.n_active_out[1] = base_fine; }
}

void launch_jacobi_update(const float *p, const float *z, float *x, JacobiState st, int n, int T, int D, int reversed,
                          float tau, int criterion, int cap, int shared_params, float refine_below, hipStream_t s) {
    if (n <= 0) return;
    hipLaunchKernelGGL(jacobi_epilogue_kernel, dim3(n), dim3(256), 0, s, p, z, x, st, T, D, reversed, tau, criterion,
                       cap, shared_params, refine_below);
}

void launch_jacobi_compact(JacobiState st, int n_listed, int keep_all, hipStream_t s) {
    if (n_listed <= 0) return;
    hipLaunchKernelGGL(compact_active_kernel, dim3(1), dim3(256), 0, s, st, n_listed, keep_all);
}

__global__ __launch_bounds__(256) void jacobi_init_kernel(const float *__restrict__ z, float *__restrict__ x,
                                                          JacobiState st, int B, size_t n_per_sample, int init) {
    const size_t n = (size_t)B * n_per_sample;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (size_t)gridDim.x * 256)
        if (init != 2) x[e] = init == 1 ? z[e] : 0.f;   // init 2: the caller's x^0 is already in x
    if (blockIdx.x == 0) {
        for (int b = threadIdx.x; b < B; b += 256) {
            st.iters[b] = 0; st.done[b] = 0; st.fine[b] = 0; st.delta[b] = 0.f; st.active_in[b] = b; st.active_out[b] = b;
        }
        if (threadIdx.x == 0) { st.n_active_out[0] = B; st.n_active_out[1] = 0; *st.nonfinite = 0; }
    }
}

void launch_jacobi_init(const float *z, float *x, JacobiState st, int B, int T, int D, int init, hipStream_t s) {
    const size_t n = (size_t)B * T * D;
    int grid = (int)((n + 255) / 256);
    if (grid > 2048) grid = 2048;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(jacobi_init_kernel, dim3(grid), dim3(256), 0, s, z, x, st, B, (size_t)T * D, init);
}

// Per-pass convergence record: delta of the pass just made and the l2 distance of the newest
// iterate to a reference solution, one workgroup per sample (fixed summation order).
__global__ __launch_bounds__(256) void jacobi_trace_kernel(const float *__restrict__ x, const float *__restrict__ x_ref,
                                                           JacobiState st, float *__restrict__ delta_out,
                                                           float *__restrict__ err_out, int n) {
    __shared__ float part[4];
    const int b = blockIdx.x;
    if (threadIdx.x == 0) delta_out[b] = st.delta[b];
    if (!x_ref) return;
    float acc = 0.f;
    for (int e = threadIdx.x; e < n; e += 256) {
        const float d = x[(size_t)b * n + e] - x_ref[(size_t)b * n + e];
        acc = fmaf(d, d, acc);
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) err_out[b] = sqrtf(((part[0] + part[1]) + part[2]) + part[3]);
}

void launch_jacobi_trace(const float *x, const float *x_ref, JacobiState st, float *delta_out, float *err_out, int B,
                         int T, int D, hipStream_t s) {
    if (B <= 0) return;
    hipLaunchKernelGGL(jacobi_trace_kernel, dim3(B), dim3(256), 0, s, x, x_ref, st, delta_out, err_out, T * D);
}

// ------------------------------------------------------------------------------------------------
// Forward map of one block (eq. 4) from the head output of one conditioner pass on the block's
// input: y = (x - mu) * exp(-alpha) with the one-token shift, and log |det dy/dx| = -sum alpha
// (eq. 1's change-of-variables term).  One workgroup per sample; fixed summation order.
__global__ __launch_bounds__(256) void forward_epilogue_kernel(const float *__restrict__ p, const float *__restrict__ x,
                                                               float *__restrict__ y, float *__restrict__ logdet,
                                                               int T, int D, int reversed, int accumulate) {
    __shared__ float part[4];
    const int b = blockIdx.x;
    const int n = T * D;
    const float *pr = p + (size_t)b * T * 2 * D;
    float acc = 0.f;
    for (int e = threadIdx.x; e < n; e += 256) {
        const int l = e / D, d = e - l * D;
        const int tok = reversed ? T - 1 - l : l;
        const size_t idx = ((size_t)b * T + tok) * D + d;
        float v = x[idx];
        if (l > 0) {
            const float mu = pr[(size_t)(l - 1) * 2 * D + d];
            const float al = pr[(size_t)(l - 1) * 2 * D + D + d];
            v = (v - mu) * expf(-al);
            acc += al;
        }
        y[idx] = v;
    }
    if (!logdet) return;
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float ld = -(((part[0] + part[1]) + part[2]) + part[3]);
        logdet[b] = accumulate ? logdet[b] + ld : ld;
    }
}

void launch_forward_epilogue(const float *p, const float *x, float *y, float *logdet, int B, int T, int D, int reversed,
                             int accumulate, hipStream_t s) {
    if (B <= 0) return;
    hipLaunchKernelGGL(forward_epilogue_kernel, dim3(B), dim3(256), 0, s, p, x, y, logdet, T, D, reversed, accumulate);
}

// ------------------------------------------------------------------------------------------------
// Sequential step epilogue (eq. 5, one token of every sample).
__global__ void decode_epilogue_kernel(const float *__restrict__ p, const float *__restrict__ z, float *__restrict__ x,
                                       int T, int D, int t, int reversed) {
    const int b = blockIdx.x;
    const int l = t + 1;
    const int tok = reversed ? T - 1 - l : l;
    for (int d = threadIdx.x; d < D; d += blockDim.x) {
        const size_t idx = ((size_t)b * T + tok) * D + d;
        float xn = z[idx];
        if (l > 0) xn = fmaf(xn, expf(p[(size_t)b * 2 * D + D + d]), p[(size_t)b * 2 * D + d]);
        x[idx] = xn;
    }
}

void launch_decode_epilogue(const float *p, const float *z, float *x, int B, int T, int D, int t, int reversed,
                            hipStream_t s) {
    if (B <= 0) return;
    hipLaunchKernelGGL(decode_epilogue_kernel, dim3(B), dim3(64), 0, s, p, z, x, T, D, t, reversed);
}

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void split_params_kernel(const float *__restrict__ p, float *__restrict__ mu,
                                                           float *__restrict__ alpha, int T, int D, int reversed) {
    const int b = blockIdx.x;
    for (int e = threadIdx.x; e < T * D; e += 256) {
        const int l = e / D, d = e - l * D;
        const int tok = reversed ? T - 1 - l : l;
        const size_t idx = ((size_t)b * T + tok) * D + d;
        float m = 0.f, a = 0.f;
        if (l > 0) {
            m = p[((size_t)b * T + l - 1) * 2 * D + d];
            a = p[((size_t)b * T + l - 1) * 2 * D + D + d];
        }
        mu[idx] = m;
        alpha[idx] = a;
    }
}

void launch_split_params(const float *p, float *mu, float *alpha, int B, int T, int D, int reversed, hipStream_t s) {
    if (B <= 0) return;
    hipLaunchKernelGGL(split_params_kernel, dim3(B), dim3(256), 0, s, p, mu, alpha, T, D, reversed);
}

// ------------------------------------------------------------------------------------------------
// dst[n, k] = HT(src[k, n]) for n < N, k < K; zero elsewhere (rows up to n_rows_padded, row length ldb)
template <typename HT>
__global__ __launch_bounds__(256) void transpose_to_h16_kernel(const float *__restrict__ src, HT *__restrict__ dst,
                                                               int K, int N, int ldb, int n_rows_padded) {
    __shared__ float tile[32][33];
    const int k0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        const int k = k0 + r, n = n0 + tx;
        tile[r][tx] = (k < K && n < N) ? src[(size_t)k * N + n] : 0.f;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int n = n0 + r, k = k0 + tx;
        if (n < n_rows_padded && k < ldb) dst[(size_t)n * ldb + k] = from_f32<HT>(tile[tx][r]);
    }
}

template <typename HT>
void launch_transpose_to_h16(const float *src, HT *dst, int K, int N, int ldb, int n_rows_padded, hipStream_t s) {
    dim3 grid((ldb + 31) / 32, (n_rows_padded + 31) / 32);
    hipLaunchKernelGGL(transpose_to_h16_kernel<HT>, grid, dim3(256), 0, s, src, dst, K, N, ldb, n_rows_padded);
}
template void launch_transpose_to_h16<bf16>(const float *, bf16 *, int, int, int, int, hipStream_t);
template void launch_transpose_to_h16<f16>(const float *, f16 *, int, int, int, int, hipStream_t);

// Fragment-major weight copy for the skinny kernels: dst holds, for column block nb = n/16 and
// k-step ks = k/32, the 64 x 8 elements lane = 16*((k%32)/8) + n%16, e = k%8 contiguously
// (dst[((nb*KS + ks)*64 + lane)*8 + e] = src[k, n]); columns up to n_rows_padded, zero filled.
template <typename HT>
__global__ __launch_bounds__(256) void weights_to_frag_kernel(const float *__restrict__ src, HT *__restrict__ dst, int K,
                                                              int N, int n_rows_padded) {
    const int KS = K / 32;
    const size_t total = (size_t)n_rows_padded * K;
    for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (size_t)gridDim.x * 256) {
        const int e = idx & 7;
        const int lane = (idx >> 3) & 63;
        const size_t fr = idx >> 9;
        const int ks = (int)(fr % KS), nb = (int)(fr / KS);
        const int n = nb * 16 + (lane & 15);
        const int k = ks * 32 + (lane >> 4) * 8 + e;
        dst[idx] = from_f32<HT>(n < N ? src[(size_t)k * N + n] : 0.f);
    }
}

template <typename HT>
void launch_weights_to_frag(const float *src, HT *dst, int K, int N, int n_rows_padded, hipStream_t s) {
    const size_t total = (size_t)n_rows_padded * K;
    int grid = (int)((total + 255) / 256);
    if (grid > 8192) grid = 8192;
    hipLaunchKernelGGL(weights_to_frag_kernel<HT>, dim3(grid), dim3(256), 0, s, src, dst, K, N, n_rows_padded);
}
template void launch_weights_to_frag<bf16>(const float *, bf16 *, int, int, int, hipStream_t);
template void launch_weights_to_frag<f16>(const float *, f16 *, int, int, int, hipStream_t);

}  // namespace sjd
