// Host side of the library: the handle, weight loading, and the entry points declared in sjd.h.
// Every arithmetic step runs in the HIP kernels of this directory; the host only sequences
// launches and reads one integer per Jacobi pass (the number of samples still iterating).
#include "../../include/sjd.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <map>
#include <mutex>
#include <new>
#include <tuple>
#include <vector>

#include "common.h"

using namespace sjd;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                                  \
    do {                                                                                               \
        hipError_t e_ = (expr);                                                                        \
        if (e_ != hipSuccess) return fail(SJD_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), \
                                          __FILE__, __LINE__);                                         \
    } while (0)

struct LayerW {
    const float *ln1_g, *ln1_b, *b_qkv, *b_o, *ln2_g, *ln2_b, *b_fc1, *b_fc2;
    const float *w_qkv, *w_o, *w_fc1, *w_fc2;      // float32 [in, out] (views into the device blob)
    void *t_qkv, *t_o, *t_fc1, *t_fc2;             // 16-bit transposed [out (padded), in]
    void *f_qkv, *f_o, *f_fc1, *f_fc2;             // 16-bit fragment-major copies for single-token steps
    void *p_qkv = nullptr, *p_o = nullptr, *p_fc1 = nullptr, *p_fc2 = nullptr;   // 32x32x16 fragment order for the panel / streaming kernels (W = 512)
};
struct BlockW {
    const float *w_in, *b_in, *pos, *lnf_g, *lnf_b, *w_head, *b_head;
    void *t_head, *f_head;
    std::vector<LayerW> layer;
};

constexpr int SJD_ELAUNCH_RETRY = -1000;  // internal: the persistent kernel could not be launched

struct ProfSpan { hipEvent_t a, b; int fam; };

}  // namespace

struct sjd_flow {
    sjd_config cfg;
    int device = 0;
    bool loaded = false;
    size_t bytes = 0;
    std::vector<void *> allocs;
    float *blob = nullptr;       // whole float32 blob on the device
    void *arena = nullptr;       // transposed 16-bit matrices
    void *arena_frag = nullptr;  // the same matrices in fragment-major order (sequential fast path)
    void *arena_panel = nullptr; // QKV, attention-output and MLP-input matrices in the panel kernels' order
    int proj_path = 0;           // 0 automatic, 1 tile kernels only, 2 panel kernels wherever they apply
    bool stream_ok = false;      // the streaming MLP-output kernel reproduced the tile kernel's bits at load time
    std::vector<BlockW> block;
    // workspaces (element type depends on dtype: float or bf16 for a, qkv, o, f and the cache)
    float *h = nullptr, *p = nullptr;
    void *a = nullptr, *qkv = nullptr, *o = nullptr, *f = nullptr;
    void *kcache = nullptr, *vcache = nullptr;  // [N][B][T][W]
    float *pp[2] = {nullptr, nullptr};          // block outputs inside sjd_sample
    JacobiState st{};
    int32_t *active[2] = {nullptr, nullptr};
    float *trace = nullptr;                     // per-pass record: delta [T][B], then l2 error [T][B]
    // float32 activation workspaces of a 16-bit flow for refined passes (sjd_jacobi_opts.refine_below), allocated
    // on first use for r32_samples samples at a time
    void *r32_a = nullptr, *r32_qkv = nullptr, *r32_o = nullptr, *r32_f = nullptr;
    int r32_samples = 0;
    int32_t *host_pin = nullptr;                // pinned: [0] n_active, [1] n_fine, [2] nonfinite, [3..] iters[B]
    // sequential fast path: device step counter, ticket, capture stream, one graph per (block, batch)
    int32_t *t_dev = nullptr;
    uint32_t *ticket = nullptr;
    hipStream_t cap_stream = nullptr;
    std::map<std::tuple<int, int, const void *, const void *>, hipGraphExec_t> step_graphs;
    int use_graphs = 1;
    int mask_nearest = 0;        // o of the masked-dependency probe (eq. 6); 0: plain causal attention
    int seq_path = 0;            // 0 automatic, 1 per-step launches (graph replay), 2 persistent kernel, 3 the same, plain launch
    int *psync = nullptr;        // synchronisation words of the persistent kernel (1024 ints)
    int n_cus = 0, n_cus_device = 0, coop = 0;   // workgroups of the persistent kernel; CUs of the device
    hipEvent_t ev[SJD_MAX_BLOCKS + 1] = {};
    // profiling
    uint32_t prof_mask = 0;
    std::vector<ProfSpan> spans;
    std::vector<hipEvent_t> free_events;
    sjd_profile prof{};
    float prof_overhead_ms = -1.f;   // what an empty event pair measures on this device (calibrated on first use)
};

namespace {

size_t act_bytes(const sjd_flow *f) { return f->cfg.dtype == SJD_DTYPE_F32 ? 4 : 2; }

int dev_alloc(sjd_flow *f, void **out, size_t nbytes) {
    if (nbytes == 0) nbytes = 256;
    hipError_t e = hipMalloc(out, nbytes);
    if (e != hipSuccess) return fail(SJD_ENOMEM, "hipMalloc of %zu bytes failed: %s", nbytes, hipGetErrorString(e));
    f->allocs.push_back(*out);
    f->bytes += nbytes;
    return SJD_OK;
}

size_t round_up(size_t v, size_t m) { return (v + m - 1) / m * m; }

size_t block_floats(const sjd_config &c) {
    size_t D = c.token_dim, W = c.width, T = c.seq_len, R = c.mlp_ratio, N = c.n_layers;
    size_t per_layer = 2 * W + W * 3 * W + 3 * W + W * W + W + 2 * W + W * R * W + R * W + R * W * W + W;
    return D * W + W + T * W + N * per_layer + 2 * W + W * 2 * D + 2 * D;
}

constexpr size_t kNPad = 256;  // transposed weights are padded to this many rows per matrix

// the panel projection kernels cover 16-bit flows of width 512 whose matrices have multiples of 256 columns
bool panel_ok(const sjd_config &c) {
    return c.dtype != SJD_DTYPE_F32 && c.width == 512 && ((size_t)c.mlp_ratio * c.width) % 256 == 0;
}

size_t arena_elems_per_block(const sjd_config &c) {
    size_t W = c.width, R = c.mlp_ratio, D = c.token_dim;
    size_t per_layer = round_up(3 * W, kNPad) * W + round_up(W, kNPad) * W + round_up(R * W, kNPad) * W +
                       round_up(W, kNPad) * R * W;
    return c.n_layers * per_layer + round_up(2 * D, kNPad) * W;
}

// ---- profiling helpers ---------------------------------------------------------------------------
// An event pair around nothing does not measure zero: the markers themselves take a few microseconds, which is
// as much as a single-token kernel.  The empty pair is measured once (median of 33) and taken off every span.
void calibrate_profile(sjd_flow *f, hipStream_t s) {
    f->prof_overhead_ms = 0.f;
    constexpr int N = 33;
    hipEvent_t a[N], b[N];
    int made = 0;
    for (; made < N; ++made)
        if (hipEventCreate(&a[made]) != hipSuccess || hipEventCreate(&b[made]) != hipSuccess) break;
    if (made == N) {
        for (int i = 0; i < N; ++i) { (void)hipEventRecord(a[i], s); (void)hipEventRecord(b[i], s); }
        float ms[N];
        bool ok = hipStreamSynchronize(s) == hipSuccess;
        for (int i = 0; ok && i < N; ++i) ok = hipEventElapsedTime(&ms[i], a[i], b[i]) == hipSuccess;
        if (ok) {
            for (int i = 1; i < N; ++i)            // insertion sort: 33 values
                for (int j = i; j > 0 && ms[j] < ms[j - 1]; --j) { const float t = ms[j]; ms[j] = ms[j - 1]; ms[j - 1] = t; }
            f->prof_overhead_ms = ms[N / 2];
        }
    }
    for (int i = 0; i < made; ++i) { (void)hipEventDestroy(a[i]); (void)hipEventDestroy(b[i]); }
    (void)hipGetLastError();
}

struct ProfScope {
    sjd_flow *f; int fam; hipStream_t s; bool on; hipEvent_t a{}, b{};
    ProfScope(sjd_flow *f_, int fam_, double flops, double bytes, hipStream_t s_) : f(f_), fam(fam_), s(s_) {
        on = (f->prof_mask >> fam) & 1u;
        if (!on) return;
        if (f->prof_overhead_ms < 0.f) calibrate_profile(f, s);
        auto get = [&]() {
            hipEvent_t e;
            if (!f->free_events.empty()) { e = f->free_events.back(); f->free_events.pop_back(); }
            else if (hipEventCreate(&e) != hipSuccess) { e = nullptr; }
            return e;
        };
        a = get(); b = get();
        if (!a || !b) { on = false; return; }
        f->prof.flops[fam] += flops;
        f->prof.bytes[fam] += bytes;
        f->prof.launches[fam] += 1;
        (void)hipEventRecord(a, s);
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(b, s);
        f->spans.push_back({a, b, fam});
    }
};

int drain_profile(sjd_flow *f) {
    for (auto &sp : f->spans) {
        HIP_TRY(hipEventSynchronize(sp.b));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, sp.a, sp.b));
        ms -= f->prof_overhead_ms;
        f->prof.ms[sp.fam] += ms > 0.f ? ms : 0.f;
        f->free_events.push_back(sp.a);
        f->free_events.push_back(sp.b);
    }
    f->spans.clear();
    return SJD_OK;
}

// The streaming MLP-output kernel issues its weight loads as inline assembly with hand-counted waits.  Once per
// load_weights it is run beside the tile kernel on one small problem with the flow's own weights (block 0, layer 0;
// 256 rows of ones; the residual stream starts at zero); unless the two give the same bits the flow keeps to the
// tile kernels.  Uses the workspaces f and h, which no call is using yet.
int stream_self_check(sjd_flow *f) {
    const sjd_config &c = f->cfg;
    const int W = c.width, RW = c.mlp_ratio * c.width, M = 256;
    if (!gemm_stream_applicable(M, W, RW) || (size_t)c.max_batch * c.seq_len < 2 * (size_t)M) return SJD_OK;   // not used by this flow
    const LayerW &lw = f->block[0].layer[0];
    const size_t a_bytes = (size_t)M * RW * 2, h_bytes = (size_t)M * W * 4;
    // 0x3C3C is 1.0586 as IEEE half and 0.0115 as bf16: a constant left operand, so every stale or misplaced
    // weight fragment changes a sum
    HIP_TRY(hipMemset(f->f, 0x3C, a_bytes));
    HIP_TRY(hipMemset(f->h, 0, 2 * h_bytes));
    float *h0 = f->h, *h1 = f->h + (size_t)M * W;
    if (c.dtype == SJD_DTYPE_BF16) {
        launch_gemm_stream_resid<bf16>((const bf16 *)f->f, (const bf16 *)lw.p_fc2, lw.b_fc2, h0, M, W, RW, 0);
        launch_gemm_h16<bf16, float>((const bf16 *)f->f, (const bf16 *)lw.t_fc2, lw.b_fc2, h1, h1, M, W, RW, EPI_BIAS_RESIDUAL, 0, 3);
    } else {
        launch_gemm_stream_resid<f16>((const f16 *)f->f, (const f16 *)lw.p_fc2, lw.b_fc2, h0, M, W, RW, 0);
        launch_gemm_h16<f16, float>((const f16 *)f->f, (const f16 *)lw.t_fc2, lw.b_fc2, h1, h1, M, W, RW, EPI_BIAS_RESIDUAL, 0, 3);
    }
    std::vector<float> host(2 * (size_t)M * W);
    HIP_TRY(hipMemcpy(host.data(), f->h, 2 * h_bytes, hipMemcpyDeviceToHost));
    HIP_TRY(hipGetLastError());
    f->stream_ok = memcmp(host.data(), host.data() + (size_t)M * W, h_bytes) == 0;
    return SJD_OK;
}

// ---- one projection, in the flow's precision ----------------------------------------------------
template <typename HT>
void project16(const void *A, const void *wt, const float *bias, void *C, int M, int N, int K, Epi epi, bool out_f32,
               hipStream_t s) {
    if (out_f32)
        launch_gemm_h16<HT, float>((const HT *)A, (const HT *)wt, bias,
                                   epi == EPI_BIAS_RESIDUAL ? (const float *)C : nullptr, (float *)C, M, N, K, epi, s);
    else
        launch_gemm_h16<HT, HT>((const HT *)A, (const HT *)wt, bias, nullptr, (HT *)C, M, N, K, epi, s);
}

// in: A [M, K]; out: C [M, N]; residual variant accumulates into the float32 stream h in place.
void project(sjd_flow *f, int fam, const void *A, const float *w32, const void *wt, const float *bias, void *C, int M,
             int N, int K, Epi epi, bool out_f32, hipStream_t s) {
    const int dt = f->cfg.dtype;
    const double in_b = dt == SJD_DTYPE_F32 ? 4.0 : 2.0, out_b = (dt != SJD_DTYPE_F32 && !out_f32) ? 2.0 : 4.0;
    double bytes = (double)M * K * in_b + (double)K * N * in_b + (double)M * N * out_b + (double)N * 4;
    if (epi == EPI_BIAS_RESIDUAL) bytes += (double)M * N * 4;
    ProfScope ps(f, fam, 2.0 * M * (double)N * K, bytes, s);
    if (dt == SJD_DTYPE_F32)
        launch_gemm_f32((const float *)A, w32, bias, epi == EPI_BIAS_RESIDUAL ? (const float *)C : nullptr, (float *)C,
                        M, N, K, epi, s);
    else if (dt == SJD_DTYPE_BF16) project16<bf16>(A, wt, bias, C, M, N, K, epi, out_f32, s);
    else project16<f16>(A, wt, bias, C, M, N, K, epi, out_f32, s);
}

void layernorm(sjd_flow *f, const float *x, const float *g, const float *b, void *y, int rows, hipStream_t s) {
    const int W = f->cfg.width;
    ProfScope ps(f, SJD_PROF_OTHER, 0.0, (double)rows * W * (4.0 + act_bytes(f)), s);
    if (f->cfg.dtype == SJD_DTYPE_BF16) launch_layernorm<bf16>(x, g, b, (bf16 *)y, rows, W, s);
    else if (f->cfg.dtype == SJD_DTYPE_F16) launch_layernorm<f16>(x, g, b, (f16 *)y, rows, W, s);
    else launch_layernorm<float>(x, g, b, (float *)y, rows, W, s);
}

// LayerNorm + projection in one launch (16-bit flows of width 512): C = epi(LayerNorm(H) W + bias)
void ln_project_panel(sjd_flow *f, const float *H, const float *g, const float *b, const void *wf, const float *bias,
                      void *C, int M, int N, Epi epi, hipStream_t s) {
    const int W = f->cfg.width;
    ProfScope ps(f, epi == EPI_BIAS_GELU ? SJD_PROF_GEMM_FC1 : SJD_PROF_GEMM, 2.0 * M * (double)N * W, (double)M * W * 4.0 + (double)W * N * 2.0 + (double)M * N * 2.0 + N * 4.0, s);
    if (f->cfg.dtype == SJD_DTYPE_BF16) launch_ln_gemm_panel<bf16>(H, g, b, (const bf16 *)wf, bias, (bf16 *)C, M, N, epi, s);
    else launch_ln_gemm_panel<f16>(H, g, b, (const f16 *)wf, bias, (f16 *)C, M, N, epi, s);
}

// H += A W + bias on the panel kernel
void project_panel_resid(sjd_flow *f, const void *A, const void *wf, const float *bias, float *H, int M, int N,
                         hipStream_t s) {
    const int W = f->cfg.width;
    ProfScope ps(f, SJD_PROF_GEMM_RESID, 2.0 * M * (double)N * W, (double)M * W * 2.0 + (double)W * N * 2.0 + (double)M * N * 8.0 + N * 4.0, s);
    if (f->cfg.dtype == SJD_DTYPE_BF16) launch_gemm_panel_resid<bf16>((const bf16 *)A, (const bf16 *)wf, bias, H, M, N, s);
    else launch_gemm_panel_resid<f16>((const f16 *)A, (const f16 *)wf, bias, H, M, N, s);
}

// whole-sequence causal attention on the fused qkv buffer [n*T, 3W] -> o [n*T, W]
template <typename AT>
void attention_full(const void *qkv, void *o, int n, int T, int W, int H, int mask_o, hipStream_t s) {
    const AT *q = (const AT *)qkv;
    if constexpr (sizeof(AT) == 2) {
        if (W / H == 64 && mask_o == 0) { launch_flash_attention_h16<AT>(q, (AT *)o, n, T, H, s); return; }
    } else {
        if (W / H == 64 && mask_o == 0) { launch_flash_attention_f32(q, (float *)o, n, T, H, s); return; }
    }
    // the masked probe (a diagnostic) takes the row-wise kernel in every mode
    launch_attention_rows<AT, AT>(q, 3 * W, q + W, q + 2 * W, 3 * W, (int64_t)T * 3 * W, (AT *)o, W, n, T, 0, H, W / H,
                                  mask_o, s);
}

template <typename AT>
void attention_step(sjd_flow *f, int l, int B, int t, hipStream_t s) {
    const sjd_config &c = f->cfg;
    const size_t layer_off = (size_t)l * c.max_batch * c.seq_len * c.width;
    launch_decode_attention<AT>((const AT *)f->qkv, (AT *)f->kcache + layer_off, (AT *)f->vcache + layer_off,
                                (AT *)f->o, B, c.seq_len, t, c.n_heads, c.width / c.n_heads, f->mask_nearest, s);
}

// Whole-sequence conditioner pass on `n` samples listed in `active` (device, nullable = identity).
// Leaves the head output in f->p: [n*T, 2D], row r of a sample = parameters of position r+1.
void conditioner_pass(sjd_flow *f, int j, const float *x, int n, const int32_t *active, hipStream_t s) {
    const sjd_config &c = f->cfg;
    const int T = c.seq_len, W = c.width, D = c.token_dim, H = c.n_heads, RW = c.mlp_ratio * c.width;
    const int M = n * T;
    const int rev = (c.reverse_mask >> j) & 1;
    const BlockW &bw = f->block[j];
    {
        ProfScope ps(f, SJD_PROF_OTHER, 2.0 * M * (double)D * W, (double)M * W * 4, s);
        launch_embed(x, bw.w_in, bw.b_in, bw.pos, f->h, M, D, W, RowMap{active, T, 0, T, rev}, s);
    }
    // Width 512: LayerNorm + projection in one activation-stationary launch where that is faster: a
    // workgroup of those kernels is 128 rows x 768..1024 columns of work, so below ~90 panels the tile
    // kernels' finer grain wins (measured on configuration C2: QKV from 10240 rows on, MLP input from 12288)
    const bool panel_any = f->arena_panel && f->proj_path != 1 && gemm_panel_applicable(M, RW, W, 2) &&
                           gemm_panel_applicable(M, 3 * W, W, 2) && gemm_panel_applicable(M, W, W, 4);
    const bool panel_qkv = panel_any && (f->proj_path == 2 || M >= 10240);
    const bool panel_fc1 = panel_any && (f->proj_path == 2 || M >= 12288);
    const bool stream_fc2 = panel_any && f->stream_ok && (f->proj_path == 2 || M >= 10240) && gemm_stream_applicable(M, W, RW);
    for (int l = 0; l < c.n_layers; ++l) {
        const LayerW &lw = bw.layer[l];
        if (panel_qkv) ln_project_panel(f, f->h, lw.ln1_g, lw.ln1_b, lw.p_qkv, lw.b_qkv, f->qkv, M, 3 * W, EPI_BIAS, s);
        else {
            layernorm(f, f->h, lw.ln1_g, lw.ln1_b, f->a, M, s);
            project(f, SJD_PROF_GEMM, f->a, lw.w_qkv, lw.t_qkv, lw.b_qkv, f->qkv, M, 3 * W, W, EPI_BIAS, false, s);
        }
        {
            const double ab = act_bytes(f);
            ProfScope ps(f, SJD_PROF_ATTENTION, 2.0 * n * (double)T * (T + 1) * W, (double)M * 4 * W * ab, s);
            if (c.dtype == SJD_DTYPE_BF16) attention_full<bf16>(f->qkv, f->o, n, T, W, H, f->mask_nearest, s);
            else if (c.dtype == SJD_DTYPE_F16) attention_full<f16>(f->qkv, f->o, n, T, W, H, f->mask_nearest, s);
            else attention_full<float>(f->qkv, f->o, n, T, W, H, f->mask_nearest, s);
        }
        if (panel_qkv) project_panel_resid(f, f->o, lw.p_o, lw.b_o, f->h, M, W, s);
        else project(f, SJD_PROF_GEMM_RESID, f->o, lw.w_o, lw.t_o, lw.b_o, f->h, M, W, W, EPI_BIAS_RESIDUAL, true, s);
        if (panel_fc1) ln_project_panel(f, f->h, lw.ln2_g, lw.ln2_b, lw.p_fc1, lw.b_fc1, f->f, M, RW, EPI_BIAS_GELU, s);
        else {
            layernorm(f, f->h, lw.ln2_g, lw.ln2_b, f->a, M, s);
            project(f, SJD_PROF_GEMM_FC1, f->a, lw.w_fc1, lw.t_fc1, lw.b_fc1, f->f, M, RW, W, EPI_BIAS_GELU, false, s);
        }
        if (stream_fc2) {
            ProfScope ps(f, SJD_PROF_GEMM_RESID, 2.0 * M * (double)W * RW, (double)M * RW * 2.0 + (double)RW * W * 2.0 + (double)M * W * 8.0 + W * 4.0, s);
            if (c.dtype == SJD_DTYPE_BF16) launch_gemm_stream_resid<bf16>((const bf16 *)f->f, (const bf16 *)lw.p_fc2, lw.b_fc2, f->h, M, W, RW, s);
            else launch_gemm_stream_resid<f16>((const f16 *)f->f, (const f16 *)lw.p_fc2, lw.b_fc2, f->h, M, W, RW, s);
        } else project(f, SJD_PROF_GEMM_RESID, f->f, lw.w_fc2, lw.t_fc2, lw.b_fc2, f->h, M, W, RW, EPI_BIAS_RESIDUAL, true, s);
    }
    layernorm(f, f->h, bw.lnf_g, bw.lnf_b, f->a, M, s);
    project(f, SJD_PROF_GEMM_HEAD, f->a, bw.w_head, bw.t_head, bw.b_head, f->p, M, 2 * D, W, EPI_BIAS, true, s);
}

// One single-token step of the sequential inverse: position t of every sample goes through all
// layers against the key/value cache; the head output parameterises position t+1.
void decode_step(sjd_flow *f, int j, const float *z, float *x, int B, int t, hipStream_t s) {
    const sjd_config &c = f->cfg;
    const int T = c.seq_len, W = c.width, D = c.token_dim, RW = c.mlp_ratio * c.width;
    const int rev = (c.reverse_mask >> j) & 1;
    const BlockW &bw = f->block[j];
    const size_t ab = act_bytes(f);
    {
        ProfScope ps(f, SJD_PROF_OTHER, 2.0 * B * (double)D * W, (double)B * W * 4, s);
        launch_embed(x, bw.w_in, bw.b_in, bw.pos, f->h, B, D, W, RowMap{nullptr, 1, t, T, rev}, s);
    }
    for (int l = 0; l < c.n_layers; ++l) {
        const LayerW &lw = bw.layer[l];
        layernorm(f, f->h, lw.ln1_g, lw.ln1_b, f->a, B, s);
        project(f, SJD_PROF_DECODE_GEMM, f->a, lw.w_qkv, lw.t_qkv, lw.b_qkv, f->qkv, B, 3 * W, W, EPI_BIAS, false, s);
        {
            ProfScope ps(f, SJD_PROF_DECODE_ATTN, 4.0 * B * (double)(t + 1) * W,
                         (double)B * (2.0 * (t + 1) * W + 4.0 * W) * ab, s);
            if (c.dtype == SJD_DTYPE_BF16) attention_step<bf16>(f, l, B, t, s);
            else if (c.dtype == SJD_DTYPE_F16) attention_step<f16>(f, l, B, t, s);
            else attention_step<float>(f, l, B, t, s);
        }
        project(f, SJD_PROF_DECODE_GEMM, f->o, lw.w_o, lw.t_o, lw.b_o, f->h, B, W, W, EPI_BIAS_RESIDUAL, true, s);
        layernorm(f, f->h, lw.ln2_g, lw.ln2_b, f->a, B, s);
        project(f, SJD_PROF_DECODE_GEMM, f->a, lw.w_fc1, lw.t_fc1, lw.b_fc1, f->f, B, RW, W, EPI_BIAS_GELU, false, s);
        project(f, SJD_PROF_DECODE_GEMM, f->f, lw.w_fc2, lw.t_fc2, lw.b_fc2, f->h, B, W, RW, EPI_BIAS_RESIDUAL, true, s);
    }
    layernorm(f, f->h, bw.lnf_g, bw.lnf_b, f->a, B, s);
    project(f, SJD_PROF_DECODE_GEMM, f->a, bw.w_head, bw.t_head, bw.b_head, f->p, B, 2 * D, W, EPI_BIAS, true, s);
    {
        ProfScope ps(f, SJD_PROF_EPILOGUE, 0.0, (double)B * D * 16.0, s);
        launch_decode_epilogue(f->p, z, x, B, T, D, t, rev, s);
    }
}

int check_call(const sjd_flow *f, int block, const void *z, const void *x, int batch) {
    if (!f) return fail(SJD_EINVAL, "null flow handle");
    if (!f->loaded) return fail(SJD_ESTATE, "weights have not been loaded");
    if (!z || !x) return fail(SJD_EINVAL, "null device pointer");
    if (batch < 0 || batch > f->cfg.max_batch)
        return fail(SJD_EINVAL, "batch %d outside 0..max_batch=%d", batch, f->cfg.max_batch);
    if (block < 0 || block >= f->cfg.n_blocks) return fail(SJD_EINVAL, "block %d outside 0..%d", block, f->cfg.n_blocks - 1);
    const size_t n = (size_t)batch * f->cfg.seq_len * f->cfg.token_dim * sizeof(float);
    const char *a = (const char *)z, *b = (const char *)x;
    if (n && a < b + n && b < a + n) return fail(SJD_EINVAL, "input and output buffers overlap");
    return SJD_OK;
}

int check_opts(const sjd_jacobi_opts *o) {
    if (!o) return fail(SJD_EINVAL, "null options");
    if (o->tau != o->tau) return fail(SJD_EINVAL, "tau is NaN");
    if (o->criterion != 0 && o->criterion != 1) return fail(SJD_EINVAL, "criterion must be 0 or 1");
    if (o->init < 0 || o->init > 2) return fail(SJD_EINVAL, "init must be 0 (zeros), 1 (block input) or 2 (x_dev as passed)");
    if (o->max_iters < 0) return fail(SJD_EINVAL, "max_iters is negative");
    if (!(o->refine_below >= 0.f)) return fail(SJD_EINVAL, "refine_below is negative or NaN");
    return SJD_OK;
}

// Alg. 1 for one block.  iters_pin (pinned host, [batch]) receives per-sample pass counts.
// With `trace` every pass also records each sample's delta and (x_ref given) the l2 distance of its
// newest iterate to x_ref into f->trace.
// Float32 workspaces for refined passes of a 16-bit flow: about 8192 rows at a time.
int ensure_refine_workspace(sjd_flow *f) {
    if (f->r32_samples) return SJD_OK;
    const sjd_config &c = f->cfg;
    int n = 8192 / c.seq_len;
    n = n < 1 ? 1 : (n > c.max_batch ? c.max_batch : n);
    const size_t M = (size_t)n * c.seq_len, W = c.width, R = c.mlp_ratio;
    int rc;
    if ((rc = dev_alloc(f, &f->r32_a, M * W * 4)) || (rc = dev_alloc(f, &f->r32_qkv, M * 3 * W * 4)) ||
        (rc = dev_alloc(f, &f->r32_o, M * W * 4)) || (rc = dev_alloc(f, &f->r32_f, M * R * W * 4)))
        return rc;
    f->r32_samples = n;
    return SJD_OK;
}

// A whole-sequence conditioner pass of a 16-bit flow in float32 arithmetic: the float32 weights of the blob, the
// float32 kernels, float32 activations in the refinement workspaces.  n <= f->r32_samples.
void conditioner_pass_f32(sjd_flow *f, int j, const float *x, int n, const int32_t *active, hipStream_t s) {
    const int dtype = f->cfg.dtype;
    void *a = f->a, *qkv = f->qkv, *o = f->o, *ff = f->f, *panel = f->arena_panel;
    f->cfg.dtype = SJD_DTYPE_F32;
    f->a = f->r32_a; f->qkv = f->r32_qkv; f->o = f->r32_o; f->f = f->r32_f; f->arena_panel = nullptr;
    conditioner_pass(f, j, x, n, active, s);
    f->cfg.dtype = dtype;
    f->a = a; f->qkv = qkv; f->o = o; f->f = ff; f->arena_panel = panel;
}

int run_jacobi(sjd_flow *f, int j, const float *z, float *x, int batch, const sjd_jacobi_opts *opts, int *passes_out,
               bool *nonfinite_out, hipStream_t s, bool trace = false, const float *x_ref = nullptr) {
    const sjd_config &c = f->cfg;
    const int T = c.seq_len, D = c.token_dim;
    const int rev = (c.reverse_mask >> j) & 1;
    const int cap = (opts->max_iters > 0 && opts->max_iters < T) ? opts->max_iters : T;
    *passes_out = 0;
    *nonfinite_out = false;
    if (batch == 0) return SJD_OK;
    JacobiState st = f->st;
    st.active_in = f->active[0];
    st.active_out = f->active[1];
    launch_jacobi_init(z, x, st, batch, T, D, opts->init, s);
    // refinement: a sample marked fine (its delta fell below opts->refine_below) runs in float32 from then on;
    // the compaction puts those samples at the end of the list
    const float refine = c.dtype != SJD_DTYPE_F32 ? opts->refine_below : 0.f;
    if (refine > 0.f) { int rc = ensure_refine_workspace(f); if (rc) return rc; }
    int n_live = batch, n_listed = batch, n_fine = 0, passes = 0;
    while (n_live > 0 && passes < cap) {
        // Alg. 1 starts every sample from the same iterate, x^0 = 0, and the conditioner sees nothing else: the
        // parameters of the first pass are the same for all samples.  That pass therefore runs on the rows of one
        // sample (sample 0, still all zero) and its head output serves the whole batch - the same bits as running
        // it on every sample, since a row's result does not depend on which other rows are in the pass.
        const bool shared_first = passes == 0 && opts->init == 0 && n_listed > 1;
        auto update = [&](JacobiState part, int n, int shared) {
            ProfScope ps(f, SJD_PROF_EPILOGUE, 0.0, (double)n * T * D * 24.0, s);
            launch_jacobi_update(f->p, z, x, part, n, T, D, rev, opts->tau, opts->criterion, cap, shared, refine, s);
        };
        if (shared_first) {
            conditioner_pass(f, j, x, 1, nullptr, s);
            update(st, n_listed, 1);
        } else {
            const int n16 = n_listed - n_fine;
            if (n16 > 0) {
                conditioner_pass(f, j, x, n16, st.active_in, s);
                update(st, n16, 0);
            }
            for (int off = n16; off < n_listed; off += f->r32_samples) {
                const int n = n_listed - off < f->r32_samples ? n_listed - off : f->r32_samples;
                JacobiState part = st;
                part.active_in = st.active_in + off;
                conditioner_pass_f32(f, j, x, n, part.active_in, s);
                update(part, n, 0);
            }
        }
        launch_jacobi_compact(st, n_listed, opts->drop_converged ? 0 : 1, s);
        if (trace)
            launch_jacobi_trace(x, x_ref, st, f->trace + (size_t)passes * batch,
                                f->trace + ((size_t)T + passes) * batch, batch, T, D, s);
        HIP_TRY(hipMemcpyAsync(f->host_pin, st.n_active_out, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        HIP_TRY(hipGetLastError());
        n_live = f->host_pin[0];
        n_fine = f->host_pin[1];
        if (n_live < 0 || n_live > batch || n_fine < 0 || n_fine > n_live)
            return fail(SJD_EHIP, "active-sample counts %d, %d are out of range", n_live, n_fine);
        if (opts->drop_converged) n_listed = n_live;
        int32_t *t = st.active_in; st.active_in = st.active_out; st.active_out = t;
        ++passes;
    }
    HIP_TRY(hipMemcpyAsync(f->host_pin + 2, st.nonfinite, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipMemcpyAsync(f->host_pin + 3, st.iters, sizeof(int32_t) * batch, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    *passes_out = passes;
    *nonfinite_out = f->host_pin[2] != 0;
    return SJD_OK;
}

// ---- sequential fast path (16-bit modes, head size 64) ------------------------------------------
bool fast_decode_ok(const sjd_flow *f) {
    return f->cfg.dtype != SJD_DTYPE_F32 && f->cfg.width / f->cfg.n_heads == 64 && f->cfg.max_batch <= 256;
}
// Fragment-major operands: a width the fused LayerNorm projection covers.
bool frag_ok(const sjd_flow *f, int batch) {
    const int W = f->cfg.width;
    (void)batch;
    return fast_decode_ok(f) && (W == 256 || W == 512 || W == 768 || W == 1024);
}

// Launches of one step (all layers, head, advance) for position *t_dev, on stream s.
template <typename HT>
void fast_step(sjd_flow *f, int j, const float *z, float *x, int B, bool frag, hipStream_t s) {
    const sjd_config &c = f->cfg;
    const int T = c.seq_len, W = c.width, D = c.token_dim, H = c.n_heads, RW = c.mlp_ratio * c.width;
    const int rev = (c.reverse_mask >> j) & 1;
    const BlockW &bw = f->block[j];
    HT *a = (HT *)f->a, *qkv = (HT *)f->qkv, *o = (HT *)f->o, *ff = (HT *)f->f;
    const double wb = 2.0;
    auto gemm_bytes = [&](int N, int K, double outb) { return (double)K * N * wb + (double)B * K * wb + (double)B * N * outb; };
    // LayerNorm + projection: fused when the operands are fragment-major, else two launches
    auto ln_project = [&](const float *g, const float *be, const void *wt, const void *wf, const float *bias, void *out,
                          int N, Epi epi, bool out_f32) {
        ProfScope ps(f, out_f32 ? SJD_PROF_DECODE_HEAD : (epi == EPI_BIAS_GELU ? SJD_PROF_DECODE_FC1 : SJD_PROF_DECODE_GEMM),
                     2.0 * B * (double)N * W, gemm_bytes(N, W, out_f32 ? 4 : 2), s);
        if (frag) {
            bool ok = out_f32 ? launch_skinny_ln_gemm<HT, float>(f->h, g, be, (const HT *)wf, bias, (float *)out, B, N, W, epi, s)
                              : launch_skinny_ln_gemm<HT, HT>(f->h, g, be, (const HT *)wf, bias, (HT *)out, B, N, W, epi, s);
            (void)ok;  // frag_ok() admits only widths the fused kernel covers
        } else {
            launch_layernorm<HT>(f->h, g, be, a, B, W, s);
            if (out_f32) launch_skinny_gemm<HT, float>(a, (const HT *)wt, bias, nullptr, (float *)out, B, N, W, epi, false, s);
            else launch_skinny_gemm<HT, HT>(a, (const HT *)wt, bias, nullptr, (HT *)out, B, N, W, epi, false, s);
        }
    };
    for (int l = 0; l < c.n_layers; ++l) {
        const LayerW &lw = bw.layer[l];
        const size_t layer_off = (size_t)l * c.max_batch * T * W;
        ln_project(lw.ln1_g, lw.ln1_b, lw.t_qkv, lw.f_qkv, lw.b_qkv, qkv, 3 * W, EPI_BIAS, false);
        {
            // mean prefix length T/2: keys and values read once
            ProfScope ps(f, SJD_PROF_DECODE_ATTN, 4.0 * B * (T / 2.0) * W, (double)B * (T / 2.0) * W * 2 * wb, s);
            launch_decode_attention_h16<HT>(qkv, (HT *)f->kcache + layer_off, (HT *)f->vcache + layer_off, o, f->t_dev, B,
                                            T, H, frag, s);
        }
        {
            ProfScope ps(f, SJD_PROF_DECODE_RESID, 2.0 * B * (double)W * W, gemm_bytes(W, W, 8), s);
            launch_skinny_gemm<HT, float>(o, (const HT *)(frag ? lw.f_o : lw.t_o), lw.b_o, f->h, f->h, B, W, W,
                                          EPI_BIAS_RESIDUAL, frag, s);
        }
        ln_project(lw.ln2_g, lw.ln2_b, lw.t_fc1, lw.f_fc1, lw.b_fc1, ff, RW, EPI_BIAS_GELU, false);
        {
            ProfScope ps(f, SJD_PROF_DECODE_RESID, 2.0 * B * (double)RW * W, gemm_bytes(W, RW, 8), s);
            launch_skinny_gemm<HT, float>(ff, (const HT *)(frag ? lw.f_fc2 : lw.t_fc2), lw.b_fc2, f->h, f->h, B, W, RW,
                                          EPI_BIAS_RESIDUAL, frag, s);
        }
    }
    ln_project(bw.lnf_g, bw.lnf_b, bw.t_head, bw.f_head, bw.b_head, f->p, 2 * D, EPI_BIAS, true);
    {
        ProfScope ps(f, SJD_PROF_EPILOGUE, 0.0, (double)B * (D * 16.0 + W * 4.0), s);
        launch_decode_advance(f->p, z, x, bw.w_in, bw.b_in, bw.pos, f->h, f->t_dev, f->ticket, B, T, D, W, rev, 0, frag, s);
    }
}

void fast_step_any(sjd_flow *f, int j, const float *z, float *x, int B, bool frag, hipStream_t s) {
    if (f->cfg.dtype == SJD_DTYPE_BF16) fast_step<bf16>(f, j, z, x, B, frag, s);
    else fast_step<f16>(f, j, z, x, B, frag, s);
}

int run_sequential_fast(sjd_flow *f, int j, const float *z, float *x, int batch, hipStream_t s) {
    const sjd_config &c = f->cfg;
    const int T = c.seq_len, D = c.token_dim, W = c.width;
    const int rev = (c.reverse_mask >> j) & 1;
    const BlockW &bw = f->block[j];
    const bool frag = frag_ok(f, batch);
    launch_decode_advance(f->p, z, x, bw.w_in, bw.b_in, bw.pos, f->h, f->t_dev, f->ticket, batch, T, D, W, rev, 1, frag, s);
    if (T == 1) return SJD_OK;
    const bool eager = f->prof_mask != 0 || !f->use_graphs;
    if (eager) {
        for (int t = 0; t + 1 < T; ++t) fast_step_any(f, j, z, x, batch, frag, s);
        HIP_TRY(hipGetLastError());
        return SJD_OK;
    }
    hipGraphExec_t exec = nullptr;
    // a captured step holds z and x as kernel arguments, so they are part of the key
    auto key = std::make_tuple(j, batch, (const void *)z, (const void *)x);
    auto it = f->step_graphs.find(key);
    if (it != f->step_graphs.end()) {
        exec = it->second;
    } else {
        // captured on the handle's own stream: the caller's may be the legacy default stream, which
        // cannot be captured
        if (f->step_graphs.size() >= 64) {
            for (auto &kv : f->step_graphs) (void)hipGraphExecDestroy(kv.second);
            f->step_graphs.clear();
        }
        hipGraph_t graph = nullptr;
        HIP_TRY(hipStreamBeginCapture(f->cap_stream, hipStreamCaptureModeThreadLocal));
        fast_step_any(f, j, z, x, batch, frag, f->cap_stream);
        HIP_TRY(hipStreamEndCapture(f->cap_stream, &graph));
        hipError_t e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (e != hipSuccess) return fail(SJD_EHIP, "hipGraphInstantiate failed: %s", hipGetErrorString(e));
        f->step_graphs[key] = exec;
    }
    for (int t = 0; t + 1 < T; ++t) HIP_TRY(hipGraphLaunch(exec, s));
    return SJD_OK;
}

// The persistent kernel covers: 16-bit modes, head size 64, W in {256, 512, 768, 1024}, MLP ratio 4, batch <= 256,
// a cooperative launch of one workgroup per CU, and per-layer caches below 4 GiB (32-bit offsets).
bool persistent_ok(const sjd_flow *f, int batch) {
    const sjd_config &c = f->cfg;
    return frag_ok(f, batch) && f->coop && f->n_cus >= 8 && batch <= 256 && c.token_dim <= 64 && c.mlp_ratio == 4 && c.n_layers <= kSeqMaxLayers &&
           (size_t)c.max_batch * c.seq_len * c.width * 2 < ((size_t)1 << 32) &&
           seq_persistent_lds_bytes(batch <= 128 ? 1 : 2, c.seq_len, c.token_dim) <= 160 * 1024;
}

int run_sequential_persistent(sjd_flow *f, int j, const float *z, float *x, int batch, hipStream_t s) {
    const sjd_config &c = f->cfg;
    const BlockW &bw = f->block[j];
    const int MB = batch <= 128 ? 1 : 2;
    SeqArgs a{};
    a.n_layers = c.n_layers; a.ratio = c.mlp_ratio;
    for (int l = 0; l < c.n_layers; ++l) {
        const LayerW &lw = bw.layer[l];
        a.layers[l] = SeqLayer{lw.ln1_g, lw.ln1_b, lw.b_qkv, lw.b_o, lw.ln2_g, lw.ln2_b, lw.b_fc1, lw.b_fc2,
                               lw.f_qkv, lw.f_o, lw.f_fc1, lw.f_fc2};
    }
    a.lnf_g = bw.lnf_g; a.lnf_b = bw.lnf_b; a.b_head = bw.b_head; a.f_head = bw.f_head;
    a.w_in = bw.w_in; a.b_in = bw.b_in; a.pos = bw.pos;
    a.z = z; a.x = x;
    a.hs = f->h; a.qkv = f->qkv; a.o = f->o; a.ff = f->f; a.p = f->p;
    a.kcache = f->kcache; a.vcache = f->vcache;
    a.kv_layer_stride = (size_t)c.max_batch * c.seq_len * c.width;
    a.B = batch; a.T = c.seq_len; a.D = c.token_dim; a.reversed = (c.reverse_mask >> j) & 1;
    a.sync = f->psync;
    a.spin_max = 1 << 21;  // a poll takes ~0.5 us: about a second before a barrier gives up
    const double steps = c.seq_len - 1.0, W = c.width, R = c.mlp_ratio;
    const double wbytes = c.n_layers * (4.0 + 2.0 * R) * W * W * 2.0 + 2.0 * c.token_dim * W * 2.0;
    const double kvbytes = (double)c.n_layers * batch * (c.seq_len / 2.0) * W * 2.0 * 2.0;
    ProfScope ps(f, SJD_PROF_DECODE_FUSED, steps * 2.0 * batch * (c.n_layers * (4.0 + 2.0 * R) * W * W + 2.0 * c.token_dim * W) +
                                               steps * 4.0 * batch * (c.seq_len / 2.0) * W * c.n_layers,
                 steps * (wbytes + kvbytes), s);
    HIP_TRY(hipMemsetAsync(f->psync, 0, 1024 * sizeof(int), s));
    hipError_t e = launch_seq_persistent(c.dtype == SJD_DTYPE_BF16, a, MB, c.width / 256, f->n_cus, f->seq_path != 3, s);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        // e.g. the device cannot hold one workgroup per CU right now: nothing has run yet, so in
        // automatic mode the caller falls back to per-step launches
        fail(SJD_EHIP, "persistent sequential kernel: launch failed: %s", hipGetErrorString(e));
        return SJD_ELAUNCH_RETRY;
    }
    HIP_TRY(hipMemcpyAsync(f->host_pin, f->psync + 9, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipGetLastError());
    if (f->host_pin[0] != 0) {
        fail(SJD_EHIP, "persistent sequential kernel: %s",
             f->host_pin[0] == 2 ? "fewer XCD groups than planned for" : "a group barrier timed out");
        // every wave has left the kernel (bounded waits); z is untouched and x, the caches and the workspaces are
        // simply written again, so in automatic mode the caller runs the block by per-step launches instead
        return SJD_ELAUNCH_RETRY;
    }
    return SJD_OK;
}

int run_sequential(sjd_flow *f, int j, const float *z, float *x, int batch, hipStream_t s) {
    const int T = f->cfg.seq_len, D = f->cfg.token_dim;
    const int rev = (f->cfg.reverse_mask >> j) & 1;
    if (batch == 0) return SJD_OK;
    if (f->mask_nearest == 0) {   // the masked probe takes the plain per-step path below in every mode
        if (f->seq_path >= 2 && !persistent_ok(f, batch))
            return fail(SJD_EINVAL, "the persistent sequential kernel does not cover this configuration");
        // automatic choice: the persistent kernel, except for long sequences at the largest width, where its
        // attention stage (two pairs at a time per CU) and the eightfold weight traffic lose to per-step
        // launches (measured: T = 1024, W = 1024, 32 samples: 541 ms against 505 ms)
        const bool prefer_steps = f->seq_path == 0 && f->cfg.seq_len > 512 && f->cfg.width >= 1024;
        if (f->seq_path != 1 && !prefer_steps && persistent_ok(f, batch)) {
            const int rc = run_sequential_persistent(f, j, z, x, batch, s);
            if (rc != SJD_ELAUNCH_RETRY) return rc;
            if (f->seq_path != 0) return SJD_EHIP;      // the persistent kernel was asked for explicitly
        }
        if (fast_decode_ok(f)) return run_sequential_fast(f, j, z, x, batch, s);
    }
    launch_decode_epilogue(f->p, z, x, batch, T, D, -1, rev, s);  // x_1 = y_1
    for (int t = 0; t + 1 < T; ++t) decode_step(f, j, z, x, batch, t, s);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

}  // namespace

// ================================================================================================
extern "C" {

const char *sjd_last_error(void) { return g_err; }

int sjd_flow_create(const sjd_config *cfg, sjd_flow **out) {
    if (!cfg || !out) return fail(SJD_EINVAL, "null argument");
    *out = nullptr;
    const sjd_config &c = *cfg;
    if (c.n_blocks < 1 || c.n_blocks > SJD_MAX_BLOCKS) return fail(SJD_EINVAL, "n_blocks must be 1..%d", SJD_MAX_BLOCKS);
    if (c.n_layers < 1 || c.width < 1 || c.n_heads < 1 || c.mlp_ratio < 1 || c.seq_len < 1 || c.token_dim < 1 ||
        c.max_batch < 1)
        return fail(SJD_EINVAL, "all sizes must be positive");
    if (c.width % c.n_heads) return fail(SJD_EINVAL, "width %d is not a multiple of n_heads %d", c.width, c.n_heads);
    if (c.width % 4) return fail(SJD_EINVAL, "width %d is not a multiple of 4", c.width);
    if (c.dtype != SJD_DTYPE_F32 && c.dtype != SJD_DTYPE_BF16 && c.dtype != SJD_DTYPE_F16)
        return fail(SJD_EINVAL, "unknown dtype %d", c.dtype);
    if (c.dtype != SJD_DTYPE_F32 && c.width % 64) return fail(SJD_EINVAL, "16-bit modes need width %% 64 == 0");
    if (c.seq_len > 4096) return fail(SJD_EINVAL, "seq_len above 4096 is not supported");
    if (c.token_dim > 1024) return fail(SJD_EINVAL, "token_dim above 1024 is not supported");
    if ((double)c.max_batch * c.seq_len > 1.0e9) return fail(SJD_EINVAL, "max_batch * seq_len is too large");

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(SJD_EHIP, "no HIP device is available");
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(SJD_EHIP, "device %d is %s; this library is built for gfx950 only", dev, prop.gcnArchName);

    sjd_flow *f = new (std::nothrow) sjd_flow();
    if (!f) return fail(SJD_ENOMEM, "host allocation failed");
    f->cfg = c;
    f->device = dev;
    const size_t T = c.seq_len, W = c.width, D = c.token_dim, R = c.mlp_ratio, B = c.max_batch, N = c.n_layers;
    const size_t M = B * T > 512 ? B * T : 512, ab = act_bytes(f);  // the single-token paths work on up to 8 x 32 rows; the persistent kernel keeps two copies of its residual stream
    int rc = SJD_OK;
    auto A = [&](void **p, size_t n) { if (rc == SJD_OK) rc = dev_alloc(f, p, n); };
    A((void **)&f->blob, (size_t)c.n_blocks * block_floats(c) * sizeof(float));
    if (c.dtype != SJD_DTYPE_F32) A(&f->arena, (size_t)c.n_blocks * arena_elems_per_block(c) * 2);
    if (fast_decode_ok(f)) A(&f->arena_frag, (size_t)c.n_blocks * arena_elems_per_block(c) * 2);
    if (panel_ok(c)) A(&f->arena_panel, (size_t)c.n_blocks * c.n_layers * (3 * W + W + 2 * R * W) * W * 2);
    A((void **)&f->h, M * W * 4);
    A((void **)&f->p, M * 2 * D * 4);
    A(&f->a, M * W * ab);
    A(&f->qkv, M * 3 * W * ab);
    A(&f->o, M * W * ab);
    A(&f->f, M * R * W * ab);
    A(&f->kcache, N * B * T * W * ab);
    A(&f->vcache, N * B * T * W * ab);
    A((void **)&f->pp[0], M * D * 4);
    A((void **)&f->pp[1], M * D * 4);
    A((void **)&f->st.delta, B * 4);
    A((void **)&f->st.iters, B * 4);
    A((void **)&f->st.done, B * 4);
    A((void **)&f->st.nonfinite, 4);
    A((void **)&f->st.n_active_out, 8);
    A((void **)&f->st.fine, B * 4);
    A((void **)&f->active[0], B * 4);
    A((void **)&f->active[1], B * 4);
    A((void **)&f->trace, 2 * T * B * 4);
    A((void **)&f->psync, 1024 * sizeof(int));
    {
        hipDeviceProp_t prop;
        if (rc == SJD_OK && hipGetDeviceProperties(&prop, f->device) == hipSuccess) {
            f->n_cus = f->n_cus_device = prop.multiProcessorCount;
            f->coop = prop.cooperativeLaunch;
        }
    }
    f->st.ticket = nullptr;
    A((void **)&f->t_dev, 4);
    A((void **)&f->ticket, 4);
    if (rc == SJD_OK && hipMemset(f->ticket, 0, 4) != hipSuccess) rc = fail(SJD_EHIP, "hipMemset failed");
    if (rc == SJD_OK && hipStreamCreateWithFlags(&f->cap_stream, hipStreamNonBlocking) != hipSuccess)
        rc = fail(SJD_EHIP, "hipStreamCreate failed");
    if (rc == SJD_OK && hipHostMalloc((void **)&f->host_pin, (B + 3) * sizeof(int32_t)) != hipSuccess)
        rc = fail(SJD_ENOMEM, "pinned host allocation failed");
    for (int i = 0; rc == SJD_OK && i <= c.n_blocks; ++i)
        if (hipEventCreate(&f->ev[i]) != hipSuccess) rc = fail(SJD_EHIP, "hipEventCreate failed");
    if (rc != SJD_OK) { sjd_flow_destroy(f); return rc; }
    *out = f;
    return SJD_OK;
}

void sjd_flow_destroy(sjd_flow *f) {
    if (!f) return;
    (void)hipDeviceSynchronize();
    for (auto &kv : f->step_graphs) (void)hipGraphExecDestroy(kv.second);
    if (f->cap_stream) (void)hipStreamDestroy(f->cap_stream);
    for (void *p : f->allocs) (void)hipFree(p);
    if (f->host_pin) (void)hipHostFree(f->host_pin);
    for (auto &e : f->ev) if (e) (void)hipEventDestroy(e);
    for (auto &sp : f->spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
    for (auto &e : f->free_events) (void)hipEventDestroy(e);
    delete f;
}

size_t sjd_flow_device_bytes(const sjd_flow *f) { return f ? f->bytes : 0; }

int sjd_flow_load_weights(sjd_flow *f, const void *host_blob, size_t nbytes) {
    if (!f || !host_blob) return fail(SJD_EINVAL, "null argument");
    const sjd_config &c = f->cfg;
    const size_t bf = block_floats(c);
    const size_t want = (size_t)c.n_blocks * bf * sizeof(float);
    if (nbytes != want) return fail(SJD_EINVAL, "weight blob has %zu bytes, the configuration implies %zu", nbytes, want);
    HIP_TRY(hipMemcpy(f->blob, host_blob, nbytes, hipMemcpyHostToDevice));
    const size_t D = c.token_dim, W = c.width, T = c.seq_len, R = c.mlp_ratio;
    const int dt = c.dtype;
    f->block.assign(c.n_blocks, BlockW());
    char *ar = (char *)f->arena;
    auto prep = [&](const float *src, size_t K, size_t N) -> void * {  // [K, N] float -> [N padded, K] 16-bit
        if (dt == SJD_DTYPE_F32) return nullptr;
        void *dst = ar;
        const size_t rows = round_up(N, kNPad);
        if (dt == SJD_DTYPE_BF16) launch_transpose_to_h16<bf16>(src, (bf16 *)dst, (int)K, (int)N, (int)K, (int)rows, 0);
        else launch_transpose_to_h16<f16>(src, (f16 *)dst, (int)K, (int)N, (int)K, (int)rows, 0);
        ar += rows * K * 2;
        return dst;
    };
    char *arf = (char *)f->arena_frag;
    auto prep_frag = [&](const float *src, size_t K, size_t N) -> void * {  // fragment-major 16-bit copy
        if (!f->arena_frag) return nullptr;
        void *dst = arf;
        const size_t rows = round_up(N, kNPad);
        if (dt == SJD_DTYPE_BF16) launch_weights_to_frag<bf16>(src, (bf16 *)dst, (int)K, (int)N, (int)rows, 0);
        else launch_weights_to_frag<f16>(src, (f16 *)dst, (int)K, (int)N, (int)rows, 0);
        arf += rows * K * 2;
        return dst;
    };
    char *arp = (char *)f->arena_panel;
    auto prep_panel = [&](const void *wt, size_t N) -> void * {   // from the transposed 16-bit copy
        if (!f->arena_panel) return nullptr;
        void *dst = arp;
        if (dt == SJD_DTYPE_BF16) launch_weights_to_panel_frag<bf16>((const bf16 *)wt, (bf16 *)dst, (int)N, 0);
        else launch_weights_to_panel_frag<f16>((const f16 *)wt, (f16 *)dst, (int)N, 0);
        arp += N * W * 2;
        return dst;
    };
    for (int j = 0; j < c.n_blocks; ++j) {
        const float *p = f->blob + (size_t)j * bf;
        BlockW &bw = f->block[j];
        bw.w_in = p; p += D * W;
        bw.b_in = p; p += W;
        bw.pos = p; p += T * W;
        bw.layer.resize(c.n_layers);
        for (int l = 0; l < c.n_layers; ++l) {
            LayerW &lw = bw.layer[l];
            lw.ln1_g = p; p += W;
            lw.ln1_b = p; p += W;
            lw.w_qkv = p; p += W * 3 * W;
            lw.b_qkv = p; p += 3 * W;
            lw.w_o = p; p += W * W;
            lw.b_o = p; p += W;
            lw.ln2_g = p; p += W;
            lw.ln2_b = p; p += W;
            lw.w_fc1 = p; p += W * R * W;
            lw.b_fc1 = p; p += R * W;
            lw.w_fc2 = p; p += R * W * W;
            lw.b_fc2 = p; p += W;
            lw.t_qkv = prep(lw.w_qkv, W, 3 * W);
            lw.t_o = prep(lw.w_o, W, W);
            lw.t_fc1 = prep(lw.w_fc1, W, R * W);
            lw.t_fc2 = prep(lw.w_fc2, R * W, W);
            lw.f_qkv = prep_frag(lw.w_qkv, W, 3 * W);
            lw.f_o = prep_frag(lw.w_o, W, W);
            lw.f_fc1 = prep_frag(lw.w_fc1, W, R * W);
            lw.f_fc2 = prep_frag(lw.w_fc2, R * W, W);
            lw.p_qkv = prep_panel(lw.t_qkv, 3 * W);
            lw.p_o = prep_panel(lw.t_o, W);
            lw.p_fc1 = prep_panel(lw.t_fc1, R * W);
            if (f->arena_panel) {                       // MLP output: [W, R W] transposed -> fragment order, k = R W
                lw.p_fc2 = arp;
                if (dt == SJD_DTYPE_BF16) launch_weights_to_frag32<bf16>((const bf16 *)lw.t_fc2, (bf16 *)arp, (int)W, (int)(R * W), 0);
                else launch_weights_to_frag32<f16>((const f16 *)lw.t_fc2, (f16 *)arp, (int)W, (int)(R * W), 0);
                arp += W * R * W * 2;
            }
        }
        bw.lnf_g = p; p += W;
        bw.lnf_b = p; p += W;
        bw.w_head = p; p += W * 2 * D;
        bw.b_head = p;
        bw.t_head = prep(bw.w_head, W, 2 * D);
        bw.f_head = prep_frag(bw.w_head, W, 2 * D);
    }
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipGetLastError());
    f->stream_ok = false;
    if (f->arena_panel) {
        int rc = stream_self_check(f);
        if (rc) return rc;
    }
    f->loaded = true;
    return SJD_OK;
}

int sjd_conditioner(sjd_flow *f, int block, const float *x_dev, float *mu_dev, float *alpha_dev, int batch,
                    void *hip_stream) {
    int rc = check_call(f, block, x_dev, mu_dev, batch);
    if (rc) return rc;
    if (!alpha_dev) return fail(SJD_EINVAL, "null device pointer");
    if ((rc = check_call(f, block, x_dev, alpha_dev, batch))) return rc;
    if ((rc = check_call(f, block, mu_dev, alpha_dev, batch))) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(hipSetDevice(f->device));
    conditioner_pass(f, block, x_dev, batch, nullptr, s);
    launch_split_params(f->p, mu_dev, alpha_dev, batch, f->cfg.seq_len, f->cfg.token_dim,
                        (f->cfg.reverse_mask >> block) & 1, s);
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_jacobi_inverse_block(sjd_flow *f, int block, const float *z_dev, float *x_dev, int batch,
                             const sjd_jacobi_opts *opts, int32_t *iters_per_sample_host, int32_t *block_iters_host,
                             void *hip_stream) {
    int rc = check_call(f, block, z_dev, x_dev, batch);
    if (rc) return rc;
    if ((rc = check_opts(opts))) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(hipSetDevice(f->device));
    int passes = 0;
    bool nonfinite = false;
    if ((rc = run_jacobi(f, block, z_dev, x_dev, batch, opts, &passes, &nonfinite, s))) return rc;
    if (iters_per_sample_host) memcpy(iters_per_sample_host, f->host_pin + 3, sizeof(int32_t) * batch);
    if (block_iters_host) *block_iters_host = passes;
    if (nonfinite) return fail(SJD_ENONFINITE, "block %d: a sample ended with a non-finite difference norm", block);
    return SJD_OK;
}

int sjd_sequential_inverse_block(sjd_flow *f, int block, const float *z_dev, float *x_dev, int batch,
                                 void *hip_stream) {
    int rc = check_call(f, block, z_dev, x_dev, batch);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(hipSetDevice(f->device));
    if ((rc = run_sequential(f, block, z_dev, x_dev, batch, s))) return rc;
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_sample(sjd_flow *f, const float *z_dev, float *x_dev, int batch, uint32_t jacobi_mask,
               const sjd_jacobi_opts *opts, sjd_stats *stats_host, int32_t *iters_host, void *hip_stream) {
    int rc = check_call(f, 0, z_dev, x_dev, batch);
    if (rc) return rc;
    const sjd_config &c = f->cfg;
    uint32_t used = c.n_blocks >= 32 ? 0xFFFFFFFFu : ((1u << c.n_blocks) - 1u);
    if ((jacobi_mask & used) && (rc = check_opts(opts))) return rc;
    if ((jacobi_mask & used) && opts->init == 2)
        return fail(SJD_EINVAL, "init 2 (caller's first iterate) is for single-block calls");
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(hipSetDevice(f->device));
    if (stats_host) memset(stats_host, 0, sizeof(*stats_host));
    const int T = c.seq_len;
    bool any_nonfinite = false;
    const float *in = z_dev;
    HIP_TRY(hipEventRecord(f->ev[0], s));
    for (int j = 0; j < c.n_blocks; ++j) {
        float *out = (j == c.n_blocks - 1) ? x_dev : f->pp[j & 1];
        if ((jacobi_mask >> j) & 1u) {
            int passes = 0;
            bool nonfinite = false;
            if ((rc = run_jacobi(f, j, in, out, batch, opts, &passes, &nonfinite, s))) return rc;
            any_nonfinite |= nonfinite;
            double sum = 0;
            for (int b = 0; b < batch; ++b) sum += f->host_pin[3 + b];
            if (iters_host) memcpy(iters_host + (size_t)j * batch, f->host_pin + 3, sizeof(int32_t) * batch);
            if (stats_host) {
                stats_host->block_iters[j] = passes;
                stats_host->mean_sample_iters[j] = batch ? (float)(sum / batch) : 0.f;
            }
        } else {
            if ((rc = run_sequential(f, j, in, out, batch, s))) return rc;
            if (iters_host) for (int b = 0; b < batch; ++b) iters_host[(size_t)j * batch + b] = T - 1;
            if (stats_host) { stats_host->block_iters[j] = T - 1; stats_host->mean_sample_iters[j] = (float)(T - 1); }
        }
        HIP_TRY(hipEventRecord(f->ev[j + 1], s));
        in = out;
    }
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipGetLastError());
    if (stats_host)
        for (int j = 0; j < c.n_blocks; ++j) HIP_TRY(hipEventElapsedTime(&stats_host->block_ms[j], f->ev[j], f->ev[j + 1]));
    if (any_nonfinite) return fail(SJD_ENONFINITE, "a sample ended a Jacobi block with a non-finite difference norm");
    return SJD_OK;
}

int sjd_jacobi_trace_block(sjd_flow *f, int block, const float *z_dev, float *x_dev, const float *x_ref_dev, int batch,
                           const sjd_jacobi_opts *opts, float *delta_trace_host, float *err_trace_host,
                           int32_t *iters_per_sample_host, int32_t *block_iters_host, void *hip_stream) {
    int rc = check_call(f, block, z_dev, x_dev, batch);
    if (rc) return rc;
    if ((rc = check_opts(opts))) return rc;
    if (!delta_trace_host) return fail(SJD_EINVAL, "null trace buffer");
    if (err_trace_host && !x_ref_dev) return fail(SJD_EINVAL, "an error trace needs the reference solution");
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(hipSetDevice(f->device));
    const int T = f->cfg.seq_len;
    int passes = 0;
    bool nonfinite = false;
    if ((rc = run_jacobi(f, block, z_dev, x_dev, batch, opts, &passes, &nonfinite, s, true, x_ref_dev))) return rc;
    if (passes > 0 && batch > 0) {
        HIP_TRY(hipMemcpyAsync(delta_trace_host, f->trace, sizeof(float) * passes * batch, hipMemcpyDeviceToHost, s));
        if (err_trace_host)
            HIP_TRY(hipMemcpyAsync(err_trace_host, f->trace + (size_t)T * batch, sizeof(float) * passes * batch,
                                   hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
    }
    if (block_iters_host) *block_iters_host = passes;
    if (iters_per_sample_host) memcpy(iters_per_sample_host, f->host_pin + 3, sizeof(int32_t) * batch);
    if (nonfinite) return fail(SJD_ENONFINITE, "block %d: a sample ended with a non-finite difference norm", block);
    return SJD_OK;
}

int sjd_forward_block(sjd_flow *f, int block, const float *x_dev, float *y_dev, float *logdet_dev, int accumulate,
                      int batch, void *hip_stream) {
    int rc = check_call(f, block, x_dev, y_dev, batch);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(hipSetDevice(f->device));
    if (batch > 0) {
        conditioner_pass(f, block, x_dev, batch, nullptr, s);
        ProfScope ps(f, SJD_PROF_EPILOGUE, 0.0, (double)batch * f->cfg.seq_len * f->cfg.token_dim * 16.0, s);
        launch_forward_epilogue(f->p, x_dev, y_dev, logdet_dev, batch, f->cfg.seq_len, f->cfg.token_dim,
                                (f->cfg.reverse_mask >> block) & 1, accumulate ? 1 : 0, s);
    }
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_forward(sjd_flow *f, const float *x_dev, float *z_dev, float *logdet_dev, int batch, void *hip_stream) {
    int rc = check_call(f, 0, x_dev, z_dev, batch);
    if (rc) return rc;
    const sjd_config &c = f->cfg;
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(hipSetDevice(f->device));
    const float *in = x_dev;
    for (int j = c.n_blocks - 1; j >= 0 && batch > 0; --j) {
        float *out = (j == 0) ? z_dev : f->pp[j & 1];
        conditioner_pass(f, j, in, batch, nullptr, s);
        ProfScope ps(f, SJD_PROF_EPILOGUE, 0.0, (double)batch * c.seq_len * c.token_dim * 16.0, s);
        launch_forward_epilogue(f->p, in, out, logdet_dev, batch, c.seq_len, c.token_dim, (c.reverse_mask >> j) & 1,
                                j != c.n_blocks - 1, s);
        in = out;
    }
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_op_linear_h16(int dtype, int kernel, const void *a_dev, const void *wt_dev, const float *bias_dev,
                      float *resid_out_dev, void *c_dev, int M, int N, int K, int epilogue, void *hip_stream) {
    if (!a_dev || !wt_dev || !bias_dev) return fail(SJD_EINVAL, "null device pointer");
    if (dtype != SJD_DTYPE_BF16 && dtype != SJD_DTYPE_F16) return fail(SJD_EINVAL, "dtype must be a 16-bit mode");
    if (M < 1 || N < 1 || K < 64 || K % 64) return fail(SJD_EINVAL, "need M, N >= 1 and K a positive multiple of 64");
    if (kernel < 0 || kernel > 4) return fail(SJD_EINVAL, "kernel must be 0..4");
    if (epilogue < 0 || epilogue > 2) return fail(SJD_EINVAL, "epilogue must be 0..2");
    if (epilogue == 2 ? !resid_out_dev : !c_dev) return fail(SJD_EINVAL, "null output pointer");
    hipStream_t s = (hipStream_t)hip_stream;
    const Epi epi = (Epi)epilogue;
    if (dtype == SJD_DTYPE_BF16) {
        if (epilogue == 2) launch_gemm_h16<bf16, float>((const bf16 *)a_dev, (const bf16 *)wt_dev, bias_dev, resid_out_dev, resid_out_dev, M, N, K, epi, s, kernel);
        else launch_gemm_h16<bf16, bf16>((const bf16 *)a_dev, (const bf16 *)wt_dev, bias_dev, nullptr, (bf16 *)c_dev, M, N, K, epi, s, kernel);
    } else {
        if (epilogue == 2) launch_gemm_h16<f16, float>((const f16 *)a_dev, (const f16 *)wt_dev, bias_dev, resid_out_dev, resid_out_dev, M, N, K, epi, s, kernel);
        else launch_gemm_h16<f16, f16>((const f16 *)a_dev, (const f16 *)wt_dev, bias_dev, nullptr, (f16 *)c_dev, M, N, K, epi, s, kernel);
    }
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

namespace {

int panel_linear_check(int dtype, const void *a_dev, const float *ln_g_dev, const float *ln_b_dev, const void *wt_dev,
                       const float *bias_dev, float *resid_out_dev, void *c_dev, int M, int N, int K, int epilogue) {
    if (!a_dev || !wt_dev || !bias_dev) return fail(SJD_EINVAL, "null device pointer");
    if (dtype != SJD_DTYPE_BF16 && dtype != SJD_DTYPE_F16) return fail(SJD_EINVAL, "dtype must be a 16-bit mode");
    if (epilogue < 0 || epilogue > 2) return fail(SJD_EINVAL, "epilogue must be 0..2");
    if (epilogue == 2 ? !resid_out_dev : (!c_dev || !ln_g_dev || !ln_b_dev)) return fail(SJD_EINVAL, "null device pointer");
    const bool stream = epilogue == 2 && K > 512;
    if (stream ? !gemm_stream_applicable(M, N, K) : !gemm_panel_applicable(M, N, K, epilogue == 2 ? 4 : 2))
        return fail(SJD_EINVAL, "need M >= 1, N a multiple of 256, K = 512 (or, residual variant, a multiple of 512) and operands below 2 GiB");
    if (epilogue == 2 && K == 512 && N > 512) return fail(SJD_EINVAL, "the residual variant with K = 512 covers N <= 512");
    return SJD_OK;
}

// The op itself: reorders the weight into `wf` (device, 2 N K bytes, every byte written before it is read) and
// launches the projection.  Asynchronous on s; allocates nothing.
void panel_linear_run(int dtype, const void *a_dev, const float *ln_g_dev, const float *ln_b_dev, const void *wt_dev,
                      const float *bias_dev, float *resid_out_dev, void *c_dev, int M, int N, int K, int epilogue,
                      void *wf, hipStream_t s) {
    const bool stream = epilogue == 2 && K > 512;
    if (dtype == SJD_DTYPE_BF16) {
        launch_weights_to_frag32<bf16>((const bf16 *)wt_dev, (bf16 *)wf, N, K, s);
        if (stream) launch_gemm_stream_resid<bf16>((const bf16 *)a_dev, (const bf16 *)wf, bias_dev, resid_out_dev, M, N, K, s);
        else if (epilogue == 2) launch_gemm_panel_resid<bf16>((const bf16 *)a_dev, (const bf16 *)wf, bias_dev, resid_out_dev, M, N, s);
        else launch_ln_gemm_panel<bf16>((const float *)a_dev, ln_g_dev, ln_b_dev, (const bf16 *)wf, bias_dev, (bf16 *)c_dev, M, N, (Epi)epilogue, s);
    } else {
        launch_weights_to_frag32<f16>((const f16 *)wt_dev, (f16 *)wf, N, K, s);
        if (stream) launch_gemm_stream_resid<f16>((const f16 *)a_dev, (const f16 *)wf, bias_dev, resid_out_dev, M, N, K, s);
        else if (epilogue == 2) launch_gemm_panel_resid<f16>((const f16 *)a_dev, (const f16 *)wf, bias_dev, resid_out_dev, M, N, s);
        else launch_ln_gemm_panel<f16>((const float *)a_dev, ln_g_dev, ln_b_dev, (const f16 *)wf, bias_dev, (f16 *)c_dev, M, N, (Epi)epilogue, s);
    }
}

}  // namespace

int sjd_op_panel_linear_h16(int dtype, const void *a_dev, const float *ln_g_dev, const float *ln_b_dev,
                            const void *wt_dev, const float *bias_dev, float *resid_out_dev, void *c_dev, int M, int N,
                            int K, int epilogue, void *hip_stream) {
    int rc = panel_linear_check(dtype, a_dev, ln_g_dev, ln_b_dev, wt_dev, bias_dev, resid_out_dev, c_dev, M, N, K, epilogue);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    void *wf = nullptr;
    HIP_TRY(hipMalloc(&wf, (size_t)N * K * 2));
    panel_linear_run(dtype, a_dev, ln_g_dev, ln_b_dev, wt_dev, bias_dev, resid_out_dev, c_dev, M, N, K, epilogue, wf, s);
    const hipError_t e1 = hipStreamSynchronize(s), e2 = hipGetLastError();
    (void)hipFree(wf);
    HIP_TRY(e1);
    HIP_TRY(e2);
    return SJD_OK;
}

// ---- the same op for callers that cannot allocate ------------------------------------------------
// The fragment-order weight copy, which sjd_op_panel_linear_h16 allocates per call, lives in a file-scope
// device array here.  In host code the array's name is only a stand-in: its device address is looked up
// once per device (each GPU holds its own copy at its own address) and that pointer is what the kernels get.
#define SJD_NOALLOC_SCRATCH_BYTES (4u << 20)
static __device__ __align__(256) unsigned char scratch[SJD_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device; resolved on the first call per device.
int scratch_address(void **out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(SJD_EINVAL, "device index %d is outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(SJD_EHIP, "hipGetSymbolAddress returned a null address for the scratch array");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SJD_OK;
}
}  // namespace

int sjd_op_panel_linear_h16_noalloc(int dtype, const void *a_dev, const float *ln_g_dev, const float *ln_b_dev,
                                    const void *wt_dev, const float *bias_dev, float *resid_out_dev, void *c_dev, int M,
                                    int N, int K, int epilogue, void *hip_stream) {
    int rc = panel_linear_check(dtype, a_dev, ln_g_dev, ln_b_dev, wt_dev, bias_dev, resid_out_dev, c_dev, M, N, K, epilogue);
    if (rc) return rc;
    if ((size_t)N * K * 2 > SJD_NOALLOC_SCRATCH_BYTES)
        return fail(SJD_EINVAL, "the weight (%d x %d, %zu bytes in 16 bits) exceeds the %u-byte scratch of the non-allocating op",
                    N, K, (size_t)N * K * 2, SJD_NOALLOC_SCRATCH_BYTES);
    void *wf = nullptr;
    if ((rc = scratch_address(&wf))) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    // every byte of the copy that the projection reads is rewritten by the reorder kernel in front of it:
    // nothing of the previous call's contents is used, so nothing needs clearing
    panel_linear_run(dtype, a_dev, ln_g_dev, ln_b_dev, wt_dev, bias_dev, resid_out_dev, c_dev, M, N, K, epilogue, wf, s);
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_op_attention_h16(int dtype, const void *qkv_dev, void *o_dev, int n_samples, int T, int H, void *hip_stream) {
    if (!qkv_dev || !o_dev) return fail(SJD_EINVAL, "null device pointer");
    if (dtype != SJD_DTYPE_BF16 && dtype != SJD_DTYPE_F16 && dtype != SJD_DTYPE_F32) return fail(SJD_EINVAL, "unknown dtype %d", dtype);
    if (n_samples < 1 || T < 1 || T > 4096 || H < 1 || H > 65535 || n_samples > 65535)
        return fail(SJD_EINVAL, "need 1 <= n_samples, H <= 65535 and 1 <= T <= 4096");
    hipStream_t s = (hipStream_t)hip_stream;
    if (dtype == SJD_DTYPE_F32) launch_flash_attention_f32((const float *)qkv_dev, (float *)o_dev, n_samples, T, H, s);
    else if (dtype == SJD_DTYPE_BF16) launch_flash_attention_h16<bf16>((const bf16 *)qkv_dev, (bf16 *)o_dev, n_samples, T, H, s);
    else launch_flash_attention_h16<f16>((const f16 *)qkv_dev, (f16 *)o_dev, n_samples, T, H, s);
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

#ifdef SJD_SEQ_TIMELINE
extern "C" __attribute__((visibility("default"))) int sjd_debug_read_sync(sjd_flow *f, int *out1024) {
    return hipMemcpy(out1024, f->psync, 1024 * sizeof(int), hipMemcpyDeviceToHost) == hipSuccess ? 0 : -1;
}
#endif

int sjd_flow_set_projection_path(sjd_flow *f, int path) {
    if (!f) return fail(SJD_EINVAL, "null flow");
    if (path < 0 || path > 2) return fail(SJD_EINVAL, "the projection path must be 0 (automatic), 1 (tile kernels) or 2 (panel kernels)");
    if (path == 2 && !f->arena_panel) return fail(SJD_EINVAL, "the panel kernels cover 16-bit flows of width 512 only");
    f->proj_path = path;
    return SJD_OK;
}

int sjd_flow_set_mask_nearest(sjd_flow *f, int o) {
    if (!f) return fail(SJD_EINVAL, "null flow");
    if (o < 0 || o > f->cfg.seq_len) return fail(SJD_EINVAL, "the mask offset must lie in 0..T");
    f->mask_nearest = o;
    return SJD_OK;
}

int sjd_flow_set_sequential_path(sjd_flow *f, int path) {
    if (!f) return fail(SJD_EINVAL, "null flow");
    if (path < 0 || path > 3)
        return fail(SJD_EINVAL, "path must be 0 (automatic), 1 (per-step launches), 2 (persistent kernel) or 3 (the same, plain launch)");
    f->seq_path = path;
    return SJD_OK;
}

int sjd_flow_set_sequential_cus(sjd_flow *f, int n_cus) {
    if (!f) return fail(SJD_EINVAL, "null flow");
    if (n_cus != 0 && (n_cus < 32 || n_cus > f->n_cus_device || n_cus % 32))
        return fail(SJD_EINVAL, "the persistent kernel's workgroup count must be 0 (one per CU of the device) or a multiple of 32 in 32..%d",
                    f->n_cus_device);
    f->n_cus = n_cus ? n_cus : f->n_cus_device;
    return SJD_OK;
}

int sjd_profile_enable(sjd_flow *f, uint32_t family_mask) {
    if (!f) return fail(SJD_EINVAL, "null flow handle");
    f->prof_mask = family_mask & ((1u << SJD_PROF_FAMILIES) - 1u);
    return SJD_OK;
}

int sjd_profile_read(sjd_flow *f, sjd_profile *out_host, int reset) {
    if (!f || !out_host) return fail(SJD_EINVAL, "null argument");
    int rc = drain_profile(f);
    if (rc) return rc;
    *out_host = f->prof;
    if (reset) memset(&f->prof, 0, sizeof(f->prof));
    return SJD_OK;
}

}  // extern "C"
