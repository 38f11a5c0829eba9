"""The activation-stationary projection kernels (LayerNorm + projection in one launch, K = 512)
against the CPU oracle's `layernorm`, `linear` and `gelu` in float64, and against the tile kernels
they replace in the whole-sequence passes of a width-512 flow (same bits).  Needs an MI355X.

Row counts span one to many 128-row panels with ragged tails; column counts give one to four column
groups per workgroup and every split of the groups over workgroups."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

K = 512
# (M, N): N / 256 = 1, 2, 3, 6, 8 column groups; M from less than a panel to 160 panels
SHAPES = [(77, 256), (300, 512), (128, 768), (1000, 1536), (2049, 2048), (4173, 1536), (20480, 512)]


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _operands(torch, M, N, dtype, seed):
    g = np.random.default_rng(seed)
    x = (g.standard_normal((M, K)) * g.uniform(0.5, 3.0, (M, 1)) + g.standard_normal((M, 1))).astype(np.float32)
    ln_g = (1.0 + 0.1 * g.standard_normal(K)).astype(np.float32)
    ln_b = (0.1 * g.standard_normal(K)).astype(np.float32)
    w = torch.from_numpy((g.standard_normal((K, N)) * 0.05).astype(np.float32)).to(dtype)
    bias = (g.standard_normal(N) * 0.1).astype(np.float32)
    wt = torch.zeros(((N + 255) // 256 * 256, K), dtype=dtype)
    wt[:N] = w.T
    return x, ln_g, ln_b, w, wt, bias


@pytest.mark.parametrize("dtype_name", ["float16", "bfloat16"])
def test_layernorm_projection_matches_oracle(torch_cuda, orc64, dtype_name):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    dtype = getattr(torch, dtype_name)
    out_eps = 2.0 ** -11 if dtype_name == "float16" else 2.0 ** -8
    for si, (M, N) in enumerate(SHAPES):
        x, ln_g, ln_b, w, wt, bias = _operands(torch, M, N, dtype, seed=40 + si)
        # the kernel rounds the normalised rows to 16 bits before the product: so does the reference
        a = torch.from_numpy(orc64.layernorm(x, ln_g, ln_b).astype(np.float32)).to(dtype).float().numpy()
        ref = orc64.linear(a, w.float().numpy(), bias)
        scale = np.abs(ref).max()
        xd, gd, bd, wd, biasd = [torch.from_numpy(t).cuda() for t in (x, ln_g, ln_b)] + [wt.cuda(), torch.from_numpy(bias).cuda()]
        c = sjd.op_panel_linear_h16(xd, wd, biasd, M, N, 0, ln_g=gd, ln_b=bd).float().cpu().numpy()
        # one output rounding, float32 accumulation, and the rare normalised value that rounds the other
        # way in float32 than in float64
        assert np.abs(c - ref).max() <= out_eps * scale + 2e-3, (dtype_name, M, N)
        cg = sjd.op_panel_linear_h16(xd, wd, biasd, M, N, 1, ln_g=gd, ln_b=bd).float().cpu().numpy()
        assert np.abs(cg - orc64.gelu(ref)).max() <= out_eps * scale + 2e-3, (dtype_name, M, N)


@pytest.mark.parametrize("dtype_name", ["float16", "bfloat16"])
def test_residual_projection_matches_oracle_and_tile_kernel(torch_cuda, orc64, dtype_name):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    dtype = getattr(torch, dtype_name)
    for si, (M, N) in enumerate([(77, 256), (300, 512), (4173, 512), (20480, 512)]):
        g = np.random.default_rng(70 + si)
        a = torch.from_numpy(g.standard_normal((M, K)).astype(np.float32)).to(dtype)
        _, _, _, w, wt, bias = _operands(torch, 1, N, dtype, seed=80 + si)
        ref = orc64.linear(a.float().numpy(), w.float().numpy(), bias)
        scale = np.abs(ref).max()
        r0 = g.standard_normal((M, N)).astype(np.float32)
        ad, wd, biasd = a.cuda(), wt.cuda(), torch.from_numpy(bias).cuda()
        rd = torch.from_numpy(r0.copy()).cuda()
        sjd.op_panel_linear_h16(ad, wd, biasd, M, N, 2, resid=rd)
        assert np.abs(rd.cpu().numpy() - (r0 + ref)).max() <= 2e-4 * scale + 1e-4, (dtype_name, M, N)
        rt = torch.from_numpy(r0.copy()).cuda()
        sjd.op_linear_h16(ad, wd, biasd, M, N, K, 2, resid=rt, kernel=3)
        assert torch.equal(rd, rt), (dtype_name, M, N)       # same instruction, same order of k: same bits


@pytest.mark.parametrize("dtype_name", ["float16", "bfloat16"])
def test_streaming_residual_projection_matches_oracle_and_tile_kernel(torch_cuda, orc64, dtype_name):
    """K > 512: the left operand streams through LDS in chunks of 256 k (2 to 8 chunk pairs here), weights
    come from L2 with hand-counted waits - any miscount shows as a wrong product."""
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    dtype = getattr(torch, dtype_name)
    for si, (M, N, Kk) in enumerate([(300, 256, 1024), (1000, 768, 1536), (4173, 512, 2048), (16389, 512, 2048), (129, 256, 4096)]):
        g = np.random.default_rng(170 + si)
        a = torch.from_numpy(g.standard_normal((M, Kk)).astype(np.float32)).to(dtype)
        w = torch.from_numpy((g.standard_normal((Kk, N)) * 0.03).astype(np.float32)).to(dtype)
        bias = (g.standard_normal(N) * 0.1).astype(np.float32)
        wt = torch.zeros(((N + 255) // 256 * 256, Kk), dtype=dtype)
        wt[:N] = w.T
        ref = orc64.linear(a.float().numpy(), w.float().numpy(), bias)
        scale = np.abs(ref).max()
        r0 = g.standard_normal((M, N)).astype(np.float32)
        ad, wd, biasd = a.cuda(), wt.cuda(), torch.from_numpy(bias).cuda()
        rd = torch.from_numpy(r0.copy()).cuda()
        sjd.op_panel_linear_h16(ad, wd, biasd, M, N, 2, K=Kk, resid=rd)
        assert np.abs(rd.cpu().numpy() - (r0 + ref)).max() <= 2e-4 * scale + 1e-4, (dtype_name, M, N, Kk)
        rt = torch.from_numpy(r0.copy()).cuda()
        sjd.op_linear_h16(ad, wd, biasd, M, N, Kk, 2, resid=rt, kernel=3)
        assert torch.equal(rd, rt), (dtype_name, M, N, Kk)       # same instruction, same order of k: same bits
        rd2 = torch.from_numpy(r0.copy()).cuda()                 # and again: nothing left over from the first launch
        sjd.op_panel_linear_h16(ad, wd, biasd, M, N, 2, K=Kk, resid=rd2)
        assert torch.equal(rd, rd2), (dtype_name, M, N, Kk)


def test_rows_do_not_depend_on_their_neighbours(torch_cuda):
    """A row gives the same bits alone and deep inside a large problem, whatever the split of the
    column groups over workgroups (it changes with the number of panels)."""
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    M, N = 16384, 1536
    x, ln_g, ln_b, w, wt, bias = _operands(torch, M, N, torch.float16, seed=7)
    xd, gd, bd, wd, biasd = [torch.from_numpy(t).cuda() for t in (x, ln_g, ln_b)] + [wt.cuda(), torch.from_numpy(bias).cuda()]
    full = sjd.op_panel_linear_h16(xd, wd, biasd, M, N, 1, ln_g=gd, ln_b=bd)
    for lo, n in ((300, 256), (5000, 1111), (16000, 384)):
        part = sjd.op_panel_linear_h16(xd[lo:lo + n].contiguous(), wd, biasd, n, N, 1, ln_g=gd, ln_b=bd)
        assert torch.equal(full[lo:lo + n], part), (lo, n)


def _flow_cfg():
    import workloads as wl
    return wl.FlowConfig("panel", n_blocks=3, n_layers=2, width=512, n_heads=8, seq_len=64, token_dim=12, batch=5,
                         bf16=True)


@pytest.mark.parametrize("dtype_name", ["f16", "bf16"])
def test_flow_gives_the_same_bits_on_both_projection_paths(torch_cuda, dtype_name):
    """Conditioner, Jacobi block and whole cascade of a width-512 flow with the tile kernels + LayerNorm
    launches (path 1) and with the activation-stationary kernels at every row count (path 2)."""
    import paper_2505_24791_amd as sjd
    import workloads as wl
    torch = torch_cuda
    cfg = _flow_cfg()
    blob = wl.make_weights(cfg)
    z = torch.from_numpy(wl.make_latent(cfg)).cuda()
    f = sjd.Flow(cfg, dtype=sjd.DTYPE_F16 if dtype_name == "f16" else sjd.DTYPE_BF16)
    f.load_weights(blob)
    out = {}
    for path in (1, 2):
        f.set_projection_path(path)
        mu, alpha = f.conditioner(1, z)
        x, iters, passes, _ = f.jacobi_inverse_block(1, z, sjd.JacobiOpts())
        xs, stats, _ = f.sample(z, 0b110, sjd.JacobiOpts())
        out[path] = (mu, alpha, x, iters.copy(), passes, xs, list(stats["block_iters"]))
    a, b = out[1], out[2]
    for i in (0, 1, 2, 5):
        assert torch.equal(a[i], b[i]), i
    assert np.array_equal(a[3], b[3]) and a[4] == b[4] and a[6] == b[6]
    f.close()


def test_headline_workload_takes_the_panel_kernels_and_gives_the_same_bits(torch_cuda):
    """Configuration C2 at its full batch (16384 rows per pass: the launch configuration that bench.py
    times): the automatic choice is the activation-stationary / streaming kernels, and a Jacobi block gives
    the bits and pass counts of the tile kernels."""
    import paper_2505_24791_amd as sjd
    import workloads as wl
    torch = torch_cuda
    cfg = wl.CONFIGS["C2"]
    f = sjd.Flow(cfg)
    f.load_weights(wl.cached_weights(cfg))
    z = torch.from_numpy(wl.make_latent(cfg)).cuda()
    out = {}
    for path in (1, 0):
        f.set_projection_path(path)
        f.profile_enable([sjd.PROF_GEMM, sjd.PROF_OTHER])
        mu, alpha = f.conditioner(2, z)
        x, iters, passes, _ = f.jacobi_inverse_block(1, z, sjd.JacobiOpts())
        prof = f.profile_read(reset=True)
        out[path] = (mu, alpha, x, iters.copy(), passes, prof)
    for i in (0, 1, 2):
        assert torch.equal(out[1][i], out[0][i]), i
    assert np.array_equal(out[1][3], out[0][3]) and out[1][4] == out[0][4]
    # the LayerNorm launches of the layers (family "other") are gone from the passes that took the panel kernels
    assert out[0][5]["gemm"]["launches"] == out[1][5]["gemm"]["launches"]
    assert out[0][5]["other"]["launches"] < out[1][5]["other"]["launches"]
    f.close()


def test_projection_path_is_validated(torch_cuda):
    import paper_2505_24791_amd as sjd
    import workloads as wl
    f = sjd.Flow(_flow_cfg())
    with pytest.raises(sjd.SjdError):
        f.set_projection_path(3)
    f.set_projection_path(2)
    f.close()
    narrow = wl.FlowConfig("narrow", n_blocks=2, n_layers=1, width=256, n_heads=4, seq_len=32, token_dim=12, batch=2,
                           bf16=True)
    f = sjd.Flow(narrow)
    with pytest.raises(sjd.SjdError):
        f.set_projection_path(2)        # width 256: the panel kernels do not apply
    f.set_projection_path(1)
    f.close()
    x = torch_cuda.zeros((10, 512), device="cuda")
    wt = torch_cuda.zeros((512, 512), dtype=torch_cuda.float16, device="cuda")
    v = torch_cuda.zeros(512, device="cuda")
    with pytest.raises(sjd.SjdError):
        sjd.op_panel_linear_h16(x, wt, v, 10, 384, 0, ln_g=v, ln_b=v)     # N not a multiple of 256
