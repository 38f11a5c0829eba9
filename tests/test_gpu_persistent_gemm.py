"""The persistent eight-wave projection kernel (256x256 tiles, workgroups that walk over their tiles)
against the CPU oracle's `linear` / `gelu` in float64 and, bit for bit, against the tile kernel it
replaces in the whole-sequence passes.  Needs an MI355X.

Shapes: one tile, a ragged last row tile, more tiles than workgroups on the device (so that workgroups
take several tiles in a row and the hand-over between tiles - operands of the next tile requested during
the last k-tile of this one - is exercised), the shortest k the kernel takes (two k-tiles) and long k."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

# (M, N, K); N % 256 == 0, K % 128 == 0
SHAPES = [(256, 256, 128), (77, 256, 256), (700, 512, 384), (1300, 768, 1024), (16640, 1536, 512), (300, 1024, 4096),
          (40000, 768, 256)]


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _operands(torch, M, N, K, dtype, seed):
    g = np.random.default_rng(seed)
    a = torch.from_numpy(g.standard_normal((M, K)).astype(np.float32)).to(dtype)
    w = torch.from_numpy((g.standard_normal((K, N)) * 0.04).astype(np.float32)).to(dtype)
    bias = torch.from_numpy(g.standard_normal(N).astype(np.float32) * 0.1)
    return a, w, w.T.contiguous(), bias


@pytest.mark.parametrize("kernel", [4])
@pytest.mark.parametrize("dtype_name", ["float16", "bfloat16"])
def test_persistent_kernel_matches_oracle_and_tile_kernel(torch_cuda, orc64, dtype_name, kernel):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    dtype = getattr(torch, dtype_name)
    out_eps = 2.0 ** -11 if dtype_name == "float16" else 2.0 ** -8
    for si, (M, N, K) in enumerate(SHAPES):
        a, w, wt, bias = _operands(torch, M, N, K, dtype, seed=300 + si)
        ad, wd, bd = a.cuda(), wt.cuda(), bias.cuda()
        # the oracle on a spread of rows when the problem is large (rows are independent)
        rows = np.arange(M) if M * N * K <= 4e8 else np.unique(np.linspace(0, M - 1, 300).astype(int))
        ref = orc64.linear(a.float().numpy()[rows], w.float().numpy(), bias.numpy())
        scale = np.abs(ref).max()
        for epi in (0, 1):
            c = sjd.op_linear_h16(ad, wd, bd, M, N, K, epi, kernel=kernel)
            want = ref if epi == 0 else orc64.gelu(ref)
            assert np.abs(c.float().cpu().numpy()[rows] - want).max() <= out_eps * scale + 1e-3, (dtype_name, M, N, K, epi)
            assert torch.equal(c, sjd.op_linear_h16(ad, wd, bd, M, N, K, epi, kernel=3)), (dtype_name, M, N, K, epi)
        r0 = np.random.default_rng(99).standard_normal((M, N)).astype(np.float32)
        rd = torch.from_numpy(r0.copy()).cuda()
        sjd.op_linear_h16(ad, wd, bd, M, N, K, 2, resid=rd, kernel=kernel)
        assert np.abs(rd.cpu().numpy()[rows] - (r0[rows] + ref)).max() <= 3e-4 * scale + 1e-4, (dtype_name, M, N, K)
        rt = torch.from_numpy(r0.copy()).cuda()
        sjd.op_linear_h16(ad, wd, bd, M, N, K, 2, resid=rt, kernel=3)
        assert torch.equal(rd, rt), (dtype_name, M, N, K)


@pytest.mark.parametrize("kernel", [4])
def test_persistent_kernel_rows_do_not_depend_on_their_neighbours(torch_cuda, kernel):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    M, N, K = 2048, 512, 256
    a, w, wt, bias = _operands(torch, M, N, K, torch.float16, seed=5)
    ad, wd, bd = a.cuda(), wt.cuda(), bias.cuda()
    full = sjd.op_linear_h16(ad, wd, bd, M, N, K, 0, kernel=kernel)
    part = sjd.op_linear_h16(ad[300:556].contiguous(), wd, bd, 256, N, K, 0, kernel=kernel)
    assert torch.equal(full[300:556], part)
