"""The matrix-core projection kernels one by one against the CPU oracle (its `linear` and `gelu`
primitives in float64 on the same 16-bit-rounded operands).  Needs an MI355X.

Shapes span several tiles of each kernel with ragged edges in M and N; the error bound is the one
float32 accumulation of 16-bit products allows plus, for 16-bit results, one output rounding."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

KERNELS = {1: "256x128x32 staged", 2: "256x256x64 LDS-direct", 3: "128x128x64", 0: "auto"}
# K values give the register-staged kernels 1..16 k-tiles: both main loops (two register sets from 4
# k-tiles on when the count is even, else one set) with zero, one and several steady-state iterations
SHAPES = [(300, 200, 128), (700, 1000, 64), (513, 257, 320), (1024, 768, 256), (400, 384, 512), (260, 130, 384)]


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _operands(torch, M, N, K, dtype, seed):
    g = np.random.default_rng(seed)
    a = torch.from_numpy(g.standard_normal((M, K)).astype(np.float32)).to(dtype)
    w = torch.from_numpy((g.standard_normal((K, N)) * 0.05).astype(np.float32)).to(dtype)
    bias = torch.from_numpy(g.standard_normal(N).astype(np.float32) * 0.1)
    n_pad = (N + 255) // 256 * 256
    wt = torch.zeros((n_pad, K), dtype=dtype)
    wt[:N] = w.T
    return a, w, wt, bias


@pytest.mark.parametrize("kernel", sorted(KERNELS), ids=[KERNELS[k].replace(" ", "_") for k in sorted(KERNELS)])
@pytest.mark.parametrize("dtype_name", ["float16", "bfloat16"])
def test_projection_kernels_match_oracle(torch_cuda, orc64, kernel, dtype_name):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    dtype = getattr(torch, dtype_name)
    out_eps = 2.0 ** -11 if dtype_name == "float16" else 2.0 ** -8
    for si, (M, N, K) in enumerate(SHAPES):
        a, w, wt, bias = _operands(torch, M, N, K, dtype, seed=10 + si)
        ref = orc64.linear(a.float().numpy(), w.float().numpy(), bias.numpy())        # float64, same rounded operands
        scale = np.abs(ref).max()
        ad, wd, bd = a.cuda(), wt.cuda(), bias.cuda()
        c = sjd.op_linear_h16(ad, wd, bd, M, N, K, 0, kernel=kernel).float().cpu().numpy()
        assert np.abs(c - ref).max() <= out_eps * scale + 1e-3, (KERNELS[kernel], M, N, K)
        cg = sjd.op_linear_h16(ad, wd, bd, M, N, K, 1, kernel=kernel).float().cpu().numpy()
        refg = orc64.gelu(ref)
        assert np.abs(cg - refg).max() <= out_eps * scale + 1e-3, (KERNELS[kernel], M, N, K)
        r0 = np.random.default_rng(99).standard_normal((M, N)).astype(np.float32)
        rd = torch.from_numpy(r0.copy()).cuda()
        sjd.op_linear_h16(ad, wd, bd, M, N, K, 2, resid=rd, kernel=kernel)
        assert np.abs(rd.cpu().numpy() - (r0 + ref)).max() <= 2e-4 * scale + 1e-4, (KERNELS[kernel], M, N, K)


def test_projection_rows_do_not_depend_on_their_neighbours(torch_cuda):
    """A row's result is the same bits whether it is computed alone in a small problem or deep
    inside a large one (what lets converged samples leave the batch without changing anything)."""
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    M, N, K = 1024, 512, 256
    a, w, wt, bias = _operands(torch, M, N, K, torch.float16, seed=5)
    ad, wd, bd = a.cuda(), wt.cuda(), bias.cuda()
    for kernel in (1, 2, 3):
        full = sjd.op_linear_h16(ad, wd, bd, M, N, K, 0, kernel=kernel)
        part = sjd.op_linear_h16(ad[300:556].contiguous(), wd, bd, 256, N, K, 0, kernel=kernel)
        assert torch.equal(full[300:556], part)
