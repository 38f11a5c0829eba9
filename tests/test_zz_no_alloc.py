"""The projection op for callers that cannot allocate (`sjd_op_panel_linear_h16_noalloc`: its temporary
weight copy lives in a device array of the library) against the allocating op it is a variant of, through
the C boundary: same bits, on two calls in a row of which the second is smaller - it finds the first
call's contents in the shared array - and for every epilogue the op has.  Needs an MI355X.

Integer-exact bar: the two entry points run the same kernels on the same operands, so the outputs must be
bit-identical; the allocating op itself is checked against the oracle in test_gpu_panel.py.
"""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _case(torch, M, N, K, dtype, seed):
    g = np.random.default_rng(seed)
    x = (g.standard_normal((M, 512)) * 1.5 + 0.3).astype(np.float32)          # float32 rows for the LayerNorm variants
    a = torch.from_numpy(g.standard_normal((M, K)).astype(np.float32)).to(dtype)   # 16-bit rows for the residual variants
    ln_g = (1.0 + 0.1 * g.standard_normal(512)).astype(np.float32)
    ln_b = (0.1 * g.standard_normal(512)).astype(np.float32)
    wt = torch.from_numpy((g.standard_normal((N, K)) * 0.05).astype(np.float32)).to(dtype)
    bias = (g.standard_normal(N) * 0.1).astype(np.float32)
    r0 = g.standard_normal((M, N)).astype(np.float32)
    return x, a, ln_g, ln_b, wt, bias, r0


def _both(torch, sjd, M, N, K, dtype, seed):
    """Runs every epilogue the shape admits through both entry points; returns [(label, alloc, noalloc)]."""
    x, a, ln_g, ln_b, wt, bias, r0 = _case(torch, M, N, K, dtype, seed)
    xd, gd, bd, biasd = (torch.from_numpy(t).cuda() for t in (x, ln_g, ln_b, bias))
    ad, wd = a.cuda(), wt.cuda()
    out = []
    if K == 512:
        for epi in (0, 1):
            ref = sjd.op_panel_linear_h16(xd, wd, biasd, M, N, epi, ln_g=gd, ln_b=bd)
            got = sjd.op_panel_linear_h16(xd, wd, biasd, M, N, epi, ln_g=gd, ln_b=bd, noalloc=True)
            out.append((f"epilogue {epi}", ref, got))
    if K > 512 or N <= 512:
        ref = torch.from_numpy(r0.copy()).cuda()
        got = torch.from_numpy(r0.copy()).cuda()
        sjd.op_panel_linear_h16(ad, wd, biasd, M, N, 2, K=K, resid=ref)
        sjd.op_panel_linear_h16(ad, wd, biasd, M, N, 2, K=K, resid=got, noalloc=True)
        out.append(("epilogue 2", ref, got))
    return out


@pytest.mark.parametrize("dtype_name", ["float16", "bfloat16"])
def test_noalloc_op_equals_allocating_op_on_consecutive_calls(torch_cuda, dtype_name):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    dtype = getattr(torch, dtype_name)
    # first a large weight (the whole 4 MiB array in use), then smaller ones that reuse the array's front part,
    # then the streaming kernel (K = 2048), then the large one again
    shapes = [(700, 2048, 512), (300, 512, 512), (77, 256, 512), (1000, 512, 2048), (129, 256, 1024), (700, 2048, 512)]
    for si, (M, N, K) in enumerate(shapes):
        for label, ref, got in _both(torch, sjd, M, N, K, dtype, seed=200 + si):
            assert torch.isfinite(got.float()).all(), (dtype_name, M, N, K, label)
            assert torch.equal(ref, got), (dtype_name, M, N, K, label)


def test_noalloc_op_rejects_what_does_not_fit(torch_cuda):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    lib = sjd.load_library()
    M, N, K = 64, 1024, 4096            # 8 MiB of weight in 16 bits: over the array's 4 MiB
    a = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    wt = torch.zeros((N, K), dtype=torch.float16, device="cuda")
    bias = torch.zeros(N, dtype=torch.float32, device="cuda")
    r = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    p = lambda t: C.c_void_p(t.data_ptr())
    rc = lib.sjd_op_panel_linear_h16_noalloc(sjd.DTYPE_F16, p(a), None, None, p(wt), p(bias), p(r), None, M, N, K, 2, None)
    assert rc == sjd.SJD_EINVAL
    assert b"scratch" in lib.sjd_last_error()
    # the allocating op takes the same call
    assert lib.sjd_op_panel_linear_h16(sjd.DTYPE_F16, p(a), None, None, p(wt), p(bias), p(r), None, M, N, K, 2, None) == 0
    # and the argument checks are shared
    assert lib.sjd_op_panel_linear_h16_noalloc(sjd.DTYPE_F16, None, None, None, p(wt), p(bias), p(r), None, M, N, K, 2, None) \
        == sjd.SJD_EINVAL
