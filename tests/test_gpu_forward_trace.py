"""The forward map with its log-determinant (eq. 4 under eq. 1), the caller-supplied first iterate
and the per-pass convergence record of Jacobi decoding, HIP path against the CPU oracle through
the C boundary.  Needs an MI355X.

Tolerances as for sampling: float32 mode 1e-4, 16-bit modes 2e-2 on values.  A log-determinant
is a sum of (T-1)*D alphas, so its bound is that many times the per-value bound of the mode's
conditioner (1e-6 float32, 2e-4 for half operands at the recipe's weight scale), stated per case."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _flow(cfg, blob, dtype=None):
    import paper_2505_24791_amd as sjd
    f = sjd.Flow(cfg, dtype=dtype)
    f.load_weights(blob)
    return f


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda()


F32 = wl.FlowConfig("ragged", n_blocks=3, n_layers=2, width=96, n_heads=3, seq_len=37, token_dim=5, batch=7, bf16=False)
H16 = wl.FlowConfig("h16", n_blocks=3, n_layers=2, width=256, n_heads=4, seq_len=70, token_dim=6, batch=5, bf16=True)


@pytest.mark.parametrize("cfg,tol,ld_tol", [(wl.CONFIGS["C1"], 1e-4, 1e-3), (F32, 1e-4, 1e-3), (H16, 2e-2, 0.1)],
                         ids=["C1", "ragged_f32", "half"])
def test_forward_and_logdet_match_oracle(torch_cuda, orc64, cfg, tol, ld_tol):
    torch = torch_cuda
    blob = wl.make_weights(cfg, perturb_affine=cfg.name != "C1")
    x = wl.make_latent(cfg, seed=11)
    f = _flow(cfg, blob)
    xd = _dev(torch, x)
    # block by block, accumulating the log-determinant on the device
    cur, ld = xd, None
    ref = x.astype(np.float64)
    ref_ld = np.zeros(cfg.batch)
    for j in range(cfg.n_blocks - 1, -1, -1):
        cur, ld = f.forward_block(j, cur, logdet=ld, accumulate=ld is not None)
        for b in range(cfg.batch):
            ref[b], l = orc64.forward_block_logdet(cfg, blob, j, ref[b])
            ref_ld[b] += l
        assert np.abs(cur.cpu().numpy() - ref).max() <= tol, j
        assert np.abs(ld.cpu().numpy() - ref_ld).max() <= ld_tol, j
    # the whole map in one call gives the same bits as the chain of block calls
    z, ld_all = f.forward(xd)
    assert torch.equal(z, cur) and torch.equal(ld_all, ld)
    rz, rld = orc64.forward_logdet(cfg, blob, x)
    assert np.abs(z.cpu().numpy() - rz).max() <= tol
    assert np.abs(ld_all.cpu().numpy() - rld).max() <= ld_tol
    assert np.abs(rld).max() > 10 * ld_tol or cfg.name == "C1"      # the comparison is not vacuous
    f.close()


def test_forward_inverts_sampling_on_the_device(torch_cuda):
    """forward(sample(z)) = z for the sequential inverse (float32: 1e-4 round trip)."""
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    cfg = wl.CONFIGS["C1"]
    blob = wl.make_weights(cfg)
    f = _flow(cfg, blob)
    z = _dev(torch, wl.make_latent(cfg))
    x, _, _ = f.sample(z, 0, sjd.JacobiOpts())
    zz, ld = f.forward(x)
    assert (zz - z).abs().max().item() <= 1e-4
    assert torch.isfinite(ld).all()
    f.close()


def test_forward_argument_errors(torch_cuda):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    cfg = wl.CONFIGS["C1"]
    f = _flow(cfg, wl.make_weights(cfg))
    x = _dev(torch, wl.make_latent(cfg))
    with pytest.raises(sjd.SjdError) as e:
        f.forward_block(cfg.n_blocks, x)
    assert e.value.code == sjd.SJD_EINVAL
    with pytest.raises(sjd.SjdError) as e:      # init 2 has no meaning inside the cascade
        f.sample(x, ~1, sjd.JacobiOpts(init=2))
    assert e.value.code == sjd.SJD_EINVAL
    f.close()


@pytest.mark.parametrize("cfg,tol", [(F32, 1e-4), (H16, 2e-2)], ids=["f32", "half"])
def test_caller_supplied_first_iterate(torch_cuda, orc32, cfg, tol):
    """x^0 drawn by the caller (N(0, I), the initialisation study of Sec. 4.3): same result and pass
    counts as the oracle from the same x^0; x^0 = zeros and x^0 = z reproduce init 0 and 1 bit for bit."""
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    blob = wl.make_weights(cfg, perturb_affine=True)
    z = wl.make_latent(cfg, seed=21)
    x0 = np.random.default_rng(5).standard_normal(z.shape).astype(np.float32)
    f = _flow(cfg, blob)
    zd = _dev(torch, z)
    tau = 1e-3
    for j in (0, 1):
        x, iters, passes, _ = f.jacobi_inverse_block(j, zd, sjd.JacobiOpts(tau=tau, init=2), x0=_dev(torch, x0))
        xs = x.cpu().numpy()
        for b in range(cfg.batch):
            rx, it, tr = orc32.jacobi_inverse_block(cfg, blob, j, z[b], tau, x0=x0[b], want_trace=True)
            if any(abs(d - tau) <= 0.01 * tau for d in tr[-2:]) and it < cfg.seq_len:
                continue                                           # knife edge: not compared
            if cfg.bf16:
                assert abs(int(iters[b]) - it) <= 1, (j, b)
            else:
                assert int(iters[b]) == it, (j, b)
            assert np.abs(xs[b] - rx).max() <= tol, (j, b)
        for init, start in ((0, torch.zeros_like(zd)), (1, zd)):
            a = f.jacobi_inverse_block(j, zd, sjd.JacobiOpts(tau=tau, init=init))
            c = f.jacobi_inverse_block(j, zd, sjd.JacobiOpts(tau=tau, init=2), x0=start)
            assert torch.equal(a[0], c[0]) and np.array_equal(a[1], c[1])
    f.close()


@pytest.mark.parametrize("cfg,tol", [(F32, 1e-4), (H16, 2e-2)], ids=["f32", "half"])
def test_convergence_record_matches_oracle(torch_cuda, orc32, cfg, tol):
    """Per-pass delta and l2 distance to the sequential solution: oracle iterates give the reference
    curve; the error never grows on the exact prefix (Prop. 3.2) and is zero at the cap in float32."""
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    blob = wl.make_weights(cfg, perturb_affine=True)
    z = wl.make_latent(cfg, seed=31)
    f = _flow(cfg, blob)
    zd = _dev(torch, z)
    n = cfg.seq_len * cfg.token_dim
    for j in (0, 1):
        xref = f.sequential_inverse_block(j, zd)
        opts = sjd.JacobiOpts(tau=0.0, max_iters=12)
        x, iters, passes, delta, err = f.jacobi_trace_block(j, zd, opts, x_ref=xref)
        assert passes == 12 and delta.shape == (12, cfg.batch) and err.shape == (12, cfg.batch)
        plain = f.jacobi_inverse_block(j, zd, opts)
        assert torch.equal(plain[0], x)                             # recording changes nothing
        for b in range(cfg.batch):
            rseq = orc32.sequential_inverse_block(cfg, blob, j, z[b])
            _, it, tr, its = orc32.jacobi_inverse_block(cfg, blob, j, z[b], 0.0, max_iters=12, want_trace=True,
                                                        want_iterates=True)
            rerr = np.sqrt(((its.astype(np.float64) - rseq[None].astype(np.float64)) ** 2).reshape(12, -1).sum(1))
            # per-value bound tol -> l2 bound tol * sqrt(n); delta is a mean of absolute differences
            assert np.abs(err[:, b] - rerr).max() <= tol * np.sqrt(n), (j, b)
            assert np.abs(delta[:, b] - tr).max() <= 2 * tol, (j, b)
        # with a threshold: entries of a stopped sample repeat
        opts = sjd.JacobiOpts(tau=1e-3)
        x, iters, passes, delta, err = f.jacobi_trace_block(j, zd, opts, x_ref=xref)
        for b in range(cfg.batch):
            k = int(iters[b])
            assert np.all(delta[k - 1:, b] == delta[k - 1, b]) and np.all(err[k - 1:, b] == err[k - 1, b])
            assert delta[k - 1, b] < 1e-3 or k == cfg.seq_len
    # float32: run to the cap T and the last iterate is the sequential solution (Prop. 3.2)
    if not cfg.bf16:
        xref = f.sequential_inverse_block(0, zd)
        _, _, passes, delta, err = f.jacobi_trace_block(0, zd, sjd.JacobiOpts(tau=0.0), x_ref=xref)
        assert passes == cfg.seq_len and err[-1].max() <= 1e-4
    f.close()


@pytest.mark.parametrize("case", ["f32", "half_ragged", "half_c2_shape"])
def test_first_pass_shared_over_the_batch_gives_the_same_bits(case):
    """Alg. 1 starts every sample from x^0 = 0, so the first pass's parameters are the same for all samples and
    the library computes them on one sample's rows.  A caller-supplied all-zero first iterate takes the ordinary
    path (every sample through the conditioner): iterates and pass counts must agree bit for bit, in float32, on
    a ragged 16-bit shape, and at configuration 2's shape (where the full pass and the one-sample pass take
    different projection kernels)."""
    import torch
    import paper_2505_24791_amd as sjd
    if case == "f32":
        cfg = wl.CONFIGS["C1"]
    elif case == "half_ragged":
        cfg = wl.FlowConfig("r", n_blocks=2, n_layers=2, width=128, n_heads=2, seq_len=70, token_dim=6, batch=9, bf16=True)
    else:
        cfg = wl.CONFIGS["C2"].with_(n_blocks=2, batch=48)
    blob = wl.make_weights(cfg, perturb_affine=(case != "half_c2_shape"))
    z = torch.from_numpy(wl.make_latent(cfg)).cuda()
    f = sjd.Flow(cfg)
    f.load_weights(blob)
    for j in range(cfg.n_blocks):
        for cap in (1, 0):
            xa, ia, pa, _ = f.jacobi_inverse_block(j, z, sjd.JacobiOpts(tau=cfg.tau, init=0, max_iters=cap))
            xb, ib, pb, _ = f.jacobi_inverse_block(j, z, sjd.JacobiOpts(tau=cfg.tau, init=2, max_iters=cap), x0=torch.zeros_like(z))
            assert torch.equal(xa, xb), (case, j, cap)
            assert np.array_equal(ia, ib) and pa == pb
    f.close()
