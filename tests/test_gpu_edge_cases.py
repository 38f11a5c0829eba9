"""Edge cases and invariants of the HIP path, through the C boundary.  Needs an MI355X.

What is checked here is what the method fixes regardless of weights (Alg. 1, Props. 3.1/3.2 and the
readings listed in the design notes): the cap of T passes, tau = 0 and tau = inf, exactness after T
passes, batch independence, the effect-free dropping of converged samples, determinism, options,
error codes.  Values are compared with the CPU oracle where a value is asserted.
"""
import ctypes as C

import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda()


SMALL_F32 = wl.FlowConfig("edge_f32", n_blocks=3, n_layers=2, width=64, n_heads=2, seq_len=12, token_dim=4, batch=6,
                          bf16=False)
SMALL_H16 = wl.FlowConfig("edge_h16", n_blocks=3, n_layers=2, width=256, n_heads=4, seq_len=24, token_dim=8, batch=9,
                          bf16=True)


def _make(cfg, **kw):
    import paper_2505_24791_amd as sjd
    # float32: stronger weights than the workloads' recipe, so that the context matters more; 16-bit:
    # the recipe's scale (the 2e-2 bound on final samples is stated for it), biases and gains perturbed
    if cfg.bf16:
        blob = wl.make_weights(cfg, perturb_affine=True)
    else:
        blob = wl.make_weights(cfg, perturb_affine=True, std=0.05, head_std=0.03)
    f = sjd.Flow(cfg, **kw)
    f.load_weights(blob)
    return f, blob


@pytest.mark.parametrize("cfg", [SMALL_F32, SMALL_H16], ids=["f32", "h16"])
def test_tau_zero_runs_T_passes_and_equals_sequential(torch_cuda, orc64, cfg):
    """tau = 0: delta < tau never holds, every sample takes exactly T passes (the cap) and, by
    Prop. 3.2, the result is the sequential inverse."""
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    f, blob = _make(cfg)
    z = wl.make_latent(cfg)
    zd = _dev(torch, z)
    for j in range(cfg.n_blocks):
        x, iters, passes, rc = f.jacobi_inverse_block(j, zd, sjd.JacobiOpts(tau=0.0))
        assert rc == 0 and passes == cfg.seq_len and np.all(iters == cfg.seq_len)
        ref = np.stack([orc64.sequential_inverse_block(cfg, blob, j, z[b]) for b in range(cfg.batch)])
        tol = 1e-4 if not cfg.bf16 else 2e-2
        assert np.abs(x.cpu().numpy() - ref).max() <= tol
        # the GPU's own sequential path agrees as well
        xs = f.sequential_inverse_block(j, zd).cpu().numpy()
        assert np.abs(xs - ref).max() <= tol
    f.close()


def test_T_passes_reach_the_same_bits_from_either_initial_guess(torch_cuda):
    """After t passes token t is final and depends only on final earlier tokens (proof of
    Prop. 3.2), whatever the start was.  Because a row's arithmetic here does not depend on which
    other rows share its tile, the T-pass results from x0 = 0 and from x0 = input must agree bit
    for bit - in the 16-bit modes too."""
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    for cfg in (SMALL_F32, SMALL_H16):
        f, _ = _make(cfg)
        zd = _dev(torch, wl.make_latent(cfg))
        for j in range(cfg.n_blocks):
            a, ia, _, _ = f.jacobi_inverse_block(j, zd, sjd.JacobiOpts(tau=0.0, init=0))
            b, ib, _, _ = f.jacobi_inverse_block(j, zd, sjd.JacobiOpts(tau=0.0, init=1))
            assert np.all(ia == cfg.seq_len) and np.all(ib == cfg.seq_len)
            assert torch.equal(a, b)
        f.close()


@pytest.mark.parametrize("cfg", [SMALL_F32, SMALL_H16], ids=["f32", "h16"])
def test_tau_infinite_is_one_pass_of_F_from_zero(torch_cuda, orc64, cfg):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    f, blob = _make(cfg)
    z = wl.make_latent(cfg)
    x, iters, passes, rc = f.jacobi_inverse_block(0, _dev(torch, z), sjd.JacobiOpts(tau=float("inf")))
    assert passes == 1 and np.all(iters == 1)
    ref = np.stack([orc64.jacobi_map(cfg, blob, 0, z[b], np.zeros_like(z[b])) for b in range(cfg.batch)])
    assert np.abs(x.cpu().numpy() - ref).max() <= (1e-4 if not cfg.bf16 else 5e-3)
    f.close()


def test_max_iters_lowers_the_cap_and_init_from_input(torch_cuda, orc64):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    cfg = SMALL_F32
    f, blob = _make(cfg)
    z = wl.make_latent(cfg)
    zd = _dev(torch, z)
    x, iters, passes, _ = f.jacobi_inverse_block(2, zd, sjd.JacobiOpts(tau=0.0, max_iters=3))
    assert passes == 3 and np.all(iters == 3)
    for b in range(cfg.batch):
        ref, it = orc64.jacobi_inverse_block(cfg, blob, 2, z[b], 0.0, max_iters=3)
        assert it == 3 and np.abs(x[b].cpu().numpy() - ref).max() <= 1e-4
    # initial guess = the block's input (initialisation study of Sec. 4.3): same fixed point, own pass counts
    x1, it1, _, _ = f.jacobi_inverse_block(2, zd, sjd.JacobiOpts(tau=1e-4, init=1))
    for b in range(cfg.batch):
        ref, it = orc64.jacobi_inverse_block(cfg, blob, 2, z[b], 1e-4, x0=z[b])
        assert it1[b] == it and np.abs(x1[b].cpu().numpy() - ref).max() <= 1e-4
    f.close()


def test_max_norm_criterion_matches_oracle(torch_cuda, orc64):
    """criterion 1: the stopping rule exactly as Alg. 1 prints it (infinity norm)."""
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    cfg = SMALL_F32
    f, blob = _make(cfg)
    z = wl.make_latent(cfg)
    x, iters, _, _ = f.jacobi_inverse_block(1, _dev(torch, z), sjd.JacobiOpts(tau=3e-3, criterion=1))
    for b in range(cfg.batch):
        ref, it, tr = orc64.jacobi_inverse_block(cfg, blob, 1, z[b], 3e-3, criterion=1, want_trace=True)
        if min(abs(d - 3e-3) for d in tr[-2:]) < 3e-5:
            continue  # within 1 % of tau: either count is legitimate
        assert iters[b] == it and np.abs(x[b].cpu().numpy() - ref).max() <= 1e-4
    f.close()


@pytest.mark.parametrize("cfg", [SMALL_F32, SMALL_H16], ids=["f32", "h16"])
def test_dropping_converged_samples_changes_nothing(torch_cuda, cfg):
    """Converged samples leave the batch the conditioner runs on; that is a pure optimisation:
    results and pass counts are bit-identical with drop_converged = 0, and a sample alone gives the
    same bits as inside the batch."""
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    f, _ = _make(cfg)
    z = wl.make_latent(cfg)
    z[1] *= 0.05          # a sample that converges much earlier than the others
    zd = _dev(torch, z)
    mask = (1 << cfg.n_blocks) - 1
    a, sa, ia = f.sample(zd, mask, sjd.JacobiOpts(tau=cfg.tau, drop_converged=1))
    b, sb, ib = f.sample(zd, mask, sjd.JacobiOpts(tau=cfg.tau, drop_converged=0))
    assert np.array_equal(ia, ib) and torch.equal(a, b)
    assert len(set(ia[0].tolist())) > 1, "the batch should not converge in lock-step for this test to bite"
    for s in (0, 1, cfg.batch - 1):
        c, _, ic = f.sample(zd[s:s + 1].contiguous(), mask, sjd.JacobiOpts(tau=cfg.tau))
        assert np.array_equal(ic[:, 0], ia[:, s]) and torch.equal(c[0], a[s])
    f.close()


def test_two_runs_are_bitwise_identical_and_graph_replay_equals_eager(torch_cuda):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    cfg = SMALL_H16
    f, _ = _make(cfg)
    f.set_sequential_path(1)                             # per-step launches, replayed as a graph
    zd = _dev(torch, wl.make_latent(cfg))
    sel = ~1 & ((1 << cfg.n_blocks) - 1)
    a, _, ia = f.sample(zd, sel, sjd.JacobiOpts(tau=cfg.tau))
    for _ in range(3):                                   # replays of the captured step graph, with eager work between
        b, _, ib = f.sample(zd, sel, sjd.JacobiOpts(tau=cfg.tau))
        torch.cuda.synchronize()
        assert torch.equal(a, b) and np.array_equal(ia, ib)
    # with kernel timing on, the sequential block runs without the graph: same bits
    f.profile_enable(range(sjd.PROF_FAMILIES))
    c, _, ic = f.sample(zd, sel, sjd.JacobiOpts(tau=cfg.tau))
    prof = f.profile_read()
    f.profile_enable([])
    assert torch.equal(a, c) and np.array_equal(ia, ic)
    assert prof["decode_gemm"]["launches"] > 0 and prof["gemm"]["ms"] > 0
    # other buffers, other batch: new graphs, same values for the shared samples
    z2 = zd[:5].clone()
    d, _, _ = f.sample(z2, sel, sjd.JacobiOpts(tau=cfg.tau))
    assert torch.equal(d, a[:5])
    # the persistent kernel: also the same bits run after run, with and without kernel timing
    f.set_sequential_path(2)
    p1, _, ip1 = f.sample(zd, sel, sjd.JacobiOpts(tau=cfg.tau))
    f.profile_enable(range(sjd.PROF_FAMILIES))
    p2, _, ip2 = f.sample(zd, sel, sjd.JacobiOpts(tau=cfg.tau))
    prof = f.profile_read()
    f.profile_enable([])
    assert torch.equal(p1, p2) and np.array_equal(ip1, ip2)
    assert prof["decode_fused"]["launches"] == 1 and prof["decode_gemm"]["launches"] == 0
    assert (p1 - a).abs().max().item() <= 2e-2
    f.close()


def test_batch_of_one_and_single_token(torch_cuda, orc32):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    cfg = wl.FlowConfig("one", n_blocks=2, n_layers=1, width=64, n_heads=1, seq_len=1, token_dim=3, batch=1, bf16=True)
    f, blob = _make(cfg)
    z = wl.make_latent(cfg)
    x, st, iters = f.sample(_dev(torch, z), 0b10, sjd.JacobiOpts(tau=1e-3))
    assert np.array_equal(x.cpu().numpy(), z)            # one token: the block copies its input (x_1 = y_1)
    assert iters.tolist() == [[0], [1]]                  # T-1 = 0 sequential steps; one Jacobi pass (cap T = 1)
    f.close()


def test_identity_flow_when_head_is_zero(torch_cuda):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    for cfg in (SMALL_F32, SMALL_H16):
        blob = wl.make_weights(cfg, perturb_affine=True)
        for v in wl.blob_views(cfg, blob):
            v["w_head"][...] = 0; v["b_head"][...] = 0
        f = sjd.Flow(cfg); f.load_weights(blob)
        z = wl.make_latent(cfg)
        x, st, iters = f.sample(_dev(torch, z), (1 << cfg.n_blocks) - 1, sjd.JacobiOpts(tau=1e-3))
        assert np.array_equal(x.cpu().numpy(), z) and np.all(iters == 2)   # delta_1 = mean|z|, delta_2 = 0
        f.close()


def test_nan_input_terminates_at_the_cap_with_an_error_code(torch_cuda):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    cfg = SMALL_F32
    f, _ = _make(cfg)
    z = wl.make_latent(cfg)
    z[2, 0, 0] = np.nan
    x, iters, passes, rc = f.jacobi_inverse_block(0, _dev(torch, z), sjd.JacobiOpts(tau=1e-3), allow_nonfinite=True)
    assert rc == sjd.SJD_ENONFINITE and iters[2] == cfg.seq_len and passes == cfg.seq_len
    assert np.all(iters[[0, 1, 3, 4, 5]] < cfg.seq_len)        # the other samples are unaffected
    assert np.all(np.isfinite(x.cpu().numpy()[[0, 1, 3, 4, 5]]))
    with pytest.raises(sjd.SjdError) as e:
        f.jacobi_inverse_block(0, _dev(torch, z), sjd.JacobiOpts(tau=1e-3))
    assert e.value.code == sjd.SJD_ENONFINITE
    f.close()


def test_argument_errors(torch_cuda):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    cfg = SMALL_F32
    f = sjd.Flow(cfg, max_batch=4)
    z = _dev(torch, wl.make_latent(cfg, batch=4))
    with pytest.raises(sjd.SjdError) as e:                      # weights not loaded
        f.sequential_inverse_block(0, z)
    assert e.value.code == sjd.SJD_ESTATE
    blob = wl.make_weights(cfg)
    with pytest.raises(sjd.SjdError) as e:                      # wrong blob size
        f.load_weights(blob[:-1])
    assert e.value.code == sjd.SJD_EINVAL
    f.load_weights(blob)
    lib = f.lib
    x = torch.empty_like(z)
    opts = sjd.SjdJacobiOpts(1e-3, 0, 0, 0, 1)
    vp = lambda t: C.c_void_p(t.data_ptr())
    assert lib.sjd_sequential_inverse_block(f._h, 7, vp(z), vp(x), 4, None) == sjd.SJD_EINVAL       # block index
    assert lib.sjd_sequential_inverse_block(f._h, 0, vp(z), vp(x), 5, None) == sjd.SJD_EINVAL       # batch > max_batch
    assert lib.sjd_sequential_inverse_block(f._h, 0, vp(z), vp(z), 4, None) == sjd.SJD_EINVAL       # overlap
    assert lib.sjd_sequential_inverse_block(f._h, 0, None, vp(x), 4, None) == sjd.SJD_EINVAL        # null
    bad = sjd.SjdJacobiOpts(float("nan"), 0, 0, 0, 1)
    assert lib.sjd_jacobi_inverse_block(f._h, 0, vp(z), vp(x), 4, C.byref(bad), None, None, None) == sjd.SJD_EINVAL
    bad = sjd.SjdJacobiOpts(1e-3, 2, 0, 0, 1)
    assert lib.sjd_jacobi_inverse_block(f._h, 0, vp(z), vp(x), 4, C.byref(bad), None, None, None) == sjd.SJD_EINVAL
    assert lib.sjd_jacobi_inverse_block(f._h, 0, vp(z), vp(x), 4, None, None, None, None) == sjd.SJD_EINVAL
    assert b"" != lib.sjd_last_error()
    # batch 0 is a no-op
    assert lib.sjd_sample(f._h, vp(z), vp(x), 0, 0xE, C.byref(opts), None, None, None) == sjd.SJD_OK
    f.close()


def test_sample_stats_and_modes(torch_cuda, orc64):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    cfg = SMALL_H16
    f, blob = _make(cfg)
    z = wl.make_latent(cfg)
    zd = _dev(torch, z)
    K = cfg.n_blocks
    for mask in (0, ~1 & ((1 << K) - 1), (1 << K) - 1, 0b010):
        x, st, iters = f.sample(zd, mask, sjd.JacobiOpts(tau=cfg.tau))
        rx, riters, _ = orc64.sample(cfg, blob, z, mask, cfg.tau)
        assert np.abs(x.cpu().numpy() - rx).max() <= 2e-2
        for j in range(K):
            if (mask >> j) & 1:
                assert st["block_iters"][j] == iters[j].max()
                assert abs(st["mean_sample_iters"][j] - iters[j].mean()) < 1e-4
                assert np.abs(iters[j].astype(int) - riters[j]).max() <= 1
            else:
                assert st["block_iters"][j] == cfg.seq_len - 1 and np.all(iters[j] == cfg.seq_len - 1)
            assert st["block_ms"][j] > 0
    f.close()
