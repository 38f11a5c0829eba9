"""HIP path against the CPU oracle, element by element, through the C boundary.  Needs an MI355X.

Tolerances (the benchmark spec): float32 mode max |err| <= 1e-4 with identical per-sample
pass counts in every block; bf16 mode max |err| <= 2e-2 on final samples.  A seed whose oracle
delta at the deciding pass (or the one before) lies within 1 % of tau could legitimately stop one
pass apart in the two implementations; such seeds are reported and skipped over, never compared
with a loosened rule.
"""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 2e-2


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _flow(cfg, blob, max_batch=None, dtype=None):
    import paper_2505_24791_amd as sjd
    f = sjd.Flow(cfg, max_batch=max_batch, dtype=dtype)
    f.load_weights(blob)
    return f


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda()


def _knife_edge(orc, cfg, blob, z, mask, tau):
    """True if any sample's deciding delta (or the one before) is within 1 % of tau in the oracle."""
    cur = z.astype(orc.dtype)
    for j in range(cfg.n_blocks):
        nxt = np.empty_like(cur)
        for b in range(cur.shape[0]):
            if (mask >> j) & 1:
                x, it, tr = orc.jacobi_inverse_block(cfg, blob, j, cur[b], tau, want_trace=True)
                near = [d for d in tr[-2:] if abs(d - tau) <= 0.01 * tau]
                if near and it < cfg.seq_len:
                    return True
                nxt[b] = x
            else:
                nxt[b] = orc.sequential_inverse_block(cfg, blob, j, cur[b])
        cur = nxt
    return False


# ------------------------------------------------------------------------------------------------
# float32 mode: configuration 1 and ragged small shapes

F32_CASES = [
    ("C1", wl.CONFIGS["C1"], False),
    ("ragged", wl.FlowConfig("ragged", n_blocks=3, n_layers=2, width=96, n_heads=3, seq_len=37, token_dim=5,
                             batch=7, bf16=False), True),
    ("one_token", wl.FlowConfig("one_token", n_blocks=2, n_layers=1, width=32, n_heads=2, seq_len=1, token_dim=4,
                                batch=3, bf16=False), True),
    # head size 64: whole-sequence attention runs on the float32 matrix-instruction kernel (two query tiles, ragged)
    ("dh64", wl.FlowConfig("dh64", n_blocks=2, n_layers=2, width=128, n_heads=2, seq_len=150, token_dim=6,
                           batch=3, bf16=False), True),
]


@pytest.mark.parametrize("name,cfg,perturb", F32_CASES, ids=[c[0] for c in F32_CASES])
def test_f32_conditioner_matches_oracle(torch_cuda, orc32, orc64, name, cfg, perturb):
    torch = torch_cuda
    blob = wl.make_weights(cfg, perturb_affine=perturb)
    x = wl.make_latent(cfg, seed=3)
    f = _flow(cfg, blob)
    for j in range(cfg.n_blocks):
        mu, al = f.conditioner(j, _dev(torch, x))
        mu, al = mu.cpu().numpy(), al.cpu().numpy()
        rev = (cfg.reverse_mask >> j) & 1
        for b in range(cfg.batch):
            xb = x[b][::-1] if rev else x[b]
            rmu, ral = orc64.cond(cfg, blob, j, xb)           # processing order
            if rev:
                rmu, ral = rmu[::-1], ral[::-1]
            assert np.abs(mu[b] - rmu).max() <= 2e-5, (name, j, b)
            assert np.abs(al[b] - ral).max() <= 2e-5, (name, j, b)
    f.close()


@pytest.mark.parametrize("name,cfg,perturb", F32_CASES, ids=[c[0] for c in F32_CASES])
@pytest.mark.parametrize("mode", ["selective", "sequential", "all_jacobi"])
def test_f32_sample_matches_oracle(torch_cuda, orc32, orc64, name, cfg, perturb, mode):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    mask = {"selective": ~1, "sequential": 0, "all_jacobi": ~0}[mode] & ((1 << cfg.n_blocks) - 1)
    blob = wl.make_weights(cfg, perturb_affine=perturb)
    f = _flow(cfg, blob)
    seed = wl.LATENT_SEED
    while _knife_edge(orc64, cfg, blob, wl.make_latent(cfg, seed=seed), mask, cfg.tau):
        print(f"seed {seed} is knife-edge for {name}/{mode}; trying the next one")
        seed += 1
    z = wl.make_latent(cfg, seed=seed)
    x, stats, iters = f.sample(_dev(torch, z), mask, sjd.JacobiOpts(tau=cfg.tau))
    x = x.cpu().numpy()
    for orc in (orc32, orc64):
        rx, riters, _ = orc.sample(cfg, blob, z, mask, cfg.tau)
        assert np.array_equal(iters, riters), (name, mode, iters, riters)
        assert np.abs(x - rx).max() <= TOL_F32
    assert stats["block_iters"] == [int(v) for v in riters.max(axis=1)]
    np.testing.assert_allclose(stats["mean_sample_iters"], riters.mean(axis=1), rtol=1e-6)
    f.close()


def test_f32_block_calls_match_oracle(torch_cuda, orc64):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    cfg = wl.CONFIGS["C1"]
    blob = wl.make_weights(cfg); z = wl.make_latent(cfg)
    f = _flow(cfg, blob)
    zd = _dev(torch, z)
    for j in range(cfg.n_blocks):
        xs = f.sequential_inverse_block(j, zd).cpu().numpy()
        xj, iters, passes, rc = f.jacobi_inverse_block(j, zd, sjd.JacobiOpts(tau=cfg.tau))
        xj = xj.cpu().numpy()
        for b in range(cfg.batch):
            rs = orc64.sequential_inverse_block(cfg, blob, j, z[b])
            rj, it = orc64.jacobi_inverse_block(cfg, blob, j, z[b], cfg.tau)
            assert np.abs(xs[b] - rs).max() <= TOL_F32
            assert np.abs(xj[b] - rj).max() <= TOL_F32
            assert iters[b] == it
        assert passes == iters.max() and rc == 0
    f.close()


# ------------------------------------------------------------------------------------------------
# 16-bit modes (dtype 2: IEEE-half operands, the default for these workloads; dtype 1: bf16
# operands): MFMA projections and flash attention on shapes spanning several tiles and ragged tails

BF16_CASES = [
    # T = 200: two 128-row query tiles with a ragged tail, four 64-key tiles; M = 5*200 = 1000 rows
    ("bf16_ragged", wl.FlowConfig("bf16_ragged", n_blocks=3, n_layers=2, width=128, n_heads=2, seq_len=200,
                                  token_dim=12, batch=5, bf16=True), True),
    # width 256, 40 samples: single-token steps on fragment-major operands, 64-row tiles (3 row blocks live)
    ("bf16_frag64", wl.FlowConfig("bf16_frag64", n_blocks=2, n_layers=2, width=256, n_heads=4, seq_len=40,
                                  token_dim=8, batch=40, bf16=True), True),
    # the same with at most 32 rows (two row blocks, 16 waves splitting K)
    ("bf16_frag32", wl.FlowConfig("bf16_frag32", n_blocks=2, n_layers=1, width=256, n_heads=4, seq_len=24,
                                  token_dim=8, batch=19, bf16=True), True),
    # 70 samples: two row groups of the single-token kernels, the second with 6 live rows
    ("bf16_frag_groups", wl.FlowConfig("bf16_frag_groups", n_blocks=2, n_layers=1, width=256, n_heads=4, seq_len=20,
                                       token_dim=8, batch=70, bf16=True), True),
    # head size 32: the generic attention path
    ("bf16_dh32", wl.FlowConfig("bf16_dh32", n_blocks=2, n_layers=1, width=64, n_heads=2, seq_len=50, token_dim=6,
                                batch=3, bf16=True), True),
]


@pytest.mark.parametrize("dtype", [2, 1], ids=["f16", "bf16"])
@pytest.mark.parametrize("name,cfg,perturb", BF16_CASES, ids=[c[0] for c in BF16_CASES])
def test_bf16_conditioner_matches_oracle(torch_cuda, orc64, name, cfg, perturb, dtype):
    torch = torch_cuda
    blob = wl.make_weights(cfg, perturb_affine=perturb)
    x = wl.make_latent(cfg, seed=3)
    f = _flow(cfg, blob, dtype=dtype)
    worst = 0.0
    for j in range(cfg.n_blocks):
        mu, al = f.conditioner(j, _dev(torch, x))
        mu, al = mu.cpu().numpy(), al.cpu().numpy()
        rev = (cfg.reverse_mask >> j) & 1
        for b in range(cfg.batch):
            xb = x[b][::-1] if rev else x[b]
            rmu, ral = orc64.cond(cfg, blob, j, xb)
            if rev:
                rmu, ral = rmu[::-1], ral[::-1]
            worst = max(worst, np.abs(mu[b] - rmu).max(), np.abs(al[b] - ral).max())
    print(f"{name} dtype {dtype}: worst conditioner error {worst:.3e}")
    # One pass of the conditioner, not final samples: the bounds are this build's own, tighter than the 2e-2 that
    # the task states for samples, and sit a factor of two above what these cases measure (IEEE half <= 3.0e-4,
    # bf16 <= 2.3e-3: eight times coarser operands)
    assert worst <= (1e-3 if dtype == 2 else 5e-3)
    f.close()


@pytest.mark.parametrize("dtype", [2, 1], ids=["f16", "bf16"])
@pytest.mark.parametrize("name,cfg,perturb", BF16_CASES, ids=[c[0] for c in BF16_CASES])
@pytest.mark.parametrize("mode", ["selective", "sequential", "all_jacobi"])
def test_bf16_sample_matches_oracle(torch_cuda, orc64, name, cfg, perturb, mode, dtype):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    mask = {"selective": ~1, "sequential": 0, "all_jacobi": ~0}[mode] & ((1 << cfg.n_blocks) - 1)
    blob = wl.make_weights(cfg, perturb_affine=perturb)
    z = wl.make_latent(cfg)
    f = _flow(cfg, blob, dtype=dtype)
    x, stats, iters = f.sample(_dev(torch, z), mask, sjd.JacobiOpts(tau=cfg.tau))
    x = x.cpu().numpy()
    rx, riters, _ = orc64.sample(cfg, blob, z, mask, cfg.tau)
    err = np.abs(x - rx).max()
    print(f"{name}/{mode} dtype {dtype}: max err {err:.3e}; passes gpu {iters.max(axis=1)} oracle {riters.max(axis=1)}")
    assert err <= TOL_BF16
    if dtype == 2:
        assert np.abs(iters.astype(int) - riters).max() <= 1  # 16-bit rounding may move a stop by one pass
    f.close()


def test_config2_subset_matches_oracle(torch_cuda, orc32):
    """Configuration 2 at its real shape on the first samples of the batch (samples are
    independent): final samples within 2e-2 of the oracle, pass counts within one."""
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    cfg = wl.CONFIGS["C2"]
    nb = 8
    blob = wl.make_weights(cfg)
    z = wl.make_latent(cfg)[:nb]
    f = _flow(cfg, blob, max_batch=nb)
    mask = ~1 & ((1 << cfg.n_blocks) - 1)
    x, stats, iters = f.sample(_dev(torch, z), mask, sjd.JacobiOpts(tau=cfg.tau))
    x = x.cpu().numpy()
    rx, riters, _ = orc32.sample(cfg, blob, z, mask, cfg.tau)
    err = np.abs(x - rx).max()
    print(f"C2 subset: max err {err:.3e}; passes gpu {iters.max(axis=1)} oracle {riters.max(axis=1)}")
    assert err <= TOL_BF16
    assert np.abs(iters.astype(int) - riters).max() <= 1
    f.close()


def test_config2_full_batch_sampled_outputs_match_oracle(torch_cuda, orc32):
    """Configuration 2 exactly as `bench.py` launches it (batch 64, selective strategy, default
    options): the oracle recomputes a spread of samples one by one (samples are independent), and
    properties that hold for every sample are checked on all of them."""
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    cfg = wl.CONFIGS["C2"]
    blob = wl.make_weights(cfg)
    z = wl.make_latent(cfg)
    f = _flow(cfg, blob)
    mask = ~1 & ((1 << cfg.n_blocks) - 1)
    zd = _dev(torch, z)
    x, stats, iters = f.sample(zd, mask, sjd.JacobiOpts(tau=cfg.tau))
    xs = x.cpu().numpy()
    picks = [0, 9, 26, 47, 63]
    rx, riters, _ = orc32.sample(cfg, blob, z[picks], mask, cfg.tau)
    err = np.abs(xs[picks] - rx).max()
    print(f"C2 full batch: max err on samples {picks}: {err:.3e}; passes {stats['block_iters']}")
    assert err <= TOL_BF16
    assert np.abs(iters[:, picks].astype(int) - riters).max() <= 1
    # every sample: finite, block 0 took T-1 steps, Jacobi blocks between 2 passes and the cap, and the
    # forward map takes the result back to the latent (Jacobi blocks stopped at tau, so to within a few tau)
    assert np.isfinite(xs).all()
    assert (iters[0] == cfg.seq_len - 1).all()
    assert (iters[1:] >= 2).all() and (iters[1:] <= cfg.seq_len).all()
    zz, logdet = f.forward(x)
    assert (zz - zd).abs().max().item() <= 0.1
    assert (zz - zd).abs().mean().item() <= 5 * cfg.tau
    assert torch.isfinite(logdet).all()
    # a second run gives the same bits
    x2, _, iters2 = f.sample(zd, mask, sjd.JacobiOpts(tau=cfg.tau))
    assert torch.equal(x, x2) and np.array_equal(iters, iters2)
    f.close()
