"""What the three arithmetic modes deliver at workload scale: configuration 2 at its real shape on the
first samples of the batch, against the float32 CPU oracle.  Needs an MI355X.

The record these tests pin (measured on the MI355X):

  mode            all-sequential sample   selective, tau = 1e-3          selective, tau = 1e-4
  float32         err 1e-5                err 1e-5, oracle's counts      err 1e-5, oracle's counts
  IEEE half       err 3e-3                err 2e-3, oracle's counts      err 3e-3, 59..79 passes (oracle 8..10)
  bf16 operands   err 2.3e-2 (> 2e-2)     err 2e-2, 21..41 passes        230..235 passes of 256

  half + float32 refinement below 1e-3 (sjd_jacobi_opts.refine_below):            err 3e-3, oracle's counts (+-1)

Every 16-bit operand is a rounding stage; Jacobi decoding iterates the map, so once the true change of
an iterate is below the rounding noise of one pass the difference norm stays at that noise: about 1.4e-4
(mean |dx|) with IEEE-half operands and 1.1e-3 with bf16 operands.  A threshold under the floor is only
met by chance, far later than in exact arithmetic - the result stays as accurate as the mode allows, the
count does not.  Hence: IEEE half is the default 16-bit mode, it is exact in the counts down to
tau = 1e-3, and below the floor (tau = 1e-4) the float32 mode reproduces the oracle's counts.
"""
import numpy as np
import pytest

import workloads as wl

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]
NB = 4


@pytest.fixture(scope="module")
def c2(orc32):
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    cfg = wl.CONFIGS["C2"]
    blob = wl.make_weights(cfg)
    z = wl.make_latent(cfg)[:NB]
    full = (1 << cfg.n_blocks) - 1
    ref = {"seq": orc32.sample(cfg, blob, z, 0, 1e-3)[0]}
    for tau in (1e-3, 1e-4):
        ref[tau] = orc32.sample(cfg, blob, z, ~1 & full, tau)
    return cfg, blob, z, torch.from_numpy(z).cuda(), full, ref


def _run(c2, dtype, tau, **opts):
    import paper_2505_24791_amd as sjd
    cfg, blob, z, zd, full, ref = c2
    f = sjd.Flow(cfg, max_batch=NB, dtype=dtype)
    f.load_weights(blob)
    xs, _, _ = f.sample(zd, 0, sjd.JacobiOpts(tau=tau))
    xj, _, iters = f.sample(zd, ~1 & full, sjd.JacobiOpts(tau=tau, **opts))
    f.close()
    err_seq = float(np.abs(xs.cpu().numpy() - ref["seq"]).max())
    err_sel = float(np.abs(xj.cpu().numpy() - ref[tau][0]).max())
    return err_seq, err_sel, iters, ref[tau][1], ref[tau][2]


def _not_knife_edge(rdel, tau):
    return ~((rdel > 0) & (np.abs(rdel - tau) <= 0.01 * tau))


def test_float32_mode_reproduces_the_oracle_counts_down_to_tau_1e_4(c2):
    for tau in (1e-3, 1e-4):
        err_seq, err_sel, iters, riters, rdel = _run(c2, 0, tau)
        print(f"float32, tau {tau:g}: err {err_seq:.2e} / {err_sel:.2e}, passes {iters[1:].tolist()}")
        assert err_seq <= 1e-4 and err_sel <= 1e-4
        ok = _not_knife_edge(rdel, tau)
        assert np.array_equal(iters[ok], riters[ok])


def test_half_mode_is_exact_in_the_counts_at_tau_1e_3_and_floor_limited_at_1e_4(c2):
    err_seq, err_sel, iters, riters, rdel = _run(c2, 2, 1e-3)
    print(f"IEEE half, tau 1e-3: err {err_seq:.2e} / {err_sel:.2e}, passes {iters[1:].tolist()}")
    assert err_seq <= 2e-2 and err_sel <= 2e-2
    ok = _not_knife_edge(rdel, 1e-3)
    assert (np.abs(iters.astype(int) - riters)[ok] <= 1).all()
    err_seq, err_sel, iters, riters, rdel = _run(c2, 2, 1e-4)
    print(f"IEEE half, tau 1e-4: err {err_sel:.2e}, passes {iters[1:].tolist()} (oracle {riters[1:].tolist()})")
    # under the noise floor of the mode: never earlier than the oracle, far later, and the samples stay accurate
    assert err_sel <= 2e-2
    assert (iters[1:] >= riters[1:]).all()
    assert iters[1:].min() >= 3 * riters[1:].max(), "the floor moved: revisit the record at the top of this file"
    assert iters[1:].max() < c2[0].seq_len, "every sample still stops by its own test, none runs to the cap"


def test_bf16_operands_miss_the_sample_bound_and_the_counts_at_workload_scale(c2):
    err_seq, err_sel, iters, riters, rdel = _run(c2, 1, 1e-3)
    print(f"bf16 operands, tau 1e-3: err {err_seq:.2e} / {err_sel:.2e}, passes {iters[1:].tolist()} (oracle {riters[1:].tolist()})")
    # measured 2.3e-2 / 2.0e-2: around the task's 2e-2, not safely under it; bounded here by twice that
    assert 5e-3 <= err_seq <= 4e-2 and err_sel <= 4e-2
    # the difference norm floors near tau: two to five times the oracle's passes
    assert (iters[1:] >= riters[1:]).all()
    assert iters[1:].min() >= 2 * riters[1:].max(), "bf16 counts came close to the oracle's: revisit the record"


def test_half_mode_with_float32_refinement_follows_the_oracle_counts_under_the_floor(c2):
    """tau = 1e-4 lies under the rounding floor of half operands.  With refine_below = 1e-3 a sample's passes run
    in float32 once its delta is under 1e-3: the float32 passes contract the rounding noise of the half passes
    away like any other error of the iterate, and the sample stops within one pass of exact arithmetic."""
    err_seq, err_sel, iters, riters, rdel = _run(c2, 2, 1e-4, refine_below=1e-3)
    print(f"IEEE half + float32 below 1e-3, tau 1e-4: err {err_sel:.2e}, passes {iters[1:].tolist()} "
          f"(oracle {riters[1:].tolist()})")
    assert err_sel <= 2e-2
    ok = _not_knife_edge(rdel, 1e-4)
    assert (np.abs(iters.astype(int) - riters)[ok] <= 1).all()


def test_refinement_is_per_sample(c2):
    """A sample switches to float32 by its own delta, so its result and count do not depend on the batch it runs
    in: each sample alone gives the bits it gives inside the batch."""
    import torch
    import paper_2505_24791_amd as sjd
    cfg, blob, z, zd, full, ref = c2
    f = sjd.Flow(cfg, max_batch=NB, dtype=2)
    f.load_weights(blob)
    opts = sjd.JacobiOpts(tau=1e-4, refine_below=1e-3)
    y = f.sequential_inverse_block(0, zd)
    xb, itb, _, _ = f.jacobi_inverse_block(1, y, opts)
    for b in (0, NB - 1):
        x1, it1, _, _ = f.jacobi_inverse_block(1, y[b:b + 1].contiguous(), opts)
        assert torch.equal(x1[0], xb[b]) and int(it1[0]) == int(itb[b])
    # keeping converged samples in the batch changes neither results nor counts
    xk, itk, _, _ = f.jacobi_inverse_block(1, y, sjd.JacobiOpts(tau=1e-4, refine_below=1e-3, drop_converged=0))
    assert torch.equal(xk, xb) and np.array_equal(itk, itb)
    f.close()


def test_max_norm_of_alg1_with_refinement_follows_the_oracle(c2):
    """The maximum norm that Alg. 1 prints is floor-limited in half at tau = 1e-3 already (the maximum over a
    sample's values of the same rounding noise is several times its mean: 63-192 passes measured).  Refined
    below 1e-2 it stops within one pass of the float32 oracle."""
    import paper_2505_24791_amd as sjd
    cfg, blob, z, zd, full, ref = c2
    f = sjd.Flow(cfg, max_batch=NB, dtype=2)
    f.load_weights(blob)
    y = f.sequential_inverse_block(0, zd)
    x, iters, _, _ = f.jacobi_inverse_block(1, y, sjd.JacobiOpts(tau=1e-3, criterion=1, refine_below=1e-2))
    yh = y.cpu().numpy()
    from oracle import Oracle
    orc = Oracle("f32")
    for b in range(NB):
        rx, rit, tr = orc.jacobi_inverse_block(cfg, blob, 1, yh[b], 1e-3, criterion=1, want_trace=True)
        print(f"max norm, sample {b}: gpu {int(iters[b])} passes, oracle {rit} (last delta {tr[rit - 1]:.3e})")
        assert np.abs(x[b].cpu().numpy() - rx).max() <= 2e-2
        if abs(tr[rit - 1] - 1e-3) > 1e-5:
            assert abs(int(iters[b]) - rit) <= 1
    f.close()
