"""The masked-dependency probe (Sec. 3.2, eq. 6: attention without the o nearest predecessors) on the
device against the CPU oracle, through the C boundary.  Needs an MI355X."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu

F32 = wl.FlowConfig("probe_f32", n_blocks=2, n_layers=2, width=96, n_heads=3, seq_len=21, token_dim=5, batch=4, bf16=False)
H16 = wl.FlowConfig("probe_h16", n_blocks=2, n_layers=2, width=256, n_heads=4, seq_len=30, token_dim=6, batch=5, bf16=True)


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


@pytest.mark.parametrize("cfg,tol", [(F32, 1e-4), (H16, 2e-2)], ids=["f32", "half"])
@pytest.mark.parametrize("o", [1, 3, 40])
def test_masked_probe_matches_oracle(torch_cuda, orc32, cfg, tol, o):
    import paper_2505_24791_amd as sjd
    torch = torch_cuda
    o = min(o, cfg.seq_len)
    blob = wl.make_weights(cfg, perturb_affine=True)
    z = wl.make_latent(cfg, seed=13)
    zd = torch.from_numpy(z).cuda()
    mcfg = cfg.with_(mask_nearest=o)
    f = sjd.Flow(cfg)
    f.load_weights(blob)
    plain = f.sequential_inverse_block(0, zd).cpu().numpy()
    f.set_mask_nearest(o)
    for j in range(cfg.n_blocks):
        # conditioner
        mu, al = f.conditioner(j, zd)
        rev = (cfg.reverse_mask >> j) & 1
        for b in range(cfg.batch):
            xb = z[b][::-1] if rev else z[b]
            rmu, ral = orc32.cond(mcfg, blob, j, xb)
            if rev:
                rmu, ral = rmu[::-1], ral[::-1]
            assert np.abs(mu[b].cpu().numpy() - rmu).max() <= tol and np.abs(al[b].cpu().numpy() - ral).max() <= tol
        # sequential inverse, and Jacobi decoding run to the cap reaches the same masked solution
        xs = f.sequential_inverse_block(j, zd).cpu().numpy()
        xj, iters, passes, _ = f.jacobi_inverse_block(j, zd, sjd.JacobiOpts(tau=0.0))
        for b in range(cfg.batch):
            ref = orc32.sequential_inverse_block(mcfg, blob, j, z[b])
            assert np.abs(xs[b] - ref).max() <= tol, (j, b)
            assert np.abs(xj[b].cpu().numpy() - ref).max() <= tol, (j, b)
        assert passes == cfg.seq_len
        # the forward map of the masked model inverts its sequential inverse
        zz, _ = f.forward_block(j, torch.from_numpy(xs).cuda())
        assert (zz - zd).abs().max().item() <= (1e-4 if not cfg.bf16 else 2e-2)
    masked0 = f.sequential_inverse_block(0, zd).cpu().numpy()
    assert np.abs(masked0 - plain).max() > 10 * tol or cfg.bf16          # the probe really changes the result
    f.set_mask_nearest(0)
    assert np.array_equal(f.sequential_inverse_block(0, zd).cpu().numpy(), plain)   # and switches off again
    with pytest.raises(sjd.SjdError):
        f.set_mask_nearest(cfg.seq_len + 1)
    f.close()
