"""Two batches in flight (sequential block of one beside the Jacobi blocks of the previous one, on
streams restricted to disjoint sets of CUs) give the bits and pass counts of plain sampling.
Needs an MI355X."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def test_pipelined_sampling_matches_plain_sampling():
    import torch
    import paper_2505_24791_amd as sjd
    from paper_2505_24791_amd.pipeline import PipelinedSampler
    assert torch.cuda.is_available(), "this test needs the GPU"
    cfg = wl.FlowConfig("pipe", n_blocks=3, n_layers=2, width=256, n_heads=4, seq_len=24, token_dim=6, batch=12, bf16=True)
    blob = wl.make_weights(cfg, perturb_affine=True)
    zs = [torch.from_numpy(wl.make_latent(cfg, seed=70 + i)).cuda() for i in range(5)]
    opts = sjd.JacobiOpts(tau=1e-3)
    f = sjd.Flow(cfg)
    f.load_weights(blob)
    ref, ref_passes = [], []
    for z in zs:
        x, st, _ = f.sample(z, 0b110, opts)
        ref.append(x.clone())
        ref_passes.append(list(st["block_iters"]))
    f.close()
    for n_seq in (128, 64):
        print(f"pipelined, {n_seq} CUs for the sequential block", flush=True)
        ps = PipelinedSampler(cfg, blob, n_seq_cus=n_seq)
        outs, passes = ps.run(zs, opts)
        ps.close()
        for i, (a, b) in enumerate(zip(outs, ref)):
            assert torch.equal(a, b), (n_seq, i)
            assert passes[i] == ref_passes[i], (n_seq, i, passes[i], ref_passes[i])


def test_sequential_workgroup_count_is_validated():
    import paper_2505_24791_amd as sjd
    cfg = wl.FlowConfig("pipe2", n_blocks=1, n_layers=1, width=256, n_heads=4, seq_len=8, token_dim=4, batch=2, bf16=True)
    f = sjd.Flow(cfg)
    for bad in (8, 48, 100, 288, -32):
        with pytest.raises(sjd.SjdError) as e:
            f.set_sequential_cus(bad)
        assert e.value.code == sjd.SJD_EINVAL
    f.set_sequential_cus(64)
    f.set_sequential_cus(0)
    f.close()
