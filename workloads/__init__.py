"""Seeded synthetic workloads for selective Jacobi decoding of a block-autoregressive flow.

This module only *draws numbers and lays them out*: flow configurations, the flat weight blob,
and latent batches.  It contains none of the method's arithmetic (no conditioner, no affine map,
no stopping rule), so that the CPU oracle and the HIP library can both be fed from it without
sharing any code of the method itself.

Weight blob (headerless, little-endian float32, one flow block after another in *sampling
order*: block 0 is the first one applied to the latent).  Matrices are row-major ``[in, out]``
so that a token row ``a`` is mapped by ``a @ W + b``:

    per block:
        w_in   [D, W]      b_in  [W]       pos  [T, W]
        per transformer layer (N of them):
            ln1_g [W]  ln1_b [W]
            w_qkv [W, 3W]  b_qkv [3W]      # columns = [q | k | v]; head h owns h*dh..(h+1)*dh of each
            w_o   [W, W]   b_o   [W]
            ln2_g [W]  ln2_b [W]
            w_fc1 [W, R*W] b_fc1 [R*W]
            w_fc2 [R*W, W] b_fc2 [W]
        lnf_g [W]  lnf_b [W]
        w_head [W, 2D]  b_head [2D]        # columns = [mu | alpha]

Recipe (the paper trains its flows; trained weights and datasets are not available, so seeded
Gaussians of the same shapes stand in for them): every matrix and the positional table ~
N(0, 0.02^2); ``w_head`` ~ N(0, 0.01^2); biases 0, LayerNorm gain 1 / shift 0.  With
``perturb_affine=True`` the biases and LayerNorm parameters are drawn at random as well, which
tests use so that a misplaced bias or gain cannot hide behind a zero.  For bf16 configurations the
drawn values are rounded to the nearest bf16 (ties to even) and stored widened back to float32, so
both consumers see bit-identical weights.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Iterator, List, Tuple

import numpy as np

WEIGHT_SEED_BASE = 20250524
LATENT_SEED = 7


@dataclass(frozen=True)
class FlowConfig:
    name: str
    n_blocks: int      # K
    n_layers: int      # N transformer layers per block
    width: int         # W
    n_heads: int       # H
    seq_len: int       # T tokens
    token_dim: int     # D
    batch: int         # B
    bf16: bool
    mlp_ratio: int = 4
    tau: float = 1e-3
    temperature: float = 1.0
    mask_nearest: int = 0   # o of the masked-dependency probe (eq. 6): attention skips the o nearest predecessors

    @property
    def head_dim(self) -> int:
        return self.width // self.n_heads

    @property
    def reverse_mask(self) -> int:
        """Bit j set: block j (sampling order) works on the reversed token order (odd blocks)."""
        m = 0
        for j in range(self.n_blocks):
            if j % 2 == 1:
                m |= 1 << j
        return m

    def with_(self, **kw) -> "FlowConfig":
        return replace(self, **kw)


CONFIGS: Dict[str, FlowConfig] = {
    # 28x28x1, patch 4
    "C1": FlowConfig("C1", n_blocks=4, n_layers=2, width=128, n_heads=4, seq_len=49, token_dim=16,
                     batch=4, bf16=False),
    # 32x32x3, patch 2
    "C2": FlowConfig("C2", n_blocks=4, n_layers=4, width=512, n_heads=8, seq_len=256, token_dim=12,
                     batch=64, bf16=True),
    "C3": FlowConfig("C3", n_blocks=8, n_layers=8, width=768, n_heads=12, seq_len=256, token_dim=12,
                     batch=256, bf16=True, temperature=0.9),
    # 64x64x3, patch 4
    "C4": FlowConfig("C4", n_blocks=8, n_layers=8, width=1024, n_heads=16, seq_len=256, token_dim=48,
                     batch=128, bf16=True),
    # 128x128x3, patch 4
    "C5": FlowConfig("C5", n_blocks=8, n_layers=8, width=1024, n_heads=16, seq_len=1024, token_dim=48,
                     batch=32, bf16=True),
}


def block_tensors(cfg: FlowConfig) -> List[Tuple[str, Tuple[int, ...]]]:
    """Names and shapes of one block's tensors, in blob order."""
    D, W, T, R = cfg.token_dim, cfg.width, cfg.seq_len, cfg.mlp_ratio
    out: List[Tuple[str, Tuple[int, ...]]] = [("w_in", (D, W)), ("b_in", (W,)), ("pos", (T, W))]
    for l in range(cfg.n_layers):
        p = f"l{l}."
        out += [
            (p + "ln1_g", (W,)), (p + "ln1_b", (W,)),
            (p + "w_qkv", (W, 3 * W)), (p + "b_qkv", (3 * W,)),
            (p + "w_o", (W, W)), (p + "b_o", (W,)),
            (p + "ln2_g", (W,)), (p + "ln2_b", (W,)),
            (p + "w_fc1", (W, R * W)), (p + "b_fc1", (R * W,)),
            (p + "w_fc2", (R * W, W)), (p + "b_fc2", (W,)),
        ]
    out += [("lnf_g", (W,)), ("lnf_b", (W,)), ("w_head", (W, 2 * D)), ("b_head", (2 * D,))]
    return out


def block_floats(cfg: FlowConfig) -> int:
    return int(sum(int(np.prod(s)) for _, s in block_tensors(cfg)))


def blob_floats(cfg: FlowConfig) -> int:
    return cfg.n_blocks * block_floats(cfg)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result is float32 again.
    (Finite inputs far from overflow, which is all this module draws.)"""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty_like(a)
    flat_in, flat_out = a.reshape(-1), out.reshape(-1)
    step = 1 << 24
    for i in range(0, flat_in.size, step):          # chunked: no blob-sized temporaries
        u = flat_in[i:i + step].view(np.uint32)
        r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
        r &= np.uint32(0xFFFF0000)
        flat_out[i:i + step] = r.view(np.float32)
    return out


def make_weights(cfg: FlowConfig, seed_base: int = WEIGHT_SEED_BASE, *, perturb_affine: bool = False,
                 std: float = 0.02, head_std: float = 0.01) -> np.ndarray:
    """The whole flow's weight blob as a flat float32 array (see the module docstring)."""
    blob = np.empty(blob_floats(cfg), dtype=np.float32)
    off = 0
    for j in range(cfg.n_blocks):
        rng = np.random.Generator(np.random.PCG64(seed_base + j))
        for name, shape in block_tensors(cfg):
            n = int(np.prod(shape))
            base = name.split(".")[-1]
            if base.startswith("w_") or base == "pos":
                s = head_std if base == "w_head" else std
                v = rng.standard_normal(n, dtype=np.float32) * np.float32(s)
            elif base.endswith("_g"):
                v = np.ones(n, np.float32)
                if perturb_affine:
                    v = v + rng.standard_normal(n, dtype=np.float32) * np.float32(0.1)
            else:  # biases and LayerNorm shifts
                v = np.zeros(n, np.float32)
                if perturb_affine:
                    v = rng.standard_normal(n, dtype=np.float32) * np.float32(std)
            blob[off:off + n] = v
            off += n
    assert off == blob.size
    if cfg.bf16:
        blob = round_to_bf16(blob)
    return blob


def cached_weights(cfg: FlowConfig, cache_dir: str | None = None) -> np.ndarray:
    """``make_weights(cfg)`` with an on-disk cache (``.npy`` under the system temp directory): the
    larger workloads draw several hundred million numbers, which takes longer than the GPU work."""
    import os
    import tempfile
    d = cache_dir or os.path.join(tempfile.gettempdir(), "sjd_workloads")
    os.makedirs(d, exist_ok=True)
    path = os.path.join(d, f"{cfg.name}_K{cfg.n_blocks}_N{cfg.n_layers}_W{cfg.width}_T{cfg.seq_len}_D{cfg.token_dim}"
                           f"_{'bf16' if cfg.bf16 else 'f32'}_{WEIGHT_SEED_BASE}.npy")
    if os.path.exists(path):
        try:
            blob = np.load(path)
            if blob.dtype == np.float32 and blob.size == blob_floats(cfg):
                return blob
        except Exception:
            pass
    blob = make_weights(cfg)
    try:
        np.save(path, blob)
    except OSError:
        pass
    return blob


def blob_views(cfg: FlowConfig, blob: np.ndarray) -> List[Dict[str, np.ndarray]]:
    """Per-block dicts of named views into ``blob`` (no copies); for tests that edit weights."""
    assert blob.dtype == np.float32 and blob.size == blob_floats(cfg)
    views = []
    off = 0
    for _ in range(cfg.n_blocks):
        d = {}
        for name, shape in block_tensors(cfg):
            n = int(np.prod(shape))
            d[name] = blob[off:off + n].reshape(shape)
            off += n
        views.append(d)
    return views


def make_latent(cfg: FlowConfig, batch: int | None = None, seed: int = LATENT_SEED) -> np.ndarray:
    """z ~ N(0, I) scaled by the config's noise temperature, float32 ``[B, T, D]``."""
    b = cfg.batch if batch is None else batch
    rng = np.random.Generator(np.random.PCG64(seed))
    z = rng.standard_normal((b, cfg.seq_len, cfg.token_dim), dtype=np.float32)
    return (z * np.float32(cfg.temperature)).astype(np.float32)


def tiny_config(T: int, D: int = 3, W: int = 16, H: int = 2, N: int = 1, K: int = 2, B: int = 2,
                bf16: bool = False, name: str = "tiny") -> FlowConfig:
    return FlowConfig(name, n_blocks=K, n_layers=N, width=W, n_heads=H, seq_len=T, token_dim=D,
                      batch=B, bf16=bf16)


def iter_configs() -> Iterator[FlowConfig]:
    return iter(CONFIGS.values())
