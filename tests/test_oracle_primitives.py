"""Pins for the oracle's building blocks: each is checked against a library routine or a closed
form that does not go through the oracle's own code.  CPU only."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as wl

RNG = np.random.default_rng(123)


@pytest.mark.parametrize("W", [1, 7, 128, 1000])
def test_layernorm_matches_library(orc64, W):
    x = RNG.standard_normal((5, W)) * 3 + 1.5
    g = RNG.standard_normal(W).astype(np.float32)
    b = RNG.standard_normal(W).astype(np.float32)
    got = orc64.layernorm(x, g, b)
    ref = F.layer_norm(torch.from_numpy(x), (W,), torch.from_numpy(g).double(), torch.from_numpy(b).double(), 1e-5)
    np.testing.assert_allclose(got, ref.numpy(), rtol=1e-12, atol=1e-12)


def test_layernorm_closed_form(orc64):
    # a row (1, -1) has mean 0 and biased variance 1: y = +-1/sqrt(1 + 1e-5)
    y = orc64.layernorm(np.array([[1.0, -1.0]]), np.ones(2, np.float32), np.zeros(2, np.float32))
    r = 1.0 / math.sqrt(1.0 + 1e-5)
    np.testing.assert_allclose(y, [[r, -r]], rtol=1e-14)
    # a constant row maps to the shift
    y = orc64.layernorm(np.full((1, 9), 4.0), np.full(9, 2.0, np.float32), np.full(9, 0.5, np.float32))
    np.testing.assert_allclose(y, np.full((1, 9), 0.5), atol=1e-12)


def test_gelu_is_the_erf_form(orc64):
    x = np.linspace(-6, 6, 241)
    got = orc64.gelu(x)
    ref = F.gelu(torch.from_numpy(x), approximate="none").numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-15)
    # x * Phi(x) with Phi from the complementary error function; and not the tanh approximation
    phi = np.array([0.5 * math.erfc(-v / math.sqrt(2)) for v in x])
    np.testing.assert_allclose(got, x * phi, rtol=1e-12, atol=1e-15)
    assert np.abs(got - F.gelu(torch.from_numpy(x), approximate="tanh").numpy()).max() > 1e-4


def test_linear_is_row_times_matrix_plus_bias(orc64):
    a = RNG.standard_normal((6, 11))
    Wm = RNG.standard_normal((11, 5)).astype(np.float32)
    b = RNG.standard_normal(5).astype(np.float32)
    got = orc64.linear(a, Wm, b)
    ref = F.linear(torch.from_numpy(a), torch.from_numpy(Wm).double().T, torch.from_numpy(b).double()).numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)
    # a non-square weight with a single 1 picks one input column: catches a transposed operand
    E = np.zeros((11, 5), np.float32); E[3, 1] = 1
    got = orc64.linear(a, E, np.zeros(5, np.float32))
    assert np.array_equal(got[:, 1], a[:, 3]) and np.count_nonzero(got) == 6


@pytest.mark.parametrize("T,W,H", [(1, 8, 2), (5, 12, 3), (17, 64, 4), (49, 128, 4)])
def test_causal_attention_matches_library(orc64, T, W, H):
    q, k, v = (RNG.standard_normal((T, W)) for _ in range(3))
    got = orc64.causal_attention(q, k, v, H)
    dh = W // H
    tq, tk, tv = (torch.from_numpy(a).reshape(T, H, dh).permute(1, 0, 2).unsqueeze(0) for a in (q, k, v))
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)  # scale = 1/sqrt(dh)
    ref = ref.squeeze(0).permute(1, 0, 2).reshape(T, W).numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)


def test_causal_attention_closed_forms(orc64):
    T, W, H = 9, 8, 2
    v = RNG.standard_normal((T, W))
    # equal keys => uniform weights over the visible prefix => running mean of the values
    q = RNG.standard_normal((T, W)); k = np.tile(RNG.standard_normal((1, W)), (T, 1))
    got = orc64.causal_attention(q, k, v, H)
    ref = np.cumsum(v, axis=0) / np.arange(1, T + 1)[:, None]
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)
    # first row sees only itself
    got = orc64.causal_attention(RNG.standard_normal((T, W)), RNG.standard_normal((T, W)), v, H)
    np.testing.assert_allclose(got[0], v[0], rtol=1e-13)
    # two tokens, one head of size 1, by hand: weights softmax([q1 k0, q1 k1])
    q = np.array([[0.3], [2.0]]); k = np.array([[1.0], [-0.5]]); vv = np.array([[10.0], [20.0]])
    e0, e1 = math.exp(2.0 * 1.0), math.exp(2.0 * -0.5)
    got = orc64.causal_attention(q, k, vv, 1)
    np.testing.assert_allclose(got[:, 0], [10.0, (e0 * 10 + e1 * 20) / (e0 + e1)], rtol=1e-13)
    # heads do not mix: changing head 1's keys leaves head 0's output alone
    q, k = RNG.standard_normal((T, W)), RNG.standard_normal((T, W))
    a = orc64.causal_attention(q, k, v, H)
    k2 = k.copy(); k2[:, W // H:] += 1.0
    b = orc64.causal_attention(q, k2, v, H)
    assert np.array_equal(a[:, :W // H], b[:, :W // H]) and not np.array_equal(a[:, W // H:], b[:, W // H:])


def _torch_conditioner(cfg, views, x):
    """The conditioner from library routines only (layer_norm, linear, sdpa, gelu), float64."""
    T, W, H, D = cfg.seq_len, cfg.width, cfg.n_heads, cfg.token_dim
    g = lambda name: torch.from_numpy(views[name]).double()
    h = F.linear(torch.from_numpy(x).double(), g("w_in").T, g("b_in")) + g("pos")
    for l in range(cfg.n_layers):
        p = f"l{l}."
        a = F.layer_norm(h, (W,), g(p + "ln1_g"), g(p + "ln1_b"), 1e-5)
        qkv = F.linear(a, g(p + "w_qkv").T, g(p + "b_qkv"))
        q, k, v = (t.reshape(T, H, W // H).permute(1, 0, 2).unsqueeze(0) for t in qkv.split(W, dim=1))
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True).squeeze(0).permute(1, 0, 2).reshape(T, W)
        h = h + F.linear(o, g(p + "w_o").T, g(p + "b_o"))
        m = F.layer_norm(h, (W,), g(p + "ln2_g"), g(p + "ln2_b"), 1e-5)
        h = h + F.linear(F.gelu(F.linear(m, g(p + "w_fc1").T, g(p + "b_fc1"))), g(p + "w_fc2").T, g(p + "b_fc2"))
    out = F.linear(F.layer_norm(h, (W,), g("lnf_g"), g("lnf_b"), 1e-5), g("w_head").T, g("b_head"))
    mu = torch.zeros(T, D, dtype=torch.float64); al = torch.zeros(T, D, dtype=torch.float64)
    mu[1:] = out[:-1, :D]; al[1:] = out[:-1, D:]
    return mu.numpy(), al.numpy()


@pytest.mark.parametrize("T,D,W,H,N", [(6, 3, 16, 2, 2), (49, 16, 128, 4, 2)])
def test_whole_conditioner_matches_library_composition(orc64, orc32, T, D, W, H, N):
    cfg = wl.tiny_config(T=T, D=D, W=W, H=H, N=N, K=2)
    blob = wl.make_weights(cfg, perturb_affine=True, std=0.08, head_std=0.05)
    views = wl.blob_views(cfg, blob)
    x = RNG.standard_normal((T, D))
    for j in range(cfg.n_blocks):
        mu, al = orc64.cond(cfg, blob, j, x)
        rmu, ral = _torch_conditioner(cfg, views[j], x)
        np.testing.assert_allclose(mu, rmu, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(al, ral, rtol=1e-10, atol=1e-12)
        assert np.all(mu[0] == 0) and np.all(al[0] == 0)
        mu32, al32 = orc32.cond(cfg, blob, j, x)
        np.testing.assert_allclose(mu32, rmu, atol=2e-5)
        np.testing.assert_allclose(al32, ral, atol=2e-5)


def test_blob_size_and_parameter_count():
    # per block: D*W + W + T*W + N*(12 W^2 + 13 W) + 2W + 2DW + 2D with the 4x MLP
    for cfg in wl.iter_configs():
        D, W, T, N = cfg.token_dim, cfg.width, cfg.seq_len, cfg.n_layers
        expect = D * W + W + T * W + N * (12 * W * W + 13 * W) + 2 * W + 2 * D * W + 2 * D
        assert wl.block_floats(cfg) == expect


def test_bf16_rounding_is_nearest_even():
    a = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, -3.14159, 0.0], np.float32)
    r = wl.round_to_bf16(a)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.0 + 2.0 ** -7) and r[3] == np.float32(1.0 + 2.0 ** -6)
    t = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r, t)
    big = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    assert np.array_equal(wl.round_to_bf16(big), torch.from_numpy(big).to(torch.bfloat16).float().numpy())
