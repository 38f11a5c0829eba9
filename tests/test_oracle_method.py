"""Pins for the oracle at the level of the method: what the paper and the mathematics fix about
the forward map (eq. 4), the sequential inverse (eq. 5), the Jacobi map F (Def. A.1) and Jacobi
decoding (Alg. 1, Props. 3.1 and 3.2).  CPU only; brute force on tiny sizes."""
import numpy as np
import pytest

import workloads as wl

TINY_T = [1, 2, 3, 5, 8]


def _flow(T, seed=0, **kw):
    kw.setdefault("K", 3)
    cfg = wl.tiny_config(T=T, **kw)
    # strong weights so that the conditioner really depends on its context
    blob = wl.make_weights(cfg, seed_base=1000 + seed, perturb_affine=True, std=0.15, head_std=0.1)
    z = wl.make_latent(cfg, batch=3, seed=seed + 5)
    return cfg, blob, z


# ---- eq. 4 / eq. 5 are mutual inverses -------------------------------------------------------

@pytest.mark.parametrize("T", TINY_T)
def test_forward_of_sequential_inverse_is_identity_tiny(orc64, orc32, T):
    cfg, blob, z = _flow(T)
    for j in range(cfg.n_blocks):
        x = orc64.sequential_inverse_block(cfg, blob, j, z[0])
        np.testing.assert_allclose(orc64.forward_block(cfg, blob, j, x), z[0], atol=1e-12)
        # and the other way round
        y = orc64.forward_block(cfg, blob, j, z[1])
        np.testing.assert_allclose(orc64.sequential_inverse_block(cfg, blob, j, y), z[1], atol=1e-11)
        x32 = orc32.sequential_inverse_block(cfg, blob, j, z[0])
        assert np.abs(orc32.forward_block(cfg, blob, j, x32) - z[0]).max() <= 1e-5


def test_forward_of_inverse_whole_flow_config1(orc64, orc32):
    cfg = wl.CONFIGS["C1"]
    blob = wl.make_weights(cfg); z = wl.make_latent(cfg)
    for orc, tol in ((orc64, 1e-12), (orc32, 1e-5)):
        x, iters, _ = orc.sample(cfg, blob, z, 0, 0.0)      # every block sequential
        assert np.all(iters == cfg.seq_len - 1)             # T-1 conditioner steps per block
        assert np.abs(orc.forward(cfg, blob, x) - z).max() <= tol
        assert np.abs(x - z).max() > 0.1                    # the flow is not the identity


def test_forward_block_formula_two_tokens(orc64):
    # y_1 = x_1;  y_2 = (x_2 - mu_2) * exp(-alpha_2), with (mu, alpha) from the conditioner on x
    cfg, blob, z = _flow(2, D=1, K=1)
    x = z[0].astype(np.float64)
    mu, al = orc64.cond(cfg, blob, 0, x)
    y = orc64.forward_block(cfg, blob, 0, x)
    assert y[0, 0] == x[0, 0]
    np.testing.assert_allclose(y[1, 0], (x[1, 0] - mu[1, 0]) * np.exp(-al[1, 0]), rtol=1e-14)
    # inverse of a token: x_2 = y_2 * exp(alpha_2) + mu_2, parameters from x_1 only
    xi = orc64.sequential_inverse_block(cfg, blob, 0, x)
    mu_i, al_i = orc64.cond(cfg, blob, 0, xi)
    np.testing.assert_allclose(xi[1, 0], x[1, 0] * np.exp(al_i[1, 0]) + mu_i[1, 0], rtol=1e-14)
    assert al[1, 0] != 0 and mu[1, 0] != 0


# ---- the two sequential implementations --------------------------------------------------------

@pytest.mark.parametrize("T", [2, 3, 5, 8, 13])
def test_cached_sequential_equals_definition(orc64, orc32, T):
    cfg, blob, z = _flow(T, N=2)
    for j in range(cfg.n_blocks):
        for orc in (orc64, orc32):
            a = orc.sequential_inverse_block_naive(cfg, blob, j, z[0], fill=0.0)
            b = orc.sequential_inverse_block_naive(cfg, blob, j, z[0], fill=123.5)   # unknown tokens cannot matter
            c = orc.sequential_inverse_block(cfg, blob, j, z[0])
            assert np.array_equal(a, b)
            assert np.array_equal(a, c)


# ---- Prop. 3.2 and its proof: finite convergence, prefix exactness, idempotence ---------------

@pytest.mark.parametrize("T", TINY_T)
def test_jacobi_reaches_sequential_in_T_passes_from_any_start(orc64, T):
    cfg, blob, z = _flow(T)
    rng = np.random.default_rng(T)
    for j in range(cfg.n_blocks):
        star = orc64.sequential_inverse_block(cfg, blob, j, z[0])
        for x0 in (np.zeros_like(z[0]), z[0], rng.standard_normal(z[0].shape) * 3):
            x = x0.astype(np.float64)
            for t in range(1, T + 1):
                x = orc64.jacobi_map(cfg, blob, j, z[0], x)
                # P(t): after t passes the first t tokens (processing order) are exact
                rev = (cfg.reverse_mask >> j) & 1
                xs, ss = (x[::-1], star[::-1]) if rev else (x, star)
                assert np.array_equal(xs[:t], ss[:t]), (j, t)
            assert np.array_equal(x, star)
            assert np.array_equal(orc64.jacobi_map(cfg, blob, j, z[0], x), x)   # stays there: difference exactly 0


def test_sequential_output_is_a_fixed_point_and_token1_is_copied(orc64):
    cfg, blob, z = _flow(8)
    star = orc64.sequential_inverse_block(cfg, blob, 0, z[0])
    assert np.array_equal(orc64.jacobi_map(cfg, blob, 0, z[0], star), star)
    junk = np.random.default_rng(1).standard_normal(z[0].shape)
    assert np.array_equal(orc64.jacobi_map(cfg, blob, 0, z[0], junk)[0], z[0][0].astype(np.float64))
    # block 1 is reversed: its first processed token is the last canonical one
    assert np.array_equal(orc64.jacobi_map(cfg, blob, 1, z[0], junk)[-1], z[0][-1].astype(np.float64))


def test_single_token_one_pass_exact(orc64, orc32):
    cfg, blob, z = _flow(1)
    for orc in (orc64, orc32):
        x, it = orc.jacobi_inverse_block(cfg, blob, 0, z[0], 1e-3)
        assert it == 1 and np.array_equal(x, z[0].astype(orc.dtype))
        xs, iters, _ = orc.sample(cfg, blob, z, ~0, 1e-3)
        assert np.all(iters == 1) and np.array_equal(xs, z.astype(orc.dtype))


@pytest.mark.parametrize("j", [0, 1])
def test_jacobi_map_is_strictly_causal(orc64, j):
    """Perturbing token p changes F only at tokens after p (strictly lower-triangular Jacobian)."""
    cfg, blob, z = _flow(8, N=2)
    rng = np.random.default_rng(3)
    x = rng.standard_normal(z[0].shape)
    base = orc64.jacobi_map(cfg, blob, j, z[0], x)
    rev = (cfg.reverse_mask >> j) & 1
    for p in range(cfg.seq_len):
        xp = x.copy()
        canon = cfg.seq_len - 1 - p if rev else p
        xp[canon] += 0.5
        out = orc64.jacobi_map(cfg, blob, j, z[0], xp)
        a, b = (out[::-1], base[::-1]) if rev else (out, base)
        assert np.array_equal(a[:p + 1], b[:p + 1])
        if p + 1 < cfg.seq_len:
            assert not np.array_equal(a[p + 1], b[p + 1])       # the very next token does react


def test_reversed_block_is_flip_conjugate(orc64):
    cfg, blob, z = _flow(6, K=2)
    nf = cfg.with_(n_blocks=2)
    # same weights, reversal switched off by describing the flow with a zero mask via a twin config
    class NoRev:
        pass
    twin = NoRev()
    for k in ("n_blocks", "n_layers", "width", "n_heads", "mlp_ratio", "seq_len", "token_dim"):
        setattr(twin, k, getattr(nf, k))
    twin.reverse_mask = 0
    a = orc64.sequential_inverse_block(cfg, blob, 1, z[0])            # block 1 is reversed in cfg
    b = orc64.sequential_inverse_block(twin, blob, 1, z[0][::-1])[::-1]
    assert np.array_equal(a, b)
    a = orc64.forward_block(cfg, blob, 1, z[1])
    b = orc64.forward_block(twin, blob, 1, z[1][::-1])[::-1]
    assert np.array_equal(a, b)


# ---- Alg. 1: stopping rule, counting, initial guesses -----------------------------------------

def test_tau_zero_runs_T_passes_and_equals_sequential(orc64, orc32):
    cfg, blob, z = _flow(8)
    for orc in (orc64, orc32):
        for j in range(cfg.n_blocks):
            x, it = orc.jacobi_inverse_block(cfg, blob, j, z[0], 0.0)
            assert it == cfg.seq_len
            assert np.array_equal(x, orc.sequential_inverse_block(cfg, blob, j, z[0]))


def test_tau_infinite_is_one_pass_of_F_from_zero(orc64):
    cfg, blob, z = _flow(8)
    x, it = orc64.jacobi_inverse_block(cfg, blob, 0, z[0], float("inf"))
    assert it == 1
    assert np.array_equal(x, orc64.jacobi_map(cfg, blob, 0, z[0], np.zeros_like(z[0])))


def test_iteration_count_is_monotone_in_tau_and_trace_is_the_stated_norm(orc64):
    cfg, blob, z = _flow(8, N=2)
    n = cfg.seq_len * cfg.token_dim
    for crit in (0, 1):
        x, it, trace, iterates = orc64.jacobi_inverse_block(cfg, blob, 0, z[0], 0.0, criterion=crit,
                                                             want_trace=True, want_iterates=True)
        assert it == cfg.seq_len
        prev = np.zeros_like(iterates[0])
        for i in range(it):
            d = np.abs(iterates[i] - prev)
            want = d.max() if crit == 1 else d.sum() / n
            np.testing.assert_allclose(trace[i], want, rtol=1e-12, atol=0)
            assert np.array_equal(iterates[i], orc64.jacobi_map(cfg, blob, 0, z[0], prev))
            prev = iterates[i]
        assert np.array_equal(iterates[-1], x)
        counts = []
        for tau in (1e-9, 1e-6, 1e-3, 1e-1, 10.0):
            xi, iti, tr = orc64.jacobi_inverse_block(cfg, blob, 0, z[0], tau, criterion=crit, want_trace=True)
            # stops at the first pass whose delta is below tau (strictly), returning that pass's iterate
            first = next((i + 1 for i, d in enumerate(trace) if d < tau), cfg.seq_len)
            assert iti == first and np.array_equal(xi, iterates[iti - 1])
            counts.append(iti)
        assert counts == sorted(counts, reverse=True)


def test_max_iters_lowers_the_cap(orc64):
    cfg, blob, z = _flow(8)
    x, it = orc64.jacobi_inverse_block(cfg, blob, 0, z[0], 0.0, max_iters=3)
    assert it == 3
    y = np.zeros_like(z[0], dtype=np.float64)
    for _ in range(3):
        y = orc64.jacobi_map(cfg, blob, 0, z[0], y)
    assert np.array_equal(x, y)


def test_all_initial_guesses_agree_at_tau_zero(orc64):
    cfg, blob, z = _flow(8)
    rng = np.random.default_rng(9)
    ref, _ = orc64.jacobi_inverse_block(cfg, blob, 1, z[0], 0.0)
    for x0 in (z[0], rng.standard_normal(z[0].shape)):
        x, it = orc64.jacobi_inverse_block(cfg, blob, 1, z[0], 0.0, x0=x0)
        assert np.array_equal(x, ref)


def test_identity_flow_when_head_is_zero(orc64, orc32):
    cfg, blob, z = _flow(5)
    for v in wl.blob_views(cfg, blob):
        v["w_head"][...] = 0; v["b_head"][...] = 0
    for orc in (orc64, orc32):
        x, iters, deltas = orc.sample(cfg, blob, z, ~0, 1e-3)
        assert np.array_equal(x, z.astype(orc.dtype))
        assert np.all(iters == 2) and np.all(deltas == 0)       # delta_1 = mean|z|, delta_2 = 0
        xs, _, _ = orc.sample(cfg, blob, z, 0, 1e-3)
        assert np.array_equal(xs, z.astype(orc.dtype))


def test_context_free_chain(orc64):
    """With the attention output and MLP output projections zeroed the residual stream of a token
    never sees another token, so the parameters of token l depend on token l-1 alone: the
    conditioner on a sequence equals the one-token conditioner applied position by position, and
    Jacobi decoding needs all T passes (each pass fixes exactly one more token)."""
    T = 6
    cfg, blob, z = _flow(T, K=1)
    v = wl.blob_views(cfg, blob)[0]
    for l in range(cfg.n_layers):
        for k in ("w_o", "b_o", "w_fc2", "b_fc2"):
            v[f"l{l}.{k}"][...] = 0
    x = np.random.default_rng(4).standard_normal((T, cfg.token_dim))
    mu, al = orc64.cond(cfg, blob, 0, x)
    one = cfg.with_(seq_len=1)
    for l in range(1, T):
        b1 = wl.make_weights(one, seed_base=1)            # right size; overwrite with this block's weights
        v1 = wl.blob_views(one, b1)[0]
        for name in v1:
            v1[name][...] = v[name][l - 1:l] if name == "pos" else v[name]
        # the one-token flow's head row 0 would parameterise its (absent) second token: read it
        # through a two-token twin whose second position reuses the same weights
        two = cfg.with_(seq_len=2)
        b2 = wl.make_weights(two, seed_base=1)
        v2 = wl.blob_views(two, b2)[0]
        for name in v2:
            v2[name][...] = np.concatenate([v[name][l - 1:l], v[name][l - 1:l]]) if name == "pos" else v[name]
        m2, a2 = orc64.cond(two, b2, 0, np.stack([x[l - 1], x[l - 1]]))
        np.testing.assert_allclose(mu[l], m2[1], rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(al[l], a2[1], rtol=1e-13, atol=1e-15)
    xj, it, trace = orc64.jacobi_inverse_block(cfg, blob, 0, z[0], 1e-14, want_trace=True)
    assert it == T and np.all(trace[:-1] > 0)
    assert np.array_equal(xj, orc64.sequential_inverse_block(cfg, blob, 0, z[0]))


def test_superlinear_error_decay_near_the_solution(orc64):
    """Prop. 3.1: e_{t+1} = o(e_t).  On the seeded near-identity flow every pass shrinks the error
    by a factor well below one and the factor itself falls as the iterate closes in."""
    cfg = wl.CONFIGS["C1"]
    blob = wl.make_weights(cfg); z = wl.make_latent(cfg)
    star = orc64.sequential_inverse_block(cfg, blob, 1, z[0])
    _, it, iterates = orc64.jacobi_inverse_block(cfg, blob, 1, z[0], 0.0, max_iters=12, want_iterates=True)
    err = np.array([np.linalg.norm(iterates[i] - star) for i in range(it)])
    ratio = err[1:] / err[:-1]
    assert np.all(ratio < 0.2), ratio
    assert ratio[-1] < ratio[0]
    assert err[-1] < 1e-8 * err[0]


# ---- the cascade and the batch -----------------------------------------------------------------

def test_sample_is_the_composition_of_block_calls(orc64):
    cfg, blob, z = _flow(8, K=3)
    mask = 0b110
    x, iters, deltas = orc64.sample(cfg, blob, z, mask, 1e-4)
    for b in range(z.shape[0]):
        cur = z[b]
        for j in range(cfg.n_blocks):
            if (mask >> j) & 1:
                cur, it, tr = orc64.jacobi_inverse_block(cfg, blob, j, cur, 1e-4, want_trace=True)
                assert iters[j, b] == it and deltas[j, b] == tr[-1]
            else:
                cur = orc64.sequential_inverse_block(cfg, blob, j, cur)
                assert iters[j, b] == cfg.seq_len - 1
        assert np.array_equal(cur, x[b])


def test_sample_with_block_input_as_first_iterate_is_the_composition_of_block_calls(orc64):
    """`sample(init=1)` starts every Jacobi block from that block's own input (Sec. 4.3's alternative
    initialisation), in the order the block processes its tokens: on a flow with reversed blocks it must
    equal the chain of single-block calls with x0 = the block's (canonical-order) input, pass counts
    included - handing the block the un-flipped input as x0 would change the counts of the reversed
    blocks.  The single-block call is itself pinned (flip conjugacy, Prop. 3.2 from any start)."""
    cfg, blob, z = _flow(8, K=4, seed=3)
    assert cfg.reverse_mask == 0b1010
    mask = 0b1110
    tau = 1e-3
    x, iters, deltas = orc64.sample(cfg, blob, z, mask, tau, init=1)
    x0, iters0, _ = orc64.sample(cfg, blob, z, mask, tau, init=0)
    differs = False
    for b in range(z.shape[0]):
        cur = z[b]
        for j in range(cfg.n_blocks):
            if (mask >> j) & 1:
                nxt, it, tr = orc64.jacobi_inverse_block(cfg, blob, j, cur, tau, x0=cur, want_trace=True)
                assert iters[j, b] == it and deltas[j, b] == tr[-1], (j, b)
                # the wrong reading (x0 in the other token order) is a different run
                wrong, it_w, tr_w = orc64.jacobi_inverse_block(cfg, blob, j, cur, tau, x0=cur[::-1].copy(), want_trace=True)
                differs |= (tr_w[0] != tr[0])
                cur = nxt
            else:
                cur = orc64.sequential_inverse_block(cfg, blob, j, cur)
        assert np.array_equal(cur, x[b])
    assert differs
    # both initialisations approximate the same sequential solution: results agree to a few tau
    assert np.abs(x - x0).max() < 0.05 and not np.array_equal(iters, iters0)


def test_samples_are_independent(orc64):
    cfg, blob, z = _flow(8)
    x, iters, _ = orc64.sample(cfg, blob, z, ~1, 1e-3)
    for b in range(z.shape[0]):
        xb, ib, _ = orc64.sample(cfg, blob, z[b:b + 1], ~1, 1e-3)
        assert np.array_equal(xb[0], x[b]) and np.array_equal(ib[:, 0], iters[:, b])


def test_selective_result_close_to_sequential_within_tau_scale(orc64):
    """Reconstruction-consistency idea of App. E.4 on synthetic data: forward(x) then selective
    Jacobi inverse comes back to x up to the stopping tolerance."""
    cfg = wl.CONFIGS["C1"]
    blob = wl.make_weights(cfg)
    x = wl.make_latent(cfg, seed=11)
    z = orc64.forward(cfg, blob, x)
    xr, iters, _ = orc64.sample(cfg, blob, z, ~1, 1e-3)
    assert np.abs(xr - x).mean() < 1e-3
    assert np.all(iters[1:] < 10) and np.all(iters[0] == cfg.seq_len - 1)
    xr0, _, _ = orc64.sample(cfg, blob, z, ~1, 0.0)
    assert np.abs(xr0 - x).max() < 1e-11


# ---- log-determinant of the forward map (eq. 1's change-of-variables term for eq. 4) -----------

def _numerical_jacobian(fn, x, h=1e-6):
    n = x.size
    J = np.empty((n, n))
    for i in range(n):
        e = np.zeros(n); e[i] = h
        J[:, i] = (fn((x.reshape(-1) + e).reshape(x.shape)).reshape(-1)
                   - fn((x.reshape(-1) - e).reshape(x.shape)).reshape(-1)) / (2 * h)
    return J


@pytest.mark.parametrize("T,D", [(3, 2), (5, 1), (4, 3)])
def test_logdet_equals_log_determinant_of_the_numerical_jacobian(orc64, T, D):
    cfg, blob, z = _flow(T, seed=3, D=D)
    x = z[0].astype(np.float64)
    total = 0.0
    cur = x
    for j in range(cfg.n_blocks - 1, -1, -1):
        y, ld = orc64.forward_block_logdet(cfg, blob, j, cur)
        J = _numerical_jacobian(lambda v: orc64.forward_block(cfg, blob, j, v), cur)
        sign, logabs = np.linalg.slogdet(J)
        assert sign > 0                                   # diagonal exp(-alpha) > 0
        assert abs(logabs - ld) <= 1e-6
        np.testing.assert_array_equal(y, orc64.forward_block(cfg, blob, j, cur))
        total += ld
        cur = y
    # the whole flow: Jacobians multiply, log-determinants add
    zf, ld_all = orc64.forward_logdet(cfg, blob, x[None])
    np.testing.assert_array_equal(zf[0], cur)
    assert abs(ld_all[0] - total) <= 1e-12
    Jf = _numerical_jacobian(lambda v: orc64.forward(cfg, blob, v[None])[0], x)
    assert abs(np.linalg.slogdet(Jf)[1] - total) <= 1e-5


def test_logdet_closed_forms(orc64, orc32):
    """Head weights zero: alpha is the head's bias for every token but the first, whatever the
    input, so logdet = -(T-1) * sum_d b_alpha[d] per block; zero bias too: volume preserving."""
    cfg = wl.tiny_config(T=6, D=3, K=3)
    blob = wl.make_weights(cfg, seed_base=77, perturb_affine=True, std=0.1)
    views = wl.blob_views(cfg, blob)
    expect = 0.0
    for j, v in enumerate(views):
        v["w_head"][...] = 0.0
        v["b_head"][...] = 0.0
        v["b_head"][cfg.token_dim:] = np.float32(0.1 * (j + 1)) * np.arange(1, cfg.token_dim + 1, dtype=np.float32)
        expect += -(cfg.seq_len - 1) * float(v["b_head"][cfg.token_dim:].astype(np.float64).sum())
    x = wl.make_latent(cfg, batch=2, seed=1)
    for orc, tol in ((orc64, 1e-12), (orc32, 1e-5)):
        _, ld = orc.forward_logdet(cfg, blob, x)
        np.testing.assert_allclose(ld, [expect, expect], atol=tol * 10)
    for v in views:
        v["b_head"][...] = 0.0
    z, ld = orc64.forward_logdet(cfg, blob, x)
    np.testing.assert_array_equal(ld, [0.0, 0.0])
    np.testing.assert_array_equal(z, x.astype(np.float64))


# ---- masked-dependency probe (eq. 6): attention without the o nearest predecessors ---------------

def _masked(cfg, o):
    return cfg.with_(mask_nearest=o)


def test_masked_probe_zero_offset_is_the_plain_model(orc64):
    cfg, blob, z = _flow(6, seed=9)
    for j in range(cfg.n_blocks):
        np.testing.assert_array_equal(orc64.sequential_inverse_block(_masked(cfg, 0), blob, j, z[0]),
                                      orc64.sequential_inverse_block(cfg, blob, j, z[0]))


@pytest.mark.parametrize("o", [1, 2, 4])
def test_masked_probe_dependency_structure(orc64, o):
    """With the o nearest predecessors masked, the parameters of token l (head row l-1) come from
    token l-1 itself (residual path) and from tokens <= l-1-o (attention): changing token j must
    leave rows q with j < q < j+o bit-identical and change row j and rows q >= j+o."""
    T = 9
    cfg, blob, z = _flow(T, seed=4, K=1)
    cfg = _masked(cfg, o)
    x = z[0].astype(np.float64)
    mu0, al0 = orc64.cond(cfg, blob, 0, x)                 # row l: parameters of token l (from head row l-1)
    for j in range(T - 1):
        xp = x.copy(); xp[j] += 0.37
        mu1, al1 = orc64.cond(cfg, blob, 0, xp)
        changed = [l for l in range(T) if not (np.array_equal(mu0[l], mu1[l]) and np.array_equal(al0[l], al1[l]))]
        # head row q = l-1 depends on token q and tokens <= q-o
        expect = [l for l in range(1, T) if (l - 1 == j) or (l - 1 - o >= j)]
        assert changed == expect, (o, j, changed, expect)


def test_masked_probe_with_everything_masked_equals_no_attention(orc64):
    """o >= T: no row sees any key, attention contributes only its output bias - the same map as
    the plain model with the attention output projection set to zero."""
    T = 7
    cfg, blob, z = _flow(T, seed=6)
    blob0 = blob.copy()
    for v in wl.blob_views(cfg, blob0):
        for l in range(cfg.n_layers):
            v[f"l{l}.w_o"][...] = 0.0
    for j in range(cfg.n_blocks):
        a = orc64.sequential_inverse_block(_masked(cfg, T), blob, j, z[0])
        b = orc64.sequential_inverse_block(cfg, blob0, j, z[0])
        np.testing.assert_allclose(a, b, atol=1e-13)
        # and Jacobi decoding of the masked model reaches the masked sequential result (same triangular structure)
        xj, it = orc64.jacobi_inverse_block(_masked(cfg, 2), blob, j, z[0], 0.0)
        np.testing.assert_allclose(xj, orc64.sequential_inverse_block(_masked(cfg, 2), blob, j, z[0]), atol=1e-11)


def test_masked_probe_forward_inverts_masked_inverse(orc64):
    cfg, blob, z = _flow(8, seed=2)
    cfg = _masked(cfg, 3)
    for j in range(cfg.n_blocks):
        x = orc64.sequential_inverse_block(cfg, blob, j, z[0])
        np.testing.assert_allclose(orc64.forward_block(cfg, blob, j, x), z[0], atol=1e-12)
        np.testing.assert_allclose(orc64.sequential_inverse_block_naive(cfg, blob, j, z[0]), x, atol=1e-12)
