"""Pins of the oracle's batched verify()/resample() against the paper (no GPU).

verify() is a deterministic function of the supplied uniforms; fed with seeded uniforms its
outputs must follow the laws the paper proves: the target law when nothing is relaxed
(Theorem 1), the exactly enumerated law when relaxed, and the expected accepted length of
Eq. token_exp.
"""
import numpy as np
import pytest
import scipy.stats


def u24(rng, shape):
    return (rng.integers(0, 1 << 24, shape).astype(np.float32) * np.float32(2.0 ** -24))


def draw_tokens(rng, q_rows, n):
    """Drafting stage for prefix-independent rows: x~_i ~ q_i (numpy sampler, input side)."""
    L, V = q_rows.shape
    return np.stack([rng.choice(V, size=n, p=q_rows[i]) for i in range(L)], axis=1).astype(np.int32)


def setup_rows(oracle, rng, L, V, sharp=1.5, noise=0.8):
    lt = (sharp * rng.standard_normal((L + 1, V))).astype(np.float32)
    ld = (lt[:L] + noise * rng.standard_normal((L, V))).astype(np.float32)
    p = np.stack([oracle.softmax(r.astype(np.float64)) for r in lt])
    q = np.stack([oracle.softmax(r.astype(np.float64)) for r in ld])
    return lt, ld, p, q


def run_verify(oracle, lt, ld, tokens, omega, ua, ur, **kw):
    n = tokens.shape[0]
    T = np.broadcast_to(lt, (n,) + lt.shape)
    D = np.broadcast_to(ld, (n,) + ld.shape)
    return oracle.verify(T, D, tokens, np.asarray(omega, np.float32), ua, ur, num_threads=4, **kw)


def chi2_p(counts, probs):
    exp = probs * counts.sum()
    stat = ((counts - exp) ** 2 / exp).sum()
    return scipy.stats.chi2.sf(stat, len(probs) - 1)


def test_lossless_chi_square_V8(oracle):
    """Theorem 1 (and its omega<1 extension with G*): every emitted position follows the target."""
    rng = np.random.default_rng(42)
    L, V, n = 2, 8, 200_000
    lt, ld, p, q = setup_rows(oracle, rng, L, V)
    for omega in ([1.0, 1.0], [1.0, 0.3]):
        tokens = draw_tokens(rng, q, n)
        out = run_verify(oracle, lt, ld, tokens, omega, u24(rng, (n, L)), u24(rng, n))
        tau, nxt = out["accept_len"], out["next_token"]
        assert tau.min() >= 0 and tau.max() <= L and (tau == L).any() and (tau == 0).any()
        # position 1: the draft token if accepted, else the resampled one
        x1 = np.where(tau >= 1, tokens[:, 0], nxt)
        assert chi2_p(np.bincount(x1, minlength=V), p[0]) > 1e-3
        # position 2 given position 1 was accepted (rows are prefix independent)
        m = tau >= 1
        x2 = np.where(tau[m] >= 2, tokens[m, 1], nxt[m])
        assert chi2_p(np.bincount(x2, minlength=V), p[1]) > 1e-3
        # bonus token when everything was accepted
        m = tau == L
        assert chi2_p(np.bincount(nxt[m], minlength=V), p[2]) > 1e-3
        # accepted prefix is the draft's own tokens: nothing to check beyond tau; next_token valid
        assert nxt.min() >= 0 and nxt.max() < V


def test_relaxed_single_position_matches_enumerated_law(oracle):
    """omega > 1, L = 1: emitted token ~ q f + G* rho (Algorithm 1 written out), chi-square."""
    rng = np.random.default_rng(43)
    V, n, om = 8, 200_000, 2.0
    lt, ld, p, q = setup_rows(oracle, rng, 1, V, noise=1.2)
    f = np.array([oracle.accept_prob(p[0][x], q[0][x], om) for x in range(V)])
    g, R = oracle.residual(p[0], q[0], om)
    law = q[0] * f + (g / R) * np.sum((1 - f) * q[0])
    assert abs(law.sum() - 1) < 1e-12 and 0.5 * np.abs(law - p[0]).sum() > 1e-3
    tokens = draw_tokens(rng, q, n)
    out = run_verify(oracle, lt, ld, tokens, [om], u24(rng, (n, 1)), u24(rng, n))
    x1 = np.where(out["accept_len"] >= 1, tokens[:, 0], out["next_token"])
    counts = np.bincount(x1, minlength=V)
    assert chi2_p(counts, law) > 1e-3
    assert chi2_p(counts, p[0]) < 1e-6          # and it is measurably not the target


def test_exact_measure_on_uniform_grid(oracle):
    """Deterministic version of the lossless pin: integrate verify() over a regular grid of
    (r_1, u) for every draft token; the induced law of x_1 equals p_1 up to the grid step."""
    rng = np.random.default_rng(44)
    V, N = 8, 256
    lt, ld, p, q = setup_rows(oracle, rng, 1, V)
    grid = ((np.arange(N) + 0.5) / N).astype(np.float32)
    ua, ur = np.meshgrid(grid, grid, indexing="ij")
    ua, ur = ua.reshape(-1, 1), ur.reshape(-1)
    law = np.zeros(V)
    for xt in range(V):
        tokens = np.full((N * N, 1), xt, np.int32)
        out = run_verify(oracle, lt, ld, tokens, [1.0], ua, ur)
        x1 = np.where(out["accept_len"] >= 1, xt, out["next_token"])
        law += q[0][xt] * np.bincount(x1, minlength=V) / (N * N)
    assert np.abs(law - p[0]).max() < 2.0 / N


def test_expected_accept_length(oracle):
    """Eq. token_exp for prefix-independent rows: E[tau] = sum_i prod_{j<=i} alpha_j,
    alpha_j = sum_x q_j(x) f_j(x)."""
    rng = np.random.default_rng(45)
    L, V, n = 4, 16, 200_000
    lt, ld, p, q = setup_rows(oracle, rng, L, V, noise=1.0)
    omega = oracle.schedule(oracle.SCHED_EXP, L, 1.5, 0.7)
    alpha = [sum(q[i][x] * oracle.accept_prob(p[i][x], q[i][x], np.float32(omega[i])) for x in range(V))
             for i in range(L)]
    e_tau = float(np.sum(np.cumprod(alpha)))
    # the batched diagnostics (logits in, alpha out) give the same factors
    a_rows, b_rows = oracle.diagnostics(lt[None], ld[None], omega)
    np.testing.assert_allclose(a_rows[0], alpha, rtol=1e-12)
    assert (b_rows >= -1e-15).all() and (b_rows[0][np.asarray(omega) > 1.0] > 0).all()
    tokens = draw_tokens(rng, q, n)
    out = run_verify(oracle, lt, ld, tokens, omega, u24(rng, (n, L)), u24(rng, n))
    tau = out["accept_len"].astype(np.float64)
    se = tau.std() / np.sqrt(n)
    assert abs(tau.mean() - e_tau) < 5 * se
    # P(tau >= i) = prod_{j<=i} alpha_j, position by position
    for i in range(1, L + 1):
        pi = float(np.prod(alpha[:i]))
        assert abs((tau >= i).mean() - pi) < 5 * np.sqrt(pi * (1 - pi) / n)


def test_verify_rowwise_outputs_and_first_rejection(oracle):
    """tau is the index before the first rejected position; diagnostics are per-row values."""
    rng = np.random.default_rng(46)
    B, L, V = 64, 6, 32
    T = (2 * rng.standard_normal((B, L + 1, V))).astype(np.float32)
    D = (T[:, :L] + rng.standard_normal((B, L, V))).astype(np.float32)
    tok = rng.integers(0, V, (B, L)).astype(np.int32)
    omega = oracle.schedule(oracle.SCHED_EXP, L, 1.1, 0.7).astype(np.float32)
    ua, ur = u24(rng, (B, L)), u24(rng, B)
    out = oracle.verify(T, D, tok, omega, ua, ur)
    for b in range(B):
        acc = []
        for i in range(L):
            p = oracle.softmax(T[b, i].astype(np.float64))
            q = oracle.softmax(D[b, i].astype(np.float64))
            x = tok[b, i]
            assert out["p_tok"][b, i] == p[x] and out["q_tok"][b, i] == q[x]
            f = min(1.0, float(omega[i]) * p[x] / q[x])
            assert out["f"][b, i] == pytest.approx(f, rel=1e-15)
            acc.append(ua[b, i] <= f)
            assert out["acc"][b, i] == acc[-1]
        tau = L if all(acc) else acc.index(False)
        assert out["accept_len"][b] == tau
        if tau < L:
            p = oracle.softmax(T[b, tau].astype(np.float64))
            q = oracle.softmax(D[b, tau].astype(np.float64))
            g = np.maximum(p - np.minimum(q, float(omega[tau]) * p), 0)
        else:
            g = oracle.softmax(T[b, L].astype(np.float64))
        R = 0.0
        for v in g:
            R += v
        assert out["resid_mass"][b] == pytest.approx(R, rel=1e-14)
        C = np.cumsum(g)
        assert out["next_token"][b] == int(np.nonzero(C > float(ur[b]) * R)[0][0])
    # no bonus row: tau = L gives next_token = -1
    out2 = oracle.verify(T[:, :L], D, tok, np.full(L, 1e6, np.float32), ua, ur)
    assert np.all(out2["accept_len"] == L) and np.all(out2["next_token"] == -1)
    # per-sequence omega [B, L] is honoured
    om2 = np.tile(omega, (B, 1))
    om2[::2] = 0.0
    out3 = oracle.verify(T, D, tok, om2, ua, ur)
    assert np.all(out3["accept_len"][::2] == 0)
    np.testing.assert_array_equal(out3["accept_len"][1::2], out["accept_len"][1::2])
    # thread count does not change anything
    out4 = oracle.verify(T, D, tok, omega, ua, ur, num_threads=4)
    for k in out:
        np.testing.assert_array_equal(out[k], out4[k])


def test_resample_standalone_equals_verify_path(oracle):
    rng = np.random.default_rng(47)
    B, V = 16, 50
    T = (2 * rng.standard_normal((B, V))).astype(np.float32)
    D = (T + rng.standard_normal((B, V))).astype(np.float32)
    om = rng.choice([0.3, 1.0, 1.5], B).astype(np.float32)
    u = u24(rng, B)
    tok, mass, g = oracle.resample(T, D, om, u, want_g=True)
    for b in range(B):
        # a verify call that rejects at position 1 (omega-scaled p cannot reach r=1-2^-24 only if f<1;
        # force the rejection with a token of zero target probability instead)
        p = oracle.softmax(T[b].astype(np.float64))
        q = oracle.softmax(D[b].astype(np.float64))
        gg, R = oracle.residual(p, q, float(om[b]))
        np.testing.assert_array_equal(g[b], gg)
        assert mass[b] == R and tok[b] == oracle.inverse_cdf(gg, float(u[b]) * R)
    tok_b, mass_b = oracle.resample(T, None, None, u)
    for b in range(B):
        p = oracle.softmax(T[b].astype(np.float64))
        assert tok_b[b] == int(np.nonzero(np.cumsum(p) > float(u[b]) * mass_b[b])[0][0])
        assert abs(mass_b[b] - 1) < 1e-14


def test_verify_with_guidance_and_topk(oracle):
    """Config-3 style options: supports differ; p(x~)=0 rejects, q(x~)=0 accepts (0/0 := 1 included)."""
    rng = np.random.default_rng(48)
    B, L, V, k = 8, 3, 64, 5
    Tu = rng.standard_normal((B, L + 1, V)).astype(np.float32)
    Tc = (Tu + rng.standard_normal((B, L + 1, V))).astype(np.float32)
    Du = (Tu[:, :L] + rng.standard_normal((B, L, V))).astype(np.float32)
    Dc = (Tc[:, :L] + rng.standard_normal((B, L, V))).astype(np.float32)
    tok = rng.integers(0, V, (B, L)).astype(np.int32)
    ua, ur = u24(rng, (B, L)), u24(rng, B)
    om = np.array([2.0, 1.0, 0.5], np.float32)
    out = oracle.verify(Tc, Dc, tok, om, ua, ur, target_uncond=Tu, draft_uncond=Du,
                        cfg_scale=4.0, temperature=0.8, top_k=k)
    for b in range(B):
        for i in range(L):
            p = oracle.softmax(oracle.transform_row(Tc[b, i], Tu[b, i], 4.0, 0.8, k))
            q = oracle.softmax(oracle.transform_row(Dc[b, i], Du[b, i], 4.0, 0.8, k))
            assert (p > 0).sum() == k and (q > 0).sum() == k
            x = tok[b, i]
            assert out["p_tok"][b, i] == p[x] and out["q_tok"][b, i] == q[x]
            if q[x] == 0:
                assert out["acc"][b, i] == 1 and out["f"][b, i] == 1.0
            elif p[x] == 0:
                assert out["f"][b, i] == 0.0 and out["acc"][b, i] == (ua[b, i] == 0)
        j = out["accept_len"][b]
        pj = oracle.softmax(oracle.transform_row(Tc[b, j], Tu[b, j], 4.0, 0.8, k))
        assert pj[out["next_token"][b]] > 0          # resampled / bonus token lies in the target's support
