"""Pins of the oracle's LANTERN-style variant (aggregated acceptance over latent neighbours,
Eq. p_lantern / Eq. f_lantern / Eq. g_lantern, and the ablation that resamples with G*).

No GPU.  What fixes the functions here: a hand-worked row, a brute-force statement of the
neighbour-set rule, the reduction to vanilla speculative decoding at lambda = 0, the identity
G* = G^van for f >= f^van (Proposition on the design of G), the exact output law at L = 1 with
the closed-form total variation of Theorem 2 / Proposition LP, and sampling tests of the whole
verify call against that enumerated law.
"""
import numpy as np
import pytest
import scipy.stats

RNG = np.random.default_rng(20260209)


def random_table(V, k, rng, pad=0.0, self_entries=False):
    """k distinct neighbours per token, nearest first; optionally padding (-1) and self entries."""
    nbr = np.empty((V, k), np.int32)
    for x in range(V):
        others = np.array([y for y in range(V) if y != x])
        row = rng.permutation(others)[:k]
        if len(row) < k:
            row = np.concatenate([row, -np.ones(k - len(row), np.int64)])
        nbr[x] = row
    if pad > 0:
        nbr[rng.random((V, k)) < pad] = -1
    if self_entries:
        for x in range(V):
            nbr[x, rng.integers(0, k)] = x
    return nbr


def test_hand_worked_row(oracle):
    """Eq. p_lantern, Eq. f_lantern, Eq. g_lantern on a row small enough to do by hand.
    p(1) = 0.1, lambda = 3: neighbours of token 1 are 2, 3, 4 with p = 0.2, 0.25, 0.05.
    0.2 < 0.3 keeps token 2; 0.2 + 0.25 = 0.45 is not below 0.3, so A = {1, 2}, the aggregated
    probability is 0.3, f = min{1, 0.3 / 0.5} = 0.6, P^{k,lambda} = (0.4, 0.3, 0, 0.25, 0.05) and
    [P^{k,lambda} - q]_+ = (0.3, 0, 0, 0.05, 0)."""
    p = np.array([0.4, 0.1, 0.2, 0.25, 0.05])
    q = np.array([0.1, 0.5, 0.1, 0.2, 0.1])
    nbr = np.array([[1, 2, 3], [2, 3, 4], [0, 1, 3], [0, 1, 2], [0, 1, 2]], np.int32)
    m, agg, members = oracle.lantern_set(p, 1, nbr[1], 3.0)
    assert m == 1 and members.tolist() == [2]
    assert agg == pytest.approx(0.3, abs=1e-15)
    assert oracle.lantern_accept_prob(p, q, 1, nbr, 3.0) == pytest.approx(0.6, abs=1e-15)
    g, R = oracle.lantern_residual(p, q, nbr, 3.0, oracle.RESAMPLE_LANTERN, 1)
    np.testing.assert_allclose(g, [0.3, 0.0, 0.0, 0.05, 0.0], atol=1e-15)
    assert R == pytest.approx(0.35, abs=1e-15)
    # token 0 (p = 0.4, q = 0.1) merges all three neighbours (0.1, 0.3, 0.55 < 1.2): the aggregated
    # 0.95 sits on token 0, its neighbours are emptied, token 4 keeps 0.05 < q
    g0, R0 = oracle.lantern_residual(p, q, nbr, 3.0, oracle.RESAMPLE_LANTERN, 0)
    np.testing.assert_allclose(g0, [0.85, 0.0, 0.0, 0.0, 0.0], atol=1e-15)
    assert R0 == pytest.approx(0.85, abs=1e-15)
    # a larger lambda takes the next neighbour too; lambda = 0 takes none
    assert oracle.lantern_set(p, 1, nbr[1], 5.5)[0] == 3          # 0.5 < 0.55
    assert oracle.lantern_set(p, 1, nbr[1], 4.8)[0] == 2          # 0.45 < 0.48, 0.5 is not
    assert oracle.lantern_set(p, 1, nbr[1], 4.0)[0] == 1          # 0.45 < 0.4 is false
    assert oracle.lantern_set(p, 1, nbr[1], 0.0)[:2] == (0, 0.1)
    # the inequality is strict: a neighbour that would bring the sum to exactly lambda p(x) stays out
    pt = np.array([0.25, 0.25, 0.5])
    assert oracle.lantern_set(pt, 0, np.array([1, 2], np.int32), 1.0)[0] == 0
    assert oracle.lantern_set(pt, 0, np.array([1, 2], np.int32), 1.5)[0] == 1
    assert oracle.lantern_set(pt, 0, np.array([1, 2], np.int32), 3.0)[0] == 1     # 0.75 < 0.75 is false


def test_neighbour_set_rule_against_brute_force(oracle):
    """Largest prefix (nearest first) whose summed probability stays below lambda p(x); padding
    and self entries are skipped."""
    for V, k in ((8, 3), (32, 10), (64, 63)):
        nbr = random_table(V, k, RNG, pad=0.2, self_entries=True)
        for _ in range(20):
            p = oracle.softmax(2.0 * RNG.standard_normal(V))
            lam = float(RNG.choice([0.0, 0.05, 0.5, 2.0, 50.0]))
            for x in range(V):
                valid = [int(n) for n in nbr[x] if n >= 0 and n != x]
                cum = np.cumsum(p[valid]) if valid else np.zeros(0)
                below = cum < lam * p[x]
                m_ref = int(np.argmin(below)) if not below.all() else len(valid)
                m, agg, members = oracle.lantern_set(p, x, nbr[x], lam)
                assert m == m_ref
                assert members.tolist() == valid[:m_ref]
                assert agg == pytest.approx(p[x] + (cum[m_ref - 1] if m_ref else 0.0), rel=1e-14)


def test_acceptance_dominates_vanilla_and_grows_with_lambda(oracle):
    V, k = 24, 6
    nbr = random_table(V, k, RNG)
    for _ in range(10):
        p = oracle.softmax(2.0 * RNG.standard_normal(V))
        q = oracle.softmax(2.0 * RNG.standard_normal(V))
        prev = np.array([oracle.accept_prob(p[x], q[x], 1.0) for x in range(V)])     # Eq. f_tsd
        for lam in (0.0, 0.1, 1.0, 2.0, 100.0):
            f = np.array([oracle.lantern_accept_prob(p, q, x, nbr, lam) for x in range(V)])
            assert np.all(f >= prev - 1e-15)
            prev = f
        if lam == 0.0:
            np.testing.assert_array_equal(f, prev)


def _workload(B, L, V, rng, sharp=2.0, noise=1.0, bonus=True):
    t = (sharp * rng.standard_normal((B, L + int(bonus), V))).astype(np.float32)
    d = (t[:, :L] + noise * rng.standard_normal((B, L, V))).astype(np.float32)
    tok = np.empty((B, L), np.int32)
    for b in range(B):
        for i in range(L):
            q = scipy.special.softmax(d[b, i].astype(np.float64))
            tok[b, i] = rng.choice(V, p=q)
    ua = (rng.integers(0, 1 << 24, (B, L)) * 2.0 ** -24).astype(np.float32)
    ur = (rng.integers(0, 1 << 24, B) * 2.0 ** -24).astype(np.float32)
    return t, d, tok, ua, ur


def test_lambda_zero_is_vanilla_speculative_decoding(oracle):
    """With lambda = 0 (or no neighbours) A = {x~}: Eq. f_lantern is Eq. f_tsd and both resampling
    laws are Eq. g_tsd, so the call must agree with the Cool-SD call at omega = 1."""
    B, L, V = 40, 4, 50
    t, d, tok, ua, ur = _workload(B, L, V, RNG)
    nbr = random_table(V, 5, RNG)
    ref = oracle.verify(t, d, tok, np.ones(L, np.float32), ua, ur, resample_mode=oracle.RESAMPLE_VANILLA)
    for mode in (oracle.RESAMPLE_OPT, oracle.RESAMPLE_VANILLA, oracle.RESAMPLE_LANTERN):
        for kw in (dict(nbr=nbr, lam=0.0), dict(nbr=np.zeros((V, 0), np.int32), lam=2.0)):
            out = oracle.verify_lantern(t, d, tok, kw["nbr"], kw["lam"], ua, ur, resample_mode=mode)
            for key in ("accept_len", "next_token", "acc"):
                np.testing.assert_array_equal(out[key], ref[key])
            for key in ("p_tok", "q_tok", "f", "resid_mass"):
                np.testing.assert_allclose(out[key], ref[key], rtol=1e-15, atol=0)
            np.testing.assert_array_equal(out["count"], 0)
            np.testing.assert_allclose(out["p_agg"], ref["p_tok"], rtol=0, atol=0)


def test_optimal_law_equals_vanilla_law(oracle):
    """Proposition on the design of G: f >= f^van implies G* = G^van.  Eq. f_lantern never falls
    below Eq. f_tsd (the set always holds x~ itself), so Eq. opt_G evaluated token by token with
    each token's own neighbour set must give exactly [p - q]_+."""
    differs = 0
    for V, k in ((8, 3), (40, 10), (100, 25)):
        nbr = random_table(V, k, RNG, pad=0.1)
        for _ in range(10):
            p = oracle.softmax(2.5 * RNG.standard_normal(V))
            q = oracle.softmax(2.5 * RNG.standard_normal(V))
            lam = float(RNG.choice([0.1, 1.0, 2.0, 10.0]))
            g, R = oracle.lantern_residual(p, q, nbr, lam, oracle.RESAMPLE_OPT, 0)
            gv, Rv = oracle.residual(p, q, 1.0, oracle.RESAMPLE_VANILLA)
            np.testing.assert_array_equal(g, gv)
            assert R == Rv
            # the law of Eq. g_lantern is in general a different one
            x = int(np.argmax(q))
            gl, Rl = oracle.lantern_residual(p, q, nbr, lam, oracle.RESAMPLE_LANTERN, x)
            assert np.all(gl >= 0) and Rl > 0
            differs += not np.allclose(gl / Rl, gv / Rv)
    assert differs > 0


def _output_law_L1(oracle, p, q, nbr, lam, mode):
    """Exact law of the single emitted token of one round at L = 1 (no bonus needed: the emitted
    token is x~ when accepted, else a draw from G(. | x~))."""
    V = p.shape[0]
    f = np.array([oracle.lantern_accept_prob(p, q, x, nbr, lam) for x in range(V)])
    law = q * f
    for xd in range(V):
        rej = q[xd] * (1.0 - f[xd])
        if rej > 0:
            g, R = oracle.lantern_residual(p, q, nbr, lam, mode, xd)
            law = law + rej * g / R
    return law, f


def test_exact_tv_at_one_position(oracle):
    """L = 1: the bound of Theorem 2 is the exact total variation, and with G* it has the closed
    form sum_x [q f - p]_+ (Proposition LP: G* attains the infimum over G).  The law of
    Eq. g_lantern depends on the rejected token; its mixture over rejected tokens is one more
    admissible G, so it cannot do better (it often ties: its support avoids the tokens whose
    target mass is already exceeded)."""
    for V, k in ((6, 2), (12, 4), (30, 8)):
        nbr = random_table(V, k, RNG)
        for _ in range(8):
            p = oracle.softmax(2.0 * RNG.standard_normal(V))
            q = oracle.softmax(2.0 * RNG.standard_normal(V))
            lam = float(RNG.choice([0.5, 2.0, 8.0]))
            law_opt, f = _output_law_L1(oracle, p, q, nbr, lam, oracle.RESAMPLE_OPT)
            law_lan, _ = _output_law_L1(oracle, p, q, nbr, lam, oracle.RESAMPLE_LANTERN)
            assert abs(law_opt.sum() - 1) < 1e-12 and abs(law_lan.sum() - 1) < 1e-12
            tv_opt = 0.5 * np.abs(law_opt - p).sum()
            tv_lan = 0.5 * np.abs(law_lan - p).sum()
            closed = np.maximum(q * f - p, 0.0).sum()
            assert tv_opt == pytest.approx(closed, abs=1e-13)
            assert tv_lan >= tv_opt - 1e-13


@pytest.mark.parametrize("mode", [0, 2])
def test_verify_call_samples_the_enumerated_law(oracle, mode):
    """The whole verify call (accept test, break, resampling draw) at L = 1 on one fixed row
    pair, driven by seeded uniforms and draft tokens drawn from q: acceptance rate against
    sum_x q f (the factor of Eq. token_exp) and the emitted token against the enumerated law."""
    V, k, lam, N = 8, 3, 2.0, 120000
    rng = np.random.default_rng(77 + mode)
    nbr = random_table(V, k, rng)
    lt = (1.5 * rng.standard_normal(V)).astype(np.float32)
    ld = (lt + rng.standard_normal(V)).astype(np.float32)
    p, q = oracle.softmax(lt), oracle.softmax(ld)
    law, f = _output_law_L1(oracle, p, q, nbr, lam, mode)
    t = np.broadcast_to(lt, (N, 1, V)).copy()
    d = np.broadcast_to(ld, (N, 1, V)).copy()
    tok = rng.choice(V, size=(N, 1), p=q).astype(np.int32)
    ua = rng.random((N, 1)).astype(np.float32)
    ur = rng.random(N).astype(np.float32)
    out = oracle.verify_lantern(t, d, tok, nbr, lam, ua, ur, resample_mode=mode, num_threads=8)
    alpha = float((q * f).sum())
    acc = out["accept_len"].mean()
    assert abs(acc - alpha) < 5 * np.sqrt(alpha * (1 - alpha) / N)
    emitted = np.where(out["accept_len"] == 1, tok[:, 0], out["next_token"])
    counts = np.bincount(emitted, minlength=V)
    chi2 = ((counts - N * law) ** 2 / (N * law)).sum()
    assert chi2 < scipy.stats.chi2.ppf(1 - 1e-4, V - 1)
    # and the per-position outputs are the row-wise definitions
    m, agg, _ = oracle.lantern_set(p, int(tok[0, 0]), nbr[tok[0, 0]], lam)
    assert out["count"][0, 0] == m and out["p_agg"][0, 0] == pytest.approx(agg, rel=1e-14)
    assert out["f"][0, 0] == pytest.approx(min(1.0, agg / q[tok[0, 0]]), rel=1e-14)


def test_break_and_bonus_follow_algorithm_1(oracle):
    """Several positions: the first rejected position ends the round and is resampled there;
    when nothing is rejected the bonus token comes from p_{L+1}."""
    B, L, V = 300, 3, 12
    t, d, tok, ua, ur = _workload(B, L, V, RNG, noise=0.8)
    nbr = random_table(V, 4, RNG)
    out = oracle.verify_lantern(t, d, tok, nbr, 2.0, ua, ur, resample_mode=oracle.RESAMPLE_LANTERN)
    seen = set()
    for b in range(B):
        acc = [ua[b, i] <= out["f"][b, i] for i in range(L)]
        tau = acc.index(False) if False in acc else L
        assert out["accept_len"][b] == tau
        seen.add(tau)
        if tau < L:
            p = oracle.softmax(t[b, tau].astype(np.float64))
            q = oracle.softmax(d[b, tau].astype(np.float64))
            g, R = oracle.lantern_residual(p, q, nbr, 2.0, oracle.RESAMPLE_LANTERN, int(tok[b, tau]))
        else:
            g = oracle.softmax(t[b, L].astype(np.float64))
            R = g.sum()
        assert out["resid_mass"][b] == pytest.approx(R, rel=1e-14)
        assert out["next_token"][b] == oracle.inverse_cdf(g, float(ur[b]) * R)
    assert seen == {0, 1, 2, 3}
