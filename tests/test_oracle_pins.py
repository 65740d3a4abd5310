"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test names the passage it checks.  The enumeration helpers below are written from
Algorithm 1 and the definition of the virtually extended output law, and use the oracle
only for its building blocks (softmax, f, G), so a mistake in one of those fails a pin.
"""
import itertools

import numpy as np
import pytest
import scipy.special
import scipy.stats

RNG = np.random.default_rng(20260127)


# ----------------------------------------------------------------------------- helpers
def random_kernels(V, L, rng, sharp=1.5, noise=0.7):
    """Prefix-dependent logit tables: P_i[prefix] and Q_i[prefix] for i = 1..L+1 / 1..L."""
    P, Q = [], []
    for i in range(L + 1):
        shape = (V,) * i + (V,)
        lt = sharp * rng.standard_normal(shape)
        P.append(lt)
        if i < L:
            Q.append(lt + noise * rng.standard_normal(shape))
    return P, Q


def rows_of(O, table):
    flat = table.reshape(-1, table.shape[-1])
    out = np.stack([O.softmax(r) for r in flat])
    return out.reshape(table.shape)


def output_law(O, P, Q, omega, mode=0):
    """Exact law of x_{1:L+1} produced by Algorithm 1 followed by the virtual extension
    (remaining tokens drawn from P).  Sum over tau = j of
       Q(x_{1:j}) prod_{k<=j} f_k * rho_{j+1}(x_{1:j}) * G_{j+1}(x_{j+1}|x_{1:j}) * P(x_{j+2:L+1}|...)
    plus the all-accepted term Q(x_{1:L}) prod f_k * P(x_{L+1}|x_{1:L})."""
    L = len(Q)
    V = P[0].shape[-1]
    law = np.zeros((V,) * (L + 1))
    target = np.zeros((V,) * (L + 1))
    for xs in itertools.product(range(V), repeat=L + 1):
        pt = 1.0
        for i in range(L + 1):
            pt *= P[i][xs[:i]][xs[i]]
        target[xs] = pt
        total = 0.0
        acc_path = 1.0                      # Q(x_{1:j}) prod f_k(x_{1:k})
        for j in range(L + 1):
            if j == L:
                total += acc_path * P[L][xs[:L]][xs[L]]
                break
            p_row, q_row = P[j][xs[:j]], Q[j][xs[:j]]
            f_row = np.array([O.accept_prob(p_row[x], q_row[x], omega[j]) for x in range(V)])
            rho = float(np.sum((1.0 - f_row) * q_row))
            g, R = O.residual(p_row, q_row, omega[j], mode)
            tail = 1.0
            for i in range(j + 1, L + 1):
                tail *= P[i][xs[:i]][xs[i]]
            total += acc_path * rho * (g[xs[j]] / R) * tail
            acc_path *= q_row[xs[j]] * f_row[xs[j]]
        law[xs] = total
    return law, target


def tv_bound(O, P, Q, omega, mode=0):
    """Right-hand side of the TV upper bound of Theorem 2 for given f (via omega) and G."""
    L = len(Q)
    V = P[0].shape[-1]
    bound = 0.0
    for i in range(L):
        for xs in itertools.product(range(V), repeat=i):
            w = 1.0
            for k in range(i):
                p_k, q_k = P[k][xs[:k]], Q[k][xs[:k]]
                w *= q_k[xs[k]] * O.accept_prob(p_k[xs[k]], q_k[xs[k]], omega[k])
            p_row, q_row = P[i][xs], Q[i][xs]
            f_row = np.array([O.accept_prob(p_row[x], q_row[x], omega[i]) for x in range(V)])
            rho = float(np.sum((1.0 - f_row) * q_row))
            g, R = O.residual(p_row, q_row, omega[i], mode)
            bound += 0.5 * w * float(np.sum(np.abs(q_row * f_row - p_row + (g / R) * rho)))
    return bound


# ----------------------------------------------------------------------------- softmax
def test_softmax_matches_library_and_masks(oracle):
    for V in (1, 2, 8, 1000):
        l = 5.0 * RNG.standard_normal(V)
        if V >= 8:
            l[RNG.integers(0, V, V // 4)] = -np.inf
            l[0] = 1.0
        p = oracle.softmax(l)
        ref = scipy.special.softmax(l)
        np.testing.assert_allclose(p, ref, rtol=1e-13, atol=0)
        assert abs(p.sum() - 1.0) < 1e-13
        assert np.all(p[np.isneginf(l)] == 0.0)
    # shift invariance and a hand value
    np.testing.assert_allclose(oracle.softmax(np.array([0.0, np.log(3.0)])), [0.25, 0.75], rtol=1e-15)


# ----------------------------------------------------------------------------- schedules
@pytest.mark.parametrize("L", [1, 2, 4, 8, 16, 64])
@pytest.mark.parametrize("delta", [1.0, 1.1, 2.0, 4.0])
def test_exp_schedule_closed_form(oracle, L, delta):
    """Eq. sdar: the normaliser makes the weights sum to L, so sum omega = delta*L, and
    omega_i = delta*L*exp(-nu i)/sum_j exp(-nu j); consecutive ratio exp(-nu)."""
    nu = 0.7
    om = oracle.schedule(oracle.SCHED_EXP, L, delta, nu)
    assert om.shape == (L,)
    assert abs(om.sum() - delta * L) < 1e-12 * delta * L
    i = np.arange(1, L + 1)
    # geometric series: sum_j e^{-nu j} = e^{-nu}(1-e^{-nu L})/(1-e^{-nu})
    geo = np.exp(-nu) * (1 - np.exp(-nu * L)) / (1 - np.exp(-nu))
    np.testing.assert_allclose(om, delta * L * np.exp(-nu * i) / geo, rtol=1e-12)
    if L > 1:
        np.testing.assert_allclose(om[1:] / om[:-1], np.exp(-nu), rtol=1e-12)
        assert np.all(np.diff(om) < 0)
    assert np.all(om > 0)


def test_uniform_and_linear_schedules(oracle):
    np.testing.assert_array_equal(oracle.schedule(oracle.SCHED_UNIFORM, 5, 1.3), np.full(5, 1.3))
    # linear: w_i = (ell-i)/(ell(ell+1)); only the ratios matter after normalisation
    L, ell, delta = 4, 8, 2.0
    om = oracle.schedule(oracle.SCHED_LINEAR, L, delta, ell)
    w = np.array([ell - i for i in range(1, L + 1)], dtype=float)
    np.testing.assert_allclose(om, delta * L * w / w.sum(), rtol=1e-13)
    assert abs(om.sum() - delta * L) < 1e-12
    om8 = oracle.schedule(oracle.SCHED_LINEAR, 8, 1.0, 8)
    assert om8[-1] == 0.0 and np.all(np.diff(om8) < 0)
    with pytest.raises(ValueError):
        oracle.schedule(oracle.SCHED_LINEAR, 9, 1.0, 8)      # negative weight
    with pytest.raises(ValueError):
        oracle.schedule(oracle.SCHED_EXP, 4, 1.0, 0.0)
    with pytest.raises(ValueError):
        oracle.schedule(7, 4, 1.0, 0.7)


# ----------------------------------------------------------------------------- accept prob
def test_accept_prob_cases(oracle):
    """Eq. relax with the 0/0 := 1 convention; omega = 1 is the vanilla criterion."""
    assert oracle.accept_prob(0.2, 0.4, 1.0) == 0.5
    assert oracle.accept_prob(0.2, 0.4, 1.5) == pytest.approx(0.75)
    assert oracle.accept_prob(0.2, 0.4, 3.0) == 1.0
    assert oracle.accept_prob(0.4, 0.2, 1.0) == 1.0
    assert oracle.accept_prob(0.0, 0.0, 1.0) == 1.0
    assert oracle.accept_prob(0.3, 0.0, 1.0) == 1.0
    assert oracle.accept_prob(0.0, 0.3, 5.0) == 0.0
    assert oracle.accept(0.5, 0.2, 0.4, 1.0) and not oracle.accept(0.5000001, 0.2, 0.4, 1.0)
    assert oracle.accept(0.0, 0.0, 0.3, 1.0)            # r = 0 <= f = 0


# ----------------------------------------------------------------------------- Theorem 1 & omega<=1
@pytest.mark.parametrize("L,V,omega", [
    (1, 8, [1.0]), (2, 8, [1.0, 1.0]),                       # vanilla SD is lossless (Theorem 1)
    (2, 6, [1.0, 0.4]), (2, 6, [0.7, 0.05]), (3, 4, [1.0, 0.5, 0.25]),   # omega<1 with G* stays lossless
])
def test_output_law_equals_target_when_not_relaxed(oracle, L, V, omega):
    P, Q = random_kernels(V, L, np.random.default_rng(L * 100 + V))
    P = [rows_of(oracle, t) for t in P]
    Q = [rows_of(oracle, t) for t in Q]
    law, target = output_law(oracle, P, Q, omega)
    assert abs(law.sum() - 1.0) < 1e-12
    np.testing.assert_allclose(law, target, rtol=0, atol=1e-12)


def test_vanilla_resampling_is_biased_when_omega_below_one(oracle):
    """With omega<1 the vanilla law Norm([p-q]_+) no longer corrects the bias; G* does.
    (Separates the two resample modes.)"""
    P, Q = random_kernels(6, 1, np.random.default_rng(5))
    P = [rows_of(oracle, t) for t in P]
    Q = [rows_of(oracle, t) for t in Q]
    law_opt, target = output_law(oracle, P, Q, [0.5], mode=oracle.RESAMPLE_OPT)
    law_van, _ = output_law(oracle, P, Q, [0.5], mode=oracle.RESAMPLE_VANILLA)
    assert np.abs(law_opt - target).max() < 1e-12
    assert np.abs(law_van - target).max() > 1e-3


# ----------------------------------------------------------------------------- Proposition (G* = G^van)
def test_opt_equals_vanilla_iff_relaxed_upwards(oracle):
    rng = np.random.default_rng(7)
    for _ in range(20):
        V = int(rng.integers(2, 40))
        p = oracle.softmax(2 * rng.standard_normal(V))
        q = oracle.softmax(2 * rng.standard_normal(V))
        for om in (1.0, 1.1, 2.0, 7.5):
            g1, R1 = oracle.residual(p, q, om, oracle.RESAMPLE_OPT)
            g2, R2 = oracle.residual(p, q, om, oracle.RESAMPLE_VANILLA)
            np.testing.assert_array_equal(g1, g2)
            assert R1 == R2
            np.testing.assert_allclose(g2, np.maximum(p - q, 0.0), rtol=0, atol=0)
        g1, _ = oracle.residual(p, q, 0.5, oracle.RESAMPLE_OPT)
        g2, _ = oracle.residual(p, q, 0.5, oracle.RESAMPLE_VANILLA)
        assert np.abs(g1 - g2).max() > 0
        # the law as the theorem prints it, [p - q f]_+ with the quotient inside f
        for om in (0.5, 1.0, 1.7):
            g1, _ = oracle.residual(p, q, om, oracle.RESAMPLE_OPT)
            f = np.array([oracle.accept_prob(p[x], q[x], om) for x in range(V)])
            np.testing.assert_allclose(g1, np.maximum(p - q * f, 0.0), rtol=0, atol=1e-15)


def test_residual_is_distribution_and_mass_bounds(oracle):
    """Norm(g) is a distribution; mass R >= rejection probability (ieq. in the proof of Prop. LP);
    for omega <= 1 they are equal."""
    rng = np.random.default_rng(11)
    for _ in range(50):
        V = int(rng.integers(2, 64))
        p = oracle.softmax(3 * rng.standard_normal(V))
        q = oracle.softmax(3 * rng.standard_normal(V))
        om = float(rng.choice([0.03, 0.5, 1.0, 1.1, 2.0, 4.0]))
        g, R = oracle.residual(p, q, om)
        f = np.array([oracle.accept_prob(p[x], q[x], om) for x in range(V)])
        rho = np.sum((1 - f) * q)
        assert np.all(g >= 0) and R > 0
        assert abs((g / R).sum() - 1.0) < 1e-12
        assert R >= rho - 1e-15
        if om <= 1.0:
            assert abs(R - rho) < 1e-14
    # bonus position: g = p
    g, R = oracle.residual(p, None, 1.0)
    np.testing.assert_array_equal(g, p)
    assert abs(R - 1.0) < 1e-14
    # degenerate: identical rows, omega >= 1 -> residual vanishes, falls back to p
    g, R = oracle.residual(p, p, 1.5)
    np.testing.assert_array_equal(g, p)


# ----------------------------------------------------------------------------- Theorem 2: TV bound
@pytest.mark.parametrize("L,V,omega", [(1, 4, [1.7]), (2, 4, [2.0, 1.2]), (2, 3, [3.0, 0.6]), (2, 4, [1.1, 1.1])])
def test_exact_tv_respects_bound(oracle, L, V, omega):
    P, Q = random_kernels(V, L, np.random.default_rng(31 * L + V), sharp=1.0, noise=1.0)
    P = [rows_of(oracle, t) for t in P]
    Q = [rows_of(oracle, t) for t in Q]
    law, target = output_law(oracle, P, Q, omega)
    tv = 0.5 * np.abs(law - target).sum()
    bound = tv_bound(oracle, P, Q, omega)
    assert tv > 1e-4                       # the relaxation really biases the law
    assert tv <= bound + 1e-12
    if L == 1:
        assert abs(tv - bound) < 1e-12     # single position: the bound is the TV itself
    # at the vanilla criterion the bound collapses to zero
    assert tv_bound(oracle, P, Q, [1.0] * L) < 1e-12


def test_single_position_tv_closed_form(oracle):
    """L=1, G*: TV(P^, P) = sum_x [min(q, omega p) - p]_+ (from Prop. LP with sum(p - q f) = rho)."""
    rng = np.random.default_rng(3)
    for om in (1.0, 1.3, 2.0, 4.0):
        V = 8
        P, Q = random_kernels(V, 1, rng)
        P = [rows_of(oracle, t) for t in P]
        Q = [rows_of(oracle, t) for t in Q]
        law, target = output_law(oracle, P, Q, [om])
        tv = 0.5 * np.abs(law - target).sum()
        p, q = P[0], Q[0]
        assert abs(tv - np.maximum(np.minimum(q, om * p) - p, 0).sum()) < 1e-12


def test_position_diagnostics_against_enumeration(oracle):
    """Theorem 2 diagnostics.  beta is the bracket of the G* bound (proof Step 2), so
    (a) at L = 1 it is the exact TV of the enumerated output law;
    (b) summed over prefixes with weight Q(x_{1:i}) prod f_k it is the enumerated bound;
    (c) it vanishes at omega <= 1; and alpha at omega = 1 is the textbook acceptance rate
        of speculative decoding, 1 - TV(p, q)."""
    rng = np.random.default_rng(77)
    V = 5
    for om in (0.6, 1.0, 1.4, 2.5):
        P, Q = random_kernels(V, 1, rng, sharp=1.0, noise=1.0)
        P = [rows_of(oracle, t) for t in P]
        Q = [rows_of(oracle, t) for t in Q]
        alpha, beta = oracle.position_diagnostics(P[0], Q[0], om)
        law, target = output_law(oracle, P, Q, [om])
        if om >= 1.0:
            assert abs(0.5 * np.abs(law - target).sum() - beta) < 1e-12          # (a)
            f = np.array([oracle.accept_prob(P[0][x], Q[0][x], om) for x in range(V)])
            if om in (1.0, 1.4):   # rejections still happen here, so both sums of the bracket matter
                assert np.sum((1.0 - f) * Q[0]) > 1e-3
        else:
            assert abs(beta) < 1e-15                                               # (c)
        assert abs(alpha - np.minimum(Q[0], om * P[0]).sum()) < 1e-14
        if om == 1.0:
            assert abs(alpha - (1.0 - 0.5 * np.abs(P[0] - Q[0]).sum())) < 1e-14   # (c)
    # (b) two positions, prefix-dependent rows
    omega = [2.0, 1.3]
    P, Q = random_kernels(4, 2, rng, sharp=1.0, noise=1.0)
    P = [rows_of(oracle, t) for t in P]
    Q = [rows_of(oracle, t) for t in Q]
    total = oracle.position_diagnostics(P[0], Q[0], omega[0])[1]
    for x1 in range(4):
        w = Q[0][x1] * oracle.accept_prob(P[0][x1], Q[0][x1], omega[0])
        total += w * oracle.position_diagnostics(P[1][x1], Q[1][x1], omega[1])[1]
    assert abs(total - tv_bound(oracle, P, Q, omega)) < 1e-12


def test_prop_lp_value_and_optimality(oracle):
    """Prop. LP: for 1 >= f >= min{1,p/q}, inf_G sum|p - q f - G rho| = sum|p - q f| - rho, attained by G*."""
    rng = np.random.default_rng(17)
    for _ in range(30):
        V = int(rng.integers(2, 12))
        p = oracle.softmax(2 * rng.standard_normal(V))
        q = oracle.softmax(2 * rng.standard_normal(V))
        om = float(rng.uniform(1.0, 3.0))
        f = np.array([oracle.accept_prob(p[x], q[x], om) for x in range(V)])
        rho = np.sum((1 - f) * q)
        value = np.abs(p - q * f).sum() - rho
        g, R = oracle.residual(p, q, om)
        obj = lambda G: np.abs(p - q * f - G * rho).sum()
        assert abs(obj(g / R) - value) < 1e-13
        for _ in range(20):
            G = rng.dirichlet(np.ones(V))
            assert obj(G) >= value - 1e-13


# ----------------------------------------------------------------------------- inverse CDF / top-k / transform
def test_inverse_cdf_bruteforce(oracle):
    rng = np.random.default_rng(23)
    for _ in range(200):
        V = int(rng.integers(1, 50))
        g = rng.random(V) * (rng.random(V) < 0.6)
        if g.sum() == 0:
            g[rng.integers(0, V)] = 1.0
        R = 0.0
        for x in g:
            R += x
        for u in (0.0, 0.25, 0.999999, float(rng.random())):
            v = u * R
            C = np.cumsum(g)                      # sequential fp64, same order
            k = oracle.inverse_cdf(g, v)
            cand = np.nonzero(C > v)[0]
            want = int(cand[0]) if len(cand) else int(np.nonzero(g > 0)[0][-1])
            assert k == want and g[k] > 0
    assert oracle.inverse_cdf(np.array([0.0, 0.5, 0.0, 0.5]), 0.0) == 1      # u=0 -> first positive
    assert oracle.inverse_cdf(np.array([0.0, 0.5, 0.0, 0.5]), 0.5) == 3      # boundary goes up (strict >)
    assert oracle.inverse_cdf(np.array([0.0, 0.5, 0.0, 0.5, 0.0]), 1.0) == 3  # nothing exceeds -> last positive


def test_transform_topk_ties_and_guidance(oracle):
    rng = np.random.default_rng(29)
    V = 300
    # bf16-like coarse values make ties at the threshold
    lc = (np.round(rng.standard_normal(V) * 4) / 4).astype(np.float32)
    for k in (1, 7, 50, V):
        out = oracle.transform_row(lc, None, 1.0, 1.0, k)
        thr = np.sort(lc)[::-1][k - 1]
        keep = lc >= thr
        assert keep.sum() >= k
        np.testing.assert_array_equal(np.isfinite(out), keep)
        np.testing.assert_array_equal(out[keep], lc[keep].astype(np.float64))
    # k = 0 leaves the row alone
    np.testing.assert_array_equal(oracle.transform_row(lc, None, 1.0, 1.0, 0), lc.astype(np.float64))
    # guidance, evaluated in fp32: s = 4 (exact product) equals numpy fp32 arithmetic
    lu = rng.standard_normal(V).astype(np.float32)
    lc = (lu + rng.standard_normal(V).astype(np.float32)).astype(np.float32)
    out = oracle.transform_row(lc, lu, 4.0, 1.0, 0)
    np.testing.assert_array_equal(out, (lu + np.float32(4.0) * (lc - lu)).astype(np.float64))
    # general s: one rounding of s*d + l_u with d = fl32(l_c - l_u)
    s = np.float32(2.7)
    out = oracle.transform_row(lc, lu, float(s), 1.0, 0)
    d = (lc - lu).astype(np.float64)
    exact = np.float64(s) * d + lu.astype(np.float64)
    assert np.abs(out - exact).max() <= np.spacing(np.abs(exact).max().astype(np.float32)) / 2 + 1e-12
    assert np.mean(out == exact.astype(np.float32).astype(np.float64)) > 0.999
    # s = 1 returns the conditional logits up to the rounding of the difference
    np.testing.assert_allclose(oracle.transform_row(lc, lu, 1.0, 1.0, 0), lc, rtol=1e-6, atol=1e-6)
    # temperature: multiply by fl32(1/T)
    out = oracle.transform_row(lc, None, 1.0, 0.5, 0)
    np.testing.assert_array_equal(out, (lc * np.float32(2.0)).astype(np.float64))
    # guidance then top-k: threshold taken on the guided values
    out = oracle.transform_row(lc, lu, 4.0, 1.0, 10)
    guided = lu + np.float32(4.0) * (lc - lu)
    np.testing.assert_array_equal(np.isfinite(out), guided >= np.sort(guided)[::-1][9])


def test_transform_keeps_excluded_tokens_excluded(oracle):
    """A token that carries -inf on both inputs (excluded upstream) stays -inf under guidance, also
    when truncation sorts the row; the k-th largest is taken over what remains."""
    rng = np.random.default_rng(31)
    V = 200
    lu = rng.standard_normal(V).astype(np.float32)
    lc = (lu + rng.standard_normal(V).astype(np.float32)).astype(np.float32)
    gone = rng.random(V) < 0.3
    lc[gone] = -np.inf
    lu[gone] = -np.inf
    guided = np.where(gone, -np.inf, lu + np.float32(4.0) * (lc - np.where(gone, 0, lu))).astype(np.float32)
    guided[gone] = -np.inf
    out = oracle.transform_row(lc, lu, 4.0, 1.0, 0)
    assert not np.isnan(out).any()
    np.testing.assert_array_equal(out, guided.astype(np.float64))
    for k in (1, 10, int((~gone).sum()), V):
        out = oracle.transform_row(lc, lu, 4.0, 1.0, k)
        assert not np.isnan(out).any()
        thr = np.sort(guided)[::-1][k - 1]            # -inf once k exceeds the finite entries
        np.testing.assert_array_equal(np.isfinite(out), (guided >= thr) & ~gone)
        p = oracle.softmax(out)
        assert abs(p.sum() - 1) < 1e-12 and np.all(p[gone] == 0)
