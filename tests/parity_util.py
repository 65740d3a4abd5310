"""GPU-vs-oracle comparison with the tolerances the benchmark spec fixes.

  * accept lengths and token indices: bit-exact, except where a uniform lies within 1e-6 of
    the threshold it is compared with (such cases are counted and must be explained by that
    exemption): for the accept test the threshold is f_i, for the resampled token the two
    boundaries C_{k-1}/R and C_k/R of the law's CDF around the oracle's token, in units of u,
    whatever the law's mass R is;
  * probabilities, acceptance probabilities and residual masses: 1e-5 relative (fp32 vs fp64).
"""
import numpy as np

U_TOL = 1e-6
REL_TOL = 1e-5
ABS_FLOOR = 1e-37          # below fp32's normal range the GPU flushes to zero
# A law whose exact mass is below this is not determined by fp64 arithmetic either: the masses
# [p - q f]_+ are then rounding residue of probabilities that coincide to nine digits and more.  fp64
# probabilities near 1 carry ~1e-15 of rounding (a few ulp from the exponential and the normaliser),
# so two correct fp64 evaluations (the oracle's and the library's, which sum in different orders)
# agree on R only to ~1e-15 absolute: the 1e-5 relative tolerance on the mass needs R >= 1e-10, the
# 1e-6 band on the token (1e-6 R in units of mass) needs R >= 1e-9.  Seen: R = 1.4195e-12 on a
# two-token vocabulary, reported as 1.4194e-12 (7.8e-5 apart).  What the paper fixes there (proof
# of the proposition on the optimal G, App.): when the rejection mass sum_x (1 - f(x)) q(x) vanishes
# any G attains the infimum of the bound, and a row is reached with exactly that probability; the
# oracle's fall-back to p is one such choice.  The sampled token is then only required to be valid
# (in range, positive probability under p), and the reported mass to be either that residue or the
# fall-back's 1.
R_FLOOR = 1e-9


def token_band(R):
    """How far, in units of u, the uniform may lie from the boundary of the oracle's CDF where the GPU
    picks the neighbouring token: the task's 1e-6, whatever the law's mass R."""
    return U_TOL


def _close(gpu, ref, what, abs_tol=ABS_FLOOR):
    gpu = np.asarray(gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    err = np.abs(gpu - ref)
    bad = err > REL_TOL * np.abs(ref) + abs_tol
    assert not bad.any(), "%s: %d values off, worst rel %.3g at %s (gpu %r ref %r)" % (
        what, bad.sum(), (err / np.maximum(np.abs(ref), 1e-300)).max(), np.argwhere(bad)[0],
        gpu[tuple(np.argwhere(bad)[0])], ref[tuple(np.argwhere(bad)[0])])


def mass_close(gpu_R, ref_R, exact_R, what="resid_mass"):
    """A residual mass against the oracle's: 1e-5 relative.  A law whose exact mass is zero (p and
    q f coincide: any law is optimal there and the oracle falls back to p, mass 1) or below what
    fp64 resolves (R_FLOOR) may look either way: rounding residue, which is sampled from and
    reported, or an exact zero, after which p takes its place and the mass is 1."""
    g = float(gpu_R)
    if exact_R < R_FLOOR and (0.0 <= g <= 10 * R_FLOOR or abs(g - 1.0) <= REL_TOL):
        return
    _close(np.asarray([gpu_R]), np.asarray([ref_R]), what)


def exact_residual_mass(p, q, omega, mode):
    """sum_x [p - q f]_+ in fp64 before any fallback (q None: the law is p, mass 1)."""
    if q is None:
        return 1.0
    qf = q if mode == 1 else np.minimum(q, omega * p)
    return float(np.maximum(p - qf, 0.0).sum())


def subset(w, idx):
    """The sequences idx of a workload, as a workload of its own (for oracle checks of samples)."""
    import copy
    import torch
    idx = torch.as_tensor(idx, device=w.target.device)
    s = copy.copy(w)
    s.B = len(idx)
    for name in ("target", "draft", "draft_tokens", "u_accept", "u_resample", "target_uncond", "draft_uncond"):
        t = getattr(w, name)
        setattr(s, name, None if t is None else t.index_select(0, idx))
    return s


def run_oracle(O, w, omega, resample_mode=0, num_threads=16):
    t, d, tu, du = w.logits_f32_numpy()
    return O.verify(t, d, w.draft_tokens.cpu().numpy(), omega, w.u_accept.cpu().numpy(),
                    w.u_resample.cpu().numpy(), target_uncond=tu, draft_uncond=du,
                    cfg_scale=w.cfg_scale, temperature=w.temperature, top_k=w.top_k,
                    resample_mode=resample_mode, num_threads=num_threads)


def _oracle_row_law(O, w, b, j, omega_bj, resample_mode):
    """Unnormalised resampling law of row j (0-based; j == L is the bonus row) of sequence b."""
    t, d, tu, du = w.logits_f32_numpy()
    bonus = j == w.L
    tok, mass, g = O.resample(
        t[b:b + 1, j], None if bonus else d[b:b + 1, j], None if bonus else np.array([omega_bj], np.float32),
        w.u_resample.cpu().numpy()[b:b + 1],
        target_uncond=None if tu is None else tu[b:b + 1, j],
        draft_uncond=None if (du is None or bonus) else du[b:b + 1, j],
        cfg_scale=w.cfg_scale, temperature=w.temperature, top_k=w.top_k,
        resample_mode=resample_mode, want_g=True)
    return int(tok[0]), float(mass[0]), g[0]


def early_exit_form(P, w, has_bonus=True):
    """What cool_sd_early_exit_form says for a verify call on workload w with COOL_SD_FLAG_EARLY_EXIT
    (rows of torch tensors: 16-byte aligned whenever V is a multiple of the vector width)."""
    params = P.make_params(w.target, w.draft, top_k=w.top_k, cfg_scale=w.cfg_scale, temperature=w.temperature,
                           flags=P.COOL_SD_FLAG_EARLY_EXIT)
    vec = 8 if w.dtype == "bf16" else 4
    return P.cool_sd_early_exit_form(params, w.V % vec == 0)


def compare_verify(O, w, omega, gpu, ref=None, resample_mode=0, has_bonus=True, early_exit=False):
    """Assert parity of one verify call.  gpu: dict of numpy arrays.  Returns counters.
    early_exit: the per-position outputs after the rejected position must be NaN (never evaluated)."""
    omega = np.asarray(omega, np.float32)
    if ref is None:
        ref = run_oracle(O, w, omega, resample_mode)
    B, L = w.B, w.L
    ua = w.u_accept.cpu().numpy().astype(np.float64)
    ur = w.u_resample.cpu().numpy().astype(np.float64)
    if "p_tok" in gpu and early_exit:
        gpu = dict(gpu)
        later = np.arange(L)[None, :] > gpu["accept_len"][:, None]
        for k in ("p_tok", "q_tok", "f"):
            assert np.isnan(gpu[k][later]).all() and not np.isnan(gpu[k][~later]).any(), k
            gpu[k] = np.where(later, ref[k], gpu[k])
    if "p_tok" in gpu:
        _close(gpu["p_tok"], ref["p_tok"], "p_tok")
        _close(gpu["q_tok"], ref["q_tok"], "q_tok")
        _close(gpu["f"], ref["f"], "f")
    ambiguous = np.abs(ua - ref["f"]) <= U_TOL
    stats = dict(tau_exempt=0, token_exempt=0, sequences=B)
    for b in range(B):
        om_b = omega if omega.ndim == 1 else omega[b]
        # accepted lengths that the exemption allows
        allowed = set()
        tau = L
        for i in range(L):
            if ambiguous[b, i]:
                allowed.add(i)                     # may be rejected here ...
                continue                           # ... or accepted
            if not ref["acc"][b, i]:
                tau = i
                break
        else:
            tau = L
        allowed.add(tau)
        tg = int(gpu["accept_len"][b])
        assert tg in allowed, "seq %d: accept_len gpu %d, oracle %d, allowed %s" % (
            b, tg, ref["accept_len"][b], sorted(allowed))
        if tg != ref["accept_len"][b]:
            stats["tau_exempt"] += 1
        xg = int(gpu["next_token"][b])
        if tg == L and not has_bonus:
            assert xg == -1
            continue
        def exact_R():
            p, q = _oracle_rows(O, w, b, tg)
            return exact_residual_mass(p, q, float(om_b[min(tg, L - 1)]), resample_mode)
        if tg == ref["accept_len"][b] and xg == ref["next_token"][b]:
            if abs(float(gpu["resid_mass"][b]) - float(ref["resid_mass"][b])) > REL_TOL * abs(float(ref["resid_mass"][b])):
                mass_close(gpu["resid_mass"][b], ref["resid_mass"][b], exact_R())
            continue
        # token differs (or tau took the exempt branch): check against the oracle's law of that row
        xo, R, g = _oracle_row_law(O, w, b, tg, om_b[min(tg, L - 1)], resample_mode)
        mass_close(gpu["resid_mass"][b], R, exact_R())
        if xg != xo and min(R, exact_R()) < R_FLOOR:      # (R is 1 where the oracle fell back to p)
            p, _ = _oracle_rows(O, w, b, tg)
            assert 0 <= xg < w.V and p[xg] > 0, "seq %d: gpu token %d has no probability" % (b, xg)
            stats["token_exempt"] += 1
            continue
        if xg != xo:
            assert 0 <= xg < w.V and g[xg] > 0, "seq %d: gpu token %d has zero mass" % (b, xg)
            C = np.cumsum(g)
            v = ur[b] * R
            if xg < xo:
                gap = (v - C[xg]) / R              # oracle: C[xg] <= v
            else:
                gap = (C[xg - 1] - v) / R          # oracle: C[xo] > v already
            assert 0 <= gap <= token_band(R), "seq %d: token gpu %d oracle %d, u is %.3g away from the boundary" % (
                b, xg, xo, gap)
            stats["token_exempt"] += 1
    return stats


def to_numpy(out):
    return {k: v.detach().cpu().numpy() for k, v in out.items()}


# ------------------------------------------------------------------ aggregated acceptance (neighbour sets)
SET_TOL = 1e-12            # a running neighbour sum this close (relative) to lambda p(x~) may fall on either side:
                           # both sides decide in fp64, in different summation orders


def _oracle_rows(O, w, b, i):
    """p_i, q_i of sequence b at position i (0-based; i == L: bonus row, q is None), in fp64."""
    t, d, tu, du = w.logits_f32_numpy()
    p = O.softmax(O.transform_row(t[b, i], None if tu is None else tu[b, i], w.cfg_scale, w.temperature, w.top_k))
    if i >= w.L:
        return p, None
    q = O.softmax(O.transform_row(d[b, i], None if du is None else du[b, i], w.cfg_scale, w.temperature, w.top_k))
    return p, q


def compare_verify_lantern(O, w, nbr, lam, gpu, resample_mode=0, num_threads=16):
    """Assert parity of one cool_sd_verify_lantern call with the oracle.  Integer outputs are exact
    except where a uniform is within U_TOL of its threshold or a neighbour sum within SET_TOL of
    lambda p(x~); floating-point outputs to REL_TOL."""
    t, d, tu, du = w.logits_f32_numpy()
    tok = w.draft_tokens.cpu().numpy()
    ua = w.u_accept.cpu().numpy().astype(np.float64)
    ur = w.u_resample.cpu().numpy().astype(np.float64)
    ref = O.verify_lantern(t, d, tok, nbr, lam, ua, ur, target_uncond=tu, draft_uncond=du, cfg_scale=w.cfg_scale,
                           temperature=w.temperature, top_k=w.top_k, resample_mode=resample_mode,
                           num_threads=num_threads)
    B, L, V = w.B, w.L, w.V
    _close(gpu["p_tok"], ref["p_tok"], "p_tok")
    _close(gpu["q_tok"], ref["q_tok"], "q_tok")
    # positions whose neighbour set is decided within rounding
    loose = np.zeros((B, L), bool)
    differ = np.argwhere(gpu["count"] != ref["count"])
    for b, i in differ:
        p, _ = _oracle_rows(O, w, b, i)
        x = int(tok[b, i])
        valid = [int(n) for n in nbr[x] if 0 <= n < V and n != x]
        cum = np.cumsum(p[valid])
        thr = lam * p[x]
        assert np.any(np.abs(cum - thr) <= SET_TOL * thr), "seq %d pos %d: count gpu %d oracle %d" % (
            b, i, gpu["count"][b, i], ref["count"][b, i])
        loose[b, i] = True
    keep = ~loose
    _close(np.where(keep, gpu["p_agg"], 0), np.where(keep, ref["p_agg"], 0), "p_agg")
    _close(np.where(keep, gpu["f"], 0), np.where(keep, ref["f"], 0), "f")
    ambiguous = (np.abs(ua - ref["f"]) <= U_TOL) | loose
    stats = dict(tau_exempt=0, token_exempt=0, set_exempt=int(loose.sum()), sequences=B,
                 members=int(ref["count"].sum()))
    for b in range(B):
        allowed = set()
        tau = L
        for i in range(L):
            if ambiguous[b, i]:
                allowed.add(i)
                continue
            if not ref["acc"][b, i]:
                tau = i
                break
        allowed.add(tau)
        tg = int(gpu["accept_len"][b])
        assert tg in allowed, "seq %d: accept_len gpu %d, oracle %d" % (b, tg, ref["accept_len"][b])
        if tg != ref["accept_len"][b]:
            stats["tau_exempt"] += 1
        xg = int(gpu["next_token"][b])
        if tg == ref["accept_len"][b] and xg == ref["next_token"][b] and not loose[b, min(tg, L - 1)]:
            _close(gpu["resid_mass"][b:b + 1], ref["resid_mass"][b:b + 1], "resid_mass")
            continue
        p, q = _oracle_rows(O, w, b, tg)
        if q is None:
            g, R = p, p.sum()
        else:
            g, R = O.lantern_residual(p, q, nbr, lam, resample_mode, int(tok[b, tg]))
        if loose[b, min(tg, L - 1)] and resample_mode == 2:
            continue                              # the law itself depends on the undecided set
        _close(gpu["resid_mass"][b:b + 1], [R], "resid_mass")
        xo = O.inverse_cdf(g, ur[b] * R)
        if xg != xo:
            assert 0 <= xg < V and g[xg] > 0, "seq %d: gpu token %d has zero mass" % (b, xg)
            Cs = np.cumsum(g)
            v = ur[b] * R
            gap = (v - Cs[xg]) / R if xg < xo else (Cs[xg - 1] - v) / R
            assert 0 <= gap <= token_band(R), "seq %d: token gpu %d oracle %d, u is %.3g away from the boundary" % (
                b, xg, xo, gap)
            stats["token_exempt"] += 1
    return stats


# ------------------------------------------------------------------ Theorem 2 diagnostics
def oracle_diagnostics(oracle, w, om):
    """alpha[B, L], beta[B, L] of a workload from the oracle."""
    kw = dict(cfg_scale=w.cfg_scale, temperature=w.temperature, top_k=w.top_k)
    tu = None if w.target_uncond is None else w.target_uncond.float().cpu().numpy()
    du = None if w.draft_uncond is None else w.draft_uncond.float().cpu().numpy()
    return oracle.diagnostics(w.target.float().cpu().numpy(), w.draft.float().cpu().numpy(), om,
                              target_uncond=tu, draft_uncond=du, **kw)


def verify_diagnostics_call(P, w, om, mode=0):
    """cool_sd_verify_diagnostics on a workload; returns (verify outputs as numpy dict, alpha, beta)."""
    import torch
    omega = torch.from_numpy(np.ascontiguousarray(om, dtype=np.float32)).cuda()
    params = P.make_params(w.target, w.draft, top_k=w.top_k, cfg_scale=w.cfg_scale, temperature=w.temperature,
                           resample_mode=mode, omega_stride_b=0 if omega.dim() == 1 else omega.stride(0))
    ws = torch.empty(max(P.cool_sd_workspace_bytes(params), 256), dtype=torch.uint8, device="cuda")
    B, L = w.B, w.L
    out = dict(accept_len=torch.full((B,), -9, dtype=torch.int32, device="cuda"),
               next_token=torch.full((B,), -9, dtype=torch.int32, device="cuda"),
               p_tok=torch.zeros((B, L), device="cuda"), q_tok=torch.zeros((B, L), device="cuda"),
               f=torch.zeros((B, L), device="cuda"), resid_mass=torch.zeros(B, device="cuda"))
    alpha, beta = torch.zeros((B, L), device="cuda"), torch.zeros((B, L), device="cuda")
    P.cool_sd_verify_diagnostics(params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, omega,
                                 w.u_accept, w.u_resample, out["accept_len"], out["next_token"], out["p_tok"],
                                 out["q_tok"], out["f"], out["resid_mass"], alpha, beta, ws)
    torch.cuda.synchronize()
    return to_numpy(out), alpha.cpu().numpy().astype(np.float64), beta.cpu().numpy().astype(np.float64)
