"""ctypes front end of the fp64 C oracle (oracle/cool_sd_oracle.c).

TEST INFRASTRUCTURE.  Arrays in, arrays out (numpy); no arithmetic of the method
lives here -- every number comes from the C functions, which cite the paper.
Logits are passed as float32 (a bf16 input is widened exactly by the caller).
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

SCHED_UNIFORM, SCHED_EXP, SCHED_LINEAR = 0, 1, 2
RESAMPLE_OPT, RESAMPLE_VANILLA, RESAMPLE_LANTERN = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            path = _build.build()
        L = C.CDLL(path)
        dp, fp, ip, u8p = (C.POINTER(C.c_double), C.POINTER(C.c_float), C.POINTER(C.c_int),
                           C.POINTER(C.c_ubyte))
        L.csd_oracle_schedule.argtypes = [C.c_int, C.c_int, C.c_double, C.c_double, dp]
        L.csd_oracle_schedule.restype = C.c_int
        L.csd_oracle_transform_row.argtypes = [fp, fp, C.c_int, C.c_float, C.c_float, C.c_int, dp]
        L.csd_oracle_transform_row.restype = C.c_int
        L.csd_oracle_softmax.argtypes = [dp, C.c_int, dp]
        L.csd_oracle_softmax.restype = None
        L.csd_oracle_accept_prob.argtypes = [C.c_double] * 3
        L.csd_oracle_accept_prob.restype = C.c_double
        L.csd_oracle_accept.argtypes = [C.c_double] * 4
        L.csd_oracle_accept.restype = C.c_int
        L.csd_oracle_residual.argtypes = [dp, dp, C.c_int, C.c_double, C.c_int, dp]
        L.csd_oracle_residual.restype = C.c_double
        L.csd_oracle_position_diagnostics.argtypes = [dp, dp, C.c_int, C.c_double, dp, dp]
        L.csd_oracle_position_diagnostics.restype = None
        L.csd_oracle_inverse_cdf.argtypes = [dp, C.c_int, C.c_double]
        L.csd_oracle_inverse_cdf.restype = C.c_int
        L.csd_oracle_verify.argtypes = [
            C.c_int, C.c_int, C.c_int, C.c_int,
            fp, fp, C.c_longlong, C.c_longlong,
            fp, fp, C.c_longlong, C.c_longlong,
            C.c_float, C.c_float, C.c_int, C.c_int,
            ip, fp, C.c_longlong, fp, fp,
            ip, ip, dp, dp, dp, dp, u8p, C.c_int]
        L.csd_oracle_verify.restype = C.c_int
        L.csd_oracle_resample.argtypes = [
            C.c_int, C.c_int, fp, fp, C.c_longlong, fp, fp, C.c_longlong,
            C.c_float, C.c_float, C.c_int, C.c_int, fp, fp, ip, dp, dp]
        L.csd_oracle_resample.restype = C.c_int
        L.csd_oracle_lantern_set.argtypes = [dp, C.c_int, C.c_int, ip, C.c_int, C.c_double, dp, ip]
        L.csd_oracle_lantern_set.restype = C.c_int
        L.csd_oracle_lantern_accept_prob.argtypes = [dp, dp, C.c_int, C.c_int, ip, C.c_int, C.c_double]
        L.csd_oracle_lantern_accept_prob.restype = C.c_double
        L.csd_oracle_lantern_residual.argtypes = [dp, dp, C.c_int, ip, C.c_int, C.c_double, C.c_int, C.c_int, dp]
        L.csd_oracle_lantern_residual.restype = C.c_double
        L.csd_oracle_verify_lantern.argtypes = [
            C.c_int, C.c_int, C.c_int, C.c_int,
            fp, fp, C.c_longlong, C.c_longlong,
            fp, fp, C.c_longlong, C.c_longlong,
            C.c_float, C.c_float, C.c_int, C.c_int,
            ip, ip, C.c_int, C.c_float, fp, fp,
            ip, ip, dp, dp, dp, dp, u8p, dp, ip, C.c_int]
        L.csd_oracle_verify_lantern.restype = C.c_int
        L.csd_oracle_max_threads.argtypes = []
        L.csd_oracle_max_threads.restype = C.c_int
        _lib = L
    return _lib


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a, ty):
    return None if a is None else a.ctypes.data_as(C.POINTER(ty))


def schedule(kind, L, delta, param=0.0):
    out = np.empty(L, dtype=np.float64)
    rc = lib().csd_oracle_schedule(kind, L, float(delta), float(param), _ptr(out, C.c_double))
    if rc != 0:
        raise ValueError("csd_oracle_schedule: invalid arguments")
    return out


def transform_row(l_cond, l_uncond=None, cfg_scale=1.0, temperature=1.0, top_k=0):
    lc, lu = _f32(l_cond), _f32(l_uncond)
    out = np.empty(lc.shape[0], dtype=np.float64)
    rc = lib().csd_oracle_transform_row(_ptr(lc, C.c_float), _ptr(lu, C.c_float), lc.shape[0],
                                        cfg_scale, temperature, top_k, _ptr(out, C.c_double))
    if rc != 0:
        raise ValueError("csd_oracle_transform_row rc=%d" % rc)
    return out


def softmax(l):
    l = np.ascontiguousarray(l, dtype=np.float64)
    p = np.empty_like(l)
    lib().csd_oracle_softmax(_ptr(l, C.c_double), l.shape[0], _ptr(p, C.c_double))
    return p


def accept_prob(p_x, q_x, omega):
    return lib().csd_oracle_accept_prob(float(p_x), float(q_x), float(omega))


def accept(r, p_x, q_x, omega):
    return bool(lib().csd_oracle_accept(float(r), float(p_x), float(q_x), float(omega)))


def residual(p, q, omega, mode=RESAMPLE_OPT):
    """Unnormalised resampling law g and its mass R for one position (q=None: bonus)."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    qq = None if q is None else np.ascontiguousarray(q, dtype=np.float64)
    g = np.empty_like(p)
    R = lib().csd_oracle_residual(_ptr(p, C.c_double), _ptr(qq, C.c_double), p.shape[0],
                                  float(omega), mode, _ptr(g, C.c_double))
    return g, R


def position_diagnostics(p, q, omega):
    """(alpha, beta) of one position: acceptance probability and half the TV-bound bracket."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    q = np.ascontiguousarray(q, dtype=np.float64)
    out = np.empty(2, dtype=np.float64)
    lib().csd_oracle_position_diagnostics(_ptr(p, C.c_double), _ptr(q, C.c_double), p.shape[0], float(omega),
                                          _ptr(out[0:1], C.c_double), _ptr(out[1:2], C.c_double))
    return float(out[0]), float(out[1])


def diagnostics(target, draft, omega, *, target_uncond=None, draft_uncond=None, cfg_scale=1.0,
                temperature=1.0, top_k=0):
    """alpha[B, L], beta[B, L] (Theorem 2) of every drafted position: transform, softmax and
    position_diagnostics per row pair.  target may carry a bonus row, which is ignored."""
    t, d = _f32(target), _f32(draft)
    tu, du = _f32(target_uncond), _f32(draft_uncond)
    B, L, V = d.shape
    assert t.shape[0] == B and t.shape[1] in (L, L + 1) and t.shape[2] == V
    assert (tu is None) == (du is None) and (tu is None or (tu.shape == t.shape and du.shape == d.shape))
    om = np.broadcast_to(_f32(omega), (B, L))
    alpha = np.empty((B, L), np.float64)
    beta = np.empty((B, L), np.float64)
    for b in range(B):
        for i in range(L):
            p = softmax(transform_row(t[b, i], None if tu is None else tu[b, i], cfg_scale, temperature, top_k))
            q = softmax(transform_row(d[b, i], None if du is None else du[b, i], cfg_scale, temperature, top_k))
            alpha[b, i], beta[b, i] = position_diagnostics(p, q, om[b, i])
    return alpha, beta


def inverse_cdf(g, v):
    g = np.ascontiguousarray(g, dtype=np.float64)
    return lib().csd_oracle_inverse_cdf(_ptr(g, C.c_double), g.shape[0], float(v))


def verify(target, draft, draft_tokens, omega, u_accept, u_resample, *, target_uncond=None,
           draft_uncond=None, cfg_scale=1.0, temperature=1.0, top_k=0,
           resample_mode=RESAMPLE_OPT, num_threads=1):
    """Algorithm 1's verification stage on [B, L(+1), V] / [B, L, V] float32 logits.

    Returns a dict: accept_len[B], next_token[B], resid_mass[B], p_tok/q_tok/f[B,L], acc[B,L].
    """
    t, d = _f32(target), _f32(draft)
    tu, du = _f32(target_uncond), _f32(draft_uncond)
    B, Lt, V = t.shape
    L = d.shape[1]
    assert d.shape == (B, L, V) and Lt in (L, L + 1)
    assert (tu is None) == (du is None) and (tu is None or (tu.shape == t.shape and du.shape == d.shape))
    has_bonus = int(Lt == L + 1)
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32).reshape(B, L)
    om = _f32(omega)
    om_sb = 0 if om.ndim == 1 else L
    ua = _f32(u_accept).reshape(B, L)
    ur = _f32(u_resample).reshape(B)
    out = dict(accept_len=np.empty(B, np.int32), next_token=np.empty(B, np.int32),
               resid_mass=np.empty(B, np.float64), p_tok=np.empty((B, L), np.float64),
               q_tok=np.empty((B, L), np.float64), f=np.empty((B, L), np.float64),
               acc=np.empty((B, L), np.uint8))
    rc = lib().csd_oracle_verify(
        B, L, V, has_bonus,
        _ptr(t, C.c_float), _ptr(tu, C.c_float), Lt * V, V,
        _ptr(d, C.c_float), _ptr(du, C.c_float), L * V, V,
        cfg_scale, temperature, top_k, resample_mode,
        _ptr(tok, C.c_int), _ptr(om, C.c_float), om_sb, _ptr(ua, C.c_float), _ptr(ur, C.c_float),
        _ptr(out["accept_len"], C.c_int), _ptr(out["next_token"], C.c_int),
        _ptr(out["resid_mass"], C.c_double), _ptr(out["p_tok"], C.c_double),
        _ptr(out["q_tok"], C.c_double), _ptr(out["f"], C.c_double),
        _ptr(out["acc"], C.c_ubyte), num_threads)
    if rc != 0:
        raise ValueError("csd_oracle_verify rc=%d" % rc)
    return out


def resample(target_rows, draft_rows, omega_rows, u, *, target_uncond=None, draft_uncond=None,
             cfg_scale=1.0, temperature=1.0, top_k=0, resample_mode=RESAMPLE_OPT, want_g=False):
    """Stand-alone resampling of one row pair per sequence ([B, V] each; draft None = bonus)."""
    t, d = _f32(target_rows), _f32(draft_rows)
    tu, du = _f32(target_uncond), _f32(draft_uncond)
    B, V = t.shape
    om = _f32(omega_rows)
    uu = _f32(u).reshape(B)
    token = np.empty(B, np.int32)
    mass = np.empty(B, np.float64)
    g = np.empty((B, V), np.float64) if want_g else None
    rc = lib().csd_oracle_resample(B, V, _ptr(t, C.c_float), _ptr(tu, C.c_float), V,
                                   _ptr(d, C.c_float), _ptr(du, C.c_float), V,
                                   cfg_scale, temperature, top_k, resample_mode,
                                   _ptr(om, C.c_float), _ptr(uu, C.c_float),
                                   _ptr(token, C.c_int), _ptr(mass, C.c_double),
                                   _ptr(g, C.c_double))
    if rc != 0:
        raise ValueError("csd_oracle_resample rc=%d" % rc)
    return (token, mass, g) if want_g else (token, mass)


def _nbr(nbr, V):
    nbr = np.ascontiguousarray(nbr, dtype=np.int32)
    assert nbr.ndim == 2 and nbr.shape[0] == V
    return nbr


def lantern_set(p, x, nbr_row, lam):
    """Neighbour set of token x under the row p: (m, aggregated probability, selected neighbours)."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    row = np.ascontiguousarray(nbr_row, dtype=np.int32)
    agg = np.empty(1, np.float64)
    member = np.empty(max(1, row.shape[0]), np.int32)
    m = lib().csd_oracle_lantern_set(_ptr(p, C.c_double), p.shape[0], int(x), _ptr(row, C.c_int), row.shape[0],
                                     float(lam), _ptr(agg, C.c_double), _ptr(member, C.c_int))
    return m, float(agg[0]), member[:m].copy()


def lantern_accept_prob(p, q, x, nbr, lam):
    p = np.ascontiguousarray(p, dtype=np.float64)
    q = np.ascontiguousarray(q, dtype=np.float64)
    nbr = _nbr(nbr, p.shape[0])
    return lib().csd_oracle_lantern_accept_prob(_ptr(p, C.c_double), _ptr(q, C.c_double), p.shape[0], int(x),
                                                _ptr(nbr, C.c_int), nbr.shape[1], float(lam))


def lantern_residual(p, q, nbr, lam, mode, x_draft):
    """Unnormalised resampling law g and its mass R after the draft token x_draft was rejected."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    q = np.ascontiguousarray(q, dtype=np.float64)
    nbr = _nbr(nbr, p.shape[0])
    g = np.empty_like(p)
    R = lib().csd_oracle_lantern_residual(_ptr(p, C.c_double), _ptr(q, C.c_double), p.shape[0], _ptr(nbr, C.c_int),
                                          nbr.shape[1], float(lam), mode, int(x_draft), _ptr(g, C.c_double))
    return g, R


def verify_lantern(target, draft, draft_tokens, nbr, lam, u_accept, u_resample, *, target_uncond=None,
                   draft_uncond=None, cfg_scale=1.0, temperature=1.0, top_k=0,
                   resample_mode=RESAMPLE_OPT, num_threads=1):
    """Algorithm 1's verification stage with the aggregated acceptance probability (Eq. f_lantern).

    Returns the dict of verify() plus p_agg[B, L] and count[B, L]."""
    t, d = _f32(target), _f32(draft)
    tu, du = _f32(target_uncond), _f32(draft_uncond)
    B, Lt, V = t.shape
    L = d.shape[1]
    assert d.shape == (B, L, V) and Lt in (L, L + 1)
    assert (tu is None) == (du is None) and (tu is None or (tu.shape == t.shape and du.shape == d.shape))
    has_bonus = int(Lt == L + 1)
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32).reshape(B, L)
    nbr = _nbr(nbr, V)
    ua = _f32(u_accept).reshape(B, L)
    ur = _f32(u_resample).reshape(B)
    out = dict(accept_len=np.empty(B, np.int32), next_token=np.empty(B, np.int32),
               resid_mass=np.empty(B, np.float64), p_tok=np.empty((B, L), np.float64),
               q_tok=np.empty((B, L), np.float64), f=np.empty((B, L), np.float64),
               acc=np.empty((B, L), np.uint8), p_agg=np.empty((B, L), np.float64),
               count=np.empty((B, L), np.int32))
    rc = lib().csd_oracle_verify_lantern(
        B, L, V, has_bonus,
        _ptr(t, C.c_float), _ptr(tu, C.c_float), Lt * V, V,
        _ptr(d, C.c_float), _ptr(du, C.c_float), L * V, V,
        cfg_scale, temperature, top_k, resample_mode,
        _ptr(tok, C.c_int), _ptr(nbr, C.c_int), nbr.shape[1], float(lam), _ptr(ua, C.c_float), _ptr(ur, C.c_float),
        _ptr(out["accept_len"], C.c_int), _ptr(out["next_token"], C.c_int),
        _ptr(out["resid_mass"], C.c_double), _ptr(out["p_tok"], C.c_double),
        _ptr(out["q_tok"], C.c_double), _ptr(out["f"], C.c_double),
        _ptr(out["acc"], C.c_ubyte), _ptr(out["p_agg"], C.c_double), _ptr(out["count"], C.c_int), num_threads)
    if rc != 0:
        raise ValueError("csd_oracle_verify_lantern rc=%d" % rc)
    return out


def max_threads():
    return lib().csd_oracle_max_threads()
