"""The fp64 path of the draw x ~ G (csrc/exact_draw.h).  The fast kernels use it only where their fp32
result cannot be trusted (u next to a boundary of the CDF, a law of small mass), which random inputs
hit a few times in a hundred thousand draws; COOL_SD_FLAG_EXACT_DRAW sends every draw through it, so
these tests check the path itself against the oracle on every kind of row: both dtypes, element-wise
loads, long rows, guidance, temperature, top-k, both laws, the bonus row, the neighbour patch of
Eq. g_lantern, the early-exit kernels and the stand-alone resampling call.  Both sides then compute
in fp64, so not a single token may differ, near a boundary or not."""
import numpy as np
import pytest
import torch

from tests.parity_util import compare_verify, compare_verify_lantern, early_exit_form, to_numpy
from workloads import make_neighbor_table, make_workload, uniforms24

pytestmark = pytest.mark.gpu

CASES = [
    # cfg, B, L, V, dtype, options
    (1, 1, 4, 16384, "f32", {}),
    (2, 6, 8, 16384, "bf16", {}),
    (2, 3, 5, 4104, "bf16", {"resample_mode": 1}),
    (2, 3, 3, 5001, "bf16", {}),                      # element-wise loads
    (1, 2, 3, 1003, "f32", {"temperature": 1.3}),
    (1, 2, 2, 8, "f32", {}),
    (2, 2, 2, 1, "bf16", {}),
    (4, 6, 16, 16384, "bf16", {}),
    (5, 4, 3, 32768, "bf16", {}),                     # the one-launch form on rows of two chunks
    (5, 3, 3, 40000, "bf16", {"temperature": 0.7}),   # long rows: chunk masses, selection
    (5, 3, 2, 262144, "bf16", {}),                    # configuration 5's rows: the search narrows twice
    (1, 2, 2, 70000, "f32", {"resample_mode": 1}),
    (3, 4, 4, 16384, "bf16", {"top_k": 1000}),        # guidance + top-k
    (3, 2, 3, 40000, "bf16", {"top_k": 300}),
    (3, 2, 2, 70001, "bf16", {"top_k": 50}),          # thresholds from the radix passes
    (3, 3, 3, 8200, "bf16", {"top_k": 0, "temperature": 0.5}),   # peaked guided rows: small residual masses
]


@pytest.mark.parametrize("cfg,B,L,V,dtype,kw", CASES)
@pytest.mark.parametrize("early", [0, 1])
def test_every_draw_in_fp64_matches_the_oracle(P, oracle, cfg, B, L, V, dtype, kw, early):
    print("case", cfg, B, L, V, dtype, kw, early, flush=True)
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, dtype=dtype, top_k=kw.get("top_k") if cfg == 3 else None)
    if "temperature" in kw:
        w.temperature = kw["temperature"]
    mode = kw.get("resample_mode", 0)
    flags = P.COOL_SD_FLAG_EXACT_DRAW | (P.COOL_SD_FLAG_EARLY_EXIT if early else 0)
    honoured = bool(early) and early_exit_form(P, w) != 0
    for delta, has_bonus in ((1.1, True), (4.0, True), (1e30, True), (0.0, True), (1.1, False)):
        if delta == 0.0:
            om = np.zeros(L, np.float32)                                  # rejection at the first position
        elif delta == 1e30:
            om = np.full(L, 1e30, np.float32)                             # everything accepted: the bonus row
        else:
            om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, L, delta, w.nu)
        if not has_bonus:
            w.target = w.target[:, :L]
            if w.target_uncond is not None:
                w.target_uncond = w.target_uncond[:, :L]
        gpu = to_numpy(P.verify_workload(w, torch.from_numpy(om).cuda(), resample_mode=mode, flags=flags))
        torch.cuda.synchronize()
        st = compare_verify(oracle, w, om, gpu, resample_mode=mode, has_bonus=has_bonus, early_exit=honoured)
        assert st["token_exempt"] == 0, st


@pytest.mark.parametrize("V,dtype,guided,top_k,temperature", [
    (16384, "bf16", True, 200, 0.9), (16384, "f32", False, 1000, 1.0), (5001, "bf16", True, 50, 1.0),
    (16384, "bf16", False, 0, 1.0), (40000, "bf16", True, 300, 1.0), (65536, "bf16", True, 2000, 1.0),
    (32768, "bf16", False, 0, 1.0), (40000, "bf16", False, 0, 1.0), (70000, "bf16", True, 500, 1.0),
])
def test_resample_entry_point_in_fp64(P, oracle, V, dtype, guided, top_k, temperature):
    """cool_sd_resample with and without a draft row, every launch form, all draws in fp64."""
    B = 12
    w = make_workload(3 if guided else 1, device="cuda", B=B, L=1, V=V, dtype=dtype, top_k=top_k if guided else None)
    t, d = w.target[:, 0].contiguous(), w.draft[:, 0].contiguous()
    tu = w.target_uncond[:, 0].contiguous() if guided else None
    du = w.draft_uncond[:, 0].contiguous() if guided else None
    scale = w.cfg_scale if guided else 1.0
    u = uniforms24(torch.Generator(device="cuda").manual_seed(9), (B,), "cuda")
    u[0] = 0.0
    u[1] = 1.0 - 2.0 ** -24
    om = torch.linspace(0.25, 3.0, B, device="cuda")
    n = lambda x: None if x is None else x.float().cpu().numpy()
    kw = dict(cfg_scale=scale, temperature=temperature, top_k=top_k, want_g=True)
    for mode in (0, 1):
        params = P.make_params(t.unsqueeze(1), d.unsqueeze(1), has_bonus=0, top_k=top_k, cfg_scale=scale,
                               temperature=temperature, resample_mode=mode, flags=P.COOL_SD_FLAG_EXACT_DRAW)
        ws = torch.empty(max(P.cool_sd_workspace_bytes(params), 256), dtype=torch.uint8, device="cuda")
        tok = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        mass = torch.zeros(B, device="cuda")
        P.cool_sd_resample(params, t, tu, d, du, om, u, tok, mass, ws)
        torch.cuda.synchronize()
        ot, R, g = oracle.resample(n(t), n(d), om.cpu().numpy(), u.cpu().numpy(), target_uncond=n(tu),
                                   draft_uncond=n(du), resample_mode=mode, **kw)
        np.testing.assert_array_equal(tok.cpu().numpy(), ot)
        np.testing.assert_allclose(mass.cpu().numpy(), R, rtol=1e-6)
        # the draft-side draw: the law is q itself
        P.cool_sd_resample(params, d, du, None, None, None, u, tok, mass, ws)
        torch.cuda.synchronize()
        ot, R, g = oracle.resample(n(d), None, None, u.cpu().numpy(), target_uncond=n(du), **kw)
        np.testing.assert_array_equal(tok.cpu().numpy(), ot)
        np.testing.assert_allclose(mass.cpu().numpy(), R, rtol=1e-6)


@pytest.mark.parametrize("cfg,B,L,V,top_k", [(2, 6, 8, 16384, 0), (5, 3, 3, 40000, 0), (3, 4, 4, 16384, 1000)])
@pytest.mark.parametrize("mode", [0, 2])
def test_neighbour_patch_in_fp64(P, oracle, cfg, B, L, V, top_k, mode):
    """Eq. g_lantern (mode 2) and G* for Eq. f_lantern (mode 0) with every draw in fp64."""
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, top_k=top_k if cfg == 3 else None)
    nbr = make_neighbor_table(V, 10, device="cuda", seed=11, pad=0.1, self_entries=True)
    params = P.make_params(w.target, w.draft, top_k=w.top_k, cfg_scale=w.cfg_scale, temperature=w.temperature,
                           resample_mode=mode, flags=P.COOL_SD_FLAG_EXACT_DRAW)
    ws = torch.empty(max(P.cool_sd_workspace_bytes(params), 256), dtype=torch.uint8, device="cuda")
    out = dict(accept_len=torch.full((B,), -7, dtype=torch.int32, device="cuda"),
               next_token=torch.full((B,), -7, dtype=torch.int32, device="cuda"),
               resid_mass=torch.zeros(B, device="cuda"), count=torch.zeros((B, L), dtype=torch.int32, device="cuda"))
    for key in ("p_tok", "q_tok", "f", "p_agg"):
        out[key] = torch.zeros((B, L), device="cuda")
    for lam in (2.0, 50.0):
        P.cool_sd_verify_lantern(params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, nbr, 10, lam,
                                 w.u_accept, w.u_resample, out["accept_len"], out["next_token"], out["p_tok"],
                                 out["q_tok"], out["f"], out["resid_mass"], out["p_agg"], out["count"], ws)
        torch.cuda.synchronize()
        st = compare_verify_lantern(oracle, w, nbr.cpu().numpy(), lam, to_numpy(out), resample_mode=mode)
        assert st["token_exempt"] == 0 and st["set_exempt"] == 0, st
