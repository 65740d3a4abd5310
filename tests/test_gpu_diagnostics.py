"""Parity of cool_sd_diagnostics (alpha_i, beta_i of Theorem 2) against the CPU oracle.

Tolerances.  alpha is a sum of non-negative terms, each with the fp32 relative error of a
probability: 1e-5 relative.  beta = sum_x [min(q, omega p) - p]_+ subtracts probabilities, so
its error is absolute: every term errs by at most a few ulp of p(x), hence |error| <= a few
1e-7 x sum_x p(x); the test allows 2e-6 absolute plus 1e-5 relative.  At omega <= 1 no term can
be positive in either arithmetic and beta must be exactly zero.
"""
import numpy as np
import pytest
import torch

from tests.parity_util import oracle_diagnostics as _oracle_diag, verify_diagnostics_call as _verify_diag
from workloads import make_workload

pytestmark = pytest.mark.gpu


def _check(P, oracle, w, om):
    omega = torch.from_numpy(np.ascontiguousarray(om, dtype=np.float32)).cuda()
    alpha, beta = P.diagnostics_workload(w, omega)
    torch.cuda.synchronize()
    alpha, beta = alpha.cpu().numpy().astype(np.float64), beta.cpu().numpy().astype(np.float64)
    a_ref, b_ref = _oracle_diag(oracle, w, om)
    np.testing.assert_allclose(alpha, a_ref, rtol=1e-5, atol=1e-9)
    np.testing.assert_allclose(beta, b_ref, rtol=1e-5, atol=2e-6)
    omb = np.broadcast_to(om, alpha.shape)
    assert (beta[omb <= 1.0] == 0.0).all()
    assert (alpha >= 0).all() and (alpha <= 1.0 + 1e-5).all() and (beta >= 0).all()
    return alpha, beta


SHAPES = [
    (1, 1, 4, 16384, "f32"),        # one chunk, fp32
    (2, 4, 8, 16384, "bf16"),       # one chunk, bf16
    (2, 3, 5, 4104, "bf16"),        # partial last tile
    (2, 3, 3, 5001, "bf16"),        # element-wise loads
    (1, 2, 3, 1003, "f32"),
    (1, 2, 2, 8, "f32"),
    (2, 2, 2, 1, "bf16"),           # single token: alpha = min(1, omega), beta = [min(1, omega) - 1]_+ = 0
    (5, 2, 3, 40000, "bf16"),       # statistics pass + five chunks of 8192, ragged tail
    (5, 2, 2, 262144, "bf16"),
    (1, 2, 2, 20000, "f32"),
    (5, 3, 2, 16392, "bf16"),
]


@pytest.mark.parametrize("cfg,B,L,V,dtype", SHAPES)
def test_diagnostics_shapes(P, oracle, cfg, B, L, V, dtype):
    print("case", cfg, B, L, V, dtype, flush=True)
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, dtype=dtype)
    om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, L, 2.0, w.nu)
    _check(P, oracle, w, om)


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_diagnostics_at_full_size(P, oracle, cfg):
    """cool_sd_diagnostics and cool_sd_verify_diagnostics on the benchmark configurations at their full
    sizes (the shapes bench.py --diagnostics times): every position's alpha and beta against the oracle."""
    from tests.parity_util import compare_verify, verify_diagnostics_call
    print("full cfg", cfg, flush=True)
    w = make_workload(cfg, device="cuda")
    om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, w.L, 2.0, w.nu)
    alpha, beta = _check(P, oracle, w, om)
    both, alpha2, beta2 = verify_diagnostics_call(P, w, om)
    compare_verify(oracle, w, om, both)
    a_ref, b_ref = _oracle_diag(oracle, w, om)
    np.testing.assert_allclose(alpha2, a_ref, rtol=1e-5, atol=1e-9)
    np.testing.assert_allclose(beta2, b_ref, rtol=1e-5, atol=2e-6)


def test_diagnostics_budgets_and_per_sequence_omega(P, oracle):
    w = make_workload(2, device="cuda", B=6, L=8, V=16384)
    for delta in (0.5, 1.0, 4.0):
        _check(P, oracle, w, P.cool_sd_schedule(P.COOL_SD_SCHED_UNIFORM, 8, delta))
    om = np.tile(P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, 8, 2.0, w.nu), (6, 1)).astype(np.float32)
    om[0] = 0.0
    om[1] *= 3.0
    alpha, beta = _check(P, oracle, w, om)
    assert (alpha[0] == 0).all() and (beta[0] == 0).all()


def test_diagnostics_guidance_topk_and_no_bonus(P, oracle):
    w = make_workload(3, device="cuda", B=3, L=4)                 # guided, top-k: thresholds from the statistics pass
    om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, 4, 2.0, w.nu)
    _check(P, oracle, w, om)
    w = make_workload(3, device="cuda", B=2, L=3, top_k=0)        # guided only: one-chunk path with the transform
    _check(P, oracle, w, om[:3])
    w = make_workload(2, device="cuda", B=3, L=4, V=16384)
    w.target = w.target[:, :4].contiguous()                       # no bonus row
    _check(P, oracle, w, om)


def test_diagnostics_predict_the_acceptance_rate(P, oracle):
    """Eq. token_exp, position 1: over many independent sequences that share one row pair, the
    fraction of accepted first tokens (drawn from q_1) tends to alpha_1."""
    w = make_workload(2, device="cuda", B=1, L=1, V=4096)
    om = np.array([1.5], np.float32)
    alpha, _ = _check(P, oracle, w, om)
    n = 20000
    g = torch.Generator(device="cuda").manual_seed(5)
    q = torch.softmax(w.draft[0, 0].float(), -1)
    tokens = torch.multinomial(q, n, replacement=True, generator=g).to(torch.int32).reshape(n, 1)
    target = w.target.expand(n, 2, 4096)
    draft = w.draft.expand(n, 1, 4096)
    params = P.make_params(target, draft)
    ws = torch.empty(P.cool_sd_workspace_bytes(params), dtype=torch.uint8, device="cuda")
    u = torch.rand((n, 1), generator=g, device="cuda")
    tau = torch.empty(n, dtype=torch.int32, device="cuda")
    nxt = torch.empty(n, dtype=torch.int32, device="cuda")
    P.cool_sd_verify(params, target, None, draft, None, tokens, torch.from_numpy(om).cuda(), u,
                     torch.rand(n, generator=g, device="cuda"), tau, nxt, None, None, None, None, ws)
    torch.cuda.synchronize()
    rate = float((tau >= 1).float().mean())
    a = float(alpha[0, 0])
    assert abs(rate - a) < 5 * np.sqrt(a * (1 - a) / n)


def test_diagnostics_topk_on_long_rows(P, oracle):
    """Truncation on rows longer than one workgroup (thresholds from the radix passes), with and
    without guidance."""
    for cfg, V, k in ((3, 40000, 1000), (2, 20001, 64)):
        w = make_workload(cfg, device="cuda", B=2, L=3, V=V, top_k=k if cfg == 3 else None)
        w.top_k = k
        print("case long top-k", cfg, V, k, flush=True)
        _check(P, oracle, w, P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, 3, 2.0, w.nu))


def test_accepted_length_matches_its_prediction_at_full_size(P):
    """Eq. token_exp on one drafted path per sequence: given the draft tokens, tau has expectation
    sum_i prod_{j<=i} f_j over the acceptance uniforms; over the 256 sequences of configuration 4
    the realised mean must agree within sampling error.  With the lossless setting (uniform
    schedule, delta = 1) every beta_i is exactly zero, with a relaxed one some are positive."""
    w = make_workload(4, device="cuda")
    params = P.make_params(w.target, w.draft)
    ws = torch.empty(P.cool_sd_workspace_bytes(params), dtype=torch.uint8, device="cuda")
    tau = torch.empty(w.B, dtype=torch.int32, device="cuda")
    nxt = torch.empty_like(tau)
    f = torch.empty((w.B, w.L), device="cuda")
    alpha, beta = torch.empty_like(f), torch.empty_like(f)
    for kind, delta in ((P.COOL_SD_SCHED_UNIFORM, 1.0), (P.COOL_SD_SCHED_EXP, 2.0)):
        om = torch.from_numpy(P.cool_sd_schedule(kind, w.L, delta, w.nu)).cuda()
        P.cool_sd_verify(params, w.target, None, w.draft, None, w.draft_tokens, om, w.u_accept, w.u_resample, tau, nxt,
                         None, None, f, None, ws)
        P.cool_sd_diagnostics(params, w.target, None, w.draft, None, om, alpha, beta, ws)
        torch.cuda.synchronize()
        pred = torch.cumprod(f.double(), 1).sum(1)
        diff = (tau.double() - pred).cpu().numpy()
        se = diff.std(ddof=1) / np.sqrt(w.B)
        print("delta", delta, "mean tau", float(tau.double().mean()), "predicted", float(pred.mean()), "se", se, flush=True)
        assert abs(diff.mean()) < 5 * se + 1e-9
        if kind == P.COOL_SD_SCHED_UNIFORM:
            assert float(beta.abs().max()) == 0.0
        else:
            assert float(beta.max()) > 0.0 and float(beta.min()) >= 0.0
        assert float(alpha.min()) > 0.0 and float(alpha.max()) <= 1.0 + 1e-6


# (cfg recipe, B, L, V, dtype, top_k): one-chunk rows take the single-pass form; top-k and long rows
# run the two calls one after the other
FUSED = [(2, 6, 8, 16384, "bf16", 0), (1, 2, 4, 16384, "f32", 0), (2, 3, 5, 4104, "bf16", 0), (2, 3, 3, 5001, "bf16", 0),
         (1, 2, 2, 8, "f32", 0), (3, 3, 4, 16384, "bf16", 0), (4, 5, 16, 16384, "bf16", 0), (2, 2, 70, 512, "bf16", 0),
         (3, 3, 4, 16384, "bf16", 800), (5, 2, 3, 40000, "bf16", 0)]


@pytest.mark.parametrize("cfg,B,L,V,dtype,top_k", FUSED)
def test_verify_and_diagnostics_in_one_call(P, oracle, cfg, B, L, V, dtype, top_k):
    from tests.parity_util import compare_verify
    print("case", cfg, B, L, V, dtype, top_k, flush=True)
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, dtype=dtype, top_k=top_k if cfg == 3 else None)
    if cfg == 3 and top_k == 0:
        w.temperature = 0.8
    for mode, delta in ((0, 2.0), (1, 0.7)):
        om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, L, delta, w.nu)
        gpu, alpha, beta = _verify_diag(P, w, om, mode)
        compare_verify(oracle, w, om, gpu, resample_mode=mode)
        a_ref, b_ref = _oracle_diag(oracle, w, om)
        np.testing.assert_allclose(alpha, a_ref, rtol=1e-5, atol=1e-9)
        np.testing.assert_allclose(beta, b_ref, rtol=1e-5, atol=2e-6)
        assert (beta[np.broadcast_to(om, beta.shape) <= 1.0] == 0.0).all()


def test_verify_and_diagnostics_without_bonus_and_with_per_sequence_omega(P, oracle):
    from tests.parity_util import compare_verify
    w = make_workload(2, device="cuda", B=5, L=6, V=16384)
    w.target = w.target[:, :6]                                    # no bonus row (a strided view)
    om = np.tile(P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, 6, 3.0, w.nu), (5, 1)).astype(np.float32)
    om[1] = 0.0
    om[3] *= 20.0
    gpu, alpha, beta = _verify_diag(P, w, om)
    compare_verify(oracle, w, om, gpu, has_bonus=False)
    a_ref, b_ref = _oracle_diag(oracle, w, om)
    np.testing.assert_allclose(alpha, a_ref, rtol=1e-5, atol=1e-9)
    np.testing.assert_allclose(beta, b_ref, rtol=1e-5, atol=2e-6)
    assert (gpu["accept_len"][1] == 0) and (alpha[1] == 0).all()
