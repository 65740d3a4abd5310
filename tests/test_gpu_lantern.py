"""Parity of cool_sd_verify_lantern (aggregated acceptance over latent neighbours, Eq. f_lantern,
with G*, vanilla or Eq. g_lantern resampling) against the CPU oracle on seeded inputs.

The neighbour table is synthetic (workloads.make_neighbor_table): the real one is derived from
a trained codebook that is not available here."""
import numpy as np
import pytest
import torch

from tests.parity_util import compare_verify, compare_verify_lantern, to_numpy
from workloads import make_neighbor_table, make_workload

pytestmark = pytest.mark.gpu


def _run(P, w, nbr, lam, mode):
    out = P.verify_lantern_workload(w, nbr, lam, resample_mode=mode)
    torch.cuda.synchronize()
    return to_numpy(out)


# (cfg recipe, B, L, V, dtype, k, lambda)
CASES = [
    (2, 8, 8, 16384, "bf16", 10, 2.0),      # the comparison system's setting (lambda = 2, k = 10)
    (2, 6, 8, 16384, "bf16", 10, 0.02),     # small lambda: most sets end inside the list
    (1, 3, 4, 16384, "f32", 100, 0.5),      # two strips of neighbours per position
    (4, 6, 16, 16384, "bf16", 64, 0.1),
    (2, 4, 5, 4104, "bf16", 7, 1.0),        # partial last tile
    (1, 3, 3, 1003, "f32", 5, 0.3),         # element-wise loads
    (1, 2, 2, 8, "f32", 3, 2.0),            # tiny vocabulary
    (3, 4, 4, 16384, "bf16", 10, 0.5),      # guidance + top-k: neighbours outside the kept set weigh nothing
    (5, 2, 3, 40000, "bf16", 10, 0.2),      # rows of several chunks
    (5, 2, 2, 70001, "bf16", 40, 0.05),     # long rows, element-wise loads, sets that end inside the list
]


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("cfg,B,L,V,dtype,k,lam", CASES)
def test_lantern_against_oracle(P, oracle, cfg, B, L, V, dtype, k, lam, mode):
    print("case", cfg, B, L, V, dtype, k, lam, mode, flush=True)
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, dtype=dtype)
    nbr = make_neighbor_table(V, k, device="cuda", seed=11 + k, pad=0.1, self_entries=k > 3)
    gpu = _run(P, w, nbr, lam, mode)
    st = compare_verify_lantern(oracle, w, nbr.cpu().numpy(), lam, gpu, resample_mode=mode)
    print(st, flush=True)
    assert st["set_exempt"] <= 1


def test_more_sequences_than_a_grid_dimension(P, oracle):
    """B beyond 65535: the statistics launch (with the aggregation's workgroups appended) falls
    back to a one-dimensional grid."""
    w = make_workload(1, device="cuda", B=70000, L=1, V=8, dtype="f32")
    nbr = make_neighbor_table(8, 3, device="cuda", seed=2)
    gpu = _run(P, w, nbr, 2.0, 0)
    st = compare_verify_lantern(oracle, w, nbr.cpu().numpy(), 2.0, gpu)
    print(st, flush=True)
    assert st["tau_exempt"] + st["token_exempt"] + st["set_exempt"] <= 8


def test_sets_are_partial_and_full(P, oracle):
    """The cases above must exercise all three outcomes: empty sets, sets that end inside the
    list and sets that take the whole list."""
    w = make_workload(2, device="cuda", B=16, L=8, V=16384)
    nbr = make_neighbor_table(16384, 10, device="cuda", seed=3)
    seen = set()
    for lam in (0.001, 0.05, 2.0):
        gpu = _run(P, w, nbr, lam, 0)
        compare_verify_lantern(oracle, w, nbr.cpu().numpy(), lam, gpu)
        c = gpu["count"]
        seen |= {"empty"} if (c == 0).any() else set()
        seen |= {"partial"} if ((c > 0) & (c < 10)).any() else set()
        seen |= {"full"} if (c == 10).any() else set()
    assert seen == {"empty", "partial", "full"}


def test_lambda_zero_equals_vanilla_call(P, oracle):
    """Without neighbours Eq. f_lantern is Eq. f_tsd: the call must return what cool_sd_verify
    returns at omega = 1 with vanilla resampling, bit for bit."""
    w = make_workload(2, device="cuda", B=12, L=8, V=16384)
    nbr = make_neighbor_table(16384, 10, device="cuda", seed=5)
    ones = torch.ones(w.L, dtype=torch.float32, device="cuda")
    ref = to_numpy(P.verify_workload(w, ones, resample_mode=P.COOL_SD_RESAMPLE_VANILLA))
    for mode in (0, 1, 2):
        gpu = _run(P, w, nbr, 0.0, mode)
        for key in ("accept_len", "next_token", "p_tok", "q_tok", "f", "resid_mass"):
            np.testing.assert_array_equal(gpu[key], ref[key], err_msg=key)
        np.testing.assert_array_equal(gpu["count"], 0)
        np.testing.assert_array_equal(gpu["p_agg"], ref["p_tok"])
    compare_verify(oracle, w, np.ones(w.L, np.float32), ref, resample_mode=1)


def test_acceptance_rises_with_lambda(P):
    """More aggregated mass can only raise f (Eq. f_lantern), hence the accepted length for the
    same uniforms."""
    w = make_workload(4, device="cuda", B=64, L=16, V=16384)
    nbr = make_neighbor_table(16384, 50, device="cuda", seed=9)
    prev_f, prev_tau = None, None
    for lam in (0.0, 0.1, 1.0, 10.0):
        gpu = _run(P, w, nbr, lam, 0)
        if prev_f is not None:
            assert (gpu["f"] >= prev_f).all() and (gpu["accept_len"] >= prev_tau).all()
        prev_f, prev_tau = gpu["f"], gpu["accept_len"]
    assert prev_tau.sum() > 0


@pytest.mark.parametrize("cfg,n_check,mode", [(2, None, 0), (2, None, 2), (4, None, 0), (4, None, 2), (5, None, 0), (5, None, 2)])
def test_full_size_configurations(P, oracle, cfg, n_check, mode):
    """Benchmark-size batches with the comparison system's setting (k = 10, lambda = 2); every
    sequence, or a seeded sample of them, against the oracle."""
    from tests.parity_util import subset
    print("full lantern cfg", cfg, mode, flush=True)
    w = make_workload(cfg, device="cuda")
    nbr = make_neighbor_table(w.V, 10, device="cuda", seed=11)
    gpu = _run(P, w, nbr, 2.0, mode)
    assert gpu["accept_len"].min() >= 0 and gpu["accept_len"].max() <= w.L
    assert gpu["next_token"].min() >= 0 and gpu["next_token"].max() < w.V
    if n_check is None:
        st = compare_verify_lantern(oracle, w, nbr.cpu().numpy(), 2.0, gpu, resample_mode=mode)
    else:
        idx = np.sort(np.random.default_rng(cfg).choice(w.B, n_check, replace=False))
        st = compare_verify_lantern(oracle, subset(w, idx), nbr.cpu().numpy(), 2.0,
                                    {k: v[idx] for k, v in gpu.items()}, resample_mode=mode)
    print("exemptions", st, flush=True)
    assert st["tau_exempt"] + st["token_exempt"] + st["set_exempt"] <= 2


def test_repeat_calls_and_graph_replays_are_identical(P):
    """Same inputs, shared workspace: every eager call and every replay of a captured call returns
    the same bits (no kernel depends on the order in which workgroups run)."""
    w = make_workload(2, device="cuda", B=16, L=8, V=16384)
    nbr = make_neighbor_table(16384, 10, device="cuda", seed=5)
    params = P.make_params(w.target, w.draft, resample_mode=P.COOL_SD_RESAMPLE_LANTERN)
    ws = torch.empty(P.cool_sd_workspace_bytes(params), dtype=torch.uint8, device="cuda")
    a = torch.zeros(w.B, dtype=torch.int32, device="cuda")
    n = torch.zeros_like(a)
    f = torch.zeros((w.B, w.L), device="cuda")
    r = torch.zeros(w.B, device="cuda")

    def call():
        P.cool_sd_verify_lantern(params, w.target, None, w.draft, None, w.draft_tokens, nbr, 10, 0.3, w.u_accept,
                                 w.u_resample, a, n, None, None, f, r, None, None, ws)
    call()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (a, n, f, r)]
    for _ in range(3):
        for t in (a, n, f, r):
            t.zero_()
        call()
        torch.cuda.synchronize()
        for t, e in zip((a, n, f, r), ref):
            assert torch.equal(t, e)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        call()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for _ in range(3):
        for t in (a, n, f, r):
            t.zero_()                      # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for t, e in zip((a, n, f, r), ref):
            assert torch.equal(t, e)
