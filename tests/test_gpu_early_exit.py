"""Parity of the early-exit form of cool_sd_verify (COOL_SD_FLAG_EARLY_EXIT) against the CPU
oracle, with the same tolerances as the all-rows form, and agreement of the two forms."""
import numpy as np
import pytest
import torch

from tests.parity_util import compare_verify, early_exit_form, run_oracle, to_numpy
from workloads import make_workload

pytestmark = pytest.mark.gpu


def _both(P, w, om, **kw):
    omega = torch.from_numpy(np.ascontiguousarray(om, dtype=np.float32)).cuda()
    early = to_numpy(P.verify_workload(w, omega, flags=P.COOL_SD_FLAG_EARLY_EXIT, **kw))
    full = to_numpy(P.verify_workload(w, omega, **kw))
    torch.cuda.synchronize()
    return early, full


SHAPES = [
    (1, 1, 4, 16384, "f32"),
    (2, 32, 8, 16384, "bf16"),      # config 2
    (2, 3, 5, 4104, "bf16"),        # partial last vector block
    (2, 3, 3, 5001, "bf16"),        # rows not 16-byte aligned: served by the all-rows path
    (1, 2, 3, 1003, "f32"),
    (1, 2, 2, 8, "f32"),
    (2, 2, 2, 1, "bf16"),
    (4, 40, 16, 16384, "bf16"),     # config 4 rows
    (2, 2, 1, 16384, "bf16"),       # L = 1
    (2, 2, 300, 512, "bf16"),       # long draft window
]


@pytest.mark.parametrize("cfg,B,L,V,dtype", SHAPES)
def test_early_exit_shapes(P, oracle, cfg, B, L, V, dtype):
    print("case", cfg, B, L, V, dtype, flush=True)
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, dtype=dtype)
    om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, L, w.delta, w.nu)
    early, full = _both(P, w, om)
    honoured = V % (8 if dtype == "bf16" else 4) == 0     # otherwise the rows are not 16-byte aligned
    assert early_exit_form(P, w) == (P.COOL_SD_EARLY_EXIT_SEQUENCE if honoured else P.COOL_SD_EARLY_EXIT_NONE)
    compare_verify(oracle, w, om, early, early_exit=honoured)
    # the two forms sum the softmax denominators in different orders, so they may differ where a
    # uniform sits on a threshold; everywhere else they agree
    same = early["accept_len"] == full["accept_len"]
    assert same.mean() >= 0.9
    assert (early["next_token"][same] == full["next_token"][same]).mean() >= 0.9


@pytest.mark.parametrize("mode", [0, 1])
def test_early_exit_modes_budgets_and_no_bonus(P, oracle, mode):
    w = make_workload(4, device="cuda", B=24, L=8, V=16384)
    for delta in (1.0, 4.0, 50.0):      # delta = 50: nearly everything is accepted, bonus draws
        om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, 8, delta, w.nu)
        early, _ = _both(P, w, om, resample_mode=mode)
        compare_verify(oracle, w, om, early, resample_mode=mode, early_exit=True)
    om = P.cool_sd_schedule(P.COOL_SD_SCHED_UNIFORM, 8, 50.0)
    w.target = w.target[:, :8].contiguous()
    early, _ = _both(P, w, om, resample_mode=mode)
    compare_verify(oracle, w, om, early, resample_mode=mode, has_bonus=False, early_exit=True)
    assert (early["next_token"][early["accept_len"] == 8] == -1).all() and (early["accept_len"] == 8).any()


def test_early_exit_per_sequence_omega_guidance_and_temperature(P, oracle):
    w = make_workload(2, device="cuda", B=9, L=6, V=16384)
    om = np.tile(P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, 6, 2.0, w.nu), (9, 1)).astype(np.float32)
    om[::3] = 0.0
    om[1::3] *= 3.0
    early, _ = _both(P, w, om)
    compare_verify(oracle, w, om, early, early_exit=True)
    assert (early["accept_len"][::3] == 0).all()
    w = make_workload(3, device="cuda", B=4, L=5, top_k=0)      # guided logits, no top-k
    w.temperature = 0.7
    om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, 5, 1.5, w.nu)
    early, _ = _both(P, w, om)
    compare_verify(oracle, w, om, early, early_exit=True)


def test_early_exit_falls_back_where_not_supported(P, oracle):
    """Under top-k the call reads every row, the query says so, and every position is filled."""
    for w in (make_workload(3, device="cuda", B=3, L=4), make_workload(3, device="cuda", B=2, L=3, V=40000, top_k=500)):
        assert early_exit_form(P, w) == P.COOL_SD_EARLY_EXIT_NONE
        om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, w.L, w.delta, w.nu)
        early, full = _both(P, w, om)
        compare_verify(oracle, w, om, early)
        for k in early:
            np.testing.assert_array_equal(early[k], full[k])


# ------------------------------------------------------------------ long rows: verification in rounds
LONG_SHAPES = [
    (5, 3, 8, 40000, "bf16"),       # rounds 1, 1, 2, 4 + bonus
    (5, 2, 5, 20001, "bf16"),       # rows not 16-byte aligned
    (5, 2, 1, 65536, "bf16"),       # L = 1: one round
    (1, 2, 3, 33000, "f32"),
    (5, 4, 2, 16392, "bf16"),       # just beyond one chunk
    (5, 2, 70, 16400, "bf16"),      # rounds up to 32 positions, the last one short
    (5, 1, 200, 17000, "bf16"),     # rounds capped at 63 positions
    (5, 2, 4, 262144, "bf16"),      # config 5 rows
    (5, 1, 2, 524288, "bf16"),      # the longest rows of this form (64 statistics chunks)
]


@pytest.mark.parametrize("cfg,B,L,V,dtype", LONG_SHAPES)
def test_rounds_shapes(P, oracle, cfg, B, L, V, dtype):
    print("case", cfg, B, L, V, dtype, flush=True)
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, dtype=dtype)
    assert early_exit_form(P, w) == P.COOL_SD_EARLY_EXIT_ROUNDS
    for delta in (w.delta, 30.0):           # delta = 30: most positions accepted, later rounds and bonus draws
        om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, L, delta, w.nu)
        ref = run_oracle(oracle, w, om, 0)
        early, full = _both(P, w, om)
        compare_verify(oracle, w, om, early, ref=ref, early_exit=True)
        compare_verify(oracle, w, om, full, ref=ref)
        # same statistics kernels, same accept formula, same draw: the two forms agree exactly
        np.testing.assert_array_equal(early["accept_len"], full["accept_len"])
        np.testing.assert_array_equal(early["next_token"], full["next_token"])


def test_rounds_reject_at_every_window_edge(P, oracle):
    """L = 130: rounds [0,1) [1,2) [2,4) [4,8) [8,16) [16,32) [32,64) [64,127) [127,131).  Sequence b accepts
    everything before position taus[b] (huge omega) and rejects there (omega = 0): first and last position
    of every round, and the fully accepted window with its bonus draw."""
    taus = [0, 1, 2, 3, 4, 7, 8, 15, 16, 31, 32, 63, 64, 126, 127, 129, 130]
    L, V = 130, 16400
    w = make_workload(5, device="cuda", B=len(taus), L=L, V=V)
    om = np.full((len(taus), L), 1e30, np.float32)
    for b, t in enumerate(taus):
        om[b, t:] = 0.0
    early, full = _both(P, w, om)
    np.testing.assert_array_equal(early["accept_len"], np.array(taus, np.int32))
    ref = run_oracle(oracle, w, om, 0)
    compare_verify(oracle, w, om, early, ref=ref, early_exit=True)
    compare_verify(oracle, w, om, full, ref=ref)
    np.testing.assert_array_equal(early["next_token"], full["next_token"])


def test_rounds_beyond_the_form_fall_back(P, oracle):
    w = make_workload(5, device="cuda", B=1, L=1, V=524296)
    assert early_exit_form(P, w) == P.COOL_SD_EARLY_EXIT_NONE
    om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, 1, w.delta, w.nu)
    early, full = _both(P, w, om)
    for k in early:
        np.testing.assert_array_equal(early[k], full[k])


@pytest.mark.parametrize("mode", [0, 1])
def test_rounds_modes_no_bonus_per_sequence_omega_and_transform(P, oracle, mode):
    w = make_workload(5, device="cuda", B=6, L=8, V=33000)
    om = np.tile(P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, 8, 3.0, w.nu), (6, 1)).astype(np.float32)
    om[0] = 0.0                              # rejected at once
    om[1] = 1e6                              # everything accepted: the bonus draw
    om[2, 3:] = 0.0                          # rejected at position 4, the first of a round
    om[3, 5:] = 0.0                          # rejected inside a round
    early, _ = _both(P, w, om, resample_mode=mode)
    compare_verify(oracle, w, om, early, resample_mode=mode, early_exit=True)
    assert early["accept_len"][0] == 0 and early["accept_len"][1] == 8
    assert early["accept_len"][2] <= 3 and early["accept_len"][3] <= 5
    w.target = w.target[:, :8].contiguous()
    early, _ = _both(P, w, om, resample_mode=mode)
    compare_verify(oracle, w, om, early, resample_mode=mode, has_bonus=False, early_exit=True)
    assert early["accept_len"][1] == 8 and early["next_token"][1] == -1
    g = make_workload(3, device="cuda", B=3, L=5, V=32768, top_k=0)      # guided logits, no top-k
    g.temperature = 0.7
    omg = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, 5, 2.0, g.nu)
    early, _ = _both(P, g, omg, resample_mode=mode)
    compare_verify(oracle, g, omg, early, resample_mode=mode, early_exit=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_early_exit_degenerate_rows(P, oracle, dtype):
    """Identical models, one-hot and flat rows, all-equal logits, large logits, a draft token the
    target excludes, u = 0 and u next to 1 -- through both early-exit kernels (1024 threads for
    fp32 rows, 256 threads for packed bf16 rows)."""
    B, L, V = 8, 4, 16384
    w = make_workload(1, device="cuda", B=B, L=L, V=V, dtype=dtype)
    t, d = w.target, w.draft
    d[0] = t[0, :L]
    t[1] = float("-inf"); t[1, :, 77] = 0.0
    d[1] = 0.0
    t[2] = 3.0; d[2] = -2.0
    t[3] = t[3] * 25.0
    d[3] = d[3] * 25.0
    t[4, :, :] = torch.where(torch.arange(V, device="cuda") % 2 == 0, t[4], torch.full_like(t[4], float("-inf")))
    w.draft_tokens[4] = torch.tensor([1, 3, 5, 2], dtype=torch.int32)
    w.u_accept[5] = 0.0
    w.u_resample[5] = 0.0
    w.u_accept[6] = 1.0 - 2.0 ** -24
    w.u_resample[6] = 1.0 - 2.0 ** -24
    w.draft_tokens[7] = V - 1
    for om in (np.ones(L, np.float32), np.array([2.0, 1.0, 0.5, 0.25], np.float32)):
        early, _ = _both(P, w, om)
        compare_verify(oracle, w, om, early, early_exit=True)
        assert early["accept_len"][0] == L or om[-1] < 1.0       # identical models: nothing rejected at omega >= 1
