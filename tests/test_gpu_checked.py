"""Checked mode of the verify calls: draft tokens outside [0, V) are a contract violation that the
release library answers with the results of the clamped token; with COOL_SD_FLAG_CHECK_TOKENS, and
always in the debug build libcool_sd_checked.so, such sequences get accept_len = next_token = -1.
Every kernel runs to its end either way."""
import numpy as np
import pytest
import torch

from tests.parity_util import compare_verify, subset, to_numpy
from workloads import make_neighbor_table, make_workload

pytestmark = pytest.mark.gpu


def _poison(w):
    V = w.V
    w.draft_tokens[1, min(3, w.L - 1)] = V                    # one past the end
    w.draft_tokens[4, 0] = -5
    w.draft_tokens[5, w.L - 1] = 2 ** 31 - 1
    return [1, 4, 5], [0, 2, 3]


@pytest.mark.parametrize("cfg,kw,flags", [
    (2, dict(B=6, L=8, V=16384), 0),                          # rows of one chunk
    (5, dict(B=6, L=4, V=40000), 0),                          # long rows: accept / masses / select
    (3, dict(B=6, L=4, V=16384), 0),                          # guidance + top-k
    (2, dict(B=6, L=8, V=16384), 1),                          # early exit
])
def test_out_of_range_tokens(P, oracle, cfg, kw, flags, monkeypatch):
    w = make_workload(cfg, device="cuda", **kw)
    om_np = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, w.L, w.delta, w.nu)
    om = torch.from_numpy(om_np).cuda()
    bad, good = _poison(w)
    # release behaviour: the clamped token, every output in range
    rel = to_numpy(P.verify_workload(w, om, flags=flags))
    torch.cuda.synchronize()
    assert (rel["accept_len"] >= 0).all() and (rel["accept_len"] <= w.L).all()
    assert (rel["next_token"] >= 0).all() and (rel["next_token"] < w.V).all()
    wc = make_workload(cfg, device="cuda", **kw)
    wc.draft_tokens = w.draft_tokens.clamp(0, w.V - 1)
    compare_verify(oracle, wc, om_np, rel, early_exit=bool(flags))

    def check(out):
        for b in bad:
            assert out["accept_len"][b] == -1 and out["next_token"][b] == -1 and out["resid_mass"][b] == 0.0
        sub = {k: v[good] for k, v in out.items()}
        compare_verify(oracle, subset(w, good), om_np, sub, early_exit=bool(flags))

    # the option bit
    check(to_numpy(P.verify_workload(w, om, flags=flags | P.COOL_SD_FLAG_CHECK_TOKENS)))
    # the debug build: the same without the bit
    monkeypatch.setattr(P.binding, "_lib", P.binding.load(P.binding.LIB_CHECKED_PATH))
    check(to_numpy(P.verify_workload(w, om, flags=flags)))


def test_checked_mode_in_the_other_verify_calls(P, oracle):
    w = make_workload(2, device="cuda", B=6, L=8, V=16384)
    om = torch.from_numpy(P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, w.L, w.delta, w.nu)).cuda()
    bad, good = _poison(w)
    params = P.make_params(w.target, w.draft, flags=P.COOL_SD_FLAG_CHECK_TOKENS)
    ws = torch.empty(P.cool_sd_workspace_bytes(params), dtype=torch.uint8, device="cuda")
    al = torch.full((6,), -7, dtype=torch.int32, device="cuda")
    nt = torch.full((6,), -7, dtype=torch.int32, device="cuda")
    alpha = torch.empty((6, 8), device="cuda")
    beta = torch.empty((6, 8), device="cuda")
    P.cool_sd_verify_diagnostics(params, w.target, None, w.draft, None, w.draft_tokens, om, w.u_accept, w.u_resample,
                                 al, nt, None, None, None, None, alpha, beta, ws)
    torch.cuda.synchronize()
    assert (al[bad] == -1).all() and (nt[bad] == -1).all() and (al[good] >= 0).all()
    nbr = make_neighbor_table(w.V, 10, device="cuda", seed=11)
    al.fill_(-7)
    nt.fill_(-7)
    P.cool_sd_verify_lantern(params, w.target, None, w.draft, None, w.draft_tokens, nbr, 10, 2.0, w.u_accept,
                             w.u_resample, al, nt, None, None, None, None, None, None, ws)
    torch.cuda.synchronize()
    assert (al[bad] == -1).all() and (nt[bad] == -1).all() and (al[good] >= 0).all() and (nt[good] >= 0).all()
    assert np.isfinite(alpha.cpu().numpy()).all()
