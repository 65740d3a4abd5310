"""cool_sd_verify_noalloc (the entry point for callers that cannot allocate: its workspace is a
static device array of the library) against cool_sd_verify on the same inputs: same kernels, so
every output must be identical bit for bit.  Two calls in a row share the array, the second on a
smaller input; then shapes beyond the array are refused."""
import numpy as np
import pytest
import torch

from tests.parity_util import compare_verify, to_numpy
from workloads import make_workload

pytestmark = pytest.mark.gpu


def _outputs(B, L):
    return dict(accept_len=torch.full((B,), -7, dtype=torch.int32, device="cuda"),
                next_token=torch.full((B,), -7, dtype=torch.int32, device="cuda"),
                resid_mass=torch.full((B,), float("nan"), device="cuda"),
                p_tok=torch.full((B, L), float("nan"), device="cuda"),
                q_tok=torch.full((B, L), float("nan"), device="cuda"),
                f=torch.full((B, L), float("nan"), device="cuda"))


def _both(P, w, om):
    params = P.make_params(w.target, w.draft, top_k=w.top_k, cfg_scale=w.cfg_scale, temperature=w.temperature)
    a, b = _outputs(w.B, w.L), _outputs(w.B, w.L)
    P.cool_sd_verify_noalloc(params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, om,
                             w.u_accept, w.u_resample, a["accept_len"], a["next_token"], a["p_tok"], a["q_tok"],
                             a["f"], a["resid_mass"])
    ws = torch.empty(max(P.cool_sd_workspace_bytes(params), 256), dtype=torch.uint8, device="cuda")
    P.cool_sd_verify(params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, om, w.u_accept,
                     w.u_resample, b["accept_len"], b["next_token"], b["p_tok"], b["q_tok"], b["f"], b["resid_mass"],
                     ws)
    torch.cuda.synchronize()
    return to_numpy(a), to_numpy(b)


@pytest.mark.parametrize("first,second", [
    ((2, dict(B=32, L=8, V=16384)), (2, dict(B=5, L=3, V=5001))),          # rows of one chunk, then element-wise loads
    ((5, dict(B=6, L=4, V=262144)), (5, dict(B=2, L=3, V=40000))),         # long rows: statistics, accept, masses, select
    ((3, dict(B=8, L=4, V=16384)), (1, dict(B=1, L=4, V=16384))),          # guidance + top-k, then fp32
])
def test_two_calls_in_a_row_match_the_workspace_entry_point(P, oracle, first, second):
    for cfg, kw in (first, second):
        print("case", cfg, kw, flush=True)
        w = make_workload(cfg, device="cuda", **kw)
        om_np = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, w.L, w.delta, w.nu)
        got, ref = _both(P, w, torch.from_numpy(om_np).cuda())
        for k in ref:
            np.testing.assert_array_equal(got[k], ref[k], err_msg=k)
        compare_verify(oracle, w, om_np, got)


def test_shapes_beyond_the_static_workspace_are_refused(P):
    w = make_workload(2, device="cuda", B=2, L=2, V=1024)
    om = torch.ones(64, device="cuda")
    o = _outputs(2, 2)
    # claim a shape whose workspace exceeds the array: refused from the params alone, nothing is launched
    params = P.make_params(w.target, w.draft)
    params.B, params.L, params.V = 4096, 64, 262144
    assert P.cool_sd_workspace_bytes(params) > P.binding.COOL_SD_NOALLOC_WORKSPACE_BYTES
    rc = P.cool_sd_verify_noalloc(params, w.target, None, w.draft, None, w.draft_tokens, om, w.u_accept, w.u_resample,
                                  o["accept_len"], o["next_token"], None, None, None, None, check=False)
    assert rc == P.binding.COOL_SD_ETOOLARGE
    torch.cuda.synchronize()
    assert (o["accept_len"] == -7).all()
    with pytest.raises(P.CoolSDError, match="static array"):
        P.cool_sd_verify_noalloc(params, w.target, None, w.draft, None, w.draft_tokens, om, w.u_accept, w.u_resample,
                                 o["accept_len"], o["next_token"], None, None, None, None)
