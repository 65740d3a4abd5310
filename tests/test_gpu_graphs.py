"""Every entry point can be captured into a HIP graph: replays, with eager work and
synchronisations in between, reproduce the eager call bit for bit (no entry point records a
memset node or depends on state left by an earlier call)."""
import pytest
import torch

from workloads import make_neighbor_table, make_workload

pytestmark = pytest.mark.gpu


def _replay_equals_eager(call, outs):
    call()
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        call()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for rep in range(3):
        for o in outs:
            o.fill_(-5)
        junk = torch.randn(1 << 18, device="cuda").sum()              # unrelated eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert junk.item() == junk.item()
        for o, e in zip(outs, eager):
            assert torch.equal(o, e) or (torch.isnan(o) == torch.isnan(e)).all() and torch.equal(
                torch.nan_to_num(o), torch.nan_to_num(e)), rep


# (cfg recipe, B, L, V, top_k): one-chunk rows, guided top-k rows, long rows, long rows with radix top-k
CASES = [(2, 8, 8, 16384, 0), (3, 4, 4, 16384, 500), (5, 3, 3, 40000, 0), (3, 2, 2, 70000, 300)]


@pytest.mark.parametrize("cfg,B,L,V,top_k", CASES)
def test_entry_points_replay(P, cfg, B, L, V, top_k):
    print("case", cfg, B, L, V, top_k, flush=True)
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, top_k=top_k if cfg == 3 else None)
    om = torch.from_numpy(P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, L, 1.5, 0.7)).cuda()
    params = P.make_params(w.target, w.draft, top_k=w.top_k, cfg_scale=w.cfg_scale, temperature=w.temperature)
    ws = torch.empty(P.cool_sd_workspace_bytes(params), dtype=torch.uint8, device="cuda")
    P.cool_sd_workspace_init(ws)
    tau = torch.zeros(B, dtype=torch.int32, device="cuda")
    nxt = torch.zeros_like(tau)
    f = torch.zeros((B, L), device="cuda")
    R = torch.zeros(B, device="cuda")

    def verify():
        P.cool_sd_verify(params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, om, w.u_accept,
                         w.u_resample, tau, nxt, None, None, f, R, ws)
    _replay_equals_eager(verify, [tau, nxt, f, R])

    params.flags = P.COOL_SD_FLAG_EARLY_EXIT
    _replay_equals_eager(verify, [tau, nxt, f, R])
    params.flags = 0

    alpha, beta = torch.zeros((B, L), device="cuda"), torch.zeros((B, L), device="cuda")
    _replay_equals_eager(lambda: P.cool_sd_diagnostics(params, w.target, w.target_uncond, w.draft, w.draft_uncond, om,
                                                       alpha, beta, ws), [alpha, beta])

    _replay_equals_eager(lambda: P.cool_sd_verify_diagnostics(params, w.target, w.target_uncond, w.draft, w.draft_uncond,
                                                              w.draft_tokens, om, w.u_accept, w.u_resample, tau, nxt,
                                                              None, None, f, R, alpha, beta, ws),
                         [tau, nxt, f, R, alpha, beta])

    nbr = make_neighbor_table(V, 10, device="cuda", seed=3)
    agg, cnt = torch.zeros((B, L), device="cuda"), torch.zeros((B, L), dtype=torch.int32, device="cuda")
    for mode in (P.COOL_SD_RESAMPLE_OPT, P.COOL_SD_RESAMPLE_LANTERN):
        params.resample_mode = mode
        _replay_equals_eager(lambda: P.cool_sd_verify_lantern(params, w.target, w.target_uncond, w.draft, w.draft_uncond,
                                                              w.draft_tokens, nbr, 10, 0.5, w.u_accept, w.u_resample,
                                                              tau, nxt, None, None, f, R, agg, cnt, ws),
                             [tau, nxt, f, R, agg, cnt])
    params.resample_mode = P.COOL_SD_RESAMPLE_OPT

    # stand-alone resampling: with a draft row, and the drafting stage's draw without one
    rp = P.make_params(w.target[:, :1], w.draft[:, :1], has_bonus=0, top_k=w.top_k, cfg_scale=w.cfg_scale,
                       temperature=w.temperature)
    rws = torch.empty(P.cool_sd_workspace_bytes(rp), dtype=torch.uint8, device="cuda")
    P.cool_sd_workspace_init(rws)
    tok, mass = torch.zeros(B, dtype=torch.int32, device="cuda"), torch.zeros(B, device="cuda")
    om_rows = torch.full((B,), 1.3, device="cuda")
    tu0 = None if w.target_uncond is None else w.target_uncond[:, 0]
    du0 = None if w.draft_uncond is None else w.draft_uncond[:, 0]
    _replay_equals_eager(lambda: P.cool_sd_resample(rp, w.target[:, 0], tu0, w.draft[:, 0], du0, om_rows, w.u_resample,
                                                    tok, mass, rws), [tok, mass])
    _replay_equals_eager(lambda: P.cool_sd_resample(rp, w.draft[:, 0], du0, None, None, None, w.u_resample, tok, mass,
                                                    rws), [tok, mass])
