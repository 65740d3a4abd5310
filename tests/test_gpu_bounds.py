"""No entry point writes outside the buffers it was given: outputs and the workspace are carved
out of larger allocations whose surroundings hold a sentinel, the workspace has exactly the size
cool_sd_workspace_bytes reports, and the sentinels must survive every call."""
import numpy as np
import pytest
import torch

from workloads import make_neighbor_table, make_workload

pytestmark = pytest.mark.gpu

GUARD = 4096            # bytes of sentinel on each side
SENT = 0xA5


class Guarded:
    """A device buffer of `nbytes` (256-byte aligned start) between two sentinel regions."""

    def __init__(self, nbytes, dtype=torch.uint8, shape=None):
        self.nbytes = int(nbytes)
        pad = (-self.nbytes) % 256
        self.raw = torch.full((GUARD + self.nbytes + pad + GUARD,), SENT, dtype=torch.uint8, device="cuda")
        assert self.raw.data_ptr() % 256 == 0
        body = self.raw[GUARD:GUARD + self.nbytes]
        self.t = body.view(dtype) if shape is None else body.view(dtype).view(shape)

    def intact(self):
        head = self.raw[:GUARD]
        tail = self.raw[GUARD + self.nbytes:]
        return bool((head == SENT).all().item()) and bool((tail == SENT).all().item())


def _outputs(B, L):
    return dict(accept_len=Guarded(B * 4, torch.int32), next_token=Guarded(B * 4, torch.int32),
                p_tok=Guarded(B * L * 4, torch.float32, (B, L)), q_tok=Guarded(B * L * 4, torch.float32, (B, L)),
                f=Guarded(B * L * 4, torch.float32, (B, L)), resid_mass=Guarded(B * 4, torch.float32))


# (cfg recipe, B, L, V, dtype, top_k): one-chunk rows, partial tiles, element-wise loads, long rows,
# both top-k paths
CASES = [
    (2, 5, 8, 16384, "bf16", 0),
    (1, 3, 4, 16384, "f32", 0),
    (2, 3, 5, 4104, "bf16", 0),
    (2, 3, 3, 5001, "bf16", 0),
    (1, 2, 2, 8, "f32", 0),
    (3, 3, 4, 16384, "bf16", 1000),
    (5, 3, 3, 40000, "bf16", 0),
    (5, 2, 2, 262144, "bf16", 0),
    (3, 2, 3, 40000, "bf16", 500),
    (5, 3, 3, 32768, "bf16", 0),          # several chunks, per-sequence step in one workgroup
    (1, 2, 3, 20004, "f32", 0),
    (3, 2, 3, 24584, "bf16", 300),        # top-k with 32 logits per thread of 1024
    (5, 2, 60, 32776, "bf16", 0),         # long window on long rows: tau found by the chunk-mass launch
    (4, 7, 70, 1024, "bf16", 0),          # more positions than one wave
]


@pytest.mark.parametrize("cfg,B,L,V,dtype,top_k", CASES)
def test_entry_points_stay_inside_their_buffers(P, cfg, B, L, V, dtype, top_k):
    print("case", cfg, B, L, V, dtype, top_k, flush=True)
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, dtype=dtype, top_k=top_k if cfg == 3 else None)
    w.top_k = top_k
    om = torch.from_numpy(P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, L, 1.1, 0.7)).cuda()
    params = P.make_params(w.target, w.draft, top_k=top_k, cfg_scale=w.cfg_scale, temperature=w.temperature)
    ws = Guarded(P.cool_sd_workspace_bytes(params))
    o = _outputs(B, L)
    everything = [ws] + list(o.values())

    for flags in (0, P.COOL_SD_FLAG_EARLY_EXIT):
        params.flags = flags
        P.cool_sd_verify(params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, om, w.u_accept,
                         w.u_resample, o["accept_len"].t, o["next_token"].t, o["p_tok"].t, o["q_tok"].t, o["f"].t,
                         o["resid_mass"].t, ws.t)
        torch.cuda.synchronize()
        assert all(g.intact() for g in everything), "cool_sd_verify flags=%d" % flags
    params.flags = 0

    alpha, beta = Guarded(B * L * 4, torch.float32, (B, L)), Guarded(B * L * 4, torch.float32, (B, L))
    P.cool_sd_diagnostics(params, w.target, w.target_uncond, w.draft, w.draft_uncond, om, alpha.t, beta.t, ws.t)
    torch.cuda.synchronize()
    assert all(g.intact() for g in everything + [alpha, beta]), "cool_sd_diagnostics"

    P.cool_sd_verify_diagnostics(params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, om,
                                 w.u_accept, w.u_resample, o["accept_len"].t, o["next_token"].t, o["p_tok"].t,
                                 o["q_tok"].t, o["f"].t, o["resid_mass"].t, alpha.t, beta.t, ws.t)
    torch.cuda.synchronize()
    assert all(g.intact() for g in everything + [alpha, beta]), "cool_sd_verify_diagnostics"

    k = min(10, V - 1)
    if k >= 1:
        nbr = make_neighbor_table(V, k, device="cuda", seed=3, pad=0.1)
        p_agg, count = Guarded(B * L * 4, torch.float32, (B, L)), Guarded(B * L * 4, torch.int32, (B, L))
        for mode in (P.COOL_SD_RESAMPLE_OPT, P.COOL_SD_RESAMPLE_LANTERN):
            params.resample_mode = mode
            P.cool_sd_verify_lantern(params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, nbr, k,
                                     0.5, w.u_accept, w.u_resample, o["accept_len"].t, o["next_token"].t, o["p_tok"].t,
                                     o["q_tok"].t, o["f"].t, o["resid_mass"].t, p_agg.t, count.t, ws.t)
            torch.cuda.synchronize()
            assert all(g.intact() for g in everything + [p_agg, count]), "cool_sd_verify_lantern mode=%d" % mode
        params.resample_mode = P.COOL_SD_RESAMPLE_OPT

    # stand-alone resample on the first position's rows
    tok, mass = Guarded(B * 4, torch.int32), Guarded(B * 4, torch.float32)
    rp = P.make_params(w.target[:, :1], w.draft[:, :1], has_bonus=0, top_k=top_k, cfg_scale=w.cfg_scale,
                       temperature=w.temperature)
    rws = Guarded(P.cool_sd_workspace_bytes(rp))
    om_rows = torch.full((B,), 1.3, device="cuda")
    P.cool_sd_resample(rp, w.target[:, 0], None if w.target_uncond is None else w.target_uncond[:, 0], w.draft[:, 0],
                       None if w.draft_uncond is None else w.draft_uncond[:, 0], om_rows, w.u_resample, tok.t, mass.t,
                       rws.t)
    torch.cuda.synchronize()
    assert all(g.intact() for g in (tok, mass, rws)), "cool_sd_resample"
    assert int(tok.t.min()) >= 0 and int(tok.t.max()) < V
    # the drafting stage's draw: no draft rows
    P.cool_sd_resample(rp, w.draft[:, 0], None if w.draft_uncond is None else w.draft_uncond[:, 0], None, None, None,
                       w.u_resample, tok.t, mass.t, rws.t)
    torch.cuda.synchronize()
    assert all(g.intact() for g in (tok, mass, rws)), "cool_sd_resample without a draft"
    assert int(tok.t.min()) >= 0 and int(tok.t.max()) < V
