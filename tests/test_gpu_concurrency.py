"""The library keeps no state between or across calls: host threads that call it at the same time on
streams, workspaces and outputs of their own get the results of the same calls made one after the
other, bit for bit."""
import threading

import pytest
import torch

from workloads import make_workload

pytestmark = pytest.mark.gpu

# (cfg recipe, B, L, V, top-k, flags by name): one-chunk rows, long rows through the one-launch tail
# (tickets in the workspace), long rows in rounds, guided top-k rows
JOBS = [
    (2, 8, 8, 16384, 0, ()),
    (5, 3, 4, 65536, 0, ()),
    (5, 3, 6, 40000, 0, ("COOL_SD_FLAG_EARLY_EXIT",)),
    (3, 4, 4, 16384, 300, ()),
    (4, 6, 16, 16384, 0, ("COOL_SD_FLAG_EARLY_EXIT",)),
    (1, 2, 3, 20000, 0, ("COOL_SD_FLAG_EXACT_DRAW",)),
]


def _prepare(P, job):
    cfg, B, L, V, top_k, flag_names = job
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, top_k=top_k if cfg == 3 else None)
    flags = 0
    for n in flag_names:
        flags |= getattr(P, n)
    params = P.make_params(w.target, w.draft, top_k=w.top_k, cfg_scale=w.cfg_scale, temperature=w.temperature, flags=flags)
    ws = torch.empty(max(P.cool_sd_workspace_bytes(params), 256), dtype=torch.uint8, device="cuda")
    P.cool_sd_workspace_init(ws)
    om = torch.from_numpy(P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, L, w.delta, w.nu)).cuda()
    out = dict(a=torch.full((B,), -5, dtype=torch.int32, device="cuda"), n=torch.full((B,), -5, dtype=torch.int32, device="cuda"),
               r=torch.zeros(B, device="cuda"), f=torch.zeros((B, L), device="cuda"))
    return dict(w=w, params=params, ws=ws, om=om, out=out, stream=torch.cuda.Stream())


def _call(P, j):
    w, o = j["w"], j["out"]
    P.cool_sd_verify(j["params"], w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, j["om"], w.u_accept,
                     w.u_resample, o["a"], o["n"], None, None, o["f"], o["r"], j["ws"], stream=j["stream"].cuda_stream)


def test_host_threads_on_their_own_streams(P):
    jobs = [_prepare(P, job) for job in JOBS]
    torch.cuda.synchronize()
    # reference: one call after the other
    for j in jobs:
        _call(P, j)
    torch.cuda.synchronize()
    ref = [{k: v.clone() for k, v in j["out"].items()} for j in jobs]
    errors = []

    def worker(j, reps):
        try:
            for _ in range(reps):
                _call(P, j)
        except BaseException as e:          # a failed call must fail the test, not only its thread
            errors.append(e)

    for round_ in range(3):
        for j in jobs:
            for v in j["out"].values():
                v.fill_(-9)
        torch.cuda.synchronize()
        threads = [threading.Thread(target=worker, args=(j, 20)) for j in jobs]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        torch.cuda.synchronize()
        assert not errors, errors
        for j, r in zip(jobs, ref):
            for k in r:
                assert torch.equal(j["out"][k], r[k]) or (k == "f" and torch.equal(torch.nan_to_num(j["out"][k], nan=-1.0),
                                                                                   torch.nan_to_num(r[k], nan=-1.0))), (round_, k)
