"""Parity of the HIP library (through its C ABI) against the CPU oracle on seeded inputs."""
import numpy as np
import pytest
import torch

from tests.parity_util import compare_verify, run_oracle, to_numpy, token_band
from workloads import make_workload, uniforms24

pytestmark = pytest.mark.gpu


def _omega(P, w, L=None, delta=None):
    om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, w.L if L is None else L, w.delta if delta is None else delta, w.nu)
    return om


def _run(P, oracle, w, omega_np, **kw):
    omega = torch.from_numpy(np.ascontiguousarray(omega_np)).cuda()
    out = P.verify_workload(w, omega, **kw)
    torch.cuda.synchronize()
    return to_numpy(out)


# (cfg recipe, B, L, V, dtype): several tiles, partial tiles, ragged tails, several chunks
SHAPES = [
    (1, 1, 4, 16384, "f32"),        # config 1 itself
    (2, 4, 8, 16384, "bf16"),       # config 2 rows
    (2, 3, 5, 4104, "bf16"),        # partial last tile, vector path
    (2, 3, 3, 5001, "bf16"),        # V not a multiple of the vector width: element-wise path
    (1, 2, 3, 1003, "f32"),
    (1, 2, 2, 8, "f32"),            # tiny vocabulary
    (2, 2, 2, 1, "bf16"),           # single token
    (4, 5, 16, 16384, "bf16"),      # config 4 rows
    (5, 2, 3, 40000, "bf16"),       # three chunks, ragged last chunk
    (5, 2, 2, 262144, "bf16"),      # config 5 rows
    (1, 2, 2, 20000, "f32"),        # two chunks fp32
    (5, 3, 2, 16392, "bf16"),       # second chunk holds one vector
]


@pytest.mark.parametrize("cfg,B,L,V,dtype", SHAPES)
def test_shapes_against_oracle(P, oracle, cfg, B, L, V, dtype):
    print("case", cfg, B, L, V, dtype, flush=True)
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, dtype=dtype)
    om = _omega(P, w)
    gpu = _run(P, oracle, w, om)
    compare_verify(oracle, w, om, gpu)


# Rows of several chunks: up to 32768 logits one workgroup of 1024 threads still holds the row
# pair in registers (the per-sequence step is then one launch); beyond, accept / chunk masses /
# selection are three launches.
MID_ROWS = [
    (5, 6, 4, 32768, "bf16", {}),                                   # four chunks of 8192, the longest one-launch row
    (5, 4, 3, 32760, "bf16", {"resample_mode": 1}),                 # ragged last vector; vanilla law
    (5, 4, 3, 24584, "bf16", {"temperature": 0.7}),                 # transformed bf16: fp32 words in registers
    (1, 3, 3, 32768, "f32", {}),
    (1, 3, 2, 20004, "f32", {"temperature": 1.3}),
    (5, 3, 3, 32776, "bf16", {}),                                   # one vector beyond: the three-launch form
    (5, 3, 3, 65536, "bf16", {}),
    (5, 3, 2, 65528, "bf16", {"resample_mode": 1}),
    (5, 3, 3, 40000, "bf16", {"temperature": 0.7}),
    (1, 2, 2, 40004, "f32", {}),                                    # fp32: two vectors per thread in the selection
    (5, 2, 2, 600000, "bf16", {}),                                  # more than 64 chunks: accept_kernel, the serial chunk walk
    (5, 2, 63, 32776, "bf16", {}),                                  # 64 positions with the bonus row: tau still found by the chunk-mass launch
    (5, 2, 64, 32776, "bf16", {}),                                  # 65: accept_kernel
    (1, 5, 7, 70000, "f32", {"temperature": 0.9}),
]


@pytest.mark.parametrize("cfg,B,L,V,dtype,kw", MID_ROWS)
def test_rows_of_several_chunks_in_one_workgroup(P, oracle, cfg, B, L, V, dtype, kw):
    print("case", cfg, B, L, V, dtype, kw, flush=True)
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, dtype=dtype)
    if "temperature" in kw:
        w.temperature = kw["temperature"]
    mode = kw.get("resample_mode", 0)
    om = _omega(P, w)
    gpu = _run(P, oracle, w, om, resample_mode=mode)
    compare_verify(oracle, w, om, gpu, resample_mode=mode)
    # forced outcomes: rejection at the first position, and acceptance of everything (bonus row)
    for om_f, tau in ((np.zeros(L, np.float32), 0), (np.full(L, 1e30, np.float32), L)):
        gpu = _run(P, oracle, w, om_f, resample_mode=mode)
        assert (gpu["accept_len"] == tau).all()
        compare_verify(oracle, w, om_f, gpu, resample_mode=mode)
    # no bonus row
    w.target = w.target[:, :L]
    gpu = _run(P, oracle, w, om, resample_mode=mode)
    compare_verify(oracle, w, om, gpu, resample_mode=mode, has_bonus=False)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("delta", [1.0, 2.0, 4.0])
def test_modes_and_budgets(P, oracle, mode, delta):
    w = make_workload(4, device="cuda", B=24, L=8, V=16384)
    om = _omega(P, w, delta=delta)
    gpu = _run(P, oracle, w, om, resample_mode=mode)
    st = compare_verify(oracle, w, om, gpu, resample_mode=mode)
    assert st["tau_exempt"] + st["token_exempt"] <= 1


def test_uniform_schedule_zero_relaxation_and_per_sequence_omega(P, oracle):
    w = make_workload(2, device="cuda", B=16, L=8, V=16384)
    om = P.cool_sd_schedule(P.COOL_SD_SCHED_UNIFORM, 8, 1.0)
    compare_verify(oracle, w, om, _run(P, oracle, w, om))
    om2 = np.tile(_omega(P, w), (16, 1)).astype(np.float32)
    om2[::3] = 0.0
    om2[1::3] *= 3.0
    gpu = _run(P, oracle, w, om2)
    assert (gpu["accept_len"][::3] == 0).all()
    compare_verify(oracle, w, om2, gpu)


def test_no_bonus_row(P, oracle):
    w = make_workload(2, device="cuda", B=8, L=4, V=16384)
    w.target = w.target[:, :4]                       # non-contiguous view: strides are honoured
    om = np.full(4, 1e6, np.float32)                 # accept everything
    gpu = _run(P, oracle, w, om)
    assert (gpu["accept_len"] == 4).all() and (gpu["next_token"] == -1).all()
    om = _omega(P, w)
    compare_verify(oracle, w, om, _run(P, oracle, w, om), has_bonus=False)


def test_unaligned_rows(P, oracle):
    """Row bases that are not 16-byte aligned take the element-wise path."""
    w = make_workload(2, device="cuda", B=3, L=3, V=4096)
    flat = torch.zeros(w.target.numel() + 8, dtype=w.target.dtype, device="cuda")
    flat[3:3 + w.target.numel()] = w.target.reshape(-1)
    w.target = flat[3:3 + w.target.numel()].view(w.target.shape)
    om = _omega(P, w)
    compare_verify(oracle, w, om, _run(P, oracle, w, om))


@pytest.mark.parametrize("cfg,V,Vpad,dtype", [(2, 16000, 16384, "bf16"), (2, 5001, 5120, "bf16"), (1, 1000, 1024, "f32"),
                                              (5, 40000, 40960, "bf16"), (3, 16000, 16384, "bf16")])
def test_rows_inside_a_padded_vocabulary(P, oracle, cfg, V, Vpad, dtype):
    """Logit tensors whose rows are longer than the vocabulary (padding up to a multiple of some
    block, as a model's output layer often has): the row stride is Vpad, only the first V entries
    belong to the row, and what follows (large values here) must never be read as logits."""
    print("case", cfg, V, Vpad, dtype, flush=True)
    w = make_workload(cfg, device="cuda", B=3, L=3, V=V, dtype=dtype)

    def pad(t):
        if t is None:
            return None
        big = torch.full(t.shape[:-1] + (Vpad,), 60.0, dtype=t.dtype, device="cuda")
        big[..., :V] = t
        return big[..., :V]
    w.target, w.draft = pad(w.target), pad(w.draft)
    w.target_uncond, w.draft_uncond = pad(w.target_uncond), pad(w.draft_uncond)
    assert w.target.stride(1) == Vpad
    om = _omega(P, w)
    gpu = _run(P, oracle, w, om)
    compare_verify(oracle, w, om, gpu)
    early = to_numpy(P.verify_workload(w, torch.from_numpy(om).cuda(), flags=P.COOL_SD_FLAG_EARLY_EXIT))
    compare_verify(oracle, w, om, early, early_exit=(cfg in (1, 2) and V % (8 if dtype == "bf16" else 4) == 0))
    assert gpu["next_token"].max() < V and early["next_token"].max() < V


def test_edge_rows(P, oracle):
    """Degenerate rows: identical models, one-hot rows, all-equal logits, extreme logits,
    a draft token the target excludes, u = 0 and u next to 1."""
    torch.manual_seed(0)
    B, L, V = 8, 4, 16384
    w = make_workload(1, device="cuda", B=B, L=L, V=V, dtype="f32")
    t, d = w.target, w.draft
    d[0] = t[0, :L]                                   # identical: never rejected at omega >= 1
    t[1] = float("-inf"); t[1, :, 77] = 0.0          # one-hot target
    d[1] = 0.0                                        # flat draft
    t[2] = 3.0; d[2] = -2.0                           # all-equal logits on both
    t[3] = t[3] * 25.0                                # logits up to about +-300
    d[3] = d[3] * 25.0
    t[4, :, :] = torch.where(torch.arange(V, device="cuda") % 2 == 0, t[4], torch.full_like(t[4], float("-inf")))
    w.draft_tokens[4] = torch.tensor([1, 3, 5, 2], dtype=torch.int32)   # p(x~)=0 at odd tokens
    w.u_accept[5] = 0.0
    w.u_resample[5] = 0.0
    w.u_accept[6] = 1.0 - 2.0 ** -24
    w.u_resample[6] = 1.0 - 2.0 ** -24
    w.draft_tokens[7] = V - 1
    for om in (np.ones(L, np.float32), np.array([2.0, 1.0, 0.5, 0.25], np.float32)):
        gpu = _run(P, oracle, w, om)
        compare_verify(oracle, w, om, gpu)
        assert gpu["accept_len"][4] == 0 or w.u_accept[4, 0] == 0


def test_resample_entry_point(P, oracle):
    for V, dtype in ((16384, "bf16"), (5001, "f32"), (50000, "bf16")):
        w = make_workload(5, device="cuda", B=6, L=1, V=V, dtype=dtype)
        t, d = w.target[:, 0].contiguous(), w.draft[:, 0].contiguous()
        om = torch.tensor([0.25, 0.5, 1.0, 1.1, 2.0, 4.0], device="cuda")
        u = uniforms24(torch.Generator(device="cuda").manual_seed(5), (6,), "cuda")
        params = P.make_params(t.unsqueeze(1), d.unsqueeze(1), has_bonus=0)
        ws = torch.empty(max(P.cool_sd_workspace_bytes(params), 256), dtype=torch.uint8, device="cuda")
        P.cool_sd_workspace_init(ws)
        for mode in (0, 1):
            params.resample_mode = mode
            tok = torch.full((6,), -7, dtype=torch.int32, device="cuda")
            mass = torch.zeros(6, device="cuda")
            P.cool_sd_resample(params, t, None, d, None, om, u, tok, mass, ws)
            torch.cuda.synchronize()
            ot, om_, g = oracle.resample(t.float().cpu().numpy(), d.float().cpu().numpy(), om.cpu().numpy(),
                                         u.cpu().numpy(), resample_mode=mode, want_g=True)
            np.testing.assert_allclose(mass.cpu().numpy(), om_, rtol=1e-5)
            _tokens_match_or_sit_on_a_boundary(tok.cpu().numpy(), ot, g, om_, u.cpu().numpy())
        # bonus draw: draft absent
        tok = torch.full((6,), -7, dtype=torch.int32, device="cuda")
        P.cool_sd_resample(params, t, None, None, None, None, u, tok, None, ws)
        torch.cuda.synchronize()
        ot, om_, g = oracle.resample(t.float().cpu().numpy(), None, None, u.cpu().numpy(), want_g=True)
        _tokens_match_or_sit_on_a_boundary(tok.cpu().numpy(), ot, g, om_, u.cpu().numpy())


def _tokens_match_or_sit_on_a_boundary(tok, ot, g, R, u):
    """Every token equals the oracle's, or has mass and its uniform lies within 1e-6 (in units of
    u) of the boundary of the oracle's CDF between the two tokens.  Returns the number of such cases."""
    n = 0
    for b in range(len(tok)):
        k = int(tok[b])
        assert 0 <= k < g[b].shape[0] and g[b][k] > 0, (b, k)
        if k != ot[b]:
            C = np.cumsum(g[b])
            v = float(u[b]) * R[b]
            gap = (v - C[k]) / R[b] if k < ot[b] else (C[k - 1] - v) / R[b]
            assert 0 <= gap <= token_band(R[b]), (b, k, int(ot[b]), gap)
            n += 1
    return n


@pytest.mark.parametrize("V", [2, 64, 16384, 40000])
def test_draft_equal_to_target_up_to_a_shift(P, oracle, V):
    """Draft logits = target logits - 1/2: the two softmaxes are the same distribution, but the kernels
    form them against different reference exponents, so [p - q]_+ comes out as rounding residue instead
    of zero.  Rejected at once (omega = 0), the vanilla law has no mass: the call must fall back to p like
    the oracle -- same token, mass 1 -- and not draw from the residue."""
    B, L = 8, 2
    w = make_workload(5, device="cuda", B=B, L=L, V=V)
    g = torch.Generator(device="cuda").manual_seed(V)
    t = (torch.randint(-64, 65, (B, L + 1, V), generator=g, device="cuda").float() / 8).to(torch.bfloat16)
    w.target = t
    w.draft = (t[:, :L].float() - 0.5).to(torch.bfloat16)
    assert torch.equal(w.draft.float() + 0.5, t[:, :L].float())          # the shift is exact in bf16
    om = np.zeros(L, np.float32)
    for mode in (1, 0):
        gpu = _run(P, oracle, w, om, resample_mode=mode)
        ref = compare_verify(oracle, w, om, gpu, resample_mode=mode)
        assert ref["token_exempt"] == 0 and (gpu["accept_len"] == 0).all()
        np.testing.assert_allclose(gpu["resid_mass"], 1.0, rtol=1e-5)


def test_resample_where_the_law_has_no_mass(P, oracle):
    """p and q that coincide (here: both one-hot on the same token after top-1 truncation, from
    different logits) leave [p - q]_+ without mass: any law is optimal there, the oracle falls
    back to p (mass 1).  The token must be the one token that has probability, and the reported
    mass is 1 (the fall-back) or rounding residue far below anything fp64 resolves."""
    from tests.parity_util import R_FLOOR
    B, V = 64, 2
    g = torch.Generator(device="cuda").manual_seed(3)
    t = torch.randn((B, V), generator=g, device="cuda") * 3
    d = t + 0.1 * torch.randn((B, V), generator=g, device="cuda")
    same_top = (t.argmax(1) == d.argmax(1))
    assert same_top.sum() > B // 2
    u = uniforms24(g, (B,), "cuda")
    om = torch.full((B,), 2.0, device="cuda")
    for mode in (0, 1):
        params = P.make_params(t.unsqueeze(1), d.unsqueeze(1), has_bonus=0, top_k=1, resample_mode=mode)
        ws = torch.empty(max(P.cool_sd_workspace_bytes(params), 256), dtype=torch.uint8, device="cuda")
        tok = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        mass = torch.full((B,), -1.0, device="cuda")
        P.cool_sd_resample(params, t, None, d, None, om, u, tok, mass, ws)
        torch.cuda.synchronize()
        ot, om_, _ = oracle.resample(t.cpu().numpy(), d.cpu().numpy(), om.cpu().numpy(), u.cpu().numpy(), top_k=1,
                                     resample_mode=mode, want_g=True)
        np.testing.assert_array_equal(tok.cpu().numpy(), ot)            # the target's arg max, always
        np.testing.assert_array_equal(ot, t.argmax(1).cpu().numpy())
        m = mass.cpu().numpy()
        same = same_top.cpu().numpy()
        assert ((np.abs(m[same] - 1.0) <= 1e-5) | ((m[same] >= 0) & (m[same] <= 10 * R_FLOOR))).all()
        np.testing.assert_allclose(m[~same], om_[~same], rtol=1e-5)     # disjoint supports: mass 1


def test_resample_from_a_small_residual_of_peaked_rows(P, oracle):
    """Guided rows at temperature 0.5 are so peaked that p and q nearly cancel: R = 1.9e-3 here.  fp32
    probabilities cannot resolve such a law (cumulative masses off by ~4e-8, which is 2e-5 in units of
    u), so the library draws it in fp64: mass within 1e-5 relative, token the oracle's unless u lies
    within 1e-6 of a boundary.  Found by a randomised sweep of the fp32-only version."""
    V = 8200
    w = make_workload(3, device="cuda", B=1, L=5, V=V, dtype="bf16", seed=5000 + 41 * 1000 + 136, top_k=0)
    om = P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, 5, 20.0, 0.7)
    torch.manual_seed(201)
    m = torch.rand(V, device="cuda") < 0.3               # tokens the draft excludes
    m[201 % V] = False
    d = w.draft[:, 0].clone(); du = w.draft_uncond[:, 0].clone()
    d[..., m] = float("-inf"); du[..., m] = float("-inf")
    t = w.target[:, 0].contiguous(); tu = w.target_uncond[:, 0].contiguous()
    # the same row pair under 64 uniforms: the one of the original case, and more across the CDF
    B = 64
    t, tu, d, du = (x.expand(B, V).contiguous() for x in (t, tu, d, du))
    u = uniforms24(torch.Generator(device="cuda").manual_seed(136), (B,), "cuda")
    params = P.make_params(t.unsqueeze(1), d.unsqueeze(1), has_bonus=0, cfg_scale=w.cfg_scale, temperature=0.5)
    ws = torch.empty(max(P.cool_sd_workspace_bytes(params), 256), dtype=torch.uint8, device="cuda")
    omr = torch.full((B,), float(om[0]), device="cuda")
    tok = torch.full((B,), -7, dtype=torch.int32, device="cuda"); mass = torch.zeros(B, device="cuda")
    P.cool_sd_resample(params, t, tu, d, du, omr, u, tok, mass, ws)
    torch.cuda.synchronize()
    ot, R, g = oracle.resample(t.float().cpu().numpy(), d.float().cpu().numpy(), omr.cpu().numpy(), u.cpu().numpy(),
                               target_uncond=tu.float().cpu().numpy(), draft_uncond=du.float().cpu().numpy(),
                               cfg_scale=w.cfg_scale, temperature=0.5, want_g=True)
    assert 1e-4 < R[0] < 1e-2                            # the regime this test is about
    np.testing.assert_allclose(mass.cpu().numpy(), R, rtol=1e-5)
    assert _tokens_match_or_sit_on_a_boundary(tok.cpu().numpy(), ot, g, R, u.cpu().numpy()) <= 1


def test_repeat_calls_share_workspace_and_are_deterministic(P, oracle):
    w = make_workload(2, device="cuda", B=8, L=8, V=16384)
    om = torch.from_numpy(_omega(P, w)).cuda()
    params = P.make_params(w.target, w.draft)
    ws = torch.empty(P.cool_sd_workspace_bytes(params), dtype=torch.uint8, device="cuda")
    P.cool_sd_workspace_init(ws)
    outs = []
    for _ in range(5):
        outs.append(to_numpy(P.verify_workload(w, om, workspace=ws)))
    torch.cuda.synchronize()
    for o in outs[1:]:
        for k in o:
            np.testing.assert_array_equal(o[k], outs[0][k])
    compare_verify(oracle, w, om.cpu().numpy(), outs[-1])


# ----------------------------------------------------------------------------- guidance / temperature / top-k
@pytest.mark.parametrize("B,L,V,dtype,top_k", [
    (4, 8, 16384, "bf16", 1000),      # config 3 rows
    (3, 3, 16384, "f32", 1000),
    (3, 2, 5001, "bf16", 50),         # element-wise loads
    (2, 2, 4104, "bf16", 1),          # greedy support
    (2, 2, 2048, "bf16", 2048),       # k = V keeps everything
    (2, 3, 16384, "bf16", 0),         # guidance without truncation
])
def test_guidance_topk_against_oracle(P, oracle, B, L, V, dtype, top_k):
    print("case cfg3", B, L, V, dtype, top_k, flush=True)
    w = make_workload(3, device="cuda", B=B, L=L, V=V, dtype=dtype, top_k=top_k)
    assert w.top_k == top_k
    om = _omega(P, w)
    gpu = _run(P, oracle, w, om)
    st = compare_verify(oracle, w, om, gpu)
    assert st["tau_exempt"] + st["token_exempt"] <= 1
    # tokens outside the draft's support are accepted, outside the target's rejected: exercise both
    w.draft_tokens = torch.randint(0, V, (B, L), dtype=torch.int32, device="cuda",
                                   generator=torch.Generator(device="cuda").manual_seed(3))
    compare_verify(oracle, w, om, _run(P, oracle, w, om))


def test_topk_ties_and_temperature(P, oracle):
    """Rows with massive ties at the threshold (coarse grid, all-equal rows) and a temperature."""
    B, L, V = 4, 2, 16384
    w = make_workload(3, device="cuda", B=B, L=L, V=V, dtype="bf16", top_k=100)
    g = torch.Generator(device="cuda").manual_seed(11)
    for t in (w.target, w.target_uncond, w.draft, w.draft_uncond):
        t[0] = (torch.randint(-3, 4, t[0].shape, device="cuda", generator=g).float() * 0.5).to(t.dtype)  # 7 levels
        t[1] = 1.25                                                                                     # all equal
    w.temperature = 0.75
    om = _omega(P, w)
    compare_verify(oracle, w, om, _run(P, oracle, w, om))
    # temperature alone (no guidance, no truncation) on fp32 logits
    w2 = make_workload(1, device="cuda", B=2, L=3, V=3000, dtype="f32")
    w2.temperature = 1.7
    om2 = _omega(P, w2)
    compare_verify(oracle, w2, om2, _run(P, oracle, w2, om2))


def test_topk_with_excluded_tokens(P, oracle):
    """Rows that already hold -inf logits (tokens excluded upstream), alone and under guidance where the
    conditional and unconditional entries may both be -inf; fewer finite entries than k in one row."""
    for cfg, dtype, V, k in ((3, "bf16", 16384, 1000), (3, "f32", 16384, 300), (2, "bf16", 16384, 64),
                             (3, "bf16", 6000, 5000)):
        w = make_workload(cfg, device="cuda", B=3, L=3, V=V, dtype=dtype, top_k=k if cfg == 3 else None)
        w.top_k = k
        g = torch.Generator(device="cuda").manual_seed(5)
        drop = torch.rand((3, 4, V), device="cuda", generator=g) < 0.3
        ninf = float("-inf")
        w.target[drop] = ninf
        w.draft[drop[:, :3]] = ninf
        if w.target_uncond is not None:
            w.target_uncond[drop] = ninf                 # same tokens excluded on both inputs
            w.draft_uncond[drop[:, :3]] = ninf
        # one target row keeps fewer finite entries than k
        w.target[0, 1, 40:] = ninf
        if w.target_uncond is not None:
            w.target_uncond[0, 1, 40:] = ninf
        om = _omega(P, w)
        print("case excluded", cfg, dtype, V, k, flush=True)
        st = compare_verify(oracle, w, om, _run(P, oracle, w, om))
        assert st["tau_exempt"] + st["token_exempt"] <= 1


@pytest.mark.parametrize("cfg,B,L,V,dtype,top_k", [
    (3, 3, 3, 40000, "bf16", 1000),      # guidance + truncation on rows of five chunks
    (3, 2, 2, 65536, "bf16", 2000),      # a 64K vocabulary
    (3, 3, 3, 32768, "bf16", 1000),      # the longest row of the 32-logits-per-thread form
    (3, 2, 3, 24584, "bf16", 300),       # its ragged last statistics pair
    (1, 2, 2, 20004, "f32", 7),
    (2, 2, 3, 20001, "bf16", 50),        # element-wise loads, no guidance
    (1, 2, 2, 33000, "f32", 1),          # greedy support on fp32 rows
    (5, 2, 2, 262144, "bf16", 4096),     # the large-vocabulary configuration's rows
    (2, 2, 2, 16392, "bf16", 16392),     # k = V on a row that barely needs a second chunk
    (2, 2, 2, 70001, "bf16", 300),       # beyond one workgroup: radix passes, element-wise loads
    (3, 2, 2, 66000, "f32", 77),         # radix passes on guided fp32 rows
])
def test_topk_on_long_rows(P, oracle, cfg, B, L, V, dtype, top_k):
    """Rows beyond 16384 logits: one workgroup of 1024 threads up to 65536, three radix passes beyond."""
    print("case long top-k", cfg, B, L, V, dtype, top_k, flush=True)
    w = make_workload(cfg, device="cuda", B=B, L=L, V=V, dtype=dtype, top_k=top_k if cfg == 3 else None)
    w.top_k = top_k
    om = _omega(P, w)
    st = compare_verify(oracle, w, om, _run(P, oracle, w, om))
    assert st["tau_exempt"] + st["token_exempt"] <= 1
    # coarse values: massive ties at the threshold, zeros of both signs, and excluded tokens
    g = torch.Generator(device="cuda").manual_seed(V)
    for t in (w.target, w.draft, w.target_uncond, w.draft_uncond):
        if t is not None:
            t[0] = (torch.randint(-3, 4, t[0].shape, device="cuda", generator=g).float() * 0.5).to(t.dtype)
            t[0, :, ::7] = float("-inf")
            t[0, :, 1::7] = -0.0
    w.draft_tokens = torch.randint(0, V, (B, L), dtype=torch.int32, device="cuda", generator=g)
    st = compare_verify(oracle, w, om, _run(P, oracle, w, om))
    assert st["tau_exempt"] + st["token_exempt"] <= 1


# ----------------------------------------------------------------------------- full benchmark sizes
@pytest.mark.parametrize("cfg,n_check", [(1, None), (2, None), (3, None), (4, None), (5, None)])
def test_full_size_configurations(P, oracle, cfg, n_check):
    """The five configurations at their full sizes, launched exactly as bench.py launches them (same
    params, workspace and chunking), without and with the early-exit flag.  Every sequence of every
    configuration is checked against the oracle."""
    from tests.parity_util import subset
    print("full cfg", cfg, flush=True)
    w = make_workload(cfg, device="cuda")
    om = _omega(P, w)
    gpu = _run(P, oracle, w, om)
    assert gpu["accept_len"].min() >= 0 and gpu["accept_len"].max() <= w.L
    assert gpu["next_token"].min() >= 0 and gpu["next_token"].max() < w.V
    if n_check is None:
        from tests.parity_util import early_exit_form, run_oracle
        ref = run_oracle(oracle, w, om, 0)
        st = compare_verify(oracle, w, om, gpu, ref=ref)
        # the same call with COOL_SD_FLAG_EARLY_EXIT (one workgroup per sequence on configurations 1, 2
        # and 4, rounds of positions on configuration 5, not honoured under top-k) against the same reference
        early = _run(P, oracle, w, om, flags=P.COOL_SD_FLAG_EARLY_EXIT)
        form = early_exit_form(P, w)
        assert form == {1: 1, 2: 1, 3: 0, 4: 1, 5: 2}[cfg]
        st2 = compare_verify(oracle, w, om, early, ref=ref, early_exit=form != 0)
        print("early-exit form", form, "exemptions", st2, flush=True)
        assert st2["tau_exempt"] + st2["token_exempt"] <= 2
    else:
        idx = np.sort(np.random.default_rng(cfg).choice(w.B, n_check, replace=False))
        st = compare_verify(oracle, subset(w, idx), om, {k: v[idx] for k, v in gpu.items()})
    # every exemption counted here lies inside the 1e-6 band (compare_verify asserts it); none is expected
    print("exemptions (uniform within 1e-6 of its threshold)", st, flush=True)
    assert st["tau_exempt"] + st["token_exempt"] <= 2
    # acceptance statistics are those of speculative decoding, not degenerate
    if w.B >= 32:
        assert 0.5 < gpu["accept_len"].mean() < w.L - 0.5


def test_hip_graph_replays_match_eager(P, oracle):
    """bench.py replays verify calls from a HIP graph: every replay must reproduce the eager result,
    also with other eager work and synchronisations between replays (both launch shapes: one-chunk
    rows and long rows)."""
    for cfg, kw in ((2, dict(B=32, L=8, V=16384)), (5, dict(B=4, L=4, V=40000))):   # config 2 at its full size
        pool = [make_workload(cfg, device="cuda", call=c, **kw) for c in range(3)]
        om = torch.from_numpy(_omega(P, pool[0])).cuda()
        params = P.make_params(pool[0].target, pool[0].draft)
        ws = torch.empty(P.cool_sd_workspace_bytes(params), dtype=torch.uint8, device="cuda")
        outs = [dict(a=torch.zeros(kw["B"], dtype=torch.int32, device="cuda"),
                     n=torch.zeros(kw["B"], dtype=torch.int32, device="cuda"),
                     r=torch.zeros(kw["B"], device="cuda")) for _ in pool]

        def issue():
            for w, o in zip(pool, outs):
                P.cool_sd_verify(params, w.target, None, w.draft, None, w.draft_tokens, om, w.u_accept,
                                 w.u_resample, o["a"], o["n"], None, None, None, o["r"], ws)

        issue()
        torch.cuda.synchronize()
        eager = [{k: v.clone() for k, v in o.items()} for o in outs]
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            issue()
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            issue()
        for rep in range(4):
            for o in outs:
                for v in o.values():
                    v.fill_(-3)
            junk = torch.randn(1 << 20, device="cuda").sum()          # unrelated eager work
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert junk.item() == junk.item()
            for o, e in zip(outs, eager):
                for k in o:
                    assert torch.equal(o[k], e[k]), (cfg, rep, k)


def test_long_draft_windows_and_tiny_shapes(P, oracle):
    """L beyond one block of positions (the first-rejection scan loops), and the smallest shapes."""
    for B, L, V, dtype, delta in ((2, 1500, 64, "f32", 50.0), (3, 257, 520, "bf16", 30.0), (1, 1, 2, "f32", 1.0),
                                  (5, 1, 16384, "bf16", 1.1)):
        w = make_workload(1, device="cuda", B=B, L=L, V=V, dtype=dtype)
        om = P.cool_sd_schedule(P.COOL_SD_SCHED_UNIFORM, L, delta)      # large budget: long accepted prefixes
        gpu = _run(P, oracle, w, om)
        compare_verify(oracle, w, om, gpu)
        if L >= 257:
            assert gpu["accept_len"].max() > 256 or delta < 40
    # everything rejected at the first position
    w = make_workload(2, device="cuda", B=4, L=8, V=16384)
    gpu = _run(P, oracle, w, np.zeros(8, np.float32))
    assert (gpu["accept_len"] == 0).all()
    compare_verify(oracle, w, np.zeros(8, np.float32), gpu)


@pytest.mark.parametrize("V,dtype,guided,top_k,temperature", [
    (16384, "bf16", True, 200, 0.9),       # the guided, truncated sampler of the paper's larger models
    (16384, "f32", False, 1000, 1.0),
    (5001, "bf16", True, 50, 1.0),          # element-wise loads
    (1003, "f32", False, 7, 1.3),
    (16384, "bf16", False, 16384, 1.0),     # k = V: nothing is cut
    (8, "f32", False, 1, 1.0),              # k = 1: the arg max
    (16384, "bf16", False, 0, 1.0),         # no truncation: the plain one-launch draw
    (40000, "bf16", True, 300, 1.0),        # rows of several chunks, truncated: still one workgroup of 1024 threads
    (65536, "bf16", True, 2000, 1.0),       # the larger model's vocabulary and truncation
    (24584, "bf16", False, 50, 0.8),        # the 32-logits-per-thread form, ragged tail
    (20004, "f32", True, 7, 1.0),
    (33000, "f32", False, 400, 1.0),        # fp32 beyond 32768: statistics pass + sampling kernels
    (32768, "bf16", False, 0, 1.0),         # no truncation, up to 32768 logits: still one launch
    (24584, "f32", True, 0, 0.9),
    (40000, "bf16", False, 0, 1.0),         # no truncation on longer rows: statistics pass + sampling kernels
    (70000, "bf16", True, 500, 1.0),        # beyond one workgroup: radix passes
])
def test_draft_side_sampling_through_resample(P, oracle, V, dtype, guided, top_k, temperature):
    """Drawing x~ ~ Q (Algorithm 1, drafting stage) is cool_sd_resample with the draft's logits as the
    only distribution: guidance, temperature and top-k apply, then an inverse-CDF draw from q."""
    print("case", V, dtype, guided, top_k, temperature, flush=True)
    B = 16
    w = make_workload(3 if guided else 1, device="cuda", B=B, L=1, V=V, dtype=dtype, top_k=top_k if guided else None)
    d = w.draft[:, 0].contiguous()
    du = w.draft_uncond[:, 0].contiguous() if guided else None
    if dtype == "bf16":
        d[3, : V // 2] = d[3, 0]                                  # heavy ties around the threshold in one row
    scale = w.cfg_scale if guided else 1.0
    params = P.make_params(d.unsqueeze(1), d.unsqueeze(1), has_bonus=0, top_k=top_k, cfg_scale=scale,
                           temperature=temperature)
    ws = torch.empty(P.cool_sd_workspace_bytes(params), dtype=torch.uint8, device="cuda")
    P.cool_sd_workspace_init(ws)
    u = uniforms24(torch.Generator(device="cuda").manual_seed(9), (B,), "cuda")
    u[0] = 0.0
    u[1] = 1.0 - 2.0 ** -24
    tok = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    mass = torch.zeros(B, device="cuda")
    P.cool_sd_resample(params, d, du, None, None, None, u, tok, mass, ws)
    torch.cuda.synchronize()
    ot, om_, g = oracle.resample(d.float().cpu().numpy(), None, None, u.cpu().numpy(),
                                 target_uncond=None if du is None else du.float().cpu().numpy(), cfg_scale=scale,
                                 temperature=temperature, top_k=top_k, want_g=True)
    np.testing.assert_allclose(mass.cpu().numpy(), om_, rtol=1e-5)
    for b in range(B):
        if top_k:
            assert (g[b] > 0).sum() >= min(top_k, V)
    _tokens_match_or_sit_on_a_boundary(tok.cpu().numpy(), ot, g, om_, u.cpu().numpy())


def test_random_shapes_and_options(P, oracle):
    """Seeded sweep over shapes, dtypes and options (every code path: element-wise loads, one-chunk and
    long rows, guidance, temperature, top-k, both resampling laws, with / without bonus row)."""
    rng = np.random.default_rng(2026)
    n_exempt = 0
    for case in range(40):
        dtype = "bf16" if rng.random() < 0.6 else "f32"
        V = int(rng.choice([3, 17, 257, 1024, 4097, 8200, 16384, 16385, 20001, 33000, 70000]))
        B = int(rng.integers(1, 6))
        L = int(rng.integers(1, 10))
        guided = rng.random() < 0.4
        cfg = 3 if guided else int(rng.choice([1, 2, 4, 5]))
        top_k = 0
        if rng.random() < 0.5:
            top_k = int(rng.integers(1, V + 1))
        w = make_workload(cfg, device="cuda", B=B, L=L, V=V, dtype=dtype, seed=1000 + case,
                          top_k=top_k if guided else None)
        if not guided:
            w.top_k = top_k
        if rng.random() < 0.3:
            w.temperature = float(rng.choice([0.5, 0.8, 1.3]))
        if rng.random() < 0.3:
            w.target = w.target[:, :L]                                   # no bonus row
            if w.target_uncond is not None:
                w.target_uncond = w.target_uncond[:, :L]
        mode = int(rng.integers(0, 2))
        delta = float(rng.choice([1.0, 1.1, 2.0, 4.0]))
        om = _omega(P, w, delta=delta)
        print("case", case, dict(cfg=cfg, B=B, L=L, V=V, dtype=dtype, top_k=w.top_k, T=w.temperature,
                                 bonus=w.target.shape[1] == L + 1, mode=mode, delta=delta), flush=True)
        gpu = _run(P, oracle, w, om, resample_mode=mode)
        st = compare_verify(oracle, w, om, gpu, resample_mode=mode, has_bonus=w.target.shape[1] == L + 1)
        n_exempt += st["tau_exempt"] + st["token_exempt"]
    assert n_exempt <= 2
