"""Seeded synthetic workloads with the shapes and value statistics of the five configurations.

The paper's workloads are logits of trained text-to-image models on captions that are not
available here; these inputs stand in for them.  Everything is drawn from a seeded
torch.Generator on the requested device, so the same (config, seed, call, device) always
gives the same arrays, and both the CPU oracle and the HIP library are fed those arrays.

Nothing in this file belongs to the verify/resample method.  The only model-side step it
plays is the *drafting* stage that precedes verification: draft tokens are sampled from the
draft distribution by the Gumbel-max trick (argmax of logits plus Gumbel noise over the
tokens the draft model may emit), so that acceptance statistics look like real speculative
decoding.
"""
from dataclasses import dataclass, field
from typing import Optional

import torch

# name -> recipe.  B/L/V/dtype follow the benchmark configurations; the noise models are
# stated per configuration in the functions below.
CONFIGS = {
    1: dict(B=1, L=4, V=16384, dtype="f32", calls=64, delta=1.1, nu=0.7),
    2: dict(B=32, L=8, V=16384, dtype="bf16", calls=72, delta=1.1, nu=0.7),
    3: dict(B=64, L=8, V=16384, dtype="bf16", calls=72, delta=1.1, nu=0.7,
            cfg_scale=4.0, temperature=1.0, top_k=1000),
    4: dict(B=256, L=16, V=16384, dtype="bf16", calls=64, delta=1.1, nu=0.7,
            delta_sweep=(1.0, 1.1, 2.0, 3.0, 4.0)),
    5: dict(B=128, L=8, V=262144, dtype="bf16", calls=72, delta=1.1, nu=0.7),
}


@dataclass
class Workload:
    """One verify call's inputs.  Logit tensors are stored in `dtype` ("f32" | "bf16")."""
    cfg: int
    B: int
    L: int
    V: int
    dtype: str
    target: torch.Tensor                      # [B, L+1, V]
    draft: torch.Tensor                       # [B, L, V]
    draft_tokens: torch.Tensor                # [B, L] int32
    u_accept: torch.Tensor                    # [B, L] float32 in [0,1), 24-bit grid
    u_resample: torch.Tensor                  # [B]    float32 in [0,1), 24-bit grid
    target_uncond: Optional[torch.Tensor] = None
    draft_uncond: Optional[torch.Tensor] = None
    cfg_scale: float = 1.0
    temperature: float = 1.0
    top_k: int = 0
    delta: float = 1.1
    nu: float = 0.7
    extra: dict = field(default_factory=dict)

    def logits_f32_numpy(self):
        """Exact float32 copies on the host (bf16 -> fp32 widening is exact)."""
        f = lambda t: None if t is None else t.detach().float().cpu().numpy()
        return f(self.target), f(self.draft), f(self.target_uncond), f(self.draft_uncond)

    def algorithmic_bytes(self):
        """Every logit of every verified row read once."""
        s = 4 if self.dtype == "f32" else 2
        streams = 2 if self.target_uncond is not None else 1
        return (self.B * (self.L + 1) + self.B * self.L) * self.V * s * streams


def uniforms24(gen, shape, device):
    """Uniforms on the 24-bit grid n * 2^-24, n in [0, 2^24): exactly representable in fp32."""
    n = torch.randint(0, 1 << 24, shape, generator=gen, device=device, dtype=torch.int32)
    return n.to(torch.float32) * (2.0 ** -24)


def _randn(gen, shape, device):
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)


def _gumbel(gen, shape, device):
    u = torch.rand(shape, generator=gen, device=device, dtype=torch.float32)
    u = u.clamp_(1e-20, 1.0 - 1e-7)
    return -torch.log(-torch.log(u))


def _store(x, dtype):
    return x.to(torch.bfloat16) if dtype == "bf16" else x.contiguous()


def _draft_tokens(gen, draft_logits_f32, keep_top_k=0):
    """Drafting stage: x~ ~ softmax(draft logits) via Gumbel-max, restricted to the tokens the
    draft model may emit (its top-k set when truncation is on).  Chunked over rows to bound
    temporary memory."""
    B, L, V = draft_logits_f32.shape
    flat = draft_logits_f32.reshape(B * L, V)
    out = torch.empty(B * L, dtype=torch.int64, device=flat.device)
    rows_per = max(1, (1 << 25) // V)
    for r0 in range(0, B * L, rows_per):
        blk = flat[r0:r0 + rows_per]
        score = blk + _gumbel(gen, blk.shape, blk.device)
        if keep_top_k:
            kth = torch.topk(blk, keep_top_k, dim=-1).values[:, -1:]
            score = torch.where(blk >= kth, score, torch.full_like(score, float("-inf")))
        out[r0:r0 + rows_per] = score.argmax(dim=-1)
    return out.reshape(B, L).to(torch.int32)


def make_workload(cfg: int, *, device="cpu", seed: Optional[int] = None, call: int = 0,
                  B: Optional[int] = None, L: Optional[int] = None, V: Optional[int] = None,
                  dtype: Optional[str] = None, top_k: Optional[int] = None) -> Workload:
    """Inputs of one verify call of configuration `cfg` (1..5).

    B, L, V, dtype, top_k override the configuration's sizes for scaled-down parity cases.
    seed defaults to 42 + (cfg - 1) (the paper's experiments use seeds 42-46); `call`
    selects an independent call of the same sequence decode.
    """
    r = dict(CONFIGS[cfg])
    B = r["B"] if B is None else B
    L = r["L"] if L is None else L
    V = r["V"] if V is None else V
    dtype = r["dtype"] if dtype is None else dtype
    seed = 42 + (cfg - 1) if seed is None else seed
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed((seed << 20) + call)

    extra = {}
    t_u = d_u = None
    cfg_scale, temperature, k = 1.0, 1.0, 0
    if cfg == 1:        # t ~ N(0, 3^2); d = t + N(0, 1^2)
        t = 3.0 * _randn(gen, (B, L + 1, V), device)
        d = t[:, :L] + _randn(gen, (B, L, V), device)
    elif cfg == 2:      # t ~ N(0, 4^2), 5% of entries + 8; d = 0.8 t + N(0, 1.5^2)
        t = 4.0 * _randn(gen, (B, L + 1, V), device)
        boost = torch.rand((B, L + 1, V), generator=gen, device=device) < 0.05
        t = t + 8.0 * boost.to(torch.float32)
        d = 0.8 * t[:, :L] + 1.5 * _randn(gen, (B, L, V), device)
    elif cfg == 3:      # conditional / unconditional pairs, combined by guidance in the kernel
        cfg_scale, temperature = r["cfg_scale"], r["temperature"]
        k = r["top_k"] if top_k is None else top_k
        k = min(k, V)
        t_u = 3.0 * _randn(gen, (B, L + 1, V), device)
        t = t_u + _randn(gen, (B, L + 1, V), device)
        # draft noise 0.2 per tensor: after guidance with s = 4 the draft's guided logits differ
        # from the target's by N(0, (4^2 + 3^2) 0.2^2) = N(0, 1), the same mismatch as configuration 1
        d_u = t_u[:, :L] + 0.2 * _randn(gen, (B, L, V), device)
        d = t[:, :L] + 0.2 * _randn(gen, (B, L, V), device)
    elif cfg == 4:      # per-sequence correlation rho ~ U(0.3, 0.95)
        rho = 0.3 + 0.65 * torch.rand((B, 1, 1), generator=gen, device=device)
        t = 3.0 * _randn(gen, (B, L + 1, V), device)
        d = rho * t[:, :L] + torch.sqrt(1.0 - rho * rho) * 3.0 * _randn(gen, (B, L, V), device)
        extra["rho"] = rho.reshape(B).cpu()
    elif cfg == 5:      # large vocabulary: t ~ N(0, 3^2); d = t + N(0, 2^2)
        t = 3.0 * _randn(gen, (B, L + 1, V), device)
        d = t[:, :L] + 2.0 * _randn(gen, (B, L, V), device)
    else:
        raise ValueError("cfg must be 1..5")

    t, d = _store(t, dtype), _store(d, dtype)
    if t_u is not None:
        t_u, d_u = _store(t_u, dtype), _store(d_u, dtype)
        # what the draft model emits: guidance on the stored logits, then its top-k set
        dl = d_u.float() + cfg_scale * (d.float() - d_u.float())
        tokens = _draft_tokens(gen, dl, keep_top_k=k)
        del dl
    else:
        tokens = _draft_tokens(gen, d.float() if dtype == "bf16" else d)
    ua = uniforms24(gen, (B, L), device)
    ur = uniforms24(gen, (B,), device)
    return Workload(cfg=cfg, B=B, L=L, V=V, dtype=dtype, target=t, draft=d, draft_tokens=tokens,
                    u_accept=ua, u_resample=ur, target_uncond=t_u, draft_uncond=d_u,
                    cfg_scale=cfg_scale, temperature=temperature, top_k=k,
                    delta=r["delta"], nu=r["nu"], extra=extra)


def make_neighbor_table(V: int, k: int, *, device="cpu", seed: int = 7, pad: float = 0.0,
                        self_entries: bool = False) -> torch.Tensor:
    """Synthetic stand-in for the codebook's nearest-neighbour table ([V, k] int32, "nearest"
    first): the real table comes from the trained VQ codebook, which is not available.  Row x
    holds k distinct tokens other than x: x plus k distinct non-zero offsets (shared by all
    rows) in a per-row random order.  pad: fraction of entries replaced by -1; self_entries: one
    entry per row replaced by x itself (both must be skipped by a consumer)."""
    assert 1 <= k < V
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    offs = torch.randperm(V - 1, generator=gen, device=device)[:k] + 1                  # distinct, in [1, V-1]
    order = torch.rand((V, k), generator=gen, device=device).argsort(dim=1)
    x = torch.arange(V, device=device).unsqueeze(1)
    nbr = (x + offs[order]) % V
    if pad > 0:
        nbr = torch.where(torch.rand((V, k), generator=gen, device=device) < pad, torch.full_like(nbr, -1), nbr)
    if self_entries:
        col = torch.randint(0, k, (V, 1), generator=gen, device=device)
        nbr = nbr.scatter(1, col, x)
    return nbr.to(torch.int32).contiguous()
