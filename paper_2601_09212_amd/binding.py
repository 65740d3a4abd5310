"""ctypes binding of libcool_sd.so: argument marshalling only.

Every function has the name and argument order of its C entry point (include/cool_sd.h).
Tensors are torch tensors on the GPU; the binding passes their data pointers and the current
HIP stream.  There is no fallback: if the library is missing, importing a symbol raises.
"""
import ctypes as C
import os

import numpy as np

COOL_SD_F32, COOL_SD_BF16 = 0, 1
COOL_SD_SCHED_UNIFORM, COOL_SD_SCHED_EXP, COOL_SD_SCHED_LINEAR = 0, 1, 2
COOL_SD_RESAMPLE_OPT, COOL_SD_RESAMPLE_VANILLA, COOL_SD_RESAMPLE_LANTERN = 0, 1, 2
COOL_SD_FLAG_EARLY_EXIT, COOL_SD_FLAG_CHECK_TOKENS, COOL_SD_FLAG_EXACT_DRAW = 1, 2, 4
COOL_SD_OK, COOL_SD_EINVAL, COOL_SD_EWORKSPACE, COOL_SD_ELAUNCH, COOL_SD_EUNSUPPORTED = 0, -1, -2, -3, -4
COOL_SD_ETOOLARGE = -5
COOL_SD_NOALLOC_WORKSPACE_BYTES = 4 << 20
COOL_SD_EARLY_EXIT_NONE, COOL_SD_EARLY_EXIT_SEQUENCE, COOL_SD_EARLY_EXIT_ROUNDS = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcool_sd.so")
LIB_CHECKED_PATH = os.path.join(_HERE, "libcool_sd_checked.so")     # debug build: draft tokens checked on every call
LIB_BENCH_PATH = os.path.join(_HERE, "libcool_sd_bench.so")         # benchmark companion (include/cool_sd_bench.h)


class CoolSDError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, cool_sd_strerror(code), code))


class CoolSDParams(C.Structure):
    _fields_ = [("B", C.c_int32), ("L", C.c_int32), ("V", C.c_int32), ("dtype", C.c_int32),
                ("t_stride_b", C.c_int64), ("t_stride_l", C.c_int64),
                ("d_stride_b", C.c_int64), ("d_stride_l", C.c_int64),
                ("omega_stride_b", C.c_int64),
                ("has_bonus", C.c_int32), ("top_k", C.c_int32),
                ("cfg_scale", C.c_float), ("temperature", C.c_float),
                ("resample_mode", C.c_int32), ("flags", C.c_int32)]


_lib = None
_bench = None


def load(path):
    """Load a build of the C-ABI library (the product, or its checked build) and declare the entry
    points of include/cool_sd.h.  Fails loudly when the file has not been built."""
    if not os.path.exists(path):
        raise ImportError("%s is not built: run `python -m paper_2601_09212_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path" % os.path.basename(path))
    # PyTorch ships its own copy of the HIP runtime (soname libamdhip64.so.7).  Load it first so
    # that this library binds to the same runtime instance that owns torch's memory and streams;
    # two runtimes in one process do not see each other's devices.
    import torch  # noqa: F401
    L = C.CDLL(path)
    vp, pp = C.c_void_p, C.POINTER(CoolSDParams)
    L.cool_sd_schedule.argtypes = [C.c_int32, C.c_int32, C.c_float, C.c_float, C.POINTER(C.c_float)]
    L.cool_sd_schedule.restype = C.c_int
    L.cool_sd_workspace_bytes.argtypes = [pp]
    L.cool_sd_workspace_bytes.restype = C.c_size_t
    L.cool_sd_workspace_init.argtypes = [vp, C.c_size_t, vp]
    L.cool_sd_workspace_init.restype = C.c_int
    L.cool_sd_verify.argtypes = [pp] + [vp] * 14 + [vp, C.c_size_t, vp]
    L.cool_sd_verify.restype = C.c_int
    L.cool_sd_verify_noalloc.argtypes = [pp] + [vp] * 14 + [vp]
    L.cool_sd_verify_noalloc.restype = C.c_int
    L.cool_sd_verify_lantern.argtypes = ([pp] + [vp] * 6 + [C.c_int32, C.c_float] + [vp] * 10
                                         + [vp, C.c_size_t, vp])
    L.cool_sd_verify_lantern.restype = C.c_int
    L.cool_sd_verify_diagnostics.argtypes = [pp] + [vp] * 16 + [vp, C.c_size_t, vp]
    L.cool_sd_verify_diagnostics.restype = C.c_int
    L.cool_sd_resample.argtypes = [pp] + [vp] * 8 + [vp, C.c_size_t, vp]
    L.cool_sd_resample.restype = C.c_int
    L.cool_sd_diagnostics.argtypes = [pp] + [vp] * 7 + [vp, C.c_size_t, vp]
    L.cool_sd_diagnostics.restype = C.c_int
    L.cool_sd_early_exit_form.argtypes = [pp, C.c_int]
    L.cool_sd_early_exit_form.restype = C.c_int
    L.cool_sd_strerror.argtypes = [C.c_int]
    L.cool_sd_strerror.restype = C.c_char_p
    return L


def lib():
    """The loaded product library."""
    global _lib
    if _lib is None:
        _lib = load(LIB_PATH)
    return _lib


def bench_lib():
    """The benchmark companion library (only bench.py and its tests use it)."""
    global _bench
    if _bench is None:
        L = load(LIB_BENCH_PATH)
        vp, pp = C.c_void_p, C.POINTER(CoolSDParams)
        L.cool_sd_bench_row_stats.argtypes = [pp] + [vp] * 5 + [vp, C.c_size_t, vp]
        L.cool_sd_bench_row_stats.restype = C.c_int
        L.cool_sd_bench_read_probe.argtypes = [vp, C.c_size_t, vp, C.c_size_t, vp, C.c_size_t, vp]
        L.cool_sd_bench_read_probe.restype = C.c_int
        _bench = L
    return _bench


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    return C.c_void_p(stream)


def cool_sd_early_exit_form(params, rows_aligned=True):
    """How a verify call with these parameters honours COOL_SD_FLAG_EARLY_EXIT (host only)."""
    rc = lib().cool_sd_early_exit_form(C.byref(params), int(bool(rows_aligned)))
    if rc < 0:
        raise CoolSDError(rc, "cool_sd_early_exit_form")
    return rc


def cool_sd_strerror(code):
    return lib().cool_sd_strerror(int(code)).decode()


def cool_sd_schedule(kind, L, delta, param=0.0):
    """omega_1..omega_L as a float32 numpy array (host)."""
    out = np.empty(max(int(L), 1), dtype=np.float32)
    rc = lib().cool_sd_schedule(kind, L, delta, param, out.ctypes.data_as(C.POINTER(C.c_float)))
    if rc != 0:
        raise CoolSDError(rc, "cool_sd_schedule")
    return out[:L]


def cool_sd_workspace_bytes(params):
    return int(lib().cool_sd_workspace_bytes(C.byref(params)))


def cool_sd_workspace_init(workspace, stream=None):
    rc = lib().cool_sd_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _stream(stream))
    if rc != 0:
        raise CoolSDError(rc, "cool_sd_workspace_init")


def cool_sd_verify(params, target, target_uncond, draft, draft_uncond, draft_tokens, omega, u_accept,
                   u_resample, accept_len, next_token, p_tok, q_tok, f, resid_mass, workspace, stream=None,
                   check=True):
    rc = lib().cool_sd_verify(C.byref(params), _ptr(target), _ptr(target_uncond), _ptr(draft),
                              _ptr(draft_uncond), _ptr(draft_tokens), _ptr(omega), _ptr(u_accept),
                              _ptr(u_resample), _ptr(accept_len), _ptr(next_token), _ptr(p_tok), _ptr(q_tok),
                              _ptr(f), _ptr(resid_mass), _ptr(workspace),
                              0 if workspace is None else workspace.numel() * workspace.element_size(),
                              _stream(stream))
    if check and rc != 0:
        raise CoolSDError(rc, "cool_sd_verify")
    return rc


def cool_sd_verify_noalloc(params, target, target_uncond, draft, draft_uncond, draft_tokens, omega, u_accept,
                           u_resample, accept_len, next_token, p_tok, q_tok, f, resid_mass, stream=None, check=True):
    rc = lib().cool_sd_verify_noalloc(C.byref(params), _ptr(target), _ptr(target_uncond), _ptr(draft),
                                      _ptr(draft_uncond), _ptr(draft_tokens), _ptr(omega), _ptr(u_accept),
                                      _ptr(u_resample), _ptr(accept_len), _ptr(next_token), _ptr(p_tok), _ptr(q_tok),
                                      _ptr(f), _ptr(resid_mass), _stream(stream))
    if check and rc != 0:
        raise CoolSDError(rc, "cool_sd_verify_noalloc")
    return rc


def cool_sd_verify_diagnostics(params, target, target_uncond, draft, draft_uncond, draft_tokens, omega, u_accept,
                               u_resample, accept_len, next_token, p_tok, q_tok, f, resid_mass, alpha, beta, workspace,
                               stream=None, check=True):
    rc = lib().cool_sd_verify_diagnostics(C.byref(params), _ptr(target), _ptr(target_uncond), _ptr(draft),
                                          _ptr(draft_uncond), _ptr(draft_tokens), _ptr(omega), _ptr(u_accept),
                                          _ptr(u_resample), _ptr(accept_len), _ptr(next_token), _ptr(p_tok),
                                          _ptr(q_tok), _ptr(f), _ptr(resid_mass), _ptr(alpha), _ptr(beta),
                                          _ptr(workspace),
                                          0 if workspace is None else workspace.numel() * workspace.element_size(),
                                          _stream(stream))
    if check and rc != 0:
        raise CoolSDError(rc, "cool_sd_verify_diagnostics")
    return rc


def cool_sd_verify_lantern(params, target, target_uncond, draft, draft_uncond, draft_tokens, neighbors, k, lam,
                           u_accept, u_resample, accept_len, next_token, p_tok, q_tok, f, resid_mass, p_agg,
                           count, workspace, stream=None, check=True):
    rc = lib().cool_sd_verify_lantern(C.byref(params), _ptr(target), _ptr(target_uncond), _ptr(draft),
                                      _ptr(draft_uncond), _ptr(draft_tokens), _ptr(neighbors), int(k), float(lam),
                                      _ptr(u_accept), _ptr(u_resample), _ptr(accept_len), _ptr(next_token),
                                      _ptr(p_tok), _ptr(q_tok), _ptr(f), _ptr(resid_mass), _ptr(p_agg),
                                      _ptr(count), _ptr(workspace),
                                      0 if workspace is None else workspace.numel() * workspace.element_size(),
                                      _stream(stream))
    if check and rc != 0:
        raise CoolSDError(rc, "cool_sd_verify_lantern")
    return rc


def cool_sd_resample(params, target_rows, target_uncond_rows, draft_rows, draft_uncond_rows, omega_rows, u,
                     token, resid_mass, workspace, stream=None, check=True):
    rc = lib().cool_sd_resample(C.byref(params), _ptr(target_rows), _ptr(target_uncond_rows), _ptr(draft_rows),
                                _ptr(draft_uncond_rows), _ptr(omega_rows), _ptr(u), _ptr(token),
                                _ptr(resid_mass), _ptr(workspace),
                                0 if workspace is None else workspace.numel() * workspace.element_size(),
                                _stream(stream))
    if check and rc != 0:
        raise CoolSDError(rc, "cool_sd_resample")
    return rc


def cool_sd_diagnostics(params, target, target_uncond, draft, draft_uncond, omega, alpha, beta, workspace,
                        stream=None, check=True):
    rc = lib().cool_sd_diagnostics(C.byref(params), _ptr(target), _ptr(target_uncond), _ptr(draft),
                                   _ptr(draft_uncond), _ptr(omega), _ptr(alpha), _ptr(beta), _ptr(workspace),
                                   0 if workspace is None else workspace.numel() * workspace.element_size(),
                                   _stream(stream))
    if check and rc != 0:
        raise CoolSDError(rc, "cool_sd_diagnostics")
    return rc


def cool_sd_bench_read_probe(a, b, workspace, stream=None, check=True):
    """Streaming read of tensors a and b (b may be None) in one launch; see include/cool_sd_bench.h."""
    nb = lambda t: 0 if t is None else t.numel() * t.element_size()
    rc = bench_lib().cool_sd_bench_read_probe(_ptr(a), nb(a), _ptr(b), nb(b), _ptr(workspace), nb(workspace),
                                              _stream(stream))
    if check and rc != 0:
        raise CoolSDError(rc, "cool_sd_bench_read_probe")
    return rc


def cool_sd_bench_row_stats(params, target, target_uncond, draft, draft_uncond, draft_tokens, workspace, stream=None,
                            check=True):
    """The statistics pass of cool_sd_verify alone; see include/cool_sd_bench.h."""
    rc = bench_lib().cool_sd_bench_row_stats(C.byref(params), _ptr(target), _ptr(target_uncond), _ptr(draft),
                                             _ptr(draft_uncond), _ptr(draft_tokens), _ptr(workspace),
                                             0 if workspace is None else workspace.numel() * workspace.element_size(),
                                             _stream(stream))
    if check and rc != 0:
        raise CoolSDError(rc, "cool_sd_bench_row_stats")
    return rc


# ------------------------------------------------------------------ conveniences (marshalling only)
def make_params(target, draft, *, has_bonus=None, top_k=0, cfg_scale=1.0, temperature=1.0,
                resample_mode=COOL_SD_RESAMPLE_OPT, omega_stride_b=0, flags=0):
    """cool_sd_params for [B, L(+1), V] / [B, L, V] torch tensors (innermost dimension contiguous)."""
    import torch
    B, L, V = draft.shape
    if has_bonus is None:
        has_bonus = int(target.shape[1] == L + 1)
    assert target.stride(2) == 1 and draft.stride(2) == 1
    dt = {torch.float32: COOL_SD_F32, torch.bfloat16: COOL_SD_BF16}[target.dtype]
    return CoolSDParams(B=B, L=L, V=V, dtype=dt, t_stride_b=target.stride(0), t_stride_l=target.stride(1),
                        d_stride_b=draft.stride(0), d_stride_l=draft.stride(1), omega_stride_b=omega_stride_b,
                        has_bonus=has_bonus, top_k=top_k, cfg_scale=cfg_scale, temperature=temperature,
                        resample_mode=resample_mode, flags=flags)


def verify_workload(w, omega, *, resample_mode=COOL_SD_RESAMPLE_OPT, workspace=None, diagnostics=True, flags=0):
    """Allocate outputs (torch, on the inputs' device), call cool_sd_verify once, return a dict of tensors."""
    import torch
    dev = w.target.device
    params = make_params(w.target, w.draft, top_k=w.top_k, cfg_scale=w.cfg_scale, temperature=w.temperature,
                         resample_mode=resample_mode, omega_stride_b=0 if omega.dim() == 1 else omega.stride(0),
                         flags=flags)
    if workspace is None:
        workspace = torch.empty(max(cool_sd_workspace_bytes(params), 256), dtype=torch.uint8, device=dev)
        cool_sd_workspace_init(workspace)
    B, L = w.B, w.L
    out = dict(accept_len=torch.full((B,), -7, dtype=torch.int32, device=dev),
               next_token=torch.full((B,), -7, dtype=torch.int32, device=dev),
               resid_mass=torch.full((B,), float("nan"), dtype=torch.float32, device=dev))
    if diagnostics:
        for k in ("p_tok", "q_tok", "f"):
            out[k] = torch.full((B, L), float("nan"), dtype=torch.float32, device=dev)
    cool_sd_verify(params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, omega,
                   w.u_accept, w.u_resample, out["accept_len"], out["next_token"], out.get("p_tok"),
                   out.get("q_tok"), out.get("f"), out["resid_mass"], workspace)
    return out


def verify_lantern_workload(w, neighbors, lam, *, resample_mode=COOL_SD_RESAMPLE_OPT, workspace=None):
    """Allocate outputs, call cool_sd_verify_lantern once ([V, k] int32 neighbour table on the device)."""
    import torch
    dev = w.target.device
    params = make_params(w.target, w.draft, top_k=w.top_k, cfg_scale=w.cfg_scale, temperature=w.temperature,
                         resample_mode=resample_mode)
    if workspace is None:
        workspace = torch.empty(max(cool_sd_workspace_bytes(params), 256), dtype=torch.uint8, device=dev)
    B, L = w.B, w.L
    out = dict(accept_len=torch.full((B,), -7, dtype=torch.int32, device=dev),
               next_token=torch.full((B,), -7, dtype=torch.int32, device=dev),
               resid_mass=torch.full((B,), float("nan"), dtype=torch.float32, device=dev),
               count=torch.full((B, L), -7, dtype=torch.int32, device=dev))
    for key in ("p_tok", "q_tok", "f", "p_agg"):
        out[key] = torch.full((B, L), float("nan"), dtype=torch.float32, device=dev)
    assert neighbors.dtype == torch.int32 and neighbors.is_contiguous() and neighbors.shape[0] == w.V
    cool_sd_verify_lantern(params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, neighbors,
                           neighbors.shape[1], lam, w.u_accept, w.u_resample, out["accept_len"], out["next_token"],
                           out["p_tok"], out["q_tok"], out["f"], out["resid_mass"], out["p_agg"], out["count"],
                           workspace)
    return out


def diagnostics_workload(w, omega, *, workspace=None):
    """Allocate alpha / beta (torch, on the inputs' device), call cool_sd_diagnostics once."""
    import torch
    dev = w.target.device
    params = make_params(w.target, w.draft, top_k=w.top_k, cfg_scale=w.cfg_scale, temperature=w.temperature,
                         omega_stride_b=0 if omega.dim() == 1 else omega.stride(0))
    if workspace is None:
        workspace = torch.empty(max(cool_sd_workspace_bytes(params), 256), dtype=torch.uint8, device=dev)
    alpha = torch.full((w.B, w.L), float("nan"), dtype=torch.float32, device=dev)
    beta = torch.full((w.B, w.L), float("nan"), dtype=torch.float32, device=dev)
    cool_sd_diagnostics(params, w.target, w.target_uncond, w.draft, w.draft_uncond, omega, alpha, beta, workspace)
    return alpha, beta
