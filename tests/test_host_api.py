"""Host-side logic of the C-ABI library (no GPU): symbols, schedule, validation, workspace sizing."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header_name):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    return set(re.findall(r"\b(cool_sd_[a-z_]+)\s*\(", header))


def _exported(path):
    """Dynamic symbols a library defines (any kind: functions, objects, kernel handles)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True).stdout
    return {ln.split()[-1] for ln in out.splitlines() if ln.strip()}


def test_library_exports_exactly_the_declared_symbols(P):
    """libcool_sd.so exports the entry points of include/cool_sd.h and nothing else: no benchmark
    switch, no kernel handle, no mutable object."""
    names = _declared("cool_sd.h")
    assert names == {"cool_sd_schedule", "cool_sd_workspace_bytes", "cool_sd_workspace_init", "cool_sd_verify",
                     "cool_sd_verify_noalloc", "cool_sd_verify_lantern", "cool_sd_verify_diagnostics",
                     "cool_sd_resample", "cool_sd_diagnostics", "cool_sd_early_exit_form", "cool_sd_strerror"}
    assert _exported(P.binding.LIB_PATH) == names
    assert _exported(P.binding.LIB_CHECKED_PATH) == names
    raw = C.CDLL(P.binding.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n


def test_bench_library_exports_its_header_on_top(P):
    extra = _declared("cool_sd_bench.h")
    assert extra == {"cool_sd_bench_row_stats", "cool_sd_bench_read_probe"}
    assert _exported(P.binding.LIB_BENCH_PATH) == _declared("cool_sd.h") | extra


def test_product_library_has_no_writable_state():
    """No file-scope mutable object in the product library: its .data and .bss hold nothing of the
    library's own (what remains is the HIP fat-binary registration the compiler emits, named
    __hip_*), so no call can depend on an earlier one."""
    import subprocess
    from paper_2601_09212_amd import binding
    out = subprocess.run(["nm", "--defined-only", binding.LIB_PATH], capture_output=True, text=True, check=True).stdout
    own = []
    for ln in out.splitlines():
        parts = ln.split()
        if len(parts) == 3 and parts[1] in "bBdD":
            name = parts[2]
            if name.startswith("_") and not name.startswith("_Z"):
                continue          # C runtime and HIP registration bookkeeping
            if name.startswith("_Z") and "kernel" in name:
                continue          # kernel handles: constant after the loader's relocation
            if "scratch" in name:
                continue          # cool_sd_verify_noalloc: the static workspace's host-side stand-in and
                                  # its per-device address, written once to a value that never changes
            own.append(ln)
    assert not own, own


def test_struct_layout_matches_header(P):
    # 4 x int32, 5 x int64, 2 x int32, 2 x float, 2 x int32
    assert C.sizeof(P.CoolSDParams) == 16 + 40 + 8 + 8 + 8


@pytest.mark.parametrize("L,delta", [(1, 1.0), (4, 1.1), (8, 2.0), (16, 4.0), (64, 1.1)])
def test_schedule_matches_oracle(P, oracle, L, delta):
    for kind, param in ((P.COOL_SD_SCHED_EXP, 0.7), (P.COOL_SD_SCHED_EXP, 0.05), (P.COOL_SD_SCHED_UNIFORM, 0.0),
                        (P.COOL_SD_SCHED_LINEAR, float(max(L, 8)))):
        got = P.cool_sd_schedule(kind, L, delta, param)
        want = oracle.schedule(kind, L, np.float32(delta), np.float32(param))
        assert got.dtype == np.float32
        np.testing.assert_allclose(got, want, rtol=2e-7, atol=0)
    assert abs(P.cool_sd_schedule(P.COOL_SD_SCHED_EXP, L, delta, 0.7).astype(np.float64).sum() - delta * L) < 1e-5 * L


def test_schedule_rejects_bad_arguments(P):
    for args in ((P.COOL_SD_SCHED_EXP, 4, 1.0, 0.0), (P.COOL_SD_SCHED_EXP, 0, 1.0, 0.7), (7, 4, 1.0, 0.7),
                 (P.COOL_SD_SCHED_LINEAR, 9, 1.0, 8.0), (P.COOL_SD_SCHED_EXP, 4, -1.0, 0.7),
                 (P.COOL_SD_SCHED_EXP, 4, float("nan"), 0.7)):
        with pytest.raises(P.CoolSDError) as e:
            P.cool_sd_schedule(*args)
        assert e.value.code == P.binding.COOL_SD_EINVAL


def _params(P, **kw):
    base = dict(B=4, L=8, V=16384, dtype=P.COOL_SD_BF16, t_stride_b=9 * 16384, t_stride_l=16384,
                d_stride_b=8 * 16384, d_stride_l=16384, omega_stride_b=0, has_bonus=1, top_k=0,
                cfg_scale=1.0, temperature=1.0, resample_mode=0, flags=0)
    base.update(kw)
    return P.CoolSDParams(**base)


def test_workspace_bytes_and_invalid_params(P):
    small = P.cool_sd_workspace_bytes(_params(P))
    assert 0 < small < 1 << 20
    big = P.cool_sd_workspace_bytes(_params(P, V=262144, t_stride_l=262144, d_stride_l=262144,
                                            t_stride_b=9 * 262144, d_stride_b=8 * 262144))
    assert big > small
    for bad in (dict(B=0), dict(V=0), dict(dtype=3), dict(top_k=-1), dict(top_k=16385), dict(temperature=0.0),
                dict(temperature=float("inf")), dict(cfg_scale=float("nan")), dict(resample_mode=3),
                dict(flags=8), dict(flags=-1), dict(t_stride_b=-1)):
        assert P.cool_sd_workspace_bytes(_params(P, **bad)) == 0, bad
    # L out of range is still a valid stand-alone resample shape (L is ignored there)
    assert P.cool_sd_workspace_bytes(_params(P, L=0)) > 0


def test_verify_validates_before_touching_the_gpu(P):
    """Argument errors come back as status codes; nothing is launched (this runs without a GPU)."""
    lib = P.binding.lib()
    fake = C.c_void_p(0x1000)          # never dereferenced on the host
    null = C.c_void_p(0)

    def call(params, target=fake, draft=fake, tu=null, du=null, ws=null, ws_bytes=0):
        return lib.cool_sd_verify(C.byref(params), target, tu, draft, du, fake, fake, fake, fake, fake, fake,
                                  null, null, null, null, ws, ws_bytes, null)

    E = P.binding
    assert call(_params(P, L=0)) == E.COOL_SD_EINVAL
    assert call(_params(P, L=5000)) == E.COOL_SD_EINVAL
    assert call(_params(P), target=null) == E.COOL_SD_EINVAL
    assert call(_params(P), tu=fake) == E.COOL_SD_EINVAL               # guidance needs both unconditional tensors
    assert call(_params(P, has_bonus=2)) == E.COOL_SD_EINVAL
    assert call(_params(P)) == E.COOL_SD_EWORKSPACE                    # no workspace
    assert call(_params(P), ws=C.c_void_p(0x1004), ws_bytes=1 << 20) == E.COOL_SD_EWORKSPACE   # misaligned
    assert call(_params(P), ws=C.c_void_p(0x1000), ws_bytes=16) == E.COOL_SD_EWORKSPACE         # too small
    # top-k on rows longer than one workgroup (65536 logits) needs the radix-select state in the workspace
    long_rows = dict(V=70000, t_stride_l=70000, d_stride_l=70000, t_stride_b=9 * 70000, d_stride_b=8 * 70000)
    plain = P.cool_sd_workspace_bytes(_params(P, **long_rows))
    with_k = P.cool_sd_workspace_bytes(_params(P, top_k=5, **long_rows))
    assert with_k >= plain + 4 * 17 * 2048 * 4
    assert call(_params(P, top_k=5, **long_rows), ws=C.c_void_p(0x1000), ws_bytes=plain) == E.COOL_SD_EWORKSPACE
    assert lib.cool_sd_verify(None, fake, null, fake, null, fake, fake, fake, fake, fake, fake, null, null, null,
                              null, null, 0, null) == E.COOL_SD_EINVAL
    # stand-alone resample
    r = lib.cool_sd_resample(C.byref(_params(P)), null, null, fake, null, fake, fake, fake, null, null, 0, null)
    assert r == E.COOL_SD_EINVAL
    r = lib.cool_sd_resample(C.byref(_params(P)), fake, null, fake, null, null, fake, fake, null, null, 0, null)
    assert r == E.COOL_SD_EINVAL                                       # draft rows need omega
    # diagnostics
    d = lambda params, t=fake, om=fake, out=fake, ws=null, n=0: lib.cool_sd_diagnostics(
        C.byref(params), t, null, fake, null, om, out, fake, ws, n, null)
    assert d(_params(P), t=null) == E.COOL_SD_EINVAL
    assert d(_params(P), om=null) == E.COOL_SD_EINVAL
    assert d(_params(P), out=null) == E.COOL_SD_EINVAL
    assert d(_params(P)) == E.COOL_SD_EWORKSPACE
    assert d(_params(P), ws=C.c_void_p(0x1000), n=16) == E.COOL_SD_EWORKSPACE
    # verify and diagnostics in one call
    def both(params, alpha=fake, beta=fake, target=fake, ws=null, n=0):
        return lib.cool_sd_verify_diagnostics(C.byref(params), target, null, fake, null, fake, fake, fake, fake, fake,
                                              fake, null, null, null, null, alpha, beta, ws, n, null)
    assert both(_params(P), alpha=null) == E.COOL_SD_EINVAL
    assert both(_params(P), beta=null) == E.COOL_SD_EINVAL
    assert both(_params(P), target=null) == E.COOL_SD_EINVAL
    assert both(_params(P, L=0)) == E.COOL_SD_EINVAL
    assert both(_params(P)) == E.COOL_SD_EWORKSPACE
    assert both(_params(P), ws=C.c_void_p(0x1000), n=16) == E.COOL_SD_EWORKSPACE
    assert both(_params(P, top_k=5), ws=C.c_void_p(0x1000), n=16) == E.COOL_SD_EWORKSPACE     # the two-pass form
    # the benchmark library's entry points
    bl = P.binding.bench_lib()
    assert bl.cool_sd_bench_read_probe(null, 16, null, 0, fake, 64, null) == E.COOL_SD_EINVAL
    assert bl.cool_sd_bench_read_probe(fake, 24, null, 0, fake, 64, null) == E.COOL_SD_EINVAL
    assert bl.cool_sd_bench_read_probe(fake, 1 << 20, null, 0, fake, 64, null) == E.COOL_SD_EWORKSPACE
    assert bl.cool_sd_bench_row_stats(C.byref(_params(P)), null, null, fake, null, fake, null, 0, null) == E.COOL_SD_EINVAL
    assert bl.cool_sd_bench_row_stats(C.byref(_params(P)), fake, null, fake, null, fake, null, 0, null) == E.COOL_SD_EWORKSPACE
    # the allocation-free entry point: arguments first, then the size limit, both before any device call
    na = lambda params, t=fake: lib.cool_sd_verify_noalloc(C.byref(params), t, null, fake, null, fake, fake, fake, fake,
                                                           fake, fake, null, null, null, null, null)
    assert na(_params(P), t=null) == E.COOL_SD_EINVAL
    assert na(_params(P, L=0)) == E.COOL_SD_EINVAL
    huge = dict(B=4096, L=64, V=262144, t_stride_l=262144, d_stride_l=262144, t_stride_b=65 * 262144, d_stride_b=64 * 262144)
    assert na(_params(P, **huge)) == E.COOL_SD_ETOOLARGE
    assert "static" in P.cool_sd_strerror(E.COOL_SD_ETOOLARGE)
    # the checked mode is an option bit of the verify calls; unknown bits stay errors
    assert call(_params(P, flags=E.COOL_SD_FLAG_CHECK_TOKENS)) == E.COOL_SD_EWORKSPACE
    assert call(_params(P, flags=E.COOL_SD_FLAG_CHECK_TOKENS | E.COOL_SD_FLAG_EARLY_EXIT)) == E.COOL_SD_EWORKSPACE
    assert call(_params(P, flags=8)) == E.COOL_SD_EINVAL
    # aggregated acceptance over neighbours
    def lan(params, nbr=fake, k=10, lam=2.0, ws=null, n=0):
        return lib.cool_sd_verify_lantern(C.byref(params), fake, null, fake, null, fake, nbr, k, C.c_float(lam),
                                          fake, fake, fake, fake, null, null, null, null, null, null, ws, n, null)
    assert lan(_params(P), nbr=null) == E.COOL_SD_EINVAL
    assert lan(_params(P), k=0) == E.COOL_SD_EINVAL
    assert lan(_params(P), lam=-1.0) == E.COOL_SD_EINVAL
    assert lan(_params(P), lam=float("inf")) == E.COOL_SD_EINVAL
    assert lan(_params(P)) == E.COOL_SD_EWORKSPACE
    assert lan(_params(P, resample_mode=E.COOL_SD_RESAMPLE_LANTERN)) == E.COOL_SD_EWORKSPACE
    assert lan(_params(P, resample_mode=3)) == E.COOL_SD_EINVAL
    assert call(_params(P, resample_mode=E.COOL_SD_RESAMPLE_LANTERN)) == E.COOL_SD_EINVAL   # only with neighbours
    assert P.cool_sd_workspace_bytes(_params(P, resample_mode=E.COOL_SD_RESAMPLE_LANTERN)) > 0
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert isinstance(P.cool_sd_strerror(code), str) and P.cool_sd_strerror(code)


def test_early_exit_form_query(P):
    """cool_sd_early_exit_form names the form a verify call takes under COOL_SD_FLAG_EARLY_EXIT, so that
    the fall-back to reading every row is visible to the caller (host logic only)."""
    E = P
    form = lambda aligned=True, **kw: P.cool_sd_early_exit_form(_params(P, **kw), aligned)
    ee = E.COOL_SD_FLAG_EARLY_EXIT
    assert form(V=16384) == E.COOL_SD_EARLY_EXIT_NONE                              # flag clear
    assert form(V=16384, flags=ee) == E.COOL_SD_EARLY_EXIT_SEQUENCE
    assert form(V=16384, flags=ee | E.COOL_SD_FLAG_EXACT_DRAW) == E.COOL_SD_EARLY_EXIT_SEQUENCE
    assert form(False, V=16384, flags=ee) == E.COOL_SD_EARLY_EXIT_NONE             # unaligned short rows
    assert form(V=16383, flags=ee) == E.COOL_SD_EARLY_EXIT_NONE                    # V not a multiple of the vector
    assert form(V=16384, L=1025, flags=ee) == E.COOL_SD_EARLY_EXIT_NONE
    assert form(V=16384, top_k=10, flags=ee) == E.COOL_SD_EARLY_EXIT_NONE
    assert form(V=16385, flags=ee) == E.COOL_SD_EARLY_EXIT_ROUNDS
    assert form(False, V=262144, flags=ee) == E.COOL_SD_EARLY_EXIT_ROUNDS          # any alignment
    assert form(V=262144, dtype=E.COOL_SD_F32, flags=ee) == E.COOL_SD_EARLY_EXIT_ROUNDS
    assert form(V=524288, flags=ee) == E.COOL_SD_EARLY_EXIT_ROUNDS
    assert form(V=524289, flags=ee) == E.COOL_SD_EARLY_EXIT_NONE                   # more than 64 statistics chunks
    assert form(V=262144, top_k=5, flags=ee) == E.COOL_SD_EARLY_EXIT_NONE
    with pytest.raises(P.CoolSDError):
        P.cool_sd_early_exit_form(_params(P, V=0, flags=ee), True)


def test_binding_fails_loudly_without_library(P, monkeypatch):
    from paper_2601_09212_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libcool_sd.so")
    with pytest.raises(ImportError):
        binding.lib()


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2601_09212_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)


def test_header_is_plain_c_and_the_example_builds(tmp_path):
    """include/cool_sd.h must be usable from C (the boundary is a C ABI): the example program is
    compiled with gcc -std=c11 -Wall -Werror against the built library, and without arguments it
    prints its usage before touching the GPU."""
    import subprocess
    from paper_2601_09212_amd import build as hb
    if not os.path.exists(hb.LIB):
        pytest.skip("library not built")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    exe = str(tmp_path / "verify_example")
    cmd = ["gcc", "-O1", "-Wall", "-Werror", "-std=c11", "-pedantic", hb.EXAMPLE_SRC, "-D__HIP_PLATFORM_AMD__",
           "-isystem", os.path.join(rocm, "include"), "-I", os.path.join(hb.ROOT, "include"), "-L", hb.PKG, "-lcool_sd",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm", "-Wl,-rpath," + hb.PKG,
           "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert r.returncode == 1 and "usage" in r.stderr
