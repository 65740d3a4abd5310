"""The C ABI used from plain C (no Python binding in the way): the example program under
paper_2601_09212_amd/examples generates its own seeded inputs, calls cool_sd_schedule,
cool_sd_workspace_bytes, cool_sd_workspace_init and cool_sd_verify, and dumps inputs and outputs;
the oracle is then run on those inputs.  A mismatch between include/cool_sd.h and the ctypes
mirror of its structures would show up as a disagreement between this test and the others."""
import os
import subprocess

import numpy as np
import pytest
import torch

from tests.parity_util import compare_verify
from workloads.synth import Workload

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BIN = os.path.join(ROOT, "paper_2601_09212_amd", "examples", "verify_example")


@pytest.mark.parametrize("B,L,V,seed", [(4, 4, 16384, 1), (3, 5, 4100, 2), (2, 3, 20000, 3)])
def test_c_program_against_oracle(oracle, tmp_path, B, L, V, seed):
    assert os.path.exists(BIN), "build first: python -m paper_2601_09212_amd.build"
    dump = str(tmp_path / "dump.bin")
    print("case", B, L, V, seed, flush=True)
    r = subprocess.run([BIN, str(B), str(L), str(V), str(seed), dump], capture_output=True, text=True, timeout=100)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0
    assert r.stdout.count("sequence ") == B
    raw = np.fromfile(dump, dtype=np.uint8)
    head = raw[:16].view(np.int32)
    assert tuple(head) == (B, L, V, 1)
    off = 16

    def take(shape, dtype):
        nonlocal off
        n = int(np.prod(shape)) * 4
        a = raw[off:off + n].view(dtype).reshape(shape).copy()
        off += n
        return a
    target, draft = take((B, L + 1, V), np.float32), take((B, L, V), np.float32)
    tokens, omega = take((B, L), np.int32), take((L,), np.float32)
    ua, ur = take((B, L), np.float32), take((B,), np.float32)
    gpu = dict(accept_len=take((B,), np.int32), next_token=take((B,), np.int32), p_tok=take((B, L), np.float32),
               q_tok=take((B, L), np.float32), f=take((B, L), np.float32), resid_mass=take((B,), np.float32))
    assert off == raw.size
    # the program's own schedule call: Eq. sdar with delta = 1.1, nu = 0.7
    wts = np.exp(-0.7 * np.arange(1, L + 1))
    np.testing.assert_allclose(omega, 1.1 * L * wts / wts.sum(), rtol=1e-6)
    t = torch.from_numpy
    w = Workload(cfg=0, B=B, L=L, V=V, dtype="f32", target=t(target), draft=t(draft), draft_tokens=t(tokens),
                 u_accept=t(ua), u_resample=t(ur))
    st = compare_verify(oracle, w, omega, gpu)
    print(st, flush=True)
    assert 0 < gpu["accept_len"].sum() < B * L          # neither everything rejected nor everything accepted
