#!/usr/bin/env python3
"""Benchmark of the Cool-SD verify-and-resample hot path on one MI355X.

A step is one cool_sd_verify call (softmax statistics of every target and draft row, relaxed
accept test, first rejection, one draw from the optimal resampling law) on one batch of
synthetic input that is already resident in HBM.  The workload is configuration 5 of the
benchmark list, the largest one (B=128, L=8, V=262144, bf16: 1.14 GB of logits per call); steps
cycle through a pool of distinct batches and are replayed from a HIP graph so that the host's
launch cost does not hide the device time.

Prints ONE JSON line: verified draft tokens per second, with
  roofline      HBM, for the dominant kernel (row_stats_kernel, the pass that reads every logit):
                algorithmic bytes of one launch / its average duration, measured live with events
                on the launch stream around graph replays of that kernel alone
                (cool_sd_bench_row_stats of the benchmark library), over the same batches right
                after the timed region; `whole_call_frac` is the same ratio for the whole step;
                `traffic` is read from the rocprofv3 counter summary under profiles/
  cpu_baseline  the fp64 CPU oracle timed on a bounded sample of the same batches.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
_HOST_THREADS = None


def measured_traffic(workload, early_exit=False, per_call=False):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 counter summary of
    this workload (profiles/verify_<workload>_rocprofv3.md, written by
    paper_2601_09212_amd/profile_summary.py from FETCH_SIZE / WRITE_SIZE runs): the line
    `traffic_bytes_per_launch: <kernel> <bytes>` (per_call: `traffic_bytes_per_call: <bytes>`, all
    launches of one library call).  None when no summary holds one."""
    name = "verify_early_exit_%s_rocprofv3.md" % workload if early_exit else "verify_%s_rocprofv3.md" % workload
    try:
        text = open(os.path.join(ROOT, "profiles", name)).read()
    except OSError:
        return None
    if per_call:
        m = re.search(r"^traffic_bytes_per_call:\s*([0-9.eE+]+)\s*$", text, flags=re.M)
        return float(m.group(1)) if m else None
    m = re.search(r"^traffic_bytes_per_launch:\s*(\S+)\s+([0-9.eE+]+)\s*$", text, flags=re.M)
    return float(m.group(2)) if m else None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=600)
    ap.add_argument("--warmup", type=int, default=60)
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--vocab", type=int, default=0, help="the workload's recipe at another vocabulary size (e.g. 65536)")
    ap.add_argument("--batch", type=int, default=0, help="the workload's recipe with another number of sequences")
    ap.add_argument("--top-k", type=int, default=0, help="the workload's recipe with this top-k (guided recipe: cfg3)")
    ap.add_argument("--launch", default="graph", choices=["graph", "direct"])
    ap.add_argument("--pool-mb", type=float, default=0.0,
                    help="distinct input batches cycled, total size (default: 3400 for configurations 4-5, else 600)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="time budget of the CPU oracle sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-others", action="store_true",
                    help="also time the CPU oracle on the other workloads (a few seconds each; for the results table)")
    ap.add_argument("--others", action="store_true", default=True,
                    help="also time the other four configurations (extra key `other_workloads`; on by default, a "
                         "few seconds)")
    ap.add_argument("--variants", action="store_true",
                    help="with --others: also configuration 4's recipe at B = 2048 and the recipes of configurations "
                         "2 and 3 at a 65536-token vocabulary")
    ap.add_argument("--no-others", dest="others", action="store_false", help="time the named workload only")
    ap.add_argument("--early-exit", action="store_true",
                    help="time the early-exit form (COOL_SD_FLAG_EARLY_EXIT) instead of the all-rows form; the "
                         "roofline object then refers to the single kernel and to the bytes it actually needs")
    ap.add_argument("--diagnostics", action="store_true",
                    help="also time cool_sd_diagnostics (alpha, beta of every position) on the timed workloads")
    ap.add_argument("--lantern", action="store_true",
                    help="also time cool_sd_verify_lantern (k = 10 synthetic neighbours, lambda = 2, G* resampling) on "
                         "the timed workloads")
    ap.add_argument("--concurrent", action="store_true",
                    help="also time the same steps issued on two streams (independent batches, each stream with its "
                         "own workspace and outputs), so that one call's per-sequence kernel overlaps the next "
                         "call's statistics kernel; reported as extra keys, `value` stays the one-stream figure")
    ap.add_argument("--draft-sampler", action="store_true",
                    help="also time the drafting stage's sampling step (cool_sd_resample on the draft rows alone: one "
                         "call draws one token for each of the B sequences); extra key `draft_sampler`")
    ap.add_argument("--delta-sweep", action="store_true",
                    help="also report acceptance statistics of the timed workload under the lossless baseline and "
                         "the annealed schedule at delta = 1, 1.1, 2, 3, 4 (accepted length, its prediction, "
                         "estimate of the total-variation bound); extra key `delta_sweep`")
    ap.add_argument("--kernel-samples", type=int, default=200, help="instrumented calls for the per-kernel time")
    ap.add_argument("--counter-run", action="store_true",
                    help="for rocprofv3 --pmc: a plain device copy of known size (the counters' reference), then "
                         "--steps direct calls; nothing is timed or printed as a result")
    return ap.parse_args()


class Runner:
    """Pool of resident batches of one configuration plus everything a verify call needs."""

    def __init__(self, pkg, torch, cfg, pool_mb, max_pool=64, flags=0, B=None, V=None, top_k=None):
        from workloads import make_workload as mk
        over = {k: v for k, v in (("B", B), ("V", V), ("top_k", top_k)) if v}
        make_workload = (lambda c, **kw: mk(c, **over, **kw)) if over else mk
        self.pkg, self.torch, self.cfg = pkg, torch, cfg
        w0 = make_workload(cfg, device="cuda", call=0)
        self.bytes_per_step = w0.algorithmic_bytes()
        n = int(min(max_pool, max(2, -(-int(pool_mb * 1e6) // self.bytes_per_step))))
        self.pool = [w0] + [make_workload(cfg, device="cuda", call=c) for c in range(1, n)]
        self.B, self.L, self.V = w0.B, w0.L, w0.V
        self.omega_np = pkg.cool_sd_schedule(pkg.COOL_SD_SCHED_EXP, w0.L, w0.delta, w0.nu)
        self.omega = torch.from_numpy(self.omega_np).cuda()
        self.params = pkg.make_params(w0.target, w0.draft, top_k=w0.top_k, cfg_scale=w0.cfg_scale,
                                      temperature=w0.temperature, flags=flags)
        self.ws = torch.empty(max(pkg.cool_sd_workspace_bytes(self.params), 256), dtype=torch.uint8, device="cuda")
        pkg.cool_sd_workspace_init(self.ws)
        self.accept_len = torch.zeros(self.B, dtype=torch.int32, device="cuda")
        self.next_token = torch.zeros(self.B, dtype=torch.int32, device="cuda")
        self.graph = None

    def step(self, i):
        w = self.pool[i % len(self.pool)]
        self.pkg.cool_sd_verify(self.params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens,
                                self.omega, w.u_accept, w.u_resample, self.accept_len, self.next_token,
                                None, None, None, None, self.ws)

    def capture(self):
        """One HIP graph holding one pass over the pool (len(pool) steps)."""
        torch = self.torch
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            for i in range(len(self.pool)):
                self.step(i)
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(len(self.pool)):
                self.step(i)
        self.graph = g
        self.part_graphs = {}

    def _partial(self, k):
        """A graph of the first k < len(pool) steps of a pass (for step counts that are not whole passes)."""
        if k not in self.part_graphs:
            torch = self.torch
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for i in range(k):
                    self.step(i)
            self.part_graphs[k] = g
        return self.part_graphs[k]

    def run(self, steps, launch):
        """Enqueue exactly `steps` steps: whole pool passes plus, in graph mode, one replay of a
        shorter graph for the remainder (captured beforehand by prepare())."""
        if launch == "graph":
            n = len(self.pool)
            for _ in range(steps // n):
                self.graph.replay()
            if steps % n:
                self.part_graphs[steps % n].replay()
            return steps
        for i in range(steps):
            self.step(i)
        return steps

    def prepare(self, counts, launch):
        if launch == "graph":
            if self.graph is None:
                self.capture()
            for c in counts:
                if c % len(self.pool):
                    self._partial(c % len(self.pool))

    def time(self, steps, warmup, launch):
        torch = self.torch
        self.prepare((steps, warmup), launch)
        self.run(warmup, launch)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        done = self.run(steps, launch)
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return done, wall, e0.elapsed_time(e1) * 1e-3


    def time_two_streams(self, passes=8):
        """Throughput when the pool's batches (independent of each other) are verified on two streams:
        even steps on one, odd steps on the other, each with its own workspace and outputs, captured
        as one graph with a fork and a join.  Returns seconds per step."""
        pkg, torch = self.pkg, self.torch
        ws2 = torch.empty_like(self.ws)
        al2, nt2 = torch.zeros_like(self.accept_len), torch.zeros_like(self.next_token)
        side = torch.cuda.Stream()

        def body():
            main = torch.cuda.current_stream()
            side.wait_stream(main)
            for i, w in enumerate(self.pool):
                if i % 2 == 0:
                    self.step(i)
                else:
                    with torch.cuda.stream(side):
                        pkg.cool_sd_verify(self.params, w.target, w.target_uncond, w.draft, w.draft_uncond,
                                           w.draft_tokens, self.omega, w.u_accept, w.u_resample, al2, nt2,
                                           None, None, None, None, ws2)
            main.wait_stream(side)
        warm = torch.cuda.Stream()
        warm.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(warm):
            body()
        torch.cuda.current_stream().wait_stream(warm)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            body()
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(passes):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / (passes * len(self.pool))

    def _replay_time(self, issue, n):
        """Seconds per pool batch of `issue` (one pass over the pool), replayed from a HIP graph and
        bracketed by events on the launch stream (torch's current stream, the one the binding
        hands to the library)."""
        torch = self.torch
        issue()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            issue()
        reps = max(2, -(-n // len(self.pool)))
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / (reps * len(self.pool))

    def read_probe_time(self, n):
        """Yardstick for the statistics kernel: a plain streaming read of the same logit tensors in one
        launch of the same shape (cool_sd_bench_read_probe), replayed back to back from a graph
        exactly as kernel_time() replays the statistics kernel.  Guided workloads need two launches
        (conditional pair, unconditional pair).  Returns seconds per step and launches per step."""
        pkg, torch = self.pkg, self.torch
        out = torch.empty(self.bytes_per_step // 8192 + 64, dtype=torch.int32, device="cuda")

        def issue():
            for w in self.pool:
                pkg.cool_sd_bench_read_probe(w.target, w.draft, out)
                if w.target_uncond is not None:
                    pkg.cool_sd_bench_read_probe(w.target_uncond, w.draft_uncond, out)
        return self._replay_time(issue, n), 2 if self.pool[0].target_uncond is not None else 1

    def kernel_time(self, n):
        """Average duration of the statistics kernel over the pool: the benchmark library launches that
        kernel alone (cool_sd_bench_row_stats: same grid, chunking and loads as in the verify call),
        one launch per pool batch is captured into a graph, and events on the launch stream bracket
        replays of it -- back-to-back launches, so the figure is the kernel's duration plus the gap
        between two launches."""
        pkg = self.pkg

        def issue():
            for w in self.pool:
                pkg.cool_sd_bench_row_stats(self.params, w.target, w.target_uncond, w.draft, w.draft_uncond,
                                            w.draft_tokens, self.ws)
        return self._replay_time(issue, n)

    def direct_call_times(self, n):
        """Mean and median duration of one direct (not graph-replayed) verify call, each bracketed by
        its own pair of events on the launch stream; includes the dispatch latency of a lone call."""
        torch = self.torch
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for i in range(5):
            self.step(i)
        torch.cuda.synchronize()
        for i, (e0, e1) in enumerate(ev):
            e0.record()
            self.step(i)
            e1.record()
            torch.cuda.synchronize()
        t = sorted(e0.elapsed_time(e1) * 1e-3 for e0, e1 in ev)
        return sum(t) / len(t), t[len(t) // 2]


def run_diagnostics(r, n):
    """n direct cool_sd_diagnostics calls, then n cool_sd_verify_diagnostics calls, cycling through the
    pool (for profiler runs)."""
    pkg, torch = r.pkg, r.torch
    alpha = torch.empty((r.B, r.L), dtype=torch.float32, device="cuda")
    beta = torch.empty_like(alpha)
    for i in range(n):
        w = r.pool[i % len(r.pool)]
        pkg.cool_sd_diagnostics(r.params, w.target, w.target_uncond, w.draft, w.draft_uncond, r.omega, alpha, beta,
                                r.ws)
    for i in range(n):
        w = r.pool[i % len(r.pool)]
        pkg.cool_sd_verify_diagnostics(r.params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens,
                                       r.omega, w.u_accept, w.u_resample, r.accept_len, r.next_token, None, None,
                                       None, None, alpha, beta, r.ws)
    torch.cuda.synchronize()


def time_diagnostics(r, passes=6):
    """Average duration of one cool_sd_diagnostics call over the pool (direct launches, events on the
    launch stream).  Algorithmic bytes: the 2 B L drafted rows, once."""
    pkg, torch = r.pkg, r.torch
    alpha = torch.empty((r.B, r.L), dtype=torch.float32, device="cuda")
    beta = torch.empty_like(alpha)

    def one(i):
        w = r.pool[i % len(r.pool)]
        pkg.cool_sd_diagnostics(r.params, w.target, w.target_uncond, w.draft, w.draft_uncond, r.omega, alpha, beta,
                                r.ws)
    for i in range(len(r.pool)):
        one(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = passes * len(r.pool)
    e0.record()
    for i in range(n):
        one(i)
    e1.record()
    torch.cuda.synchronize()
    sec = e0.elapsed_time(e1) * 1e-3 / n
    w0 = r.pool[0]
    nbytes = 2 * r.B * r.L * r.V * w0.target.element_size() * (2 if w0.target_uncond is not None else 1)

    # the verify call and the diagnostics in one call (one pass over the logits for short rows
    # without top-k), replayed from a graph like the timed verify steps
    def both(i):
        w = r.pool[i % len(r.pool)]
        pkg.cool_sd_verify_diagnostics(r.params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens,
                                       r.omega, w.u_accept, w.u_resample, r.accept_len, r.next_token, None, None,
                                       None, None, alpha, beta, r.ws)
    for i in range(len(r.pool)):
        both(i)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(len(r.pool)):
            both(i)
    g.replay()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(passes):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    sec_both = e0.elapsed_time(e1) * 1e-3 / (passes * len(r.pool))
    return {"us_per_call": sec * 1e6, "algorithmic_bytes": nbytes, "GBps": nbytes / sec / 1e9,
            "frac": nbytes / sec / 1e9 / HBM_PEAK_GBS,
            "verify_and_diagnostics_us_per_call": sec_both * 1e6,
            "verify_and_diagnostics_GBps": r.bytes_per_step / sec_both / 1e9}


def run_lantern(r, n, k=10, lam=2.0):
    """n direct cool_sd_verify_lantern calls cycling through the pool (for profiler runs)."""
    from workloads import make_neighbor_table
    pkg, torch = r.pkg, r.torch
    nbr = make_neighbor_table(r.V, k, device="cuda", seed=11)
    for i in range(n):
        w = r.pool[i % len(r.pool)]
        pkg.cool_sd_verify_lantern(r.params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, nbr,
                                   k, lam, w.u_accept, w.u_resample, r.accept_len, r.next_token, None, None, None,
                                   None, None, None, r.ws)
    torch.cuda.synchronize()


def time_lantern(r, k=10, lam=2.0, passes=6):
    """Average duration of one cool_sd_verify_lantern call over the pool, replayed from a HIP graph.
    The neighbour table is synthetic ([V, k] distinct random tokens per row)."""
    from workloads import make_neighbor_table
    pkg, torch = r.pkg, r.torch
    nbr = make_neighbor_table(r.V, k, device="cuda", seed=11)
    w0 = r.pool[0]
    params = pkg.make_params(w0.target, w0.draft, top_k=w0.top_k, cfg_scale=w0.cfg_scale, temperature=w0.temperature)

    def one(i):
        w = r.pool[i % len(r.pool)]
        pkg.cool_sd_verify_lantern(params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, nbr, k,
                                   lam, w.u_accept, w.u_resample, r.accept_len, r.next_token, None, None, None, None,
                                   None, None, r.ws)
    for i in range(len(r.pool)):
        one(i)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(len(r.pool)):
            one(i)
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(passes):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    sec = e0.elapsed_time(e1) * 1e-3 / (passes * len(r.pool))
    return {"us_per_call": sec * 1e6, "k": k, "lambda": lam, "tokens_per_s": r.B * r.L / sec,
            "mean_accept_len": float(r.accept_len.float().mean().item())}


def time_draft_sampler(r, passes=20):
    """The drafting stage's sampling step on the same tensors (Algorithm 1, drafting loop): one
    cool_sd_resample call draws x~ ~ q for the B sequences of a batch at one position (guidance,
    temperature and top-k as configured, then an inverse-CDF draw; no target involved).  The L
    positions of every pool batch are issued in turn and replayed from a HIP graph."""
    torch, pkg = r.torch, r.pkg
    w0 = r.pool[0]
    rows = lambda w, i: (w.draft[:, i:i + 1], None if w.draft_uncond is None else w.draft_uncond[:, i:i + 1])
    d0, _ = rows(w0, 0)
    params = pkg.make_params(d0, d0, has_bonus=0, top_k=w0.top_k, cfg_scale=w0.cfg_scale, temperature=w0.temperature)
    ws = torch.empty(max(pkg.cool_sd_workspace_bytes(params), 256), dtype=torch.uint8, device="cuda")
    tok = torch.empty(r.B, dtype=torch.int32, device="cuda")

    def issue():
        for w in r.pool:
            for i in range(r.L):
                d, du = rows(w, i)
                pkg.cool_sd_resample(params, d, du, None, None, None, w.u_resample, tok, None, ws)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        issue()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        issue()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(passes):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    n = passes * len(r.pool) * r.L
    sec = e0.elapsed_time(e1) * 1e-3 / n
    nbytes = r.B * r.V * w0.draft.element_size() * (2 if w0.draft_uncond is not None else 1)
    return {"us_per_call": sec * 1e6, "draft_tokens_per_s": r.B / sec, "rows_per_call": r.B,
            "algorithmic_bytes_per_call": nbytes, "GBps": nbytes / sec / 1e9, "calls_timed": n}


def delta_sweep(r, deltas=(1.0, 1.1, 2.0, 3.0, 4.0)):
    """Acceptance statistics of the timed workload's pool under the relaxation budgets of the paper's
    speed/quality sweep: the lossless baseline (uniform schedule, delta = 1), the annealed
    schedules (exponential, Eq. sdar; linear, schedule ablation) and the uniform relaxation at each delta.  Per setting, over all sequences of the pool: the realised mean
    accepted length, its prediction sum_i prod_{j<=i} f_j (Eq. token_exp, one drafted path per
    sequence) and the same-path estimate of Theorem 2's bound with G*,
    sum_i prod_{k<i} f_k * beta_i, with beta_i from cool_sd_diagnostics.  Kernel time does not
    depend on delta (every row is read whatever the outcome), so nothing is timed here."""
    torch, pkg = r.torch, r.pkg
    w0 = r.pool[0]
    params = pkg.make_params(w0.target, w0.draft, top_k=w0.top_k, cfg_scale=w0.cfg_scale, temperature=w0.temperature)
    f = torch.empty((r.B, r.L), dtype=torch.float32, device="cuda")
    alpha, beta = torch.empty_like(f), torch.empty_like(f)
    out = []
    ell = float(max(8, r.L))          # the paper's ablation uses ell = 8; the slope must not cross zero inside the window
    settings = [(pkg.COOL_SD_SCHED_UNIFORM, "uniform", 1.0, 0.0)]                      # lossless baseline
    settings += [(pkg.COOL_SD_SCHED_EXP, "exp", d, w0.nu) for d in deltas]              # annealed, Eq. sdar
    settings += [(pkg.COOL_SD_SCHED_LINEAR, "linear", d, ell) for d in deltas]          # annealed, linear decay
    settings += [(pkg.COOL_SD_SCHED_UNIFORM, "uniform", d, 0.0) for d in deltas if d != 1.0]   # uniform relaxation
    for kind, name, delta, param in settings:
        om = torch.from_numpy(pkg.cool_sd_schedule(kind, r.L, delta, param)).cuda()
        tau_sum = pred_sum = bound_sum = 0.0
        for w in r.pool:
            pkg.cool_sd_verify(params, w.target, w.target_uncond, w.draft, w.draft_uncond, w.draft_tokens, om,
                               w.u_accept, w.u_resample, r.accept_len, r.next_token, None, None, f, None, r.ws)
            pkg.cool_sd_diagnostics(params, w.target, w.target_uncond, w.draft, w.draft_uncond, om, alpha, beta, r.ws)
            reach = torch.cumprod(f.double(), dim=1)                       # prod_{j<=i} f_j
            before = torch.cat([torch.ones_like(reach[:, :1]), reach[:, :-1]], dim=1)
            tau_sum += float(r.accept_len.double().sum())
            pred_sum += float(reach.sum())
            bound_sum += float((before * beta.double()).sum())
        n = len(r.pool) * r.B
        out.append({"schedule": name, "delta": delta, "param": param if name != "uniform" else None, "sequences": n,
                    "mean_accept_len": tau_sum / n, "tokens_per_call": tau_sum / n + 1.0,
                    "predicted_accept_len": pred_sum / n, "tv_bound_estimate": bound_sum / n})
    return out


def cpu_baseline(runner, budget_s):
    """The oracle, as it stands, on whole batches of the same pool until the time budget is used
    (OpenMP over sequences, all host cores), then on one core on the first sequences of a batch."""
    from oracle import oracle as O
    from tests.parity_util import run_oracle, subset
    global _HOST_THREADS
    if _HOST_THREADS is None:           # asked once: the single-core sample below leaves the OpenMP default at 1
        _HOST_THREADS = O.max_threads()
    threads = _HOST_THREADS
    first = subset(runner.pool[0], list(range(min(runner.B, threads))))
    run_oracle(O, first, runner.omega_np, num_threads=threads)               # page in / build
    host = [None] * len(runner.pool)        # float32 host copies are made outside the timed region

    def prepared(i):
        if host[i] is None:
            w = runner.pool[i]
            t, d, tu, du = w.logits_f32_numpy()
            host[i] = dict(t=t, d=d, tu=tu, du=du, tok=w.draft_tokens.cpu().numpy(), ua=w.u_accept.cpu().numpy(),
                           ur=w.u_resample.cpu().numpy(), w=w)
        return host[i]

    def call(h, nthreads, nseq=None):
        sl = slice(None) if nseq is None else slice(0, nseq)
        w = h["w"]
        O.verify(h["t"][sl], h["d"][sl], h["tok"][sl], runner.omega_np, h["ua"][sl], h["ur"][sl],
                 target_uncond=None if h["tu"] is None else h["tu"][sl],
                 draft_uncond=None if h["du"] is None else h["du"][sl], cfg_scale=w.cfg_scale,
                 temperature=w.temperature, top_k=w.top_k, num_threads=nthreads)

    calls, el = 0, 0.0
    while el < budget_s:
        h = prepared(calls % len(runner.pool))
        t0 = time.perf_counter()
        call(h, threads)
        el += time.perf_counter() - t0
        calls += 1
    tokens = calls * runner.B * runner.L
    # the same oracle on one core, on the first sequences of a batch
    n1 = max(1, min(runner.B, int(runner.B * (budget_s / 4) / max(el / calls * threads, 1e-9))))
    t1 = time.perf_counter()
    call(prepared(0), 1, n1)
    e1 = time.perf_counter() - t1
    return {"value": tokens / el, "unit": "verified draft tokens/s", "cores": threads, "kind": "oracle",
            "sample": "%d verify calls of the same workload (B=%d, L=%d, V=%d), %.1f s, OpenMP over sequences"
                      % (calls, runner.B, runner.L, runner.V, el),
            "single_core_value": n1 * runner.L / e1,
            "single_core_sample": "the first %d sequences of one call, %.1f s, 1 thread" % (n1, e1)}


def main():
    a = parse()
    if a.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path, run with --gpus 1")
    import torch
    import paper_2601_09212_amd as pkg
    pkg.binding.lib()
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)

    cfg = int(a.workload[3:])
    flags = pkg.COOL_SD_FLAG_EARLY_EXIT if a.early_exit else 0
    pool_mb = a.pool_mb or (3400.0 if cfg >= 4 else 600.0)
    r = Runner(pkg, torch, cfg, pool_mb, flags=flags, B=a.batch or None, V=a.vocab or None, top_k=a.top_k or None)
    variant = bool(a.batch or a.vocab or a.top_k)      # not the configuration itself: its recipe at another size
    if a.counter_run:
        # reference for the byte counters: an elementwise kernel (dst = src * 1) that moves exactly
        # 2^30 B in and 2^30 B out
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        r.run(a.steps, "direct")
        torch.cuda.synchronize()
        if a.diagnostics:
            run_diagnostics(r, a.steps)
        if a.lantern:
            run_lantern(r, a.steps)
        print(json.dumps({"counter_run": a.workload, "steps": a.steps, "copy_bytes_each_way": src.numel() * 4,
                          "bytes_per_step": r.bytes_per_step}))
        return
    done, wall, dev_s = r.time(a.steps, a.warmup, a.launch)
    tokens = done * r.B * r.L
    kern_s = r.kernel_time(a.kernel_samples)
    call_s, call_median_s = r.direct_call_times(min(a.kernel_samples, 100))
    probe_s, probe_launches = r.read_probe_time(a.kernel_samples)
    kernel_name = "row_stats_topk_kernel" if r.pool[0].top_k > 0 else "row_stats_kernel"
    kernel_bytes = r.bytes_per_step
    needed_bytes = None
    if a.early_exit:
        # Algorithmic bytes of the early-exit forms: the rows Algorithm 1 needs, i.e. both rows of every
        # position up to and including the rejected one, or all L pairs plus the bonus row
        need, taus = 0, []
        for i in range(len(r.pool)):
            r.step(i)
            tau = r.accept_len.cpu().numpy().astype("int64")
            taus.append(float(tau.mean()))
            need += int(((tau + 1).clip(max=r.L) * 2 + (tau == r.L)).sum()) * r.V * r.pool[0].target.element_size()
        needed_bytes = need / len(r.pool)
        form = pkg.cool_sd_early_exit_form(r.params, True)
        if form == pkg.COOL_SD_EARLY_EXIT_SEQUENCE:
            # one kernel per call; bf16 rows without a logit transform take the 256-thread form of it
            plain_bf16 = r.pool[0].dtype == "bf16" and r.pool[0].target_uncond is None and r.pool[0].temperature == 1.0
            kernel_name = "sequence_early_exit_tile_kernel" if plain_bf16 else "sequence_early_exit_kernel"
            kernel_bytes = needed_bytes
            kern_s = dev_s / done
        elif form == pkg.COOL_SD_EARLY_EXIT_ROUNDS:
            # several statistics launches per call, each over the rows of one round of positions: the
            # roofline figure is the whole call against the needed rows
            kernel_name = "row_stats_kernel (one launch per round of positions) + accept_window_kernel + sequence_masses_kernel + sequence_select_kernel"
            kernel_bytes = needed_bytes
            kern_s = dev_s / done
    call_bytes = needed_bytes if needed_bytes is not None else r.bytes_per_step
    achieved = kernel_bytes / kern_s / 1e9
    dtype = r.pool[0].dtype
    step_s = wall / done
    line = {
        "metric": "verified draft tokens/sec (1 GPU) + achieved HBM GB/s fraction of peak",
        "value": tokens / wall, "unit": "verified draft tokens/s", "n_gpus": 1, "steps": done, "warmup": a.warmup,
        "ms_per_step": step_s * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config %d%s: B=%d, L=%d, V=%d, %s logits%s, exp schedule delta=%.3g nu=%.3g" % (
                       cfg, "'s recipe" if variant else "", r.B, r.L, r.V, dtype,
                       ", guidance s=%g, top-k %d" % (r.pool[0].cfg_scale, r.pool[0].top_k) if r.pool[0].top_k else "",
                       r.pool[0].delta, r.pool[0].nu),
                   "input_dtype": dtype, "launch": a.launch, "early_exit": bool(a.early_exit), "pool_batches": len(r.pool),
                   "pool_mb": len(r.pool) * r.bytes_per_step / 1e6, "bytes_per_step": r.bytes_per_step},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None if variant else measured_traffic(a.workload, a.early_exit),
                     "traffic_per_call": None if variant else measured_traffic(a.workload, a.early_exit, per_call=True),
                     "early_exit_form": None if not a.early_exit else pkg.cool_sd_early_exit_form(r.params, True),
                     "early_exit_needed_bytes": needed_bytes,
                     "early_exit_mean_tau": None if not a.early_exit else sum(taus) / len(taus),
                     "kernel": kernel_name, "algorithmic_bytes_per_launch": kernel_bytes,
                     "us_per_launch": kern_s * 1e6,
                     # the whole step (every launch of the call) against the same algorithmic bytes
                     # (with --early-exit: against the rows Algorithm 1 needs)
                     "whole_call_us": step_s * 1e6, "whole_call_GBps": call_bytes / step_s / 1e9,
                     "whole_call_frac": call_bytes / step_s / 1e9 / HBM_PEAK_GBS,
                     "graph_step_us": dev_s / done * 1e6,
                     "direct_call_us": call_s * 1e6, "direct_call_median_us": call_median_s * 1e6,
                     # a plain read of the same tensors in one launch of the same shape: what the chip
                     # delivers for this many bytes per launch, start-up included
                     "read_probe": {"us": probe_s * 1e6, "GBps": r.bytes_per_step / probe_s / 1e9,
                                    "launches": probe_launches, "kernel_over_probe": kern_s / probe_s}},
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(r, a.cpu_seconds)
    if a.others:
        extra = {}
        todo = [(c, None, None, None) for c in (1, 2, 3, 4, 5)]
        if a.variants:
            # configuration 4 with eight times the sequences: the regime (B well above the number of
            # compute units) the one-workgroup early-exit form is meant for; the recipes of
            # configurations 2 and 3 at a 65536-token vocabulary (the guided one with top-k 2000):
            # rows of several chunks
            todo += [(4, 2048, None, None), (2, None, 65536, None), (3, 32, 65536, 2000)]
        for c, big, vocab, topk in todo:
            if c == cfg and not big and not vocab and not variant:
                continue
            rr = Runner(pkg, torch, c, 2400.0 if c >= 4 else 600.0, max_pool=(2 if big else 8) if c >= 4 else 64,
                        flags=flags, B=big, V=vocab, top_k=topk)
            d2, w2, s2 = rr.time(max(64, 8 * len(rr.pool)), 2 * len(rr.pool), a.launch)
            k2 = rr.kernel_time(40)
            p2, pl2 = rr.read_probe_time(40)
            name = "cfg%d" % c + ("_B%d" % big if big else "") + ("_V%d" % vocab if vocab else "") + ("_k%d" % topk if topk else "")
            extra[name] = {"tokens_per_s": d2 * rr.B * rr.L / w2, "us_per_step": s2 / d2 * 1e6,
                                  "whole_call_GBps": rr.bytes_per_step / (s2 / d2) / 1e9,
                                  "whole_call_frac": rr.bytes_per_step / (s2 / d2) / 1e9 / HBM_PEAK_GBS,
                                  "row_stats_us": k2 * 1e6, "row_stats_GBps": rr.bytes_per_step / k2 / 1e9,
                                  "row_stats_frac": rr.bytes_per_step / k2 / 1e9 / HBM_PEAK_GBS,
                                  "read_probe_us": p2 * 1e6, "read_probe_GBps": rr.bytes_per_step / p2 / 1e9,
                                  "read_probe_launches": pl2,
                                  "bytes_per_step": rr.bytes_per_step, "pool_batches": len(rr.pool)}
            if a.cpu_others and not a.no_cpu_baseline:
                extra[name]["cpu_baseline"] = cpu_baseline(rr, a.cpu_seconds / 3)
            if a.diagnostics:
                extra[name]["diagnostics"] = time_diagnostics(rr)
            if a.lantern:
                extra[name]["lantern"] = time_lantern(rr)
            if a.draft_sampler:
                extra[name]["draft_sampler"] = time_draft_sampler(rr, passes=4)
            if a.concurrent:
                sec = rr.time_two_streams(passes=4)
                extra[name]["two_streams"] = {"us_per_step": sec * 1e6, "tokens_per_s": rr.B * rr.L / sec,
                                              "whole_call_GBps": rr.bytes_per_step / sec / 1e9}
            del rr
            torch.cuda.empty_cache()
        line["other_workloads"] = extra
    if a.diagnostics:
        line["diagnostics"] = time_diagnostics(r)
    if a.lantern:
        line["lantern"] = time_lantern(r)
    if a.concurrent:
        sec = r.time_two_streams()
        line["two_streams"] = {"us_per_step": sec * 1e6, "tokens_per_s": r.B * r.L / sec,
                               "whole_call_GBps": r.bytes_per_step / sec / 1e9}
    if a.draft_sampler:
        line["draft_sampler"] = time_draft_sampler(r)
    if a.delta_sweep:
        line["delta_sweep"] = delta_sweep(r)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
