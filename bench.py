#!/usr/bin/env python3
"""Benchmark of the verify-step attention on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config IDX] [--all]

A step is one call of owl_verify_attn (split-KV pass + log-sum-exp combine)
over one batch of seeded synthetic input that is already resident in HBM.
Successive steps walk through several resident copies of the KV cache so that
more than 2 GB is touched between two uses of the same bytes: a real verify
step scans 32-80 layers' caches, so the cache is always cold, and the chip's
256 MB memory-side cache would otherwise serve the smaller shapes.

Prints ONE JSON line.  `value` is algorithmic KV bytes per second
(sum_b (L_b + N) * Hkv * D * 2 tensors * 2 bytes, divided by the time of the
whole step); `ms_per_step` is the verify-step time: wall clock over exactly
--steps steps between two synchronisations.  `roofline` prices the split-KV
kernel alone from HIP events attached to its dispatch (every eighth step of
the timed region, plus a sampling pass after it so that there are at least 32
samples whatever --steps is) against whichever of the two roofs bounds the
shape: 8 TB/s of HBM over the algorithmic K/V bytes or 2.5 PFLOP/s of dense
bf16 MFMA over the algorithmic flop; both sides are printed.  `step_us` holds
percentiles of single steps (an event after every step of a separate pass).
`others` repeats this for the other bf16 workloads (timed over at least 200
steps each: their steps are as short as 30 us).  `cpu_baseline` times the
CPU oracle on a sample of output rows on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0
MIN_ROTATION_BYTES = 2 << 30
MIN_KERNEL_SAMPLES = 32
STEP_SAMPLES = 96
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def measured_traffic(workload, kernel="splitkv_kernel"):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter runs
    (FETCH_SIZE + WRITE_SIZE, calibrated), or None if none was recorded."""
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f)[kernel][workload]["hbm_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3,
                    help="0-based index into the benchmark configurations (default 3: 128K-context hybrid verify)")
    ap.add_argument("--all", action="store_true",
                    help="also time the steps around the attention and the drafter cell ('step_kernels', 'drafter_cell')")
    ap.add_argument("--no-others", action="store_true", help="time only the --config workload (no 'others')")
    ap.add_argument("--settle-ms", type=float, default=400.0,
                    help="milliseconds of the same step run before the warm-up steps, so that the clock governor has "
                         "reached its steady state under this load when the timed region starts (0 = none)")
    ap.add_argument("--split-tokens", type=int, default=0, help="override the library's split size (tuning)")
    ap.add_argument("--dtype", choices=("bf16", "f16"), default="bf16",
                    help="storage type of q/K/V (the configurations list bf16; f16 is the paper's type)")
    ap.add_argument("--drafter", action="store_true",
                    help="also time the drafter's recurrent cell (reported under 'drafter_cell'; implied by --all)")
    ap.add_argument("--kv-head-shards", type=int, default=1,
                    help="time ONE GPU's share of the --config workload when its KV heads (with their query heads) "
                         "are spread over this many GPUs: the same lengths and tree on 1/N of the heads (still one GPU)")
    ap.add_argument("--shard-shapes", action="store_true",
                    help="also time one GPU's share of the 128K hybrid workload with its KV heads spread over 2, 4 and "
                         "8 GPUs (reported under 'kv_head_shard_shapes'; implied by --all)")
    ap.add_argument("--context-sweep", action="store_true",
                    help="also time a 60-node tree (8B heads) and the 40-node hybrid tree (70B heads) on 4K..64K contexts "
                         "(reported under 'context_sweep')")
    ap.add_argument("--draft-sweep", action="store_true",
                    help="also time a 64K-context step for 1..60 drafted tokens (reported under 'draft_count_sweep')")
    ap.add_argument("--evidence", action="store_true",
                    help="also run the experiments the design notes lean on (reported under 'evidence'): the same "
                         "launches on all-zero operands, shader cycles against duration over a series of launches, the "
                         "step probe of the matrix pipe, the cost of an empty event bracket")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true")
    return ap.parse_args()


class Rotating:
    """A verify step plus enough resident copies of its KV cache to defeat the
    caches between reuses."""

    def __init__(self, case, split_tokens=0):
        import torch
        from paper_2510_07535_amd.runner import VerifyStep
        self.torch = torch
        self.step = VerifyStep(case, split_tokens=split_tokens)
        self.kv_bytes = case.kv_bytes()
        pool_bytes = 2 * self.step.k.numel() * self.step.k.element_size()
        n = max(2, -(-MIN_ROTATION_BYTES // max(pool_bytes, 1)))
        n = min(n, 64)
        self.pools = [(self.step.k, self.step.v)]
        for _ in range(n - 1):
            self.pools.append((self.step.k.clone(), self.step.v.clone()))
        self.i = 0

    def run(self, phases=3):
        k, v = self.pools[self.i % len(self.pools)]
        self.i += 1
        self.step.run(k=k, v=v, phases=phases)

    def time_steps(self, steps, warmup):
        torch = self.torch
        for _ in range(warmup):
            self.run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.run()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def settle(self, ms):
        """Runs the step for about `ms` milliseconds (untimed): a verify step never meets an idle chip
        in use, and the power management takes some hundred milliseconds of load to settle."""
        if ms <= 0:
            return
        t_end = time.perf_counter() + ms * 1e-3
        while time.perf_counter() < t_end:
            for _ in range(16):
                self.run()
            self.torch.cuda.synchronize()

    def run_split_timed(self, timer):
        k, v = self.pools[self.i % len(self.pools)]
        self.i += 1
        self.step.run_split_timed(timer, k=k, v=v)

    def time_steps_with_kernel(self, steps, warmup, settle_ms=0.0):
        """The timed region (wall clock over exactly `steps` steps).  In every eighth step the split-KV
        kernel is launched with a pair of HIP events attached to its own dispatch (begin and end of
        the kernel on the launch stream; such a step is enqueued as its two phases: the same
        kernels).  Then, outside the region: more such launches until there are MIN_KERNEL_SAMPLES, a
        few launches bracketed by ordinary event records instead (for comparison: those read ~5 us
        more), and STEP_SAMPLES steps with an event after each for the distribution of single-step
        times.  Returns a dict of seconds."""
        torch = self.torch
        from paper_2510_07535_amd.binding import KernelTimer
        every = 8                                        # a timed launch costs its step ~10 us of host-side bookkeeping
        timers = [KernelTimer() for _ in range(max((steps + every - 1) // every, MIN_KERNEL_SAMPLES))]
        n_timed = (steps + every - 1) // every
        self.settle(settle_ms)
        for _ in range(warmup):
            self.run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            if i % every == 0:
                self.run_split_timed(timers[i // every])
                self.run(phases=2)
            else:
                self.run()
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / steps
        for tm in timers[n_timed:]:
            for _ in range(every - 1):
                self.run()
            self.run_split_timed(tm)
            self.run(phases=2)
        torch.cuda.synchronize()
        ks = sorted(tm.elapsed_ms() * 1e-3 for tm in timers)
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(16)]
        for a, b in pairs:
            for _ in range(every - 1):
                self.run()
            a.record()
            self.run(phases=1)
            b.record()
            self.run(phases=2)
        torch.cuda.synchronize()
        bracket = sorted(a.elapsed_time(b) * 1e-3 for a, b in pairs)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(STEP_SAMPLES + 1)]
        marks[0].record()
        for m in marks[1:]:
            self.run()
            m.record()
        torch.cuda.synchronize()
        ss = sorted(marks[i].elapsed_time(marks[i + 1]) * 1e-3 for i in range(STEP_SAMPLES))
        pct = lambda v, q: v[min(len(v) - 1, int(q * len(v)))]
        return {"step": sec, "kernel_avg": sum(ks) / len(ks), "kernel_p10": pct(ks, 0.1), "kernel_p50": pct(ks, 0.5),
                "kernel_p90": pct(ks, 0.9), "kernel_samples": len(ks), "kernel_samples_in_timed_region": n_timed,
                "kernel_bracketed_p50": pct(bracket, 0.5),
                "step_p10": pct(ss, 0.1), "step_p50": pct(ss, 0.5), "step_p90": pct(ss, 0.9), "step_samples": len(ss)}

def stream_probe_gbs(nbytes=1 << 30):
    import torch
    from paper_2510_07535_amd import binding as B
    bufs = [torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 255) for _ in range(3)]
    sink = torch.zeros(8192, dtype=torch.int32, device="cuda")
    best = 0.0
    for nwg in (1024, 2048, 4096):
        for _ in range(3):
            B.owl_stream_read_probe(bufs[0], sink, nwg)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        reps = 12
        for r in range(reps):
            B.owl_stream_read_probe(bufs[r % 3], sink, nwg)
        b.record()
        torch.cuda.synchronize()
        best = max(best, nbytes * reps / (a.elapsed_time(b) * 1e-3) / 1e9)
    return best


def mfma_probe_tflops(kind="random", iters=20000):
    """Sustained bf16 MFMA rate of the whole chip on operands of the given kind."""
    import torch
    from paper_2510_07535_amd import binding as B
    n = 1 << 19
    if kind == "random":
        src = (torch.randn(n, device="cuda") * 1.0).to(torch.bfloat16)
    else:
        src = torch.ones(n, device="cuda", dtype=torch.bfloat16)
    nwg = 256
    sink = torch.zeros(nwg * 512, dtype=torch.float32, device="cuda")
    ghz = torch.zeros(nwg, dtype=torch.float32, device="cuda")
    B.owl_mfma_probe(src, 2000, sink, nwg)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    B.owl_mfma_probe(src, iters, sink, nwg, clock_ghz=ghz)
    b.record()
    torch.cuda.synchronize()
    return nwg * 8 * iters * 16 * 16384.0 / (a.elapsed_time(b) * 1e-3) / 1e12, float(ghz.median().item())


def kernel_shader_clock(rot):
    """Median shader clock (GHz) over the workgroups of one split-KV launch of the timed
    workload: shader cycles per constant-rate tick across the main loop (the timeline hook)."""
    import torch
    from paper_2510_07535_amd import binding as B
    nwg = rot.step.plan.n_workgroups
    buf = torch.zeros(10 * nwg, dtype=torch.int64, device="cuda")
    B.owl_debug_set_timeline(buf)
    try:
        for _ in range(60):                              # steady state: the clock governor averages over
            rot.run()                                    # milliseconds; the last launch's record is read
        torch.cuda.synchronize()
    finally:
        B.owl_debug_set_timeline(None)
    t = buf.cpu().numpy().reshape(nwg, 10)
    t = t[(t[:, 3] - t[:, 2]) >= 200]                    # main loops of at least 2 us: the tick is 10 ns
    if len(t) == 0:
        return None
    import numpy as np
    return float(np.median((t[:, 9] - t[:, 8]) / ((t[:, 3] - t[:, 2]) * 10.0)))


def evidence(rot, case):
    """Experiments behind the statements on what bounds the tree shapes (design notes, kernel section)."""
    import numpy as np
    import torch
    from paper_2510_07535_amd import binding as B
    out = {}
    # (1) an empty event bracket: what HIP events add to a bracketed kernel
    rot.settle(200)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(32)]
    for a, b in pairs:
        rot.run()
        a.record()
        b.record()
    torch.cuda.synchronize()
    out["empty_event_bracket_us"] = float(np.median([a.elapsed_time(b) * 1e3 for a, b in pairs]))
    # (2) shader cycles of the main loop against the duration of the launch, over a series of launches
    nwg = rot.step.plan.n_workgroups
    n = 120
    bufs = [torch.zeros(10 * nwg, dtype=torch.int64, device="cuda") for _ in range(n)]
    evs = []
    try:
        for i in range(n):
            B.owl_debug_set_timeline(bufs[i])
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            rot.run(phases=1)
            b.record()
            rot.run(phases=2)
            evs.append((a, b))
    finally:
        B.owl_debug_set_timeline(None)
    torch.cuda.synchronize()
    cyc, clk, us, span, phases = [], [], [], [], []
    for i in range(n):
        t = bufs[i].cpu().numpy().reshape(nwg, 10)
        t = t[t[:, 0] > 0]
        if len(t) == 0:
            continue
        rel = (t[:, :6] - t[:, 0].min()) * 0.01
        phases.append(np.median(rel[:, 1:] - rel[:, :-1], axis=0))
        span.append(float(rel[:, 5].max()))
        tt = t[(t[:, 3] - t[:, 2]) >= 100]
        cyc.append(float(np.median(tt[:, 9] - tt[:, 8])))
        clk.append(float(np.median((tt[:, 9] - tt[:, 8]) / ((tt[:, 3] - tt[:, 2]) * 10.0))))
        us.append(evs[i][0].elapsed_time(evs[i][1]) * 1e3)
    if cyc:
        ph = np.median(np.array(phases), axis=0)
        out["launch_series"] = {
            "launches": len(cyc), "workgroups": int(nwg),
            "main_loop_cycles": {"min": min(cyc), "median": float(np.median(cyc)), "max": max(cyc)},
            "shader_clock_GHz": {"min": min(clk), "median": float(np.median(clk)), "max": max(clk)},
            "event_us": {"min": min(us), "median": float(np.median(us)), "max": max(us)},
            "device_span_us": {"min": min(span), "median": float(np.median(span)), "max": max(span),
                               "what": "first workgroup's entry to last workgroup's exit on the device's 100 MHz clock"},
            "corr_clock_vs_event_us": float(np.corrcoef(clk, us)[0, 1]) if len(cyc) > 2 else None,
            "corr_cycles_vs_event_us": float(np.corrcoef(cyc, us)[0, 1]) if len(cyc) > 2 else None,
            "phase_medians_us": {"set-up": float(ph[0]), "first stage in LDS": float(ph[1]), "fast loop": float(ph[2]),
                                 "careful tail": float(ph[3]), "epilogue": float(ph[4])},
        }
    del bufs
    # (3) the same launches on all-zero operands: same instructions, same traffic, less switching
    real = rot.time_steps_with_kernel(60, 10, 200)
    saved = [(k.clone(), v.clone()) for k, v in rot.pools[:1]]
    q_saved = rot.step.q.clone()
    for k, v in rot.pools:
        k.zero_()
        v.zero_()
    rot.step.q.zero_()
    zero = rot.time_steps_with_kernel(60, 10, 200)
    rot.step.q.copy_(q_saved)
    for (k, v) in rot.pools:
        k.copy_(saved[0][0])
        v.copy_(saved[0][1])
    out["zero_operands"] = {"kernel_us_random_data": real["kernel_avg"] * 1e6, "kernel_us_all_zero_data": zero["kernel_avg"] * 1e6,
                            "step_us_random_data": real["step"] * 1e6, "step_us_all_zero_data": zero["step"] * 1e6}
    del saved
    # (4) the step probe: how busy two wavefronts per SIMD keep the matrix pipe on the loop's instruction mix
    out["step_probe"] = step_probe_rows()
    return out


def step_probe_rows(variants=None, iters=4000, nwg=256):
    """The step probe on the whole chip: cycles per 32-key step and SIMD (the matrix pipe's busy fraction
    follows) and, from HIP events around the launch, the MFMA rate the chip sustained on that
    instruction mix under its power limit with no HBM traffic at all."""
    import torch
    from paper_2510_07535_amd import binding as B
    src = torch.randn(8192, device="cuda").to(torch.bfloat16)
    sink = torch.zeros(nwg * 512, dtype=torch.float32, device="cuda")
    cycles = torch.zeros(nwg * 8, dtype=torch.int64, device="cuda")
    rows = []
    for variant, name, tiles in B.STEP_PROBE_VARIANTS:
        if variants is not None and variant not in variants:
            continue
        for _ in range(3):
            B.owl_step_probe(variant, src, iters, sink, cycles, nwg)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        reps = 8
        for _ in range(reps):
            B.owl_step_probe(variant, src, iters, sink, cycles, nwg)
        b.record()
        torch.cuda.synchronize()
        sec = a.elapsed_time(b) * 1e-3 / reps
        per = float(cycles.double().mean().item()) / iters
        need = tiles * 17 * 16.0
        flop = nwg * 4.0 * tiles * 17 * 16384.0 * iters          # 16 of the 17 MFMAs per tile-step are algorithmic
        rows.append({"variant": name, "cycles_per_step_and_simd": per, "matrix_pipe_cycles_needed": need,
                     "matrix_pipe_busy": need / per, "TFLOPs_all_mfma": flop / sec / 1e12,
                     "TFLOPs_algorithmic": flop * 16 / 17 / sec / 1e12,
                     "shader_clock_GHz": per * iters / sec / 1e9})
    return rows


def cpu_baseline(case, budget_rows=None):
    import numpy as np
    import oracle
    oracle.build()
    total_rows = case.B * case.N * case.Hq
    # ~10-30 s of host work: the oracle does ~1e10 flop/s on a handful of cores
    flop_per_row = 4.0 * case.D * float(case.ctx_lens.astype(np.float64).mean() + case.N)
    n = budget_rows or int(max(16, min(total_rows, 1.5e11 / max(flop_per_row, 1.0))))
    rng = np.random.Generator(np.random.Philox(key=12345))
    pick = rng.choice(total_rows, size=min(n, total_rows), replace=False)
    rows = np.stack([pick // (case.N * case.Hq), (pick // case.Hq) % case.N, pick % case.Hq], axis=1).astype(np.int32)
    # at least ~10 s of host work: repeat the sample if one pass is shorter
    reps, spent = 0, 0.0
    while reps < 8 and (reps == 0 or spent < 10.0):
        t0 = time.perf_counter()
        oracle.verify_attn_case(case, rows=rows)
        spent += time.perf_counter() - t0
        reps += 1
    dt = spent / reps
    full = dt * total_rows / len(rows)
    return {
        "value": case.kv_bytes() / full / 1e9, "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": f"{len(rows)} of {total_rows} output rows of the same workload, {reps} passes of {dt:.1f} s each, "
                  f"scaled to all rows ({full:.1f} s per verify step)",
        "seconds_per_step_est": full,
    }


def bench_steps(reps=200):
    """The steps around the attention (Prepare, greedy acceptance, KV commit) on
    the batched configuration's shapes: microseconds per call, launches queued
    back to back.  They are launch-bound integer / data-movement kernels."""
    import numpy as np
    import torch
    from paper_2510_07535_amd import binding as B
    from paper_2510_07535_amd import workloads as W
    from paper_2510_07535_amd.runner import VerifyStep
    dev = "cuda:0"
    case = W.make_config(4, ctx_scale=0.05)
    Bn, N = case.B, case.N
    n = N // 2
    rng = np.random.Generator(np.random.Philox(key=99))
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    parent_n = i32(case.tree_parent[:, :n].clip(max=n - 1))
    ctx = i32(case.ctx_lens)
    p2 = torch.zeros((Bn, 2 * n), dtype=torch.int32, device=dev)
    anc = torch.zeros((Bn, 2 * n), dtype=torch.int64, device=dev)
    dep = torch.zeros_like(p2)
    pos = torch.zeros_like(p2)
    tok, tgt = i32(rng.integers(0, 3, (Bn, N))), i32(rng.integers(0, 3, (Bn, N)))
    root = i32(rng.integers(0, 3, Bn))
    par = i32(case.tree_parent)
    acc = torch.zeros((Bn, N), dtype=torch.int32, device=dev)
    na, bonus, last = (torch.zeros(Bn, dtype=torch.int32, device=dev) for _ in range(3))
    step = VerifyStep(case)
    new_ctx = torch.zeros(Bn, dtype=torch.int32, device=dev)

    def timed(fn):
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e6

    res = {"shapes": {"batch": Bn, "n_draft": N, "n_kv_heads": case.Hkv, "head_dim": case.D}}
    res["prepare_us"] = timed(lambda: B.owl_prepare_spec_tree(parent_n, ctx, p2, anc, dep, pos))
    res["accept_us"] = timed(lambda: B.owl_accept_greedy(tok, par, root, tgt, N, acc, na, bonus, last))
    B.owl_accept_greedy(tok, par, root, tgt, N, acc, na, bonus, last)
    torch.cuda.synchronize()
    res["commit_us"] = timed(lambda: B.owl_commit_kv(step.desc, step.k, step.v, step.page_table, step.ctx_lens,
                                                     acc, na, new_ctx, step.status))
    res["commit_rows_moved"] = int(na.sum().item()) * case.Hkv * 2
    res["commit_bytes"] = res["commit_rows_moved"] * case.D * 2 * 2
    return res


DRAFTER_SHAPES = (
    # name, d_in, d, states, rows: the paper's cell width (Sec. 4.1) with the ten rows of one tree
    # level (Appendix A.1: top-k 10); square W is the shape the recurrence needs, 4096 / 8192 are
    # the hidden sizes of the two target models feeding the first step
    ("owl_cell_d12288_square_level10", 12288, 12288, 10, 10),
    ("owl_cell_d12288_from8192_root10", 8192, 12288, 1, 10),
    ("owl_cell_d12288_from4096_root10", 4096, 12288, 1, 10),
)


def bench_drafter(steps=60, with_cpu=True):
    """The drafter's recurrent cell (one step = projection kernel + gate kernel) on random
    weights: us per step and achieved GB/s over the 4 d d_in weight bytes, the projection
    kernel alone against the HBM peak, and the oracle on the host for the same step."""
    import torch
    from paper_2510_07535_amd import binding as B
    from paper_2510_07535_amd import workloads as W
    from paper_2510_07535_amd.runner import DrafterStep
    out = []
    for name, d_in, d, P, M in DRAFTER_SHAPES:
        case = W.make_drafter_case(name, 31, d_in=d_in, d=d, P=P, M=M, vocab=2048)
        alpha = B.owl_drafter_alpha(8, d)
        step = DrafterStep(case, alpha)
        wbytes = case.weight_bytes()
        copies = [step.w] + [step.w.clone() for _ in range(max(1, -(-MIN_ROTATION_BYTES // wbytes)) )]
        k = [0]

        def run(phases=3):
            step.run(w=copies[k[0] % len(copies)], phases=phases)
            k[0] += 1
        for _ in range(5):
            run()
        torch.cuda.synchronize()
        every = 4                                        # the projection of every fourth timed step between events
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range((steps + every - 1) // every)]
        t0 = time.perf_counter()
        for i in range(steps):
            if i % every == 0:
                a, b = ev[i // every]
                a.record()
                run(phases=1)
                b.record()
                run(phases=2)
            else:
                run()
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / steps
        ksec = sum(a.elapsed_time(b) for a, b in ev) / len(ev) * 1e-3
        assert step.dev_status() == 0
        res = {"workload": name, "d_in": d_in, "d": d, "n_states": P, "n_rows": M, "dtype": "bf16",
               "weight_bytes": wbytes, "weight_layout": "tiled", "weight_copies_rotated": len(copies), "us_per_step": sec * 1e6,
               "GBps": wbytes / sec / 1e9,
               "roofline": {"bound": "hbm", "achieved": wbytes / ksec / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": wbytes / ksec / 1e9 / HBM_PEAK_GBS,
                            "traffic": measured_traffic(name, "drafter_proj_kernel"),
                            "kernel": "drafter_proj_kernel", "kernel_avg_us": ksec * 1e6,
                            "algorithmic_bytes_per_launch": wbytes}}
        if with_cpu and name == DRAFTER_SHAPES[0][0]:
            from oracle import drafter as OD
            t0 = time.perf_counter()
            OD.drafter_cell_case(case, alpha)
            dt = time.perf_counter() - t0
            res["cpu_baseline"] = {"value": wbytes / dt / 1e9, "unit": "GB/s", "cores": os.cpu_count(),
                                   "kind": "oracle", "sample": f"the whole step once ({dt:.1f} s)"}
        out.append(res)
        del step, copies
        torch.cuda.empty_cache()
    return out


def bench_draft_sweep(ctx=65536, counts=(1, 4, 8, 16, 24, 32, 48, 60)):
    """Cost of one verify step against the number of drafted tokens: 8B head shapes, one
    sequence of `ctx` cached tokens, chains up to 8 tokens and depth-6 trees beyond."""
    import numpy as np
    import torch
    from paper_2510_07535_amd import workloads as W
    rng = np.random.Generator(np.random.Philox(key=3))
    out = []
    for n in counts:
        tree = W.chain_tree(n) if n <= 8 else W.random_tree(n, 6, rng)
        case = W.make_case(f"sweep_n{n}", 9, dtype=W.DT_BF16, Hq=32, Hkv=8, D=128, ctx_lens=[ctx], trees=[tree])
        rot = Rotating(case)
        rot.settle(300)
        sec = rot.time_steps(150, 20)
        out.append({"n_draft": n, "rows_per_kv": rot.step.plan.rows_per_kv, "ctx": ctx, "us_per_step": sec * 1e6,
                    "GBps": rot.kv_bytes / sec / 1e9})
        del rot
        torch.cuda.empty_cache()
    return out


def bench_context_sweep(contexts=(4096, 8192, 16384, 32768, 65536)):
    """Cost of one verify step against the context length (the benchmark's range starts at 4K tokens): 8B head shapes
    with a 60-node tree, 70B head shapes with the 40-node hybrid tree, one sequence."""
    import numpy as np
    import torch
    from paper_2510_07535_amd import workloads as W
    rng = np.random.Generator(np.random.Philox(key=11))
    out = []
    for ctx in contexts:
        for name, Hq, tree in (("8b_tree60", 32, W.random_tree(60, 6, rng)), ("70b_hybrid40", 64, W.hybrid_tree(32, 8, rng))):
            case = W.make_case(f"{name}_{ctx // 1024}k", 4, dtype=W.DT_BF16, Hq=Hq, Hkv=8, D=128, ctx_lens=[ctx], trees=[tree])
            rot = Rotating(case)
            rot.settle(150)
            sec = rot.time_steps(300, 20)
            pl = rot.step.plan
            out.append({"workload": case.name, "ctx": ctx, "rows_per_kv": pl.rows_per_kv, "us_per_step": sec * 1e6,
                        "GBps": rot.kv_bytes / sec / 1e9, "split_tokens": pl.split_tokens, "row_groups": pl.row_groups,
                        "tiles_per_wave": pl.tiles_per_wave, "n_workgroups": pl.n_workgroups})
            del rot
            torch.cuda.empty_cache()
    return out


def roofline_of(case, t, workload):
    """The split-KV kernel against both roofs; `bound` names the one with the longer floor."""
    kbytes = case.kv_bytes()
    rows_per_kv = (case.Hq // case.Hkv) * case.N
    # QK^T and PV are 2*D flop each per (row, key)
    flop = 4.0 * case.D * rows_per_kv * case.Hkv * float((case.ctx_lens.astype("int64") + case.N).sum())
    ksec = t["kernel_avg"]
    t_hbm, t_mfma = kbytes / (HBM_PEAK_GBS * 1e9), flop / (MFMA_PEAK_TFLOPS * 1e12)
    hbm = {"achieved": kbytes / ksec / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": t_hbm / ksec,
           "floor_us": t_hbm * 1e6, "algorithmic_bytes_per_launch": kbytes}
    mfma = {"achieved": flop / ksec / 1e12, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": t_mfma / ksec,
            "floor_us": t_mfma * 1e6, "algorithmic_flop_per_launch": flop}
    bound = "mfma" if t_mfma > t_hbm else "hbm"
    top = dict(mfma if bound == "mfma" else hbm)
    top.pop("floor_us")
    r = {"bound": bound, **top,
         "traffic": measured_traffic(workload), "traffic_source": "profiles/hbm_traffic.json (rocprofv3 FETCH_SIZE + "
         "WRITE_SIZE of an earlier run of this workload, calibrated; not measured by this run)",
         "kernel": "splitkv_kernel", "kernel_avg_us": ksec * 1e6, "kernel_p10_us": t["kernel_p10"] * 1e6,
         "kernel_median_us": t["kernel_p50"] * 1e6, "kernel_p90_us": t["kernel_p90"] * 1e6,
         "kernel_samples": t["kernel_samples"], "kernel_samples_in_timed_region": t["kernel_samples_in_timed_region"],
         "kernel_timing": "HIP events attached to the kernel's dispatch (begin / end of the kernel on the launch stream)",
         "kernel_median_us_between_event_records": t["kernel_bracketed_p50"] * 1e6,
         "t_hbm_us": t_hbm * 1e6, "t_mfma_us": t_mfma * 1e6, "hbm": hbm, "mfma": mfma}
    return r


def bench_config(idx, args, min_steps=0, kv_shards=1):
    """`min_steps` (the `others` only): their steps are as short as 30 us, and the wall clock over the
    headline's step count (20 steps = 0.6 ms) would mostly show how the host happened to be scheduled."""
    from paper_2510_07535_amd import workloads as W
    case = W.make_config(idx, dtype={"bf16": W.DT_BF16, "f16": W.DT_F16}[args.dtype], kv_shards=kv_shards)
    rot = Rotating(case, split_tokens=args.split_tokens)
    steps = max(args.steps, min_steps)
    t = rot.time_steps_with_kernel(steps, args.warmup, args.settle_ms)
    sec = t["step"]
    res = {
        "workload": W.CONFIG_NAMES[idx] if kv_shards == 1 else case.name, "config_index": idx, "steps": steps,
        "us_per_step": sec * 1e6, "GBps": rot.kv_bytes / sec / 1e9,
        "frac_of_hbm_peak": rot.kv_bytes / sec / 1e9 / HBM_PEAK_GBS,
        "step_us": {"p10": t["step_p10"] * 1e6, "p50": t["step_p50"] * 1e6, "p90": t["step_p90"] * 1e6,
                    "samples": t["step_samples"], "how": "an event after every step of a separate pass"},
        "kv_bytes": rot.kv_bytes, "plan": rot.step.plan.as_dict(), "kv_copies_rotated": len(rot.pools),
        "launches_per_step": 2,
        "roofline": roofline_of(case, t, W.CONFIG_NAMES[idx] if kv_shards == 1 else case.name),
    }
    assert rot.step.dev_status() == 0
    return case, rot, res


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build measures ONE GPU (the per-GPU share of the path at its real shape); "
              f"--gpus {args.gpus} is not supported, run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2510_07535_amd import binding as B
    from paper_2510_07535_amd import workloads as W
    B.lib()   # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    case, rot, main_res = bench_config(args.config, args, kv_shards=args.kv_head_shards)
    kbytes = main_res["kv_bytes"]
    line = {
        "metric": "verify-step attention: achieved HBM GB/s over algorithmic KV bytes (us per step in ms_per_step)",
        "value": main_res["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["us_per_step"] / 1e3, "us_per_step": main_res["us_per_step"],
        "step_us": main_res["step_us"],
        "frac_of_hbm_peak": main_res["frac_of_hbm_peak"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {W.DT_BF16: "bf16", W.DT_F32: "f32", W.DT_F16: "f16"}[case.dtype], "data": "synthetic",
        "config": {"workload": main_res["workload"], "config_index": args.config, "batch": case.B,
                   "ctx_lens_max": int(case.ctx_lens.max()), "ctx_tokens_total": int(case.ctx_lens.sum()),
                   "n_draft": case.N, "n_q_heads": case.Hq, "n_kv_heads": case.Hkv, "head_dim": case.D,
                   "page_size": 16, "kv_bytes_per_step": kbytes, "kv_copies_rotated": main_res["kv_copies_rotated"],
                   "launches_per_step": main_res["launches_per_step"], "plan": main_res["plan"]},
        "roofline": main_res["roofline"],
    }
    if not args.no_probe:
        rl = line["roofline"]
        rl["stream_read_probe_GBps"] = stream_probe_gbs()
        # the chip is power-limited: the shader clock under load, read inside the kernels, next to the rates
        rl["shader_clock_GHz"] = {"nominal": 2.4, "splitkv_kernel": kernel_shader_clock(rot)}
        for kind, key in (("random", "probe_random_operands"), ("ones", "probe_constant_operands")):
            tf, ghz = mfma_probe_tflops(kind)
            rl["mfma"][key + "_TFLOPs"] = tf
            rl["shader_clock_GHz"]["mfma_" + key] = ghz
        # the loop's own instruction mix without the HBM side: barrier + 64-bit V reads, 3 + 2 or 2 + 2 tiles
        sp = step_probe_rows(variants=(3,) if main_res["plan"]["tiles_per_wave"] == 3 else (5,))
        rl["mfma"]["step_probe_TFLOPs_algorithmic"] = sp[0]["TFLOPs_algorithmic"]
        rl["mfma"]["step_probe_variant"] = sp[0]["variant"]
        rl["mfma"]["frac_of_step_probe"] = rl["mfma"]["achieved"] / sp[0]["TFLOPs_algorithmic"]
        # the same kernel time against what this very box sustained in the probes of this run
        ksec = rl["kernel_avg_us"] * 1e-6
        floor = max(kbytes / (rl["stream_read_probe_GBps"] * 1e9),
                    rl["mfma"]["algorithmic_flop_per_launch"] / (rl["mfma"]["probe_random_operands_TFLOPs"] * 1e12))
        rl["frac_of_measured_ceiling"] = floor / ksec
        rl["measured_ceiling"] = ("the longer of: algorithmic bytes / streaming-read probe rate, algorithmic flop / "
                                  "matrix-pipe probe rate on random operands, both from this run")
    if args.evidence:
        line["evidence"] = evidence(rot, case)
    if not args.no_others:
        others = []
        for idx in (1, 2, 3, 4):
            if idx == args.config and args.kv_head_shards == 1:
                continue
            del rot
            torch.cuda.empty_cache()
            _, rot, r = bench_config(idx, args, min_steps=200)
            others.append(r)
        line["others"] = others
    if args.all:
        line["step_kernels"] = bench_steps()
    if args.all or args.shard_shapes:
        shares = []
        for n in (2, 4, 8):
            del rot
            torch.cuda.empty_cache()
            _, rot, r = bench_config(3, args, min_steps=200, kv_shards=n)
            r["kv_head_shards"] = n
            shares.append(r)
        line["kv_head_shard_shapes"] = shares
    if args.context_sweep:
        line["context_sweep"] = bench_context_sweep()
    if args.draft_sweep:
        line["draft_count_sweep"] = bench_draft_sweep()
    if args.all or args.drafter:
        line["drafter_cell"] = bench_drafter(with_cpu=not args.no_cpu_baseline)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(case)
    else:
        line["cpu_baseline"] = None
    print(json.dumps(line))


if __name__ == "__main__":
    main()
