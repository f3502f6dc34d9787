#!/usr/bin/env python3
"""Benchmark of the attention-weight path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4]

One "step" is one call of the library on one batch of seeded synthetic input
already resident in HBM.  The headline workload (top-level ``value``) is the
fused kernel on configuration c4 (B=1 H=16 N=4096 d=128 bf16, the paper's d_k
and its largest fused n); the same JSON line carries, under ``workloads``, the
dedicated softmax on c2, the fused kernel on c3 and c5, the unfused pair
(score GEMM, then softmax) and the three-kernel pipeline (multiply, scaling,
softmax) on c3..c5 for the fused-vs-unfused ratios, and the attention output.

Timing: every timed section starts with an untimed pre-heat of about 0.4 s of
the section's own call (the shader clock starts low on an idle GPU and takes a
few hundred milliseconds of load to settle; a 5 + 20 call measurement of a
0.2 ms kernel would sit entirely inside that ramp), reported as ``preheat_ms``;
then W untimed calls, then exactly K calls bracketed by a device
synchronisation on both sides (wall clock -> ``ms_per_step`` and ``value``) and
by HIP events recorded on the stream the kernels are launched on (-> the
average launch duration used for the roofline).  ``steps`` and ``warmup`` in
the JSON line are K and W as given; without the flags W = 5 and K is sized from
a three-call pilot so that the timed region lasts about 0.3 s.  Working sets
smaller than the 256 MB last-level cache are rotated through distinct buffers
(> 1 GiB in total) so that no call finds its data on chip.  Right after the
headline section has been timed its call is launched back to back for another
1.5 s while a child process samples board power and shader clock
(``amd-smi metric -p -c``); the readings go into the line as ``power``.

The CPU oracle is timed in the same run on the host cores (``cpu_baseline``):
a reported baseline, not the target.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "attention-weight elements/s and achieved HBM GB/s (% of peak), fused vs unfused"
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
ROTATE_BYTES = 1.25 * 2 ** 30  # rotate small working sets through at least this much memory
CACHE_BYTES = 256e6


def _dev(a, dtype):
    import numpy as np
    import torch
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)


WARM_MS = 400.0   # untimed pre-heat per timed section: the shader clock needs this long under load to settle
TIMED_MS = 300.0  # default length of a timed section
LAST_PREHEAT_MS = 0.0   # wall time of the most recent section's pre-heat (reported with the headline)


class PowerSampler:
    """Board power and shader clock while a section runs: a thread that keeps calling ``amd-smi metric -p -c``
    (a child process per sample) and keeps the readings.  Absent tool or unparsable output: no samples."""

    def __init__(self, period_s=0.15):
        import threading
        self.period_s = period_s
        self.samples = []
        self._stop = threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True)

    def _run(self):
        import re
        import subprocess
        while not self._stop.is_set():
            try:
                out = subprocess.run(["amd-smi", "metric", "-p", "-c"], capture_output=True, text=True, timeout=5).stdout
            except (OSError, subprocess.SubprocessError):
                return
            block = out.split("GPU: 1")[0]
            m = re.search(r"SOCKET_POWER:\s*(\d+)", block)
            clks = [int(c) for c in re.findall(r"GFX_\d+:\s*\n\s*CLK:\s*(\d+)", block)]
            if m:
                self.samples.append((int(m.group(1)), clks))
            self._stop.wait(self.period_s)

    def start(self):
        self._thread.start()
        return self

    def stop(self):
        self._stop.set()
        self._thread.join(timeout=10)
        if not self.samples:
            return None
        top = max(self.samples, key=lambda s: s[0])
        clocks = [c for c in top[1] if c > 0]
        return {"socket_power_W": top[0], "gfx_clock_MHz_min": min(clocks) if clocks else None,
                "gfx_clock_MHz_max": max(clocks) if clocks else None, "samples": len(self.samples),
                "source": "amd-smi metric -p -c while the headline call is launched back to back for 1.5 s right "
                          "after its timed region; the sample with the highest socket power"}


POWER_WINDOW_MS = 1500.0


def _power_window(call, n_sets):
    """After a section has been timed: keep launching its call for POWER_WINDOW_MS (untimed) while board power and
    shader clock are sampled -- the state the timed calls ran in, read without disturbing them."""
    import torch
    sampler = PowerSampler().start()
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < POWER_WINDOW_MS:
        for i in range(50):
            call(i % n_sets)
        torch.cuda.synchronize()
    return sampler.stop()


def _time_calls(call, n_sets, steps, warmup):
    """call(i) launches one step on buffer set i % n_sets.  A pre-heat of about WARM_MS of calls (sized from a
    three-call pilot) comes first, whatever ``steps`` / ``warmup`` say; ``warmup`` None: 5 calls; ``steps``
    None: as many as fill TIMED_MS.  Returns (wall ms/step, event ms/step, steps, warmup)."""
    import torch
    global LAST_PREHEAT_MS
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    call(0)
    e0.record(stream)
    for i in range(3):
        call(i % n_sets)
    e1.record(stream)
    torch.cuda.synchronize()
    pilot = max(e0.elapsed_time(e1) / 3, 1e-3)
    t0 = time.perf_counter()
    batch = min(max(int(50.0 / pilot), 1), 5000)        # about 50 ms of calls between looks at the clock
    while True:
        for i in range(batch):
            call(i % n_sets)
        torch.cuda.synchronize()
        LAST_PREHEAT_MS = (time.perf_counter() - t0) * 1e3
        if LAST_PREHEAT_MS >= WARM_MS:
            break
    if warmup is None:
        warmup = 5
    if steps is None:
        steps = min(max(int(TIMED_MS / pilot), 20), 50000)
    for i in range(warmup):
        call(i % n_sets)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for i in range(steps):
        call((warmup + i) % n_sets)
    e1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps, steps, warmup


def _n_sets(set_bytes):
    if set_bytes >= 2 * CACHE_BYTES:
        return 2
    return int(math.ceil(ROTATE_BYTES / set_bytes))


def _record(name, what, elements, alg_bytes, timing, n_sets):
    wall_ms, ev_ms, steps, warmup = timing
    gbs = alg_bytes / (ev_ms * 1e-3) * 1e-9
    return {
        "workload": name, "call": what, "elements": elements, "algorithmic_bytes": alg_bytes,
        "steps": steps, "warmup": warmup,
        "preheat_ms": round(LAST_PREHEAT_MS, 1),
        "ms_per_step": round(wall_ms, 5), "kernel_ms": round(ev_ms, 5),
        "elements_per_s": elements / (wall_ms * 1e-3),
        "hbm_GBps": round(gbs, 1), "hbm_frac_of_peak": round(gbs / HBM_PEAK_GBS, 4), "buffer_sets": n_sets,
    }


def bench_softmax(cfg, steps, warmup, sample_power=False):
    import torch
    import paper_2407_13885_amd as attnw
    x = cfg()
    dt = attnw.ATTNW_BF16 if x.dtype == "bf16" else attnw.ATTNW_F32
    n_sets = _n_sets(x.algorithmic_bytes)
    S0 = _dev(x.S, x.dtype)
    S = [S0] + [S0.clone() for _ in range(n_sets - 1)]
    P = [torch.empty_like(S0) for _ in range(n_sets)]
    stream = torch.cuda.current_stream()

    def call(i):
        attnw.attnw_softmax(S[i], P[i], x.rows, x.cols, dt, stream)

    timing = _time_calls(call, n_sets, steps, warmup)
    power = _power_window(call, n_sets) if sample_power else None
    rs = float((P[0].float().sum(-1) - 1.0).abs().max().item())
    rec = _record(x.name, "attnw_softmax", x.elements, x.algorithmic_bytes, timing, n_sets)
    if sample_power:
        rec["power"] = power
    rec["max_row_sum_error"] = rs
    rec["shape"] = {"rows": x.rows, "cols": x.cols, "dtype": x.dtype}
    return rec, x


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published


def bench_fused(cfg, steps, warmup, with_unfused=True, with_attention=True, sample_power=False):
    import torch
    import paper_2407_13885_amd as attnw
    x = cfg()
    dt = attnw.ATTNW_BF16 if x.dtype == "bf16" else attnw.ATTNW_F32
    tdt = torch.bfloat16 if x.dtype == "bf16" else torch.float32
    Q, K = _dev(x.Q, x.dtype), _dev(x.K, x.dtype)
    out_bytes = x.elements * x.itemsize
    n_sets = _n_sets(out_bytes)
    shape = (x.B, x.H, x.N, x.N)
    P = [torch.empty(shape, dtype=tdt, device="cuda") for _ in range(n_sets)]
    stream = torch.cuda.current_stream()
    scale = float(x.scale)

    def call(i):
        attnw.attnw_fused(Q, K, P[i], x.B, x.H, x.N, x.d, scale, dt, stream)

    timing = _time_calls(call, n_sets, steps, warmup)
    power = _power_window(call, n_sets) if sample_power else None
    ev = timing[1]
    rec = _record(x.name, "attnw_fused", x.elements, x.algorithmic_bytes, timing, n_sets)
    if sample_power:
        rec["power"] = power
    rec["shape"] = {"B": x.B, "H": x.H, "N": x.N, "d": x.d, "dtype": x.dtype}
    rec["mfma_TFLOPs_two_pass"] = round(2 * 2.0 * x.elements * x.d / (ev * 1e-3) * 1e-12, 1)
    # row sums of every row (a property that needs no oracle)
    worst = 0.0
    for b in range(x.B):
        for h in range(x.H):
            worst = max(worst, float((P[0][b, h].float().sum(-1) - 1.0).abs().max().item()))
    rec["max_row_sum_error"] = worst

    if with_unfused:
        # unfused pair: scores round-trip through HBM in the storage dtype
        S = [torch.empty(shape, dtype=tdt, device="cuda") for _ in range(n_sets)]
        rows = x.B * x.H * x.N

        def call_gemm(i):
            attnw.attnw_gemm_scores(Q, K, S[i], x.B, x.H, x.N, x.d, scale, dt, stream)

        def call_sm(i):
            attnw.attnw_softmax(S[i], P[i], rows, x.N, dt, stream)

        def call_pair(i):
            call_gemm(i)
            call_sm(i)

        # the paper's three separate kernels: multiply (scale 1), scaling in place, softmax
        def call_scale(i):
            attnw.attnw_scale(S[i], S[i], x.elements, scale, dt, stream)

        def call_three(i):
            attnw.attnw_gemm_scores(Q, K, S[i], x.B, x.H, x.N, x.d, 1.0, dt, stream)
            call_scale(i)
            call_sm(i)

        wall_p, ev_p, _, _ = _time_calls(call_pair, n_sets, steps, warmup)
        _, ev_g, _, _ = _time_calls(call_gemm, n_sets, steps, warmup)
        _, ev_s, _, _ = _time_calls(call_sm, n_sets, steps, warmup)
        wall_3, ev_3, _, _ = _time_calls(call_three, n_sets, steps, warmup)
        _, ev_c, _, _ = _time_calls(call_scale, n_sets, steps, warmup)
        unf_bytes = x.algorithmic_bytes + 2 * out_bytes      # + write S, read S
        unf3_bytes = unf_bytes + 2 * out_bytes               # + read S, write S in the scaling kernel
        rec["unfused"] = {
            "ms_per_step": round(wall_p, 5), "kernel_ms": round(ev_p, 5),
            "gemm_scores_ms": round(ev_g, 5), "softmax_ms": round(ev_s, 5),
            "elements_per_s": x.elements / (wall_p * 1e-3),
            "algorithmic_bytes": unf_bytes, "hbm_GBps": round(unf_bytes / (ev_p * 1e-3) * 1e-9, 1),
        }
        rec["unfused_three_kernels"] = {
            "ms_per_step": round(wall_3, 5), "kernel_ms": round(ev_3, 5), "scale_ms": round(ev_c, 5),
            "scale_hbm_GBps": round(2 * out_bytes / (ev_c * 1e-3) * 1e-9, 1),
            "elements_per_s": x.elements / (wall_3 * 1e-3),
            "algorithmic_bytes": unf3_bytes, "hbm_GBps": round(unf3_bytes / (ev_3 * 1e-3) * 1e-9, 1),
        }
        rec["fused_vs_unfused_speedup"] = round(ev_p / ev, 3)
        rec["fused_vs_three_kernels_speedup"] = round(ev_3 / ev, 3)
        del S
    if with_attention and x.dtype == "bf16" and x.d % 16 == 0 and x.d <= 128:
        # the next step after the weights: O = P V with P kept on chip (nothing of size N^2 touches HBM)
        import numpy as np
        Vh = wl_value_inputs(x)
        Vd = _dev(Vh, x.dtype)
        O = torch.empty((x.B, x.H, x.N, x.d), dtype=tdt, device="cuda")

        def call_attn(i):
            attnw.attnw_attention(Q, K, Vd, O, x.B, x.H, x.N, x.d, scale, dt, stream)

        wall_a, ev_a, k_a, w_a = _time_calls(call_attn, 1, steps, warmup)
        flops = 4.0 * x.elements * x.d
        tf = flops / (ev_a * 1e-3) * 1e-12
        rec["attention_output"] = {
            "call": "attnw_attention", "ms_per_step": round(wall_a, 5), "kernel_ms": round(ev_a, 5),
            "steps": k_a, "warmup": w_a, "mfma_TFLOPs": round(tf, 1),
            "roofline": {"bound": "mfma", "kernel": "attention_kernel", "achieved": round(tf, 1),
                         "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)},
            "elements_per_s": x.elements / (wall_a * 1e-3),
        }
        del O, Vd
    del P
    torch.cuda.empty_cache()
    return rec, x


def wl_value_inputs(x):
    from paper_2407_13885_amd import workloads as wl
    return wl.value_inputs(x, seed=12345)


def cpu_baseline_fused(x, rows_per_head=4096):
    """The oracle as it stands, on the host cores, on a bounded sample of the workload."""
    import oracle
    rows_per_head = min(rows_per_head, x.N)
    # touch the library once so that its build/load is not timed
    oracle.attention_weights(x.Q[0, 0], x.K[0, 0], x.dtype, x.scale, rows=(0, 1))
    t0 = time.perf_counter()
    done = 0
    for b in range(x.B):
        for h in range(x.H):
            oracle.attention_weights(x.Q[b, h], x.K[b, h], x.dtype, x.scale, rows=(0, rows_per_head))
            done += rows_per_head
    dt = time.perf_counter() - t0
    return {
        "value": done * x.N / dt, "unit": "elements/s", "cores": oracle.threads_used(), "kind": "oracle",
        "sample": f"first {rows_per_head} query rows of each of the {x.B * x.H} heads of {x.name} "
                  f"({done} of {x.B * x.H * x.N} rows, {dt:.2f} s wall), fp64, all keys",
        "seconds": round(dt, 3),
    }


def cpu_baseline_softmax(x, rows=8192):
    import oracle
    rows = min(rows, x.rows)
    oracle.softmax(x.S, x.dtype, rows=(0, 1))
    t0 = time.perf_counter()
    oracle.softmax(x.S, x.dtype, rows=(0, rows))
    dt = time.perf_counter() - t0
    return {
        "value": rows * x.cols / dt, "unit": "elements/s", "cores": oracle.threads_used(), "kind": "oracle",
        "sample": f"first {rows} of {x.rows} rows of {x.name} ({dt:.2f} s wall), fp64",
        "seconds": round(dt, 3),
    }


# Shapes off the five configurations: ragged lengths, rows of P / S that do not start on 16-, 64- or 128-byte
# boundaries, head sizes that pad the K rows on chip, many short rows, few very long rows.
# (first five: the n x n matrices of the paper's Table I)
SHAPES_SOFTMAX = [(1024, 1024), (2048, 2048), (4096, 4096), (8192, 8192), (16384, 16384), (24576, 2048), (24576, 2047), (24576, 2040), (6000, 8200), (3000, 16385), (768, 65536), (384, 131072),
                  (96, 524288), (16, 4194304), (100000, 512), (100000, 100), (1000000, 48), (602112, 49), (2000000, 8)]
# (first five: one head of n x 128, the sizes of the paper's Table I)
SHAPES_QK = [("bf16", 1, 1, 1024, 128), ("bf16", 1, 1, 2048, 128), ("bf16", 1, 1, 4096, 128), ("bf16", 1, 1, 8192, 128),
             ("bf16", 1, 1, 16384, 128), ("bf16", 1, 2, 4096, 128), ("bf16", 1, 4, 4096, 128), ("bf16", 1, 8, 4096, 128), ("bf16", 1, 16, 4096, 128), ("bf16", 1, 24, 4096, 128), ("bf16", 1, 32, 4096, 128), ("bf16", 1, 16, 4096, 64), ("bf16", 1, 16, 4096, 96), ("bf16", 1, 16, 4096, 256),
             ("bf16", 1, 16, 4000, 128), ("bf16", 1, 16, 4072, 128), ("bf16", 1, 16, 4104, 128), ("bf16", 1, 16, 4097, 128),
             ("bf16", 1, 16, 2056, 128), ("bf16", 1, 16, 3968, 64), ("bf16", 4, 16, 2049, 64), ("bf16", 8, 16, 1025, 64),
             ("bf16", 16, 12, 577, 64), ("bf16", 16, 12, 576, 64),
             ("bf16", 8, 16, 640, 64), ("bf16", 64, 16, 128, 64), ("bf16", 64, 16, 197, 64),
             ("bf16", 4096, 3, 49, 32), ("bf16", 1024, 4, 64, 32), ("bf16", 64, 16, 100, 64), ("bf16", 64, 12, 64, 64),
             ("f32", 1, 16, 2048, 64),
             ("f32", 1, 16, 4000, 64)]
SHAPES_ATTENTION = [("bf16", 1, 16, 4096, 128), ("bf16", 1, 16, 4096, 64), ("bf16", 1, 32, 4096, 32), ("bf16", 1, 16, 4000, 128),
                    ("bf16", 1, 40, 2100, 64), ("bf16", 8, 16, 512, 64), ("bf16", 64, 16, 197, 64), ("bf16", 1, 2, 32768, 128),
                    ("bf16", 1, 1, 1024, 128), ("bf16", 1, 1, 4096, 128), ("bf16", 1, 4, 4096, 128), ("bf16", 1, 1, 16384, 128),
                    ("bf16", 1, 1, 4096, 64), ("bf16", 1, 16, 4096, 96), ("bf16", 1, 16, 4096, 256), ("bf16", 1, 16, 4096, 192),
                    ("bf16", 4096, 3, 49, 32), ("bf16", 1024, 4, 64, 32), ("bf16", 256, 16, 49, 64), ("bf16", 64, 12, 128, 64),
                    ("bf16", 4, 16, 2049, 64), ("bf16", 8, 16, 1025, 64), ("bf16", 16, 12, 577, 64), ("bf16", 1, 16, 4097, 128),
                    ("f32", 1, 16, 4096, 128), ("f32", 1, 16, 4096, 64), ("f32", 1, 16, 4096, 256), ("f32", 8, 16, 512, 64)]


def bench_shapes(steps, warmup):
    """Every entry point on the shapes above (random normal inputs made on the device, seed 0; time only --
    parity on such shapes is what the GPU tests check).  Shorter sections than the configurations get:
    0.1 s of warm-up, 0.1 s timed unless --steps / --warmup say otherwise."""
    import torch
    import paper_2407_13885_amd as attnw
    global WARM_MS, TIMED_MS
    WARM_MS, TIMED_MS = 100.0, 100.0
    torch.manual_seed(0)
    TD = {"bf16": torch.bfloat16, "f32": torch.float32}
    DT = {"bf16": attnw.ATTNW_BF16, "f32": attnw.ATTNW_F32}
    stream = torch.cuda.current_stream()
    out = []
    for dt in ("bf16", "f32"):
        es = 2 if dt == "bf16" else 4
        for rows, cols in SHAPES_SOFTMAX:
            S = torch.randn(rows, cols, device="cuda", dtype=TD[dt]) * 2.0
            P = torch.empty_like(S)
            _, ev, _, _ = _time_calls(lambda i: attnw.attnw_softmax(S, P, rows, cols, DT[dt], stream), 1, steps, warmup)
            out.append({"call": "attnw_softmax", "dtype": dt, "rows": rows, "cols": cols, "us": round(ev * 1e3, 1),
                        "hbm_GBps": round(2 * rows * cols * es / (ev * 1e-3) * 1e-9, 1)})
            print(f"[bench] {out[-1]}", file=sys.stderr, flush=True)
            del S, P
    for dt, B, H, N, d in SHAPES_QK:
        es = 2 if dt == "bf16" else 4
        Q = torch.randn(B, H, N, d, device="cuda", dtype=TD[dt])
        K = torch.randn_like(Q)
        P = torch.empty(B, H, N, N, device="cuda", dtype=TD[dt])
        alg = (B * H * N * N + 2 * B * H * N * d) * es
        for name, fn in (("attnw_fused", attnw.attnw_fused), ("attnw_gemm_scores", attnw.attnw_gemm_scores)):
            _, ev, _, _ = _time_calls(lambda i: fn(Q, K, P, B, H, N, d, d ** -0.5, DT[dt], stream), 1, steps, warmup)
            out.append({"call": name, "dtype": dt, "B": B, "H": H, "N": N, "d": d, "us": round(ev * 1e3, 1),
                        "hbm_GBps": round(alg / (ev * 1e-3) * 1e-9, 1)})
            print(f"[bench] {out[-1]}", file=sys.stderr, flush=True)
        del Q, K, P
    for dt, B, H, N, d in SHAPES_ATTENTION:
        Q = torch.randn(B, H, N, d, device="cuda", dtype=TD[dt])
        K, V = torch.randn_like(Q), torch.randn_like(Q)
        O = torch.empty_like(Q)
        _, ev, _, _ = _time_calls(lambda i: attnw.attnw_attention(Q, K, V, O, B, H, N, d, d ** -0.5, DT[dt], stream),
                                  1, steps, warmup)
        out.append({"call": "attnw_attention", "dtype": dt, "B": B, "H": H, "N": N, "d": d, "us": round(ev * 1e3, 1),
                    "mfma_TFLOPs": round(4.0 * B * H * N * N * d / (ev * 1e-3) * 1e-12, 1)})
        print(f"[bench] {out[-1]}", file=sys.stderr, flush=True)
        del Q, K, V, O
    return out


def measured_traffic(workload: str, call: str):
    """HBM bytes per launch from the committed rocprofv3 counter summary (profiles/hbm_traffic.txt), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 5 and f[0] == workload and f[1] == call:
                return int(float(f[4]))
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed calls per section (default: as many as fill about 0.3 s)")
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed calls before every timed section (default: as many as fill about 0.4 s, "
                         "the time the shader clock takes to settle under load)")
    ap.add_argument("--workload", default="c4", choices=["c2", "c3", "c4", "c5"],
                    help="configuration reported at the top level of the JSON line")
    ap.add_argument("--only", action="store_true", help="measure the headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-power", action="store_true",
                    help="do not sample board power and shader clock (the sampler starts child processes, which a "
                         "profiler that preloads itself into every process does not allow)")
    ap.add_argument("--no-unfused", action="store_true", help="skip the unfused pair (score GEMM, then softmax)")
    ap.add_argument("--no-attention", action="store_true", help="skip attnw_attention (O = P V with P kept on chip)")
    ap.add_argument("--shapes", action="store_true",
                    help="instead of the configurations, time every entry point on shapes off them (ragged lengths, "
                         "unaligned rows, padded head sizes, short and very long softmax rows); prints one JSON line")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain elementwise copy of 1 GiB (read 1 GiB, write 1 GiB): the known-size "
                         "kernel that rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (heads and query rows shard with no exchange; "
              "every GPU would write its own slab of P); run it with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_2407_13885_amd as attnw
    from paper_2407_13885_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    attnw.load_library()   # raises if libattnw.so is missing: there is no fallback
    torch.cuda.set_device(0)

    if args.shapes:
        print(json.dumps({"metric": "time per call on shapes off the configurations", "unit": "us", "n_gpus": 1,
                          "data": "synthetic", "shapes": bench_shapes(args.steps, args.warmup)}))
        return 0

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)      # one elementwise kernel: 2^30 bytes in, 2^30 bytes out
        torch.cuda.synchronize()
        del src, dst

    # (rocprofv3 preloads a library into every process: no child processes under it)
    sample = not args.no_power and "rocprof" not in os.environ.get("LD_PRELOAD", "")
    order = ["c2", "c3", "c4", "c5"]
    todo = [args.workload] if args.only else order
    results, inputs = {}, {}
    for name in todo:
        print(f"[bench] {name} ...", file=sys.stderr, flush=True)
        if name == "c2":
            results[name], inputs[name] = bench_softmax(wl.c2, args.steps, args.warmup, sample_power=sample and name == args.workload)
        else:
            results[name], inputs[name] = bench_fused(wl.CONFIGS[name], args.steps, args.warmup,
                                                      with_unfused=not args.no_unfused,
                                                      with_attention=not args.no_attention,
                                                      sample_power=sample and name == args.workload)
        if name != args.workload:
            inputs.pop(name)

    head = results[args.workload]
    x = inputs[args.workload]
    cpu = None
    if not args.no_cpu_baseline:
        print("[bench] cpu_baseline (oracle on host cores) ...", file=sys.stderr, flush=True)
        cpu = cpu_baseline_softmax(x) if args.workload == "c2" else cpu_baseline_fused(x)

    dominant = {"c2": "softmax_rows_kernel", "c3": "qk_resident_kernel"}.get(args.workload, "qk_rounds_kernel")
    line = {
        "metric": METRIC,
        "value": head["elements_per_s"],
        "unit": "elements/s",
        "n_gpus": 1, "steps": head["steps"], "warmup": head["warmup"], "preheat_ms": head["preheat_ms"],
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        # bf16 operands on the matrix cores and bf16 storage, fp32 accumulation and fp32 softmax arithmetic
        "dtype": "bf16" if head["shape"].get("dtype", "bf16") == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {head['call']} {json.dumps(head['shape'])}",
                   "generator": wl.GENERATOR_ID, "buffer_sets": head["buffer_sets"]},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": head["hbm_GBps"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": head["hbm_frac_of_peak"],
                     "traffic": measured_traffic(args.workload, head["call"]),
                     # quoted, not measured by this run: the counter summary committed with this build
                     "traffic_source": "profiles/hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this build)",
                     "kernel_source": "the library's dispatch for this shape (kernel names as in profiles/)"},
        # board power and shader clock read while the headline call ran (None: amd-smi absent or silent)
        "power": head.get("power"),
        "cpu_baseline": cpu,
        "fused_vs_unfused_speedup": {k: v.get("fused_vs_unfused_speedup") for k, v in results.items()
                                     if "fused_vs_unfused_speedup" in v},
        "fused_vs_three_kernels_speedup": {k: v.get("fused_vs_three_kernels_speedup") for k, v in results.items()
                                           if "fused_vs_three_kernels_speedup" in v},
        "workloads": results,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
