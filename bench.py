#!/usr/bin/env python3
"""Benchmark of the segment-wise gossip mixing path on one MI355X.

A step is one gossip round over the whole workload: generate the round's peer tables
(Algorithm 2, host), upload them (a few KB), and run one mixing launch over all W rows
(Algorithm 1) from one HBM-resident buffer into the other (ping-pong; --in-place updates a
single buffer instead).  The parameter matrix is resident in HBM before timing starts.
Prints ONE JSON line: the whole-step rate (`value`, algorithmic GB/s = 8 B per worker-parameter
and round; 20 B with the fused optimizer), `roofline` (the mixing kernel's own rate from events
around each launch, against the 8 TB/s HBM peak, with the profiled HBM traffic), `copy_ceiling`
(a plain copy of the same footprint), `topology_gen` (host time of the table generator) and
`cpu_baseline` (the CPU oracle timed on this host).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--all]
                    [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth


def dtype_of(kind, rows16) -> str:
    """The type the path computes in: the mixing steps in fp32, the optimizer steps in fp64 registers."""
    arith = "f64" if kind in ("fused", "hiersgd") else "f32"
    if rows16:
        return f"{arith} ({rows16} rows" + (", f32 momentum" if arith == "f64" else "") + " in HBM)"
    return arith if arith == "f32" else "f64 (f32 rows in HBM)"


def entry_point(kind, rows16) -> str:
    return {"fused": "cx_sgd_fused_mix", "hiersgd": "cx_hier_sgd_fused_mix"}.get(kind, f"cx_{kind}_mix") + (
        "_" + rows16 if rows16 else "")


def describe(wl, rows="fp32") -> str:
    s = f"{wl.name}: W={wl.W} P={wl.P} {rows} S={wl.S}"
    if wl.G > 1:
        s += f" hierarchical G={wl.G} L={wl.L}"
    if wl.layers:
        s += f" segments on {wl.layers} ragged layer boundaries"
    return s


class Runner:
    """Holds one workload's device state and issues its steps."""

    def __init__(self, wl, kind, total_rounds, in_place=False, rows16=None, ld_multiple=1024, allocator="spread"):
        import torch
        from paper_2012_15198_amd import cxmix as cx
        from paper_2012_15198_amd import workloads as WL
        self.torch, self.cx, self.wl, self.kind = torch, cx, wl, kind
        dev = "cuda:0"
        self.so_host = WL.seg_off_for(wl)
        cx.cx_check_segments(self.so_host, wl.P)
        self.so = torch.from_numpy(self.so_host).to(dev)
        # layout: rows padded to a multiple of 1024 floats (4 KB) so every row starts on a cache
        # line and DRAM page boundary; two buffers, the rounds ping-pong between them
        self.in_place = in_place
        self.ld = (wl.P + ld_multiple - 1) // ld_multiple * ld_multiple
        self.rows16 = rows16                              # None (fp32 rows), "bf16" or "f16"
        rows_dt = {None: torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[rows16]
        self.n = wl.L if kind in ("hier", "hiersgd") else wl.W
        self.S = 1 if kind == "pushsum" else wl.S
        self.mode = 1 if kind == "pushsum" else 0
        # every matrix of the job from one placement call: x and x' (one buffer when in place), and for the
        # optimizer steps the fp32 momentum v, v' and the gradients g (rows of x's type)
        full = (wl.W, self.ld)
        want = [("x", full, rows_dt)] + ([] if in_place else [("y", full, rows_dt)])
        if kind in ("fused", "hiersgd"):
            vshape = full if kind == "fused" else (wl.L, self.ld)
            want += [("v", vshape, torch.float32)] + ([] if in_place else [("v2", vshape, torch.float32)])
            want += [("g", full, rows_dt)]
        self.allocator = allocator
        if allocator == "spread":
            try:
                bufs = cx.hbm_empty([w[1] for w in want], [w[2] for w in want], device=dev)
            except (cx.CxError, RuntimeError) as e:       # placement is an optimisation: say so and go on
                print(f"bench.py: cx_hbm_alloc unavailable ({e}); using torch's allocator", file=sys.stderr)
                self.allocator = f"torch (cx_hbm_alloc failed: {e})"
                bufs = None
        if allocator != "spread" or bufs is None:
            bufs = [torch.empty(w[1], dtype=w[2], device=dev) for w in want]
        for (name, _, _), t in zip(want, bufs):
            setattr(self, name, t)
        if in_place:
            self.y = self.x
        WL.gen_matrix_device(wl.W, wl.P, wl.sigma, wl.seed, ld=self.ld, device=dev, out=self.x)
        # one pinned + one device slot per round, so the host can run ahead of the GPU
        self.tab_host = torch.empty((total_rounds, self.S, self.n), dtype=torch.int32, pin_memory=True)
        self.tab_np = self.tab_host.numpy()
        self.tab_dev = torch.empty((total_rounds, self.S, self.n), dtype=torch.int32, device=dev)
        self.bytes_per_elem = bytes_per_element(kind, wl.G, rows16)
        if kind in ("fused", "hiersgd"):
            c4 = WL.WORKLOADS["C4"]            # the hierarchical step takes C4's optimizer constants and gradient scale
            self.lr, self.mu, self.wd = c4.lr, c4.mu, c4.wd
            self.v.zero_()                                                 # the momentum stays fp32
            if in_place:
                self.v2 = self.v
            WL.gen_matrix_device(wl.W, wl.P, c4.grad_sigma, wl.seed, ld=self.ld, stream=2, device=dev, out=self.g)
        if kind == "pushsum":
            self.w = [torch.ones(wl.W, device=dev), torch.zeros(wl.W, device=dev)]
        self.round = 0
        self.ev = []
        torch.cuda.synchronize()

    def step(self, timed: bool):
        torch, cx, wl, r = self.torch, self.cx, self.wl, self.round
        cx.cx_topology_gen(wl.seed, self.n, self.S, r, 1, self.mode, out=self.tab_np[r:r + 1])
        self.tab_dev[r].copy_(self.tab_host[r], non_blocking=True)
        tab = self.tab_dev[r]
        if timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        if self.kind == "gossip" and self.rows16:
            mix16 = cx.cx_gossip_mix_bf16 if self.rows16 == "bf16" else cx.cx_gossip_mix_f16
            mix16(self.x, self.y, wl.P, self.so, tab)
        elif self.kind == "gossip":
            cx.cx_gossip_mix(self.x, self.y, wl.P, self.so, tab)
        elif self.kind == "hier" and self.rows16:
            mix16 = cx.cx_hier_mix_bf16 if self.rows16 == "bf16" else cx.cx_hier_mix_f16
            mix16(self.x, self.y, wl.P, wl.G, self.so, tab)
        elif self.kind == "hier":
            cx.cx_hier_mix(self.x, self.y, wl.P, wl.G, self.so, tab)
        elif self.kind == "fused":
            fused = {None: cx.cx_sgd_fused_mix, "bf16": cx.cx_sgd_fused_mix_bf16, "f16": cx.cx_sgd_fused_mix_f16}[self.rows16]
            fused(self.x, self.y, self.v, self.v2, self.g, wl.lr, wl.mu, wl.wd, wl.P, self.so, tab)
            self.v, self.v2 = self.v2, self.v
        elif self.kind == "hiersgd":
            hsgd = {None: cx.cx_hier_sgd_fused_mix, "bf16": cx.cx_hier_sgd_fused_mix_bf16,
                    "f16": cx.cx_hier_sgd_fused_mix_f16}[self.rows16]
            hsgd(self.x, self.y, self.v, self.v2, self.g, self.lr, self.mu, self.wd, wl.P, wl.G, self.so, tab)
            self.v, self.v2 = self.v2, self.v
        elif self.kind == "pushsum":
            hop = int((0 - int(self.tab_np[r, 0, 0])) % wl.W)
            push = {None: cx.cx_pushsum_mix, "bf16": cx.cx_pushsum_mix_bf16, "f16": cx.cx_pushsum_mix_f16}[self.rows16]
            push(self.x, self.y, self.w[r & 1], self.w[1 - (r & 1)], None, wl.P, hop)
        self.x, self.y = self.y, self.x
        if timed:
            e1.record()
            self.ev.append((e0, e1))
        self.round += 1

    def run(self, steps, warmup):
        torch = self.torch
        for _ in range(warmup):
            self.step(False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step(True)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        kernel_ms = [a.elapsed_time(b) for a, b in self.ev]
        wl = self.wl
        elems = wl.W * wl.P
        alg_bytes = int(elems * self.bytes_per_elem)
        ms_step = wall * 1e3 / steps
        k_avg = float(np.mean(kernel_ms))
        return {
            "kind": self.kind, "ms_per_step": ms_step,
            "GBps": alg_bytes / (ms_step * 1e-3) / 1e9,
            "params_mixed_per_s": elems / (ms_step * 1e-3),
            "kernel_ms_avg": k_avg, "kernel_ms_min": float(np.min(kernel_ms)),
            "kernel_ms_median": float(np.median(kernel_ms)),
            "kernel_GBps": alg_bytes / (k_avg * 1e-3) / 1e9,
            "alg_bytes_per_launch": alg_bytes,
        }

    def allocation_spread(self, count, steps):
        """The same calls on `count` further allocations of the parameter matrix, the earlier ones kept
        alive so that each lands on other physical pages: kernel time per allocation (median over `steps`
        calls, events around each call).  Shows how much of a figure is placement, not code."""
        torch = self.torch
        held, out = [], []
        alg = self.wl.W * self.wl.P * self.bytes_per_elem
        for k in range(count):
            if k:
                held.append((self.x, self.y))
                fresh = torch.empty_like(self.x).copy_(self.x)
                self.y = fresh if self.in_place else torch.empty_like(self.x)
                self.x = fresh
            for _ in range(2):
                self.step(False)
            self.ev = []
            for _ in range(steps):
                self.step(True)
            torch.cuda.synchronize()
            t = float(np.median([a.elapsed_time(b) for a, b in self.ev]))
            out.append({"address": hex(self.x.data_ptr()), "kernel_ms_median": t,
                        "frac_of_hbm_peak": alg / (t * 1e-3) / 1e9 / HBM_PEAK_GBPS})
        return out

    def buffer_pairs(self, count, steps):
        """Out-of-place calls between every ordered pair of `count` allocations of the matrix (all alive at
        once): kernel time per (source, destination), median over `steps` calls.  Shows which of the two
        buffers' placement sets the rate."""
        torch = self.torch
        keep = (self.x, self.y)
        bufs = [torch.empty_like(self.x) for _ in range(count)]       # plain allocations, one after the other
        for b in bufs:
            b.copy_(self.x)
        alg = self.wl.W * self.wl.P * self.bytes_per_elem
        out = []
        for i in range(count):
            for j in range(count):
                if i == j:
                    continue
                self.ev = []
                for k in range(steps + 1):
                    self.x, self.y = bufs[i], bufs[j]
                    self.step(k > 0)
                torch.cuda.synchronize()
                t = float(np.median([a.elapsed_time(b) for a, b in self.ev]))
                out.append({"source": i, "destination": j, "kernel_ms_median": t,
                            "frac_of_hbm_peak": alg / (t * 1e-3) / 1e9 / HBM_PEAK_GBPS})
        self.x, self.y = keep
        return {"addresses": [hex(b.data_ptr()) for b in bufs], "pairs": out}

    def whole_step_latency(self, rounds):
        """One step at a time, the device idle before and after: host clock around topology generation,
        table upload, launch and completion.  Median and minimum over `rounds` steps, in ms."""
        torch = self.torch
        lat = []
        for _ in range(rounds):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            self.step(False)
            torch.cuda.synchronize()
            lat.append((time.perf_counter() - t0) * 1e3)
        return {"median": float(np.median(lat)), "min": float(np.min(lat)), "rounds": rounds}


def kernel_source_id():
    """Short hash of the kernel sources: a profile summary carries the one it was taken with."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2012_15198_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hpp", ".hip")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def profile_name(workload, kind, in_place, rows16=None):
    return f"{workload}_{kind}{'_' + rows16 if rows16 else ''}_{'inplace' if in_place else 'pingpong'}"


def profiled_traffic(workload, kind, in_place, rows16=None, tuning=None):
    """HBM bytes per launch from the committed rocprofv3 counter summary of this workload and entry
    point (FETCH_SIZE and WRITE_SIZE, scaled by the copy-kernel calibration).  The figure is NOT measured
    in this run, so it is reported only if the summary was taken with the kernel sources as they are now
    and with default launch parameters; otherwise (None, why)."""
    name = profile_name(workload, kind, in_place, rows16) + "_pmc.txt"
    path = os.path.join(ROOT, "profiles", name)
    if tuning:
        return None, "launch parameters changed with --tune: no profile for them"
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None, f"no profiles/{name}"
    traffic = src = None
    for line in lines:
        if line.startswith("traffic_bytes_per_launch:"):
            traffic = float(line.split(":")[1])
        if line.startswith("kernel_source_id:"):
            src = line.split(":")[1].strip()
    if traffic is None:
        return None, f"profiles/{name} holds no traffic figure"
    if src != kernel_source_id():
        return None, f"profiles/{name} was taken with kernel sources {src}, these are {kernel_source_id()}"
    return traffic, f"profiles/{name} (kernel sources {src})"


def copy_ceiling(nbytes, reps=10, allocator="spread"):
    """Plain streaming copy with the same footprint split (read n/2, write n/2), its two buffers placed
    like the workload's."""
    import torch
    from paper_2012_15198_amd import cxmix as cx
    n = (nbytes // 8) // 4 * 4
    if allocator == "spread":
        src, dst = cx.hbm_empty([(n,), (n,)])
    else:
        src, dst = torch.empty(n, dtype=torch.float32, device="cuda:0"), torch.empty(n, dtype=torch.float32, device="cuda:0")
    src.normal_()
    for _ in range(2):
        cx.cx_copy_baseline(src, dst)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        cx.cx_copy_baseline(src, dst)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    return {"GBps": 8.0 * n / (ms * 1e-3) / 1e9, "ms": ms, "bytes": 8 * n}


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def topology_gen_time(runner):
    """Host time of cx_topology_gen for the workload's whole table (all its rounds), outside the timed region."""
    wl, cx = runner.wl, runner.cx
    buf = np.empty((wl.rounds, runner.S, runner.n), dtype=np.int32)
    best = float("inf")
    for _ in range(5):
        t0 = time.perf_counter()
        cx.cx_topology_gen(wl.seed, runner.n, runner.S, 0, wl.rounds, runner.mode, out=buf)
        best = min(best, time.perf_counter() - t0)
    return {"host_ms_whole_table": best * 1e3, "rounds": wl.rounds, "segments": runner.S, "ranks": runner.n,
            "host_us_per_round": best * 1e6 / wl.rounds}


def cpu_baseline(wl, kind, rows16=None, budget_s=12.0, max_bytes=8 << 30):
    """The CPU oracle, as it stands, timed on this host on the entry point's own function: full rounds of
    the workload where a round's matrices fit `max_bytes`, otherwise on the first columns of every row
    (mixing is independent per column; segments are cut at the last column taken).  Inputs are drawn on
    the host with the workload's recipe."""
    import oracle as O
    from paper_2012_15198_amd import workloads as WL
    c4 = WL.WORKLOADS["C4"]
    lr, mu, wd = (wl.lr, wl.mu, wl.wd) if wl.lr else (c4.lr, c4.mu, c4.wd)
    mats = {"gossip": 1, "hier": 1, "pushsum": 1, "fused": 3, "hiersgd": 2 + 1.0 / wl.G}[kind]
    n = wl.L if kind in ("hier", "hiersgd") else wl.W
    S = 1 if kind == "pushsum" else wl.S
    fmt = rows16
    narrow = {None: lambda a: a, "bf16": lambda a: (a.view(np.uint32) >> 16).astype(np.uint16),
              "f16": lambda a: a.astype(np.float16).view(np.uint16)}[fmt]       # input preparation only
    tabs = O.topology(wl.seed, n, S, 0, 16, 1 if kind == "pushsum" else 0)
    name = {"gossip": "oracle_gossip_mix", "hier": "oracle_hier_mix_f64", "pushsum": "oracle_pushsum_mix_f32",
            "fused": "oracle_sgd_fused_mix_f64", "hiersgd": "oracle_hier_sgd_fused_mix_f64"}[kind]
    if fmt:
        name = {"gossip": f"oracle_gossip_mix_{fmt}", "hier": "oracle_hier_mix16", "fused": "oracle_sgd_fused_mix16",
                "hiersgd": "oracle_hier_sgd_fused_mix16", "pushsum": "oracle_pushsum_mix16"}[kind]
    x = v = g = so = spare = None
    w = np.ones(wl.W, dtype=np.float32)
    P = 0

    def draw(cols):
        nonlocal x, v, g, so, P, spare
        P, spare = cols, None
        so = np.minimum(WL.seg_off_for(wl), P).astype(np.int64)
        x = narrow(WL.gen_matrix(wl.W, P, wl.sigma, wl.seed))
        if kind in ("fused", "hiersgd"):
            g = narrow(WL.gen_matrix(wl.W, P, wl.grad_sigma or c4.grad_sigma, wl.seed, stream=2))
            v = np.zeros((n if kind == "hiersgd" else wl.W, P), dtype=np.float32)

    def one_round(r):
        nonlocal x, v, w
        t = tabs[r % 16]
        nonlocal spare
        if kind == "gossip" and not fmt:
            if spare is None:
                spare = np.empty_like(x)
            spare = O.gossip_mix(x, P, so, t, out=spare)          # two buffers in turn, as on the device
            x, spare = spare, x
        elif kind == "gossip":
            x = (O.gossip_mix_bf16 if fmt == "bf16" else O.gossip_mix_f16)(x, P, so, t)
        elif kind == "hier":
            x = O.hier_mix_f64(x, P, wl.G, so, t).astype(np.float32) if not fmt else O.hier_mix16(fmt, x, P, wl.G, so, t)
        elif kind == "pushsum":
            hop = int((0 - int(t[0, 0])) % wl.W)
            x, w, _ = O.pushsum_mix16(fmt, x, w, P, hop, False) if fmt else O.pushsum_mix_f32(x, w, P, hop, False)
        elif kind == "fused":
            if fmt:
                x, v = O.sgd_fused_mix16(fmt, x, v, g, lr, mu, wd, P, so, t)
            else:
                x, v = (a.astype(np.float32) for a in O.sgd_fused_mix_f64(x, v, g, lr, mu, wd, P, so, t))
        else:
            if fmt:
                x, v = O.hier_sgd_fused_mix16(fmt, x, v, g, lr, mu, wd, P, wl.G, so, t)
            else:
                x, v = (a.astype(np.float32) for a in O.hier_sgd_fused_mix_f64(x, v, g, lr, mu, wd, P, wl.G, so, t))

    # size of the sample: what memory allows, cut down so that a round takes about a quarter of the budget
    cols = int(min(wl.P, max_bytes // (4 * wl.W * mats * 2)))           # inputs and outputs
    probe = min(cols, 16384)
    draw(probe)
    t0 = time.perf_counter()
    one_round(0)
    per_col = (time.perf_counter() - t0) / probe
    cols = int(max(probe, min(cols, budget_s / 4 / per_col)))
    draw(cols)
    one_round(0)                                                      # touch the pages
    rounds, t0 = 0, time.perf_counter()
    while True:
        one_round(rounds + 1)
        rounds += 1
        dt = time.perf_counter() - t0
        if dt > budget_s or rounds >= 40:
            break
    bpe = bytes_per_element(kind, wl.G, rows16)
    elems = wl.W * P
    what = "full rounds" if P == wl.P else f"rounds on columns [0, {P}) of every row ({100.0 * P / wl.P:.1f} % of the matrix)"
    return {"value": bpe * elems * rounds / dt / 1e9, "unit": "GB/s",
            "params_mixed_per_s": elems * rounds / dt, "s_per_round": dt / rounds,
            "s_per_full_round": dt / rounds * wl.P / P,
            "cores": 1, "kind": "oracle",
            "sample": f"{rounds} {what} of {describe(wl, rows16 or 'fp32')} ({name}, single thread, "
                      f"{os.cpu_count()} host cores visible, {cpu_model()})"}


def bytes_per_element(kind, G, rows16):
    """Algorithmic bytes per worker-parameter and round: every element read once and written once."""
    if kind == "fused":
        return 14 if rows16 else 20                   # x, v, g in; x, v out (16-bit x and g, fp32 v)
    if kind == "hiersgd":
        return 4 + 10.0 / G if rows16 else 8 + 12.0 / G
    return 4 if rows16 else 8


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--kind", default=None, choices=[None, "gossip", "hier", "fused", "pushsum", "hiersgd"],
                    help="entry point to time (default: the workload's own; C4 has fused and pushsum)")
    ap.add_argument("--all", action="store_true", help="also time the other workloads' entry points")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-copy", action="store_true")
    ap.add_argument("--bf16", action="store_true", help="bfloat16 rows (every entry point has a _bf16 variant)")
    ap.add_argument("--f16", action="store_true", help="binary16 rows (every entry point has a _f16 variant)")
    ap.add_argument("--tune", default="", metavar="KEY=VALUE[,KEY=VALUE...]",
                    help="launch parameters for cx_set_tuning (see include/cx_mix.h), e.g. 6=8,1=4")
    ap.add_argument("--allocations", type=int, default=0, metavar="K",
                    help="also time the calls on K allocations of the matrix within this process (placement spread)")
    ap.add_argument("--buffer-pairs", type=int, default=0, metavar="K",
                    help="also time out-of-place calls between every ordered pair of K allocations (gossip, hier)")
    ap.add_argument("--allocator", default=None, choices=["spread", "torch"],
                    help="where the matrices come from: cx_hbm_alloc (every buffer spread over the physical memory; "
                         "the default) or torch's allocator (hipMalloc; the default with --allocations / --buffer-pairs)")
    ap.add_argument("--in-place", action="store_true",
                    help="update the matrix in place (cycle-walk kernel) instead of ping-pong buffers")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (W simulated workers share one MI355X); "
                 "--gpus must be 1")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    from paper_2012_15198_amd import cxmix as cx
    from paper_2012_15198_amd import workloads as WL
    cx.lib()                                            # fail loudly if the library is not built
    tuning = {}
    for item in filter(None, args.tune.split(",")):
        k, v = item.split("=")
        cx.cx_set_tuning(int(k), int(v))
        tuning[int(k)] = int(v)

    wl = WL.WORKLOADS[args.workload]
    kind = args.kind or {"gossip": "gossip", "hier": "hier", "fused+pushsum": "fused"}[wl.kind]
    if args.bf16 and args.f16:
        sys.exit("bench.py: --bf16 and --f16 exclude each other")
    rows16 = "bf16" if args.bf16 else "f16" if args.f16 else None
    latency_rounds = min(wl.rounds, 20)
    spread_steps = min(args.steps, 8)
    if args.buffer_pairs and (args.in_place or kind not in ("gossip", "hier") or args.buffer_pairs < 2):
        sys.exit("bench.py: --buffer-pairs K needs K >= 2 and an out-of-place gossip or hierarchical call")
    pair_rounds = args.buffer_pairs * (args.buffer_pairs - 1) * (spread_steps + 1)
    allocator = args.allocator or ("torch" if args.allocations or args.buffer_pairs else "spread")
    runner = Runner(wl, kind, args.steps + args.warmup + latency_rounds + args.allocations * (spread_steps + 2) + pair_rounds,
                    in_place=args.in_place, rows16=rows16, allocator=allocator)
    res = runner.run(args.steps, args.warmup)
    traffic, traffic_source = profiled_traffic(wl.name, kind, args.in_place, rows16, tuning)
    out = {
        "metric": "gossip-mix HBM GB/s and params-mixed/s per round (fraction of HBM peak), 1 GPU",
        "value": res["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dtype_of(kind, rows16),
        "data": "synthetic",
        "config": {"workload": describe(wl, rows16 or "fp32") if kind != "gossip" or wl.G == 1
                   else describe(wl, rows16 or "fp32") + " (flat gossip over all rows)",
                   "entry_point": entry_point(kind, rows16),
                   "rounds_timed": args.steps, "in_place": bool(args.in_place), "ld": runner.ld,
                   "buffers": "in place" if args.in_place else "ping-pong (x_in -> x_out, swapped every round)",
                   "allocator": {"spread": "cx_hbm_alloc (each matrix in 256 MiB pieces spread over the free physical memory)",
                                 "torch": "torch (hipMalloc)"}.get(runner.allocator, runner.allocator),
                   "step": "cx_topology_gen(1 round) + table upload + one mixing launch",
                   "tuning": tuning or "defaults"},
        "params_mixed_per_s": res["params_mixed_per_s"],
        "frac_of_hbm_peak": res["GBps"] / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "achieved": res["kernel_GBps"], "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": res["kernel_GBps"] / HBM_PEAK_GBPS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "profiled_traffic_GBps": traffic / (res["kernel_ms_avg"] * 1e-3) / 1e9 if traffic else None,
                     "kernel": "mix_kernel" if args.in_place else "gather_kernel",
                     "kernel_ms_avg": res["kernel_ms_avg"],
                     "kernel_ms_min": res["kernel_ms_min"], "kernel_ms_median": res["kernel_ms_median"],
                     "alg_bytes_per_launch": res["alg_bytes_per_launch"]},
    }
    out["whole_step_latency_ms"] = runner.whole_step_latency(latency_rounds)
    out["topology_gen"] = topology_gen_time(runner)
    if args.allocations:
        out["allocation_spread"] = runner.allocation_spread(args.allocations, spread_steps)
    if args.buffer_pairs:
        out["buffer_pairs"] = runner.buffer_pairs(args.buffer_pairs, spread_steps)
    if not args.no_copy:
        out["copy_ceiling"] = copy_ceiling(res["alg_bytes_per_launch"], allocator="spread" if runner.allocator == "spread" else "torch")
    del runner
    torch.cuda.empty_cache()
    out["cpu_baseline"] = None if args.no_cpu_baseline else cpu_baseline(wl, kind, rows16)

    if args.all:
        # every other workload and entry point: events around each round's call over the workload's own
        # number of rounds (median and minimum), the whole-step latency, and the oracle on the host
        others = {}
        plan = [("C1", "gossip", None), ("C2", "gossip", None), ("C2", "gossip", "bf16"), ("C2", "gossip", "f16"),
                ("C3", "hier", None), ("C3", "hier", "bf16"), ("C3", "hiersgd", None), ("C3", "hiersgd", "bf16"),
                ("C4", "fused", None), ("C4", "fused", "bf16"), ("C4", "pushsum", None), ("C4", "pushsum", "bf16"),
                ("C5", "hier", None)]
        for name, k, r16 in plan:
            if name == args.workload and k == kind and r16 == rows16:
                continue
            w2 = WL.WORKLOADS[name]
            r = Runner(w2, k, 2 * w2.rounds + 3, in_place=args.in_place, rows16=r16, allocator=allocator)
            rr = r.run(w2.rounds, 3)
            rr["workload"] = describe(w2, r16 or "fp32")
            rr["entry_point"] = entry_point(k, r16)
            rr["rounds"] = w2.rounds
            rr["frac_of_hbm_peak_kernel"] = rr["kernel_GBps"] / HBM_PEAK_GBPS
            rr["frac_of_hbm_peak_kernel_median"] = rr["alg_bytes_per_launch"] / (rr["kernel_ms_median"] * 1e-3) / 1e9 / HBM_PEAK_GBPS
            rr["whole_step_latency_ms"] = r.whole_step_latency(w2.rounds)
            rr["traffic"], rr["traffic_source"] = profiled_traffic(name, k, args.in_place, r16, tuning)
            del r
            torch.cuda.empty_cache()
            if not args.no_cpu_baseline:
                rr["cpu_baseline"] = cpu_baseline(w2, k, r16, budget_s=5.0)
            others[f"{name}:{k}" + (f":{r16}" if r16 else "")] = rr
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
