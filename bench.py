#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: fused forward + JVP of the relaxed top-k operator.

A step is one pass of the whole path (load, sort, isotonic solve, un-sort scatter, JVP) over one
batch of the chosen synthetic workload, through the C ABI.  Inputs are resident in HBM before the
timed region.  Two regimes are timed with HIP events on the launch stream:

  cold : the steps rotate over enough distinct buffer sets (> 512 MiB) that no step finds its
         inputs in the 256 MiB Infinity Cache -- this is `value` and the roofline figure;
  warm : every step uses the same buffers (reported in `warm`, an "effective" rate).

Prints ONE JSON line.  `python bench.py --gpus 1 --steps K --warmup W [--workload NAME]`.
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

HBM_PEAK_GBPS = 8000.0            # MI355X HBM3E, published peak
BYTES_PER_ELEMENT = 16            # read theta, read tangent, write mask, write JVP (fp32 each)
METRIC = "rows/s and GB/s (% HBM peak) for topkmask fwd+JVP, 16384x64 k=2 p=2"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="moe_router")
    ap.add_argument("--op", choices=["jvp", "signed_mask_jvp", "masked_value_jvp", "loss"], default="jvp",
                    help="side run: time another entry point on the workload's inputs (mask workloads): "
                         "the operators on |x| or the Fenchel-Young loss, instead of forward + JVP")
    ap.add_argument("--mode", choices=["graph", "stream"], default="graph",
                    help="graph: the K launches are captured once in a HIP graph and replayed; "
                         "stream: K plain launches from Python")
    ap.add_argument("--cold-mib", type=int, default=640, help="footprint of the rotating buffer sets")
    ap.add_argument("--regime", choices=["both", "cold"], default="both",
                    help="cold: skip the warm (same-buffer) measurement, e.g. under a profiler")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the operator, time a plain device copy of the same footprint "
                         "(theta|tangent -> out|jvp); used to scale the rocprofv3 byte counters")
    ap.add_argument("--sweep-solvers", action="store_true",
                    help="instead of the one JSON line: forward pass of the mask (p = 2) over row "
                         "lengths 16 .. 2^22, exact solve vs 100 Dykstra iterations vs torch.topk")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the one JSON line: time the mask forward + JVP over row lengths "
                         "64 .. 2^24 at a constant 2^24 elements, k = ceil(n/10) (the paper's timing "
                         "sweep uses k = ceil(n/10)), lambda = 0.1, one JSON line per row length")
    ap.add_argument("--route", action="append", default=[], metavar="WHICH=VALUE",
                    help="tuning run: set a route control of the library (topk_set_route), e.g. 2=1")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the timing of the other four workloads (key `workloads`)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=4.0)
    return ap.parse_args()


class Runner:
    """Pre-marshalled calls into the C ABI (no allocation, no tensor checks in the timed loop)."""

    def __init__(self, w, sets, device, entry="jvp"):
        import ctypes
        import torch
        from paper_2302_01425_amd import binding
        self.torch = torch
        self.lib = binding.load()
        self.w = w
        x, t = w.inputs()
        xd, td = torch.from_numpy(x).to(device), torch.from_numpy(t).to(device)
        self.bufs = []
        for _ in range(sets):
            self.bufs.append((xd.clone(), td.clone(), torch.empty_like(xd), torch.empty_like(xd)))
        op = binding.TOPK_OP_MASK_JVP if w.op == "mask" else binding.TOPK_OP_MAG_JVP
        binding.ensure_workspace(op, w.rows, w.n, w.k, w.p, device)
        self.fn = self.lib.topk_mask_jvp if w.op == "mask" else self.lib.topkmag_jvp
        if entry != "jvp":
            if w.op != "mask":
                raise SystemExit("--op needs a mask workload")
            which = {"signed_mask_jvp": binding.TOPK_OP_SIGNED_MASK,
                     "masked_value_jvp": binding.TOPK_OP_MASKED_VALUE, "loss": binding.TOPK_OP_MASK_FWD}[entry]
            binding.ensure_workspace(which, w.rows, w.n, w.k, w.p, device)
            self.fn = {"signed_mask_jvp": self.lib.topk_signed_mask_jvp,
                       "masked_value_jvp": self.lib.topk_masked_value_jvp,
                       "loss": self.lib.topk_mask_loss}[entry]
        # (the loss takes (theta, target, .., loss_out [rows], grad_out): the first floats of the
        # third buffer hold the per-row losses)
        self.args = [(ctypes.c_void_p(a.data_ptr()), ctypes.c_void_p(b.data_ptr()),
                      ctypes.c_int64(w.rows), ctypes.c_int64(w.n), ctypes.c_int64(w.k),
                      ctypes.c_double(w.p), ctypes.c_double(w.lam),
                      ctypes.c_void_p(c.data_ptr()), ctypes.c_void_p(d.data_ptr()))
                     for (a, b, c, d) in self.bufs]
        self.ctypes = ctypes
        self.copy_mode = False
        self.copies = []

    def enable_copy_mode(self):
        """Plain copies with the operator's footprint: 2 arrays in, 2 arrays out per step."""
        torch = self.torch
        self.copy_mode = True
        for (a, b, c, d) in self.bufs:
            src = torch.cat([a.reshape(-1), b.reshape(-1)])
            self.copies.append((src, torch.empty_like(src)))

    def launch(self, i, stream_ptr):
        if self.copy_mode:
            src, dst = self.copies[i % len(self.copies)]
            self.torch.mul(src, 1.0, out=dst)   # one plain elementwise kernel: reads src, writes dst
            return
        rc = self.fn(*self.args[i % len(self.args)], stream_ptr)
        if rc != 0:
            raise RuntimeError(f"library call failed: {rc}")

    def timed(self, steps, warmup, mode, rotate, min_ms=20.0):
        """Times `steps` steps with HIP events on the launch stream and returns (milliseconds per
        step, repeats).  The K steps (one captured graph, or K plain launches) are repeated R times
        between the two events, R chosen from one untimed pass so that the timed region lasts at
        least `min_ms`: the one-off cost of starting a graph or a launch burst is then spread over
        R * K steps and the figure does not depend on K."""
        torch = self.torch
        nsets = len(self.args) if rotate else 1
        stream = torch.cuda.Stream()
        sp = self.ctypes.c_void_p(stream.cuda_stream)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            for i in range(warmup):
                self.launch(i % nsets, sp)
            stream.synchronize()
            graph = None
            if mode == "graph":
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    for i in range(steps):
                        self.launch(i % nsets, sp)
                graph.replay()                      # one untimed replay (upload, page-in)
                stream.synchronize()

            def one_pass():
                if graph is not None:
                    graph.replay()
                else:
                    for i in range(steps):
                        self.launch(i % nsets, sp)

            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            one_pass()
            e1.record(stream)
            torch.cuda.synchronize()
            repeats = max(1, min(2000, int(-(-min_ms // max(e0.elapsed_time(e1), 1e-3)))))
            e0.record(stream)
            for _ in range(repeats):
                one_pass()
            e1.record(stream)
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (repeats * steps), repeats


def cpu_baseline(w, seconds):
    """The float64 oracle, as it stands, on this machine's host cores (OpenMP over rows)."""
    import oracle
    oracle.build()
    x, t = w.inputs()
    fn = oracle.topk_mask if w.op == "mask" else oracle.topkmag
    rows_cap = w.rows
    if w.rows * w.n > (1 << 22):                       # bounded sample of very large workloads
        rows_cap = max(1, (1 << 22) // w.n)
    xs, ts = x[:rows_cap], t[:rows_cap]
    if w.rows == 1 and w.n > (1 << 22):                # a single giant row: a prefix of it
        xs, ts = x[:, : 1 << 22], t[:, : 1 << 22]
    k = min(w.k, xs.shape[1]) if xs.shape[1] == w.n else max(1, xs.shape[1] // 10)
    fn(xs, k, w.p, w.lam, tangent=ts)                  # warm the library and the caches
    reps, t0 = 0, time.perf_counter()
    while True:
        fn(xs, k, w.p, w.lam, tangent=ts)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= seconds:
            break
    rows_done = reps * xs.shape[0]
    threads = oracle.max_threads() if xs.shape[0] > 1 else 1
    return {
        "value": rows_done / dt, "unit": "rows/s", "cores": threads, "kind": "oracle",
        "sample": f"{reps} x ({xs.shape[0]} rows x {xs.shape[1]}) of the workload, fwd+JVP, "
                  f"{dt:.1f} s wall",
        "elements_per_s": rows_done * xs.shape[1] / dt,
    }


def sweep(a):
    """Row-length sweep at a constant element count (all three kernel families and the
    transitions between them).  Not the benchmark contract: one JSON line per row length."""
    import torch
    from paper_2302_01425_amd.workloads import Workload
    total = 1 << 24
    for p in (2.0, 4.0 / 3.0):
        for lg in (6, 8, 10, 11, 13, 15, 17, 18, 20, 22, 24):
            n = 1 << lg
            rows = total // n
            w = Workload(f"sweep_n{n}", "mask", rows, n, -(-n // 10), p, 0.1, 7, "normal", 1.0)
            set_bytes = 4 * 4 * rows * n
            sets = max(2, -(-a.cold_mib * (1 << 20) // set_bytes))
            r = Runner(w, sets, "cuda:0")
            steps = max(10, min(200, int(2e5 / max(50.0, 1e-6 * total))))
            ms, _ = r.timed(steps, 5, a.mode, rotate=True)
            print(json.dumps({"sweep": "mask fwd+JVP, 2^24 elements, k = ceil(n/10), lambda = 0.1",
                              "p": round(p, 4), "n": n, "rows": rows, "us_per_step": ms * 1e3,
                              "gbps": BYTES_PER_ELEMENT * total / (ms * 1e-3) / 1e9,
                              "frac_of_hbm_peak": BYTES_PER_ELEMENT * total / (ms * 1e-3) / 1e9
                              / HBM_PEAK_GBPS}), flush=True)
            del r
            torch.cuda.empty_cache()


def sweep_solvers(a):
    """Forward pass of the relaxed top-k mask (p = 2, lambda = 0.1) against the row length, with
    k = ceil(n / 10) as in the paper's run-time comparison (Sec. 5, figure "Runtime comparison"):
    the library's exact solve, 100 iterations of Dykstra's algorithm (rows up to 1024 elements;
    the general-weights kernels on rank weights up to 131072), and a hard top-k (torch.topk, the framework's own primitive).  2^22 elements per call,
    stream launches timed with events.  Not the benchmark contract: one JSON line per length."""
    import torch
    from paper_2302_01425_amd import binding
    from paper_2302_01425_amd.workloads import Workload
    total = 1 << 22
    stream = torch.cuda.Stream()

    def timed(fn, steps=20, warmup=3):
        with torch.cuda.stream(stream):
            for _ in range(warmup):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            stream.synchronize()
            e0.record(stream)
            for _ in range(steps):
                fn()
            e1.record(stream)
            stream.synchronize()
        return e0.elapsed_time(e1) / steps * 1e3

    for lg in (4, 6, 8, 10, 12, 14, 16, 18, 20, 22):
        n = 1 << lg
        rows = total // n
        k = -(-n // 10)
        w = Workload(f"solvers_n{n}", "mask", rows, n, k, 2.0, 0.1, 8, "normal", 1.0)
        x = torch.from_numpy(w.inputs()[0]).cuda()
        out = torch.empty_like(x)
        binding.ensure_workspace(binding.TOPK_OP_MASK_FWD, rows, n, k, 2.0, x.device)
        line = {"sweep": "mask fwd, p = 2, lambda = 0.1, 2^22 elements, k = ceil(n/10)", "n": n,
                "rows": rows}
        line["exact_us"] = timed(lambda: binding.topk_mask_fwd(x, k, 2.0, 0.1, out=out, stream=stream))
        if n <= 1024:
            line["dykstra100_us"] = timed(
                lambda: binding.topk_mask_dykstra_fwd(x, k, 0.1, 100, out=out, stream=stream))
            exact = binding.topk_mask_fwd(x, k, 2.0, 0.1)
            approx = binding.topk_mask_dykstra_fwd(x, k, 0.1, 100)
            line["dykstra100_max_abs_diff"] = float((exact - approx).abs().max())
        if n <= binding.TOPK_GENERAL_ROW_MAX:
            # the full PAV partition for general weights, here the relaxed ranks y(-theta, rho)
            rho = torch.arange(n, 0, -1, dtype=torch.float32, device=x.device)
            xneg = -x
            binding.ensure_workspace(binding.TOPK_OP_GENERAL, rows, n, 0, 2.0, x.device)
            line["general_w_rank_us"] = timed(
                lambda: binding.topk_general_fwd(xneg, rho, binding.TOPK_PHI_IDENTITY, 2.0, 0.1,
                                                 out=out, stream=stream))
        line["hard_topk_us"] = timed(lambda: torch.topk(x, k, dim=1))
        print(json.dumps(line), flush=True)
        del x, out
        torch.cuda.empty_cache()


def other_workloads(a, traffic_table):
    """The other four configurations, each timed like the headline one (cold, same launch mode):
    per workload the time of a step, the rate of algorithmic bytes (16 B per element) and its
    fraction of the HBM peak; for the two long-row workloads also the fraction against a byte model
    that includes a whole-row 4-pass LSD radix sort through HBM (16 + 4 + 4 x 16 B per element),
    which is what sorting the rows completely would move."""
    import torch
    from paper_2302_01425_amd.workloads import WORKLOADS
    res = {}
    for name in ("tiny", "moe_router_smooth", "expert_choice", "magnitude_pruning"):
        w = WORKLOADS[name]
        elems = w.rows * w.n
        set_bytes = 4 * 4 * elems
        sets = max(2, -(-a.cold_mib * (1 << 20) // set_bytes))
        sets = min(sets, 64)                              # tiny: 64 sets are plenty of launches
        r = Runner(w, sets, "cuda:0")
        steps = max(2, min(a.steps, int(2e8 // elems) or 2))
        ms, reps = r.timed(steps, min(a.warmup, 5), a.mode, rotate=True)
        del r
        torch.cuda.empty_cache()
        gbps = BYTES_PER_ELEMENT * elems / (ms * 1e-3) / 1e9
        e = {"ms_per_step": ms, "steps": steps, "repeats": reps, "rows_per_s": w.rows / (ms * 1e-3),
             "gbps": gbps, "frac": gbps / HBM_PEAK_GBPS}
        if w.n > 1024:
            e["frac_sort_inclusive_model"] = (16 + 4 + 4 * 16) * elems / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS
        t = traffic_table.get(name)
        if t:
            e["traffic"] = t["total_bytes"]
        res[name] = e
    return res


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (rows are independent; nothing here "
              "uses a second GPU). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2302_01425_amd.workloads import WORKLOADS
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if a.route:
        from paper_2302_01425_amd import binding
        for item in a.route:
            which, value = item.split("=")
            binding.set_route(int(which), int(value))
    if a.sweep:
        sweep(a)
        return
    if a.sweep_solvers:
        sweep_solvers(a)
        return
    w = WORKLOADS[a.workload]
    algo_bytes = BYTES_PER_ELEMENT * w.rows * w.n
    set_bytes = 4 * 4 * w.rows * w.n
    sets = min(64, max(2, -(-a.cold_mib * (1 << 20) // set_bytes)))   # (tiny: 64 sets are plenty)
    r = Runner(w, sets, "cuda:0", a.op)
    if a.op != "jvp":
        # side run: another entry point on the same inputs; its own byte model (the loss reads
        # theta and the target and writes the gradient and one float per row)
        per_b = 12.0 + 4.0 / w.n if a.op == "loss" else 16.0
        ms, reps = r.timed(a.steps, a.warmup, a.mode, rotate=True)
        print(json.dumps({"side_run": a.op, "workload": w.name, "steps": a.steps, "repeats": reps,
                          "ms_per_step": ms, "algorithmic_bytes_per_element": per_b,
                          "gbps": per_b * w.rows * w.n / (ms * 1e-3) / 1e9,
                          "frac_of_hbm_peak": per_b * w.rows * w.n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}))
        return
    if a.copy_calibration:
        r.enable_copy_mode()
        ms, reps = r.timed(a.steps, a.warmup, a.mode, rotate=True)
        print(json.dumps({"calibration": "plain copy", "bytes_read_per_step": algo_bytes // 2,
                          "bytes_written_per_step": algo_bytes // 2, "steps": a.steps,
                          "repeats": reps, "ms_per_step": ms,
                          "gbps": algo_bytes / (ms * 1e-3) / 1e9}))
        return

    per_cold, reps = r.timed(a.steps, a.warmup, a.mode, rotate=True)
    per_warm = r.timed(a.steps, a.warmup, a.mode, rotate=False)[0] if a.regime == "both" else per_cold
    del r
    torch.cuda.empty_cache()

    gbps_cold = algo_bytes / (per_cold * 1e-3) / 1e9
    gbps_warm = algo_bytes / (per_warm * 1e-3) / 1e9
    traffic_table = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic_table = json.load(f)
    entry = traffic_table.get(a.workload)
    traffic = entry["total_bytes"] if entry else None    # HBM bytes per launch (rocprofv3)

    line = {
        "metric": METRIC if a.workload == "moe_router" else f"rows/s for {w.op} fwd+JVP, {a.workload}",
        "value": w.rows / (per_cold * 1e-3),
        "unit": "rows/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "repeats": reps,
        "ms_per_step": per_cold,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: {w.rows} rows x n={w.n}, k={w.k}, p={w.p:.6g}, "
                        f"lambda={w.lam}, {w.op} forward + JVP fused, fp32 in/out",
            "regime": f"cold: {sets} rotating buffer sets, {sets * set_bytes >> 20} MiB",
            "launch": a.mode,
            "timed_region": f"{reps} x {a.steps} steps between one pair of HIP events",
            "solve_arithmetic": "f64",
        },
        "elements_per_s": w.rows * w.n / (per_cold * 1e-3),
        "gbps": gbps_cold,
        "pct_hbm_peak": 100.0 * gbps_cold / HBM_PEAK_GBPS,
        "warm": ({"ms_per_step": per_warm, "rows_per_s": w.rows / (per_warm * 1e-3),
                  "effective_gbps": gbps_warm} if a.regime == "both" else None),
        "roofline": {
            "bound": "hbm", "achieved": gbps_cold, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": gbps_cold / HBM_PEAK_GBPS, "traffic": traffic,
            "algorithmic_bytes_per_launch": algo_bytes,
        },
    }
    if a.workload == "moe_router" and not a.headline_only:
        line["workloads"] = other_workloads(a, traffic_table)
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, a.cpu_seconds)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
