#!/usr/bin/env python3
"""Benchmark of the GR-KAN group-wise rational layer (FlashKAT hot path) on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic
activations at the KAT-B shape (per-GPU batch 128, 197 tokens): the forward and
the backward of both rational layers of a Transformer block,
x1 [128,197,768] and x2 [128,197,3072], 8 groups, degrees (5,4), float32,
in training order  fwd(x1) fwd(x2) bwd(x2) bwd(x1).  (--workload selects the
other configurations; the one-tensor ones run fwd(x) bwd(x).)
`value` = elements that went through forward+backward per second, with the
inputs resident in HBM.  Successive steps rotate over several buffer sets per layer so
that no launch finds its inputs in the 256 MB last-level cache.

Prints ONE JSON line: metric/value/unit (elements per second through forward+backward),
ms_per_step, `roofline` (the dominant kernel, the backward of the widest tensor, priced
against the HBM peak for float32 I/O and against the vector-ALU issue rate for bfloat16 I/O),
`device` (what the runtime reports), `detail` (per-kernel timings), `paper_micro_benchmark`
(the shape of the paper's kernel benchmark) and `cpu_baseline` (the fp64 CPU oracle timed on
the host cores).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak
VALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12  # 39.3 T lane-operations/s: 256 CUs x 64 lanes x 2.4 GHz, unpacked float32
# The backward stage-1 kernel with 16-bit I/O, per element, at the KAT-B x2 shape:
#   first number:  vector-ALU instructions issued, measured with the SQ_INSTS_VALU counter (wave instructions x
#                  64 lanes / elements; the summary is under profiles/);
#   second number: the same instructions in issue slots of 4 clocks (the 39.3 T rate: one wave instruction per
#                  SIMD in 4 clocks).  Micro-benchmarks of independent instruction streams on this chip give, per
#                  wave instruction and SIMD: 1.05-1.4 ns (0.6-0.85 slot) when every operand is a vector register,
#                  1.7-1.9 ns (1.0-1.1 slots) with a scalar-register or literal operand (the coefficients) and for
#                  conversions / shifts, 3.45 ns (2.1 slots, about 8 clocks) for v_rcp_f32.  The hot loop's
#                  instructions (from the compiler's assembly) priced with these costs give the slot count.
# The roofline fraction uses the slots; the plain count (every instruction one slot, the reciprocal too) would
# put the kernel at 0.95 of the same peak and is an upper bound on what the peak means.
BWD_VALU_16BIT = {
    ("bf16", 3, 2): (29.52, 24.54), ("bf16", 5, 4): (43.97, 36.64), ("bf16", 7, 6): (57.93, 48.74),
    ("f16", 3, 2): (29.58, 25.02), ("f16", 5, 4): (44.03, 36.87), ("f16", 7, 6): (57.98, 48.73),
}

WORKLOAD_LABEL = {"tiny": "tiny [4,197,192]", "kat_t": "KAT-T", "kat_s": "KAT-S", "kat_b": "KAT-B",
                  "stress": "stress [256,197,3072]"}


def measured_traffic(key):
    """HBM bytes per launch of the dominant kernel as rocprofv3 --pmc counted them
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size) in an earlier,
    separate profiler run: read from the tracked summaries under profiles/, which
    carry one line `traffic_bytes_per_launch[<workload>/<dtype>/<kernel>] = <bytes>`
    per measured kernel.  Returns (bytes, file name) or (None, None): nothing is
    counted in this run itself."""
    import re

    pat = re.compile(r"^traffic_bytes_per_launch\[%s\]\s*=\s*(\d+)\s*$" % re.escape(key), re.M)
    for f in sorted((ROOT / "profiles").glob("*.txt")):
        m = pat.search(f.read_text())
        if m:
            return int(m.group(1)), "profiles/" + f.name
    return None, None


IO_CODE = {"f32": 0, "bf16": 1, "f16": 2}  # grkan_dtype_t


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="kat_b", choices=["tiny", "kat_t", "kat_s", "kat_b", "stress"])
    ap.add_argument("--groups", type=int, default=0, help="override the number of groups (stress: 1, 8 or 64)")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16", "f16"])
    ap.add_argument("--degrees", default="5,4", help="m,n of the rational function: 5,4 (the paper's), 3,2 or 7,6")
    ap.add_argument("--sets", type=int, default=0,
                    help="buffer sets each layer rotates over (0 = enough that one rotation of the smallest "
                         "kernel moves more than 1.1 GB, i.e. several times the 256 MB last-level cache)")
    ap.add_argument("--preheat-ms", type=float, default=600.0,
                    help="before the warm-up steps, run untimed steps for this long (wall-clock): a GPU that has been "
                         "idle takes some hundred launches to reach its sustained clocks (measured: the same kernel "
                         "113 us in the first hundred launches, 97 in the second, 93 in the third); 0 = none")
    ap.add_argument("--event-every", type=int, default=4,
                    help="bracket the dominant kernel with HIP events on every N-th timed step (1 = every step): an "
                         "event pair costs the stream about 11 us of idle time per step (two ~5.5 us gaps in the "
                         "kernel trace), which is instrumentation, not the workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-detail", action="store_true", help="skip the per-kernel table")
    ap.add_argument("--no-paper-micro", action="store_true",
                    help="skip the paper's kernel micro-benchmark shape [1024,197,768]")
    ap.add_argument("--alg1-baseline", action="store_true",
                    help="also time the paper's Algorithm 1 (per-element global atomics) on both layers; "
                         "float32 only, takes several seconds")
    ap.add_argument("--mlp-block", action="store_true",
                    help="also time the KAT MLP block (two GR-KAN layers, torch GEMMs) against a standard "
                         "GELU MLP block, forward+backward, at the workload's x1 shape")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the HIP-graph leg (one rotation of steps captured once and replayed: what a "
                         "launch-bound caller gains; the entry points only enqueue kernels)")
    ap.add_argument("--fused-linear", action="store_true",
                    help="measure only the fused GR-KAN layer forward out = W F(x) + bias (grkan_linear_fwd, bfloat16, "
                         "one MFMA kernel) at the workload's two layer shapes against grkan_fwd followed by torch's "
                         "matrix product, and print its own JSON line (roofline: dense bf16 MFMA peak)")
    ap.add_argument("--no-fused", action="store_true",
                    help="skip the short fused-layer measurement that is part of the default line")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain device copy of x2's size (for scaling profiler byte counters)")
    return ap.parse_args()


class Layer:
    """Device buffers of one rational layer, `sets` copies of everything."""

    def __init__(self, case, sets, torch, grkan):
        import grkan_inputs

        self.rows, self.D, self.G = case["rows"], case["D"], case["G"]
        self.M = self.rows * self.D
        self.es = 4 if case["dtype"] == "f32" else 2
        if sets <= 0:
            sets = max(2, -(-1_100_000_000 // self.fwd_bytes()))
        self.sets = sets
        first = grkan_inputs.upload(case, "cuda:0")
        self.A, self.B = first["A"], first["B"]
        self.x = [first["x"]] + [first["x"].clone() for _ in range(sets - 1)]
        self.dy = [first["dy"]] + [first["dy"].clone() for _ in range(sets - 1)]
        self.y = [torch.empty_like(first["x"]) for _ in range(sets)]
        self.dx = [torch.empty_like(first["x"]) for _ in range(sets)]
        self.dA = torch.empty_like(self.A)
        self.dB = torch.empty_like(self.B)
        io = IO_CODE[case["dtype"]]
        need = grkan.grkan_bwd_workspace_bytes(self.rows, self.D, self.G, io)
        self.ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
        self.grkan = grkan

    def fwd(self, i):
        s = i % self.sets
        self.grkan.grkan_fwd(self.x[s], self.A, self.B, out=self.y[s])

    def bwd(self, i):
        s = i % self.sets
        self.grkan.grkan_bwd(self.x[s], self.dy[s], self.A, self.B, workspace=self.ws,
                             out=(self.dx[s], self.dA, self.dB))

    def fwd_bytes(self):
        return 2 * self.es * self.M

    def bwd_bytes(self):
        return 3 * self.es * self.M


def time_launches(torch, fn, n):
    """Average device time (ms) of n launches of fn(i), from HIP events on the
    launch stream."""
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for i in range(n):
        ev[i][0].record()
        fn(i)
        ev[i][1].record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in ev)
    return sum(ts) / len(ts), ts[len(ts) // 2], ts[0]


def launch_stats(torch, fn, n):
    """As time_launches, plus the half-width of the 95 % confidence interval of
    the mean (normal approximation, 1.96 s / sqrt(n)), all in ms."""
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for i in range(n):
        ev[i][0].record()
        fn(i)
        ev[i][1].record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in ev)
    mean = sum(ts) / n
    var = sum((t - mean) ** 2 for t in ts) / max(1, n - 1)
    return mean, ts[n // 2], ts[0], 1.96 * (var / n) ** 0.5


def device_report(torch, grkan):
    """What the runtime reports about the device, and the HBM peak that
    follows from memory clock x bus width, beside the published figure the
    roofline divides by.  The reported memory clock is HBM3E's command clock;
    the data strobe runs at twice that, double data rate: 4 bits per pin per
    reported cycle (2000 MHz -> 8 Gb/s per pin)."""
    p = torch.cuda.get_device_properties(0)
    q = grkan.device_query()
    return {
        "name": p.name, "compute_units": q["compute_units"], "hbm_bytes": p.total_memory,
        "engine_clock_MHz": q["engine_clock_khz"] / 1e3, "memory_clock_MHz": q["memory_clock_khz"] / 1e3,
        "memory_bus_bits": q["memory_bus_bits"],
        "hbm_peak_from_clock_x_bus_GBs": 4.0 * q["memory_clock_khz"] * 1e3 * q["memory_bus_bits"] / 8 / 1e9,
        "published_hbm_peak_GBs": HBM_PEAK_GBS,
    }


def cpu_baseline(cases):
    """The fp64 oracle, as it stands, on the host cores: one forward+backward
    pass over the same arrays."""
    import numpy as np

    from oracle import grkan_oracle

    cores = len(os.sched_getaffinity(0))
    threads = max(1, min(cores, grkan_oracle.max_threads()))
    prepared = []
    for c in cases:
        prepared.append((c["x"].astype(np.float64), c["dy"].astype(np.float64),
                         c["A"].astype(np.float64), c["B"].astype(np.float64)))
    grkan_oracle.fwd(prepared[0][0][:64], prepared[0][2], prepared[0][3], threads=threads)  # load + warm
    passes = 0
    t0 = time.perf_counter()
    while True:
        for x, dy, A, B in prepared:
            grkan_oracle.fwd(x, A, B, threads=threads)
            grkan_oracle.bwd(x, dy, A, B, threads=threads)
        passes += 1
        dt = time.perf_counter() - t0
        if dt * threads >= 15.0 or passes >= 20:  # about 15 core-seconds of oracle work
            break
    elems = passes * sum(int(p[0].size) for p in prepared)
    # the same oracle on one thread (the sequential definition), on a bounded slice of the widest tensor
    x, dy, A, B = prepared[-1]
    rows1 = max(1, min(x.shape[0], 12_000_000 // x.shape[1]))
    t1 = time.perf_counter()
    grkan_oracle.fwd(x[:rows1], A, B, threads=1)
    grkan_oracle.bwd(x[:rows1], dy[:rows1], A, B, threads=1)
    dt1 = time.perf_counter() - t1
    return {
        "value": elems / dt, "unit": "elements/s", "cores": threads, "kind": "oracle",
        "sample": "%d fwd+bwd pass(es) of the fp64 C oracle over the whole workload (%d elements in total, %.2f s wall)"
                  % (passes, elems, dt),
        "single_thread": {"value": rows1 * x.shape[1] / dt1, "unit": "elements/s", "cores": 1,
                          "sample": "one fwd+bwd pass over the first %d rows of the widest tensor (%d elements, %.2f s)"
                                    % (rows1, rows1 * x.shape[1], dt1)},
    }


MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bfloat16 matrix peak, published


def fused_linear_bench(torch, grkan, grkan_inputs, workload, launches, layers_wanted=("x2", "x1"), copy_calibration=False,
                       preheat_ms=150.0):
    """The fused layer forward at the workload's layer shapes (x1 -> 4 D, x2 -> D / 4), bfloat16:
    grkan_linear_fwd against grkan_fwd + torch.addmm (the library matrix product) and the matrix
    product alone, each the mean of `launches` event-timed launches rotating over four input sets
    (the inputs of the wide layer are 155 MB each: no launch finds its x in the last-level cache)."""
    out = {}
    cfg = grkan_inputs.CONFIGS[workload]
    names = [t for t, _ in cfg.tensors]
    for tensor in layers_wanted:
        if tensor not in names:
            continue
        case = grkan_inputs.make_linear_case(workload, tensor)
        dev = grkan_inputs.upload_linear(case)
        rows, K, N = case["rows"], case["D_in"], case["D_out"]
        sets = 4
        xs = [dev["x"]] + [dev["x"].clone() for _ in range(sets - 1)]
        outs = [torch.empty(rows, N, device="cuda:0", dtype=torch.bfloat16) for _ in range(sets)]
        ys = [torch.empty_like(dev["x"]) for _ in range(sets)]
        bias16 = dev["bias"].to(torch.bfloat16)
        Wt = dev["W"].t()
        flop = 2.0 * rows * K * N

        def fused(i):
            grkan.grkan_linear_fwd(xs[i % sets], dev["A"], dev["B"], dev["W"], dev["bias"], out=outs[i % sets])

        def fused_packed(i):
            grkan.grkan_linear_fwd(xs[i % sets], dev["A"], dev["B"], packed_w, dev["bias"], out=outs[i % sets])

        def two_kernels(i):
            grkan.grkan_fwd(xs[i % sets], dev["A"], dev["B"], out=ys[i % sets])
            torch.addmm(bias16, ys[i % sets], Wt, out=outs[i % sets])

        def product_only(i):
            torch.addmm(bias16, ys[i % sets], Wt, out=outs[i % sets])

        res = {"shape": "[%d,%d] x [%d,%d]^T" % (rows, K, N, K), "GFLOP": flop / 1e9}
        try:
            fused(0)
        except grkan.GrkanError as exc:
            # e.g. the first layer of KAT-T / KAT-S: groups of 24 / 48 channels, not a multiple of 32
            res["fused"] = {"unsupported": str(exc)}
            out["fc2" if tensor == "x2" else "fc1"] = res
            del xs, outs, ys, dev
            torch.cuda.empty_cache()
            continue
        packed_w = grkan.grkan_linear_pack_w(dev["W"])  # the weights' packed copy (inference: made once)
        for key, fn in (("fused", fused), ("fused_packed_weights", fused_packed),
                        ("grkan_fwd_plus_library_matmul", two_kernels), ("library_matmul_alone", product_only)):
            # untimed: the clocks settle to this kernel's sustained state (the first ~100 launches after a
            # change of load run up to 20 % slower), then 5 warm-up launches
            t_pre, k = time.perf_counter(), 0
            while (time.perf_counter() - t_pre) * 1e3 < preheat_ms:
                for i in range(16):
                    fn(k + i)
                k += 16
                torch.cuda.synchronize()
            for i in range(5):
                fn(i)
            mean, med, mn, ci = launch_stats(torch, fn, launches)
            res[key] = {"avg_us": mean * 1e3, "ci95_us": ci * 1e3, "median_us": med * 1e3, "min_us": mn * 1e3,
                        "TFLOP/s": flop / (mean * 1e-3) / 1e12}
        res["fused_over_two_kernels"] = res["fused"]["avg_us"] / res["grkan_fwd_plus_library_matmul"]["avg_us"]
        res["fused_packed_over_two_kernels"] = (res["fused_packed_weights"]["avg_us"]
                                                / res["grkan_fwd_plus_library_matmul"]["avg_us"])
        res["fused_packed_over_library_matmul_alone"] = (res["fused_packed_weights"]["avg_us"]
                                                         / res["library_matmul_alone"]["avg_us"])
        # bytes the method has to move: x and W read once, out written once
        res["algorithmic_bytes"] = 2 * (rows * K + N * K + rows * N) + 4 * N
        if copy_calibration:
            for i in range(3):
                ys[i % sets].copy_(xs[i % sets])
            torch.cuda.synchronize()
        out["fc2" if tensor == "x2" else "fc1"] = res
        del xs, outs, ys, dev, packed_w
        torch.cuda.empty_cache()
    return out


def fused_linear_main(args, torch, grkan, grkan_inputs):
    res = fused_linear_bench(torch, grkan, grkan_inputs, args.workload, max(20, args.steps),
                             copy_calibration=args.copy_calibration, preheat_ms=min(args.preheat_ms, 200.0))
    supported = [v for v in res.values() if "avg_us" in v.get("fused", {})]
    if not supported:
        print("bench.py: grkan_linear_fwd covers none of this workload's layers: %s" % res, file=sys.stderr)
        sys.exit(2)
    dom = res["fc2"] if res.get("fc2") in supported else supported[0]
    best = "fused_packed_weights"  # the inference path: weights packed once
    achieved = dom[best]["TFLOP/s"]
    traffic, traffic_src = measured_traffic("%s/bf16/linear_fwd_fc2_packed" % args.workload)
    line = {
        "metric": "fused GR-KAN layer forward out = W F(x) + bias, %s shapes: time and fraction of the MFMA peak"
                  % WORKLOAD_LABEL[args.workload],
        "value": achieved, "unit": "TFLOP/s", "n_gpus": 1, "steps": max(20, args.steps), "warmup": 5,
        "ms_per_step": dom[best]["avg_us"] / 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %s" % (args.workload, "; ".join("%s %s" % (k, v["shape"]) for k, v in res.items()))},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic, "traffic_source": traffic_src,
                     "kernel": "grkan_linear_fwd_kernel (packed weights) on %s, %.1f GFLOP per launch, avg %.2f us"
                               % (dom["shape"], dom["GFLOP"], dom[best]["avg_us"])},
        "detail": res,
        "device": device_report(torch, grkan),
    }
    print(json.dumps(line))


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path has no collective); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import grkan_inputs
    import paper_2505_13813_amd as grkan

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    grkan.load_library()  # raises if the HIP library is not built: there is no fallback
    torch.cuda.set_device(0)
    if args.fused_linear:
        fused_linear_main(args, torch, grkan, grkan_inputs)
        return

    cfg = grkan_inputs.CONFIGS[args.workload]
    G = args.groups if args.groups > 0 else cfg.G
    m_deg, n_deg = (int(v) for v in args.degrees.split(","))
    if (m_deg, n_deg) not in grkan.DEGREES:
        print("bench.py: degrees must be one of %s" % (grkan.DEGREES,), file=sys.stderr)
        sys.exit(2)
    cases = [grkan_inputs.make_case(args.workload, t, G=G, dtype=args.dtype, m=m_deg, n=n_deg)
             for t, _ in cfg.tensors]
    layers = [Layer(c, args.sets, torch, grkan) for c in cases]
    names = [t for t, _ in cfg.tensors]
    dom = layers[-1]  # the widest tensor: its backward pass is the dominant kernel
    dom_name = names[-1]

    def step(i):
        for layer in layers:
            layer.fwd(i)
        for layer in reversed(layers):
            layer.bwd(i)

    # untimed: bring the clocks to their sustained state, then the W warm-up steps the contract asks for
    preheat_steps = 0
    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < args.preheat_ms:
        for i in range(8):
            step(preheat_steps + i)
        preheat_steps += 8
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # timed region: exactly `steps` steps; events bracket the dominant kernel
    # (backward of the widest tensor) on the launch stream
    every = max(1, args.event_every)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range((args.steps + every - 1) // every)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        for layer in layers:
            layer.fwd(i)
        sampled = i % every == 0
        if sampled:
            ev[i // every][0].record()
        dom.bwd(i)
        if sampled:
            ev[i // every][1].record()
        for layer in reversed(layers[:-1]):
            layer.bwd(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    ms_per_step = dt * 1e3 / args.steps
    elems_per_step = sum(layer.M for layer in layers)
    step_bytes = sum(layer.fwd_bytes() + layer.bwd_bytes() for layer in layers)
    dom_ms = sum(a.elapsed_time(b) for a, b in ev) / len(ev)
    key = "%s/%s/bwd_%s" % (args.workload, args.dtype, dom_name)
    if (m_deg, n_deg) != (5, 4):
        key += "/%d,%d" % (m_deg, n_deg)
    valu = BWD_VALU_16BIT.get((args.dtype, m_deg, n_deg))
    what = "grkan_bwd on %s [%d,%d] (stage 1 + stage 2)" % (dom_name, dom.rows, dom.D)
    hbm_gbs = dom.bwd_bytes() / (dom_ms * 1e-3) / 1e9
    if args.dtype == "f32" or valu is None:
        traffic, traffic_src = measured_traffic(key)
        roofline = {
            "bound": "hbm", "achieved": hbm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": hbm_gbs / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_src,
            "kernel": "%s, %d algorithmic bytes per launch, avg %.2f us" % (what, dom.bwd_bytes(), dom_ms * 1e3),
        }
    else:
        # 16-bit I/O halves the bytes but not the arithmetic: the backward pass is bound by the vector ALU.
        # Peak = 256 CUs x 64 lanes x 2.4 GHz: one wave instruction per SIMD in 4 clocks.
        instr, slots = valu
        achieved = slots * dom.M / (dom_ms * 1e-3) / 1e12
        roofline = {
            "bound": "alu", "achieved": achieved, "peak": VALU_PEAK_TOPS, "unit": "T lane-op/s",
            "frac": achieved / VALU_PEAK_TOPS, "traffic": None,
            "valu_instr_per_element": instr, "issue_slots_per_element": slots,
            "frac_if_every_instr_were_one_slot": instr * dom.M / (dom_ms * 1e-3) / 1e12 / VALU_PEAK_TOPS,
            "hbm_GBs": hbm_gbs, "hbm_frac_of_peak": hbm_gbs / HBM_PEAK_GBS,
            "kernel": "%s, %.2f issue slots (%.2f vector-ALU instructions) per element x %d elements per launch, "
                      "avg %.2f us" % (what, slots, instr, dom.M, dom_ms * 1e3),
        }

    if args.copy_calibration:
        # a copy of known size: reads and writes dom.M elements once each
        for i in range(3):
            dom.y[i % dom.sets].copy_(dom.x[i % dom.sets])
        torch.cuda.synchronize()

    graph_replay = None
    if not args.no_graph:
        # one rotation over the buffer sets (so that a replay touches every set once; at most 64 steps),
        # captured once.  Reported beside the eager figure, never instead of it.
        try:
            per_replay = min(64, max(layer.sets for layer in layers))
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step(0)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for i in range(per_replay):
                    step(i)
            replays = max(1, args.steps // per_replay)
            for _ in range(2):
                graph.replay()
            torch.cuda.synchronize()
            tg = time.perf_counter()
            for _ in range(replays):
                graph.replay()
            torch.cuda.synchronize()
            tg = (time.perf_counter() - tg) / (replays * per_replay)
            graph_replay = {"steps_per_replay": per_replay, "replays": replays, "us_per_step": tg * 1e6,
                            "elements_per_s": elems_per_step / tg, "eager_us_per_step": ms_per_step * 1e3}
            del graph
        except Exception as exc:  # the eager measurement above stands on its own
            graph_replay = {"error": "%s: %s" % (type(exc).__name__, exc)}

    detail = None
    if not args.no_detail:
        # per kernel: 5 warm-ups, then 100 timed launches between HIP events (the paper's protocol),
        # rotating over the buffer sets; then the same with one buffer set, labelled "warm" (its inputs
        # and outputs may still sit in the 256 MB last-level cache from the launch before)
        detail = {}
        n = 100
        for name, layer in zip(names, layers):
            for pname, fn, nbytes in (("fwd", layer.fwd, layer.fwd_bytes()), ("bwd", layer.bwd, layer.bwd_bytes())):
                for i in range(5):
                    fn(i)
                avg, med, mn, ci = launch_stats(torch, fn, n)
                for _ in range(5):
                    fn(0)
                w_avg, w_med, w_mn, w_ci = launch_stats(torch, lambda _i, fn=fn: fn(0), n)
                detail["%s_%s" % (pname, name)] = {
                    "avg_us": avg * 1e3, "ci95_us": ci * 1e3, "median_us": med * 1e3, "min_us": mn * 1e3,
                    "GB/s": nbytes / (avg * 1e-3) / 1e9, "frac_of_peak": nbytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "Gelem/s": layer.M / (avg * 1e-3) / 1e9,
                    "warm_single_buffer": {"avg_us": w_avg * 1e3, "ci95_us": w_ci * 1e3, "median_us": w_med * 1e3,
                                           "min_us": w_mn * 1e3, "GB/s": nbytes / (w_avg * 1e-3) / 1e9},
                }

    paper_micro = None
    if not args.no_paper_micro and args.dtype == "f32" and (m_deg, n_deg) == (5, 4):
        # The paper's own kernel benchmark (Sec. "Insight 2" / Table 2 and Table 3): X, dO of shape
        # [1024, 197, 768], 8 groups; it reports 4.89 ms forward (KAT CUDA kernel) and 7.33 ms backward
        # (FlashKAT, Triton; 1.03 s with the atomics) on an RTX 4060 Ti.  Seeded N(0,1) inputs drawn on the GPU.
        rows_p, D_p, G_p = 1024 * 197, 768, 8
        gen = torch.Generator(device="cuda:0").manual_seed(1000)
        A_p = (torch.rand(G_p, 6, device="cuda:0", generator=gen) * 2 - 1) / torch.arange(1, 7, device="cuda:0")
        B_p = torch.rand(G_p, 4, device="cuda:0", generator=gen) - 0.5
        xs = [torch.randn(rows_p, D_p, device="cuda:0", generator=gen) for _ in range(2)]
        dys = [torch.randn(rows_p, D_p, device="cuda:0", generator=gen) for _ in range(2)]
        outs = [torch.empty(rows_p, D_p, device="cuda:0") for _ in range(2)]
        dA_p, dB_p = torch.empty_like(A_p), torch.empty_like(B_p)
        ws_p = torch.empty(grkan.grkan_bwd_workspace_bytes(rows_p, D_p, G_p, grkan.GRKAN_F32), dtype=torch.uint8,
                           device="cuda:0")
        f_avg, _, _ = time_launches(torch, lambda i: grkan.grkan_fwd(xs[i % 2], A_p, B_p, out=outs[i % 2]), 30)
        b_avg, _, _ = time_launches(
            torch, lambda i: grkan.grkan_bwd(xs[i % 2], dys[i % 2], A_p, B_p, workspace=ws_p,
                                             out=(outs[i % 2], dA_p, dB_p)), 30)
        m_p = rows_p * D_p
        paper_micro = {
            "shape": [1024, 197, 768], "G": G_p, "elements": m_p,
            "fwd_ms": f_avg, "fwd_GBs": 8 * m_p / (f_avg * 1e-3) / 1e9,
            "bwd_ms": b_avg, "bwd_GBs": 12 * m_p / (b_avg * 1e-3) / 1e9,
            "paper": {"hardware": "RTX 4060 Ti", "fwd_ms": 4.89, "bwd_flashkat_ms": 7.33, "bwd_kat_atomics_ms": 1030.0},
        }
        del xs, dys, outs

    alg1 = None
    if args.alg1_baseline and args.dtype == "f32" and (m_deg, n_deg) == (5, 4):
        # the paper's "before": Table 3 reports 1.03 s against 7.33 ms (140.5x) on an RTX 4060 Ti
        alg1 = {}
        for name, layer in zip(names, layers):
            outs = (layer.dx[0], layer.dA, layer.dB)
            grkan.grkan_alg1_bwd(layer.x[0], layer.dy[0], layer.A, layer.B, out=outs)  # warm
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            grkan.grkan_alg1_bwd(layer.x[0], layer.dy[0], layer.A, layer.B, out=outs)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            ours_ms, _, _ = time_launches(torch, layer.bwd, 20)
            alg1["bwd_" + name] = {"alg1_ms": ms, "grkan_bwd_ms": ours_ms, "speedup": ms / ours_ms}

    block = None
    if args.mlp_block:
        # context for the paper's closing remark that FlashKAT remains roughly a quarter slower than a standard Transformer
        from paper_2505_13813_amd import nn as gnn

        block = {}
        dim = layers[0].D
        for dt_name, tdt in (("bf16", torch.bfloat16), ("f32", torch.float32)):
            xb = torch.randn(cfg.batch, 197, dim, device="cuda:0", dtype=tdt, requires_grad=True)
            gb = torch.randn(cfg.batch, 197, dim, device="cuda:0", dtype=tdt)
            std = torch.nn.Sequential(torch.nn.Linear(dim, 4 * dim), torch.nn.GELU(), torch.nn.Linear(4 * dim, dim))
            kat = gnn.KATMlp(dim, groups=cfg.G, fused="never")
            mods = [("gelu_mlp", std), ("kat_mlp", kat)]
            if tdt == torch.bfloat16:
                # the same block with the second layer's forward in the one-kernel layer (F inside the product)
                mods.append(("kat_mlp_fused_fc2", gnn.KATMlp(dim, groups=cfg.G, fused="always")))
            res = {}
            for name, mod in mods:
                mod = mod.to("cuda:0").to(tdt)

                def fb(_i, mod=mod):
                    xb.grad = None
                    mod(xb).backward(gb)

                def fwd_only(_i, mod=mod):
                    with torch.no_grad():
                        mod(xb)

                for i in range(3):
                    fb(i)
                    fwd_only(i)
                avg, med, mn = time_launches(torch, fb, 20)
                res[name + "_ms"] = med
                avg, med, mn = time_launches(torch, fwd_only, 20)
                res[name + "_forward_only_ms"] = med
            res["kat_over_gelu"] = res["kat_mlp_ms"] / res["gelu_mlp_ms"]
            block[dt_name] = res

    out = {
        "metric": "GR-KAN fwd+bwd elements/s and achieved HBM GB/s (%% of peak), %s shape"
                  % WORKLOAD_LABEL[args.workload],
        "value": elems_per_step / (dt / args.steps),
        "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "preheat_ms": args.preheat_ms,
        "preheat_steps": preheat_steps, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {
            "workload": "%s: fwd+bwd of %s, G=%d, degrees (%d,%d)"
                        % (args.workload, " and ".join("%s [%d,197,%d]" % (n, cfg.batch, l.D)
                                                       for n, l in zip(names, layers)), G, m_deg, n_deg),
            "elements_per_step": elems_per_step, "buffer_sets": {n: l.sets for n, l in zip(names, layers)},
            "hbm_GBs_whole_step": step_bytes / (dt / args.steps) / 1e9,
            "hbm_frac_of_peak_whole_step": step_bytes / (dt / args.steps) / 1e9 / HBM_PEAK_GBS,
        },
        "roofline": roofline,
        "device": device_report(torch, grkan),
    }
    roofline["event_pairs_in_timed_region"] = len(ev)
    if graph_replay is not None:
        out["graph_replay"] = graph_replay
    if detail is not None:
        out["detail"] = detail
    if paper_micro is not None:
        out["paper_micro_benchmark"] = paper_micro
    if alg1 is not None:
        out["alg1_baseline"] = alg1
    if block is not None:
        out["mlp_block"] = block
    if not args.no_fused and args.workload in ("kat_t", "kat_s", "kat_b") and (m_deg, n_deg) == (5, 4):
        # the layer one level up (Eq. "GR_KAN"): F fused into the matrix product that consumes it; the wide layer only
        try:
            del layers, dom
            torch.cuda.empty_cache()
            out["fused_layer_forward"] = fused_linear_bench(torch, grkan, grkan_inputs, args.workload, 50, ("x2",),
                                                            preheat_ms=min(args.preheat_ms, 200.0))
        except grkan.GrkanError as exc:
            out["fused_layer_forward"] = {"error": str(exc)}
        layers = dom = None
    if not args.no_cpu_baseline:
        layers = dom = None
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(cases)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
