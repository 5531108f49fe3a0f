#!/usr/bin/env python3
"""Benchmark of the NT-operation hot path on one MI355X.

A "step" is one pass of the whole path over the FC-layer NT shapes
(m, n, k) = (1024, 4096, 4096) and (4096, 4096, 1024), fp32, uniform[-1, 1) inputs from seeds:
for each shape the direct NT kernel (mtnn_nt), TNN = transpose + NN (mtnn_tnn) and the
selected path (mtnn_select + mtnn_auto).  Every call computes a full NT product, so the step's
work is 4 x sum(2mnk) flop (NT, transpose + NN, TNN through its own entry point, selected path)
and `value` is that work over the step time, in GFLOP/s.  Inputs are
resident in HBM before the timed region; nothing is allocated inside it.

Prints ONE JSON line (see the keys below).  Per-kernel durations come from HIP events recorded,
inside the timed region, on the stream the kernels are launched on.
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

PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X dense fp32 matrix peak: 256 CUs x 2.4 GHz x 256 flop/clk/CU
PEAK_HBM_GBS = 8000.0             # MI355X HBM3E peak


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (the NT path needs no exchange between "
              "GPUs: split A by rows or B by rows and run one process per GPU); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_1702_03192_amd import binding as mt
    from paper_1702_03192_amd import inputs, selector_data

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    mt.lib()
    stream = torch.cuda.current_stream()

    cfg = inputs.CONFIG2
    work = []
    for (m, n, k), seed in zip(cfg["shapes"], cfg["seeds"]):
        A, B = inputs.nt_operands(m, n, k, seed, cfg["dist"])
        w = {"shape": (m, n, k), "hA": A, "hB": B,
             "A": torch.from_numpy(A).cuda(), "B": torch.from_numpy(B).cuda(),
             "C_nt": torch.empty((m, n), dtype=torch.float32, device="cuda"),
             "C_tnn": torch.empty((m, n), dtype=torch.float32, device="cuda"),
             "C_auto": torch.empty((m, n), dtype=torch.float32, device="cuda"),
             "ws": torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda"),
             "Bt": torch.empty((k, n), dtype=torch.float32, device="cuda"),
             "flops": 2.0 * m * n * k}
        # every call of the step with its arguments resolved once (one ctypes call each in the timed region)
        w["call_nt"] = mt.prepare_nt(w["A"], w["B"], w["C_nt"])
        w["call_transpose"] = mt.prepare_transpose(w["B"], w["Bt"])
        w["call_nn"] = mt.prepare_nn(w["A"], w["Bt"], w["C_tnn"])
        w["call_tnn"] = mt.prepare_tnn(w["A"], w["B"], w["C_tnn"], w["ws"])
        w["call_auto"] = mt.prepare_auto(w["A"], w["B"], w["C_auto"], w["ws"])
        work.append(w)
    torch.cuda.synchronize()

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def step(record=None):
        for wi, w in enumerate(work):
            if record is not None:
                e = [ev() for _ in range(6)]
                e[0].record(stream)
                w["call_nt"]()                                   # a1
                e[1].record(stream)
                w["call_transpose"]()                            # a2 } a4, the same two launches
                e[2].record(stream)
                w["call_nn"]()                                   # a3 } mtnn_tnn makes
                e[3].record(stream)
                w["call_tnn"]()                                  # a4 through its own entry point
                e[4].record(stream)
                w["label"] = w["call_auto"]()                    # a5 + dispatch (mtnn_select inside mtnn_auto)
                e[5].record(stream)
                record.append((wi, e))
            else:
                w["call_nt"]()
                w["call_transpose"]()
                w["call_nn"]()
                w["call_tnn"]()
                w["label"] = w["call_auto"]()

    # NT products per shape and step: mtnn_nt, transpose+mtnn_nn, mtnn_tnn, mtnn_auto = 4
    products_per_shape = 4
    # bring the GPU out of its idle clocks before the W warm-up steps (about 0.1 s of the same work)
    pre0 = time.perf_counter()
    while time.perf_counter() - pre0 < 0.1:
        step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    records = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(records)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    total_flops = products_per_shape * sum(w["flops"] for w in work)
    value = total_flops / (ms_per_step * 1e-3) / 1e9

    # per-kernel averages from the events of the timed region
    acc = {}
    for wi, e in records:
        for name, a, b in (("nt", 0, 1), ("transpose", 1, 2), ("nn", 2, 3), ("tnn", 3, 4), ("auto", 4, 5)):
            acc.setdefault((wi, name), []).append(e[a].elapsed_time(e[b]) * 1e-3)
    per_shape = []
    kernels = []
    for wi, w in enumerate(work):
        m, n, k = w["shape"]
        t = {name: float(np.mean(acc[(wi, name)])) for name in ("nt", "transpose", "nn", "tnn", "auto")}
        fl = w["flops"]
        alg_bytes = 4.0 * (m * k + n * k + m * n)
        roof_s = max(fl / (PEAK_FP32_MFMA_TFLOPS * 1e12), alg_bytes / (PEAK_HBM_GBS * 1e9))
        per_shape.append({
            "m": m, "n": n, "k": k,
            "nt_gflops": fl / t["nt"] / 1e9, "nn_gflops": fl / t["nn"] / 1e9,
            "tnn_gflops": fl / t["tnn"] / 1e9, "mtnn_gflops": fl / t["auto"] / 1e9,
            "transpose_gbs": 8.0 * n * k / t["transpose"] / 1e9,
            "label": int(w["label"]), "nt_roofline_frac": roof_s / t["nt"], "tnn_roofline_frac": roof_s / t["tnn"],
            "nt_cfg": mt.gemm_configs()[mt.mtnn_gemm_default_config(mt.OP_NT, m, n, k)],
            "nn_cfg": mt.gemm_configs()[mt.mtnn_gemm_default_config(mt.OP_NN, m, n, k)],
        })
        kernels.append(("gemm_kernel NT %s (m,n,k)=(%d,%d,%d)" % (per_shape[-1]["nt_cfg"], m, n, k), "mfma", fl, t["nt"]))
        kernels.append(("gemm_kernel NN %s (m,n,k)=(%d,%d,%d)" % (per_shape[-1]["nn_cfg"], m, n, k), "mfma", fl, t["nn"]))
        kernels.append(("transpose_kernel %dx%d" % (n, k), "hbm", 8.0 * n * k, t["transpose"]))

    # the dominant kernel of the step: the direct NT GEMM (launched by mtnn_nt and, when selected, by
    # mtnn_auto); of the two shapes' instantiations, the one with the longer average launch
    name, bound, units, dur = max((r for r in kernels if r[0].startswith("gemm_kernel NT")), key=lambda r: r[3])
    if bound == "mfma":
        roofline = {"bound": "mfma", "achieved": units / dur / 1e12, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s"}
    else:
        roofline = {"bound": "hbm", "achieved": units / dur / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    roofline["traffic"] = selector_data.measured_traffic_bytes(name)   # from profiles/, or None
    roofline["kernel"] = name
    roofline["avg_launch_us"] = dur * 1e6
    # TNN as Algorithm 1 writes it, with the buffer for B^T obtained and released inside every call
    # (here: from PyTorch's caching allocator); the paper counts that in the transpose's time (Section III).
    # Outside the timed step, whose TNN calls use a workspace allocated once.
    for w, ps in zip(work, per_shape):
        m, n, k = w["shape"]
        nbytes = mt.mtnn_tnn_workspace_bytes(n, k)

        def tnn_with_alloc():
            ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            mt.mtnn_tnn(w["A"], w["B"], w["C_tnn"], ws)
            del ws
        for _ in range(3):
            tnn_with_alloc()
        torch.cuda.synchronize()
        a0, a1 = ev(), ev()
        a0.record(stream)
        for _ in range(10):
            tnn_with_alloc()
        a1.record(stream)
        torch.cuda.synchronize()
        ps["tnn_alloc_per_call_gflops"] = w["flops"] / (a0.elapsed_time(a1) * 1e-3 / 10) / 1e9

    # Outside the timed step, the two performance targets on the shapes they are stated for: the GEMM
    # kernels at 8192^3 (MFMA-bound, every CU busy) and the transpose on matrices that cannot be
    # cache-resident (16384^2: 1 GiB in, 1 GiB out; 8192^2 rotating over three buffer pairs = 1.5 GiB).
    def timed_calls(calls, reps):
        for _ in range(2):
            for c in calls:
                c()
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record(stream)
        for r in range(reps):
            calls[r % len(calls)]()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    big = 8192
    gen = torch.Generator(device="cuda")
    gen.manual_seed(8192)
    bA = torch.rand((big, big), generator=gen, device="cuda").mul_(2).sub_(1)
    bB = torch.rand((big, big), generator=gen, device="cuda").mul_(2).sub_(1)
    bC = torch.empty((big, big), device="cuda")
    for op_name, prep in (("NT", mt.prepare_nt), ("NN", mt.prepare_nn)):
        dur = timed_calls([prep(bA, bB, bC)], 6)
        fl = 2.0 * big ** 3
        cfg_name = mt.gemm_configs()[mt.mtnn_gemm_default_config(mt.OP_NT if op_name == "NT" else mt.OP_NN, big, big, big)]
        kernels.append(("gemm_kernel %s %s (m,n,k)=(%d,%d,%d)" % (op_name, cfg_name, big, big, big), "mfma", fl, dur))
    del bA, bB, bC
    for side, pairs, reps in ((16384, 1, 5), (8192, 3, 9)):
        bufs = [(torch.empty((side, side), device="cuda").fill_(float(i)), torch.empty((side, side), device="cuda"))
                for i in range(pairs)]
        dur = timed_calls([mt.prepare_transpose(a, b) for a, b in bufs], reps)
        kernels.append(("transpose_kernel %dx%d from HBM (%d buffer pair%s, %.1f GiB)"
                        % (side, side, pairs, "" if pairs == 1 else "s", pairs * 8.0 * side * side / 2 ** 30),
                        "hbm", 8.0 * side * side, dur))
        del bufs
    torch.cuda.empty_cache()
    other = []
    for kname, b, u, d in kernels:
        peak = PEAK_FP32_MFMA_TFLOPS if b == "mfma" else PEAK_HBM_GBS
        ach = u / d / (1e12 if b == "mfma" else 1e9)
        other.append({"kernel": kname, "bound": b, "achieved": ach, "peak": peak, "frac": ach / peak,
                      "avg_launch_us": d * 1e6})

    # known-traffic copy (counter calibration point, and the practical HBM ceiling); outside the timed region
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")        # 1 GiB: far beyond the caches
    dst = torch.empty_like(src)
    mt.mtnn_copy_bytes(src, dst)
    torch.cuda.synchronize()
    c0, c1 = ev(), ev()
    c0.record(stream)
    for _ in range(5):
        mt.mtnn_copy_bytes(src, dst)
    c1.record(stream)
    torch.cuda.synchronize()
    copy_gbs = 5 * 2.0 * src.numel() / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst

    # selector: accuracy on the stored sweep (trained through the library) and per-call cost
    selector = selector_data.selector_report()
    n_calls = 200000
    shapes = [(int(a), int(b), int(c)) for a, b, c in
              inputs.uniform_ints(7, 0, 3 * 1024, 64, 8192).reshape(-1, 3)]
    L = mt.lib()
    ts = time.perf_counter()
    for i in range(n_calls):
        s = shapes[i & 1023]
        L.mtnn_select(s[0], s[1], s[2])
    te = time.perf_counter()
    tb = time.perf_counter()
    for i in range(n_calls):
        s = shapes[i & 1023]
        L.mtnn_version()
    tf = time.perf_counter()
    selector["select_ns_per_call_incl_ctypes"] = (te - ts) / n_calls * 1e9
    selector["ctypes_call_overhead_ns"] = (tf - tb) / n_calls * 1e9

    props = torch.cuda.get_device_properties(0)
    cus, clock_khz = mt.mtnn_device_attribute(0), mt.mtnn_device_attribute(1)
    mem_khz, bus_bits = mt.mtnn_device_attribute(2), mt.mtnn_device_attribute(3)
    device = {"name": props.name, "compute_units": cus, "max_clock_mhz": clock_khz / 1e3,
              # 256 fp32 matrix flop per clock per CU (4 SIMDs x one 32x32x2 MFMA per 16 passes of 4 clocks)
              "fp32_mfma_peak_from_attributes_tflops": cus * clock_khz * 1e3 * 256 / 1e12 if cus > 0 and clock_khz > 0 else None,
              "memory_clock_mhz": mem_khz / 1e3, "memory_bus_bits": bus_bits,
              "hbm_gib": props.total_memory / 2 ** 30}
    nt_splits = [mt.mtnn_gemm_default_splits(mt.OP_NT, *w["shape"]) for w in work]
    out = {
        "metric": "NT GFLOP/s (2mnk/t, fp32)", "value": value, "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config 2: FC-layer NT shapes (1024,4096,4096) and (4096,4096,1024); per shape "
                               "mtnn_nt, mtnn_transpose+mtnn_nn, mtnn_tnn, mtnn_select+mtnn_auto",
                   "nt_products_per_step": products_per_shape * len(work), "nt_split_k": nt_splits},
        "roofline": roofline, "kernels": other, "per_shape": per_shape,
        "copy_kernel_gbs": copy_gbs, "selector": selector, "device": device,
    }

    if not args.no_cpu_baseline:
        import oracle
        tc0 = time.perf_counter()
        macs = 0.0
        for w in work:
            oracle.nt_ref(w["hA"], w["hB"])
            macs += w["flops"]
        tc1 = time.perf_counter()
        out["cpu_baseline"] = {"value": macs / (tc1 - tc0) / 1e9, "unit": "GFLOP/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": "oracle nt_ref (fp64 triple loop) once on each config-2 shape in full, "
                                         "%.1f s wall" % (tc1 - tc0)}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
