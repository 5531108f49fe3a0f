"""Measurement report over all benchmark configurations (needs the GPU).

  python -m paper_1702_03192_amd.report --out <dir>/shape_report.json [--md <dir>/shape_report.md]

For every shape of configs 1, 2 and 4 and a spread of the config-3 grid it times the direct NT kernel,
TNN (pre-allocated workspace) and the selected path (mtnn_select + mtnn_auto), and reports
GFLOP/s = 2mnk/t with the fraction of the shape's roofline
max(2mnk / fp32-MFMA peak, 4(mk + nk + mn) / HBM peak); the transposes of the report list are given in
GB/s = 8 rows cols / t; the fully connected training step (config 5) is timed in its three forward
modes; and the selector is checked by measurement: on every grid shape, is the selected path ever
slower than the worse of its two alternatives?  Timing protocol as in sweep.py.
"""
from __future__ import annotations

import argparse
import json
import statistics
import sys

PEAK_TFLOPS = 157.3
PEAK_GBS = 8000.0

TRANSPOSES = [(16384, 16384), (8192, 8192), (4096, 4096), (4096, 1024), (1024, 4096), (1024, 10), (4500, 1500)]
INPLACE_TRANSPOSES = [(16384, 16384), (8192, 8192), (4096, 4096), (8192, 4096), (4096, 8192), (4096, 1024), (1024, 4096),
                      (4500, 1500), (4099, 1009)]
LAUNCH_PATH_GEMMS = [(64, 64, 64), (256, 256, 256), (512, 512, 512), (1000, 1000, 1000), (1024, 1024, 1024),
                     (64, 64, 8192), (128, 128, 4096)]      # the last two: divided 32 ways over k
LAUNCH_PATH_TRANSPOSES = [(4096, 1024), (4500, 1500), (4096, 4096)]


def roofline_seconds(m, n, k):
    return max(2.0 * m * n * k / (PEAK_TFLOPS * 1e12), 4.0 * (m * k + n * k + m * n) / (PEAK_GBS * 1e9))


def probe_lanes(out_path):
    """Times csrc/probe.hip's kernel with matrix work only, vector work only and both (HIP events, median of 9)."""
    import torch
    from . import binding as mt
    torch.cuda.set_device(0)
    mt.lib()
    stream = torch.cuda.current_stream()
    sink = torch.zeros(512, device="cuda")

    def timed(nm, nv):
        for _ in range(3):
            mt.mtnn_probe_lanes(nm, nv, sink)
        ts = []
        for _ in range(9):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            mt.mtnn_probe_lanes(nm, nv, sink)
            b.record(stream)
            b.synchronize()
            ts.append(a.elapsed_time(b) * 1e3)
        return statistics.median(ts)

    lines = ["| matrix instructions per SIMD | vector multiply-adds per SIMD | us | matrix alone + vector alone |", "|---|---|---|---|"]
    for nm, nv in ((4096, 8192), (4096, 16384), (4096, 32768), (8192, 16384)):
        t_m, t_v, t_b = timed(nm, 0), timed(0, nv), timed(nm, nv)
        lines += [f"| {nm} | 0 | {t_m:.1f} | |", f"| 0 | {nv} | {t_v:.1f} | |", f"| {nm} | {nv} | {t_b:.1f} | {t_m + t_v:.1f} |"]
    text = "\n".join(lines) + "\n"
    with open(out_path, "w") as f:
        f.write(text)
    print(text)
    return 0


def launch_path(out_path, calls=400):
    """Short calls, to set the time per call (HIP events around `calls` back-to-back prepared launches on
    one stream) beside the time inside the kernel (what a kernel trace of this same run reports per
    dispatch): the difference is the launch path, host and GPU side."""
    import torch
    from . import binding as mt
    torch.cuda.set_device(0)
    mt.lib()
    stream = torch.cuda.current_stream()
    cfgs = mt.gemm_configs()
    rows = []

    def per_call(fn):
        for _ in range(20):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(calls):
            fn()
        b.record(stream)
        b.synchronize()
        return a.elapsed_time(b) * 1e3 / calls

    for m, n, k in LAUNCH_PATH_GEMMS:
        A = torch.rand((m, k), device="cuda")
        B = torch.rand((n, k), device="cuda")
        C = torch.empty((m, n), device="cuda")
        ws = torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda")
        for name, fn in (("mtnn_nt", mt.prepare_nt(A, B, C)), ("mtnn_auto", mt.prepare_auto(A, B, C, ws)),
                         ("mtnn_nt, plain wrapper", lambda: mt.mtnn_nt(A, B, C))):
            rows.append({"call": name, "shape": [m, n, k], "us_per_call": per_call(fn), "calls": calls + 20,
                         "config": cfgs[mt.mtnn_gemm_default_config(mt.OP_NT, m, n, k)],
                         "splits": mt.mtnn_gemm_default_splits(mt.OP_NT, m, n, k)})
            print("[launch-path]", json.dumps(rows[-1]), flush=True)
    for r, c in LAUNCH_PATH_TRANSPOSES:
        X = torch.rand((r, c), device="cuda")
        Y = torch.empty((c, r), device="cuda")
        rows.append({"call": "mtnn_transpose", "shape": [r, c], "us_per_call": per_call(mt.prepare_transpose(X, Y)), "calls": calls + 20})
        print("[launch-path]", json.dumps(rows[-1]), flush=True)
    with open(out_path, "w") as f:
        json.dump(rows, f, indent=1)
    return 0


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", required=True)
    ap.add_argument("--md", default=None)
    ap.add_argument("--samples", type=int, default=20)
    ap.add_argument("--grid-verify", action="store_true", help="time NT, TNN and auto on all 512 grid shapes")
    ap.add_argument("--probe-lanes", action="store_true",
                    help="only the overlap probe: fp32 matrix instructions against vector instructions of another wave")
    ap.add_argument("--launch-path", action="store_true",
                    help="only the short calls, timed per call; run it under a kernel trace to get the time inside the kernels")
    args = ap.parse_args(argv)
    if args.probe_lanes:
        return probe_lanes(args.out)
    if args.launch_path:
        return launch_path(args.out)

    import torch
    from . import binding as mt
    from . import inputs
    from .sweep import _time_batches

    torch.cuda.set_device(0)
    mt.lib()
    stream = torch.cuda.current_stream()
    gen = torch.Generator(device="cuda")
    cfgs = mt.gemm_configs()

    def operands(m, n, k, seed, dist):
        gen.manual_seed(seed)
        if dist == "normal":
            A = torch.randn((m, k), generator=gen, device="cuda")
            B = torch.randn((n, k), generator=gen, device="cuda")
        else:
            A = torch.rand((m, k), generator=gen, device="cuda") * 2 - 1
            B = torch.rand((n, k), generator=gen, device="cuda") * 2 - 1
        return A, B

    def time_shape(m, n, k, seed, dist, samples):
        A, B = operands(m, n, k, seed, dist)
        C = torch.empty((m, n), device="cuda")
        ws = torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda")
        # about 50 ms of this shape first: after a tiny shape the clocks are low, and the first path timed
        # would pay for that (NT read 4 % low on the first big shape of the list)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        mt.mtnn_nt(A, B, C)
        b.record(stream)
        b.synchronize()
        for _ in range(min(2000, int(50.0 / max(a.elapsed_time(b), 1e-3)))):
            mt.mtnn_nt(A, B, C)
        torch.cuda.synchronize()
        # prepared calls (arguments resolved once, one ctypes call per launch): what a training loop would hold
        t_nt, _ = _time_batches(mt.prepare_nt(A, B, C), stream, samples, 2000.0)
        t_tnn, _ = _time_batches(mt.prepare_tnn(A, B, C, ws), stream, samples, 2000.0)
        t_auto, _ = _time_batches(mt.prepare_auto(A, B, C, ws), stream, samples, 2000.0)
        label = mt.mtnn_select(m, n, k)
        fl = 2.0 * m * n * k
        roof = roofline_seconds(m, n, k)
        return {"m": m, "n": n, "k": k, "dist": dist, "t_nt_us": t_nt * 1e6, "t_tnn_us": t_tnn * 1e6,
                "t_auto_us": t_auto * 1e6, "nt_gflops": fl / t_nt / 1e9, "tnn_gflops": fl / t_tnn / 1e9,
                "mtnn_gflops": fl / t_auto / 1e9, "label": label, "nt_roofline_frac": roof / t_nt,
                "mtnn_roofline_frac": roof / t_auto,
                "bound": "mfma" if 2.0 * m * n * k / (PEAK_TFLOPS * 1e12) >= 4.0 * (m * k + n * k + m * n) / (PEAK_GBS * 1e9) else "hbm",
                "nt_cfg": cfgs[mt.mtnn_gemm_default_config(mt.OP_NT, m, n, k)],
                "nt_splits": mt.mtnn_gemm_default_splits(mt.OP_NT, m, n, k)}

    # warm the clocks
    A, B = operands(4096, 4096, 4096, 1, "uniform")
    C = torch.empty((4096, 4096), device="cuda")
    for _ in range(60):
        mt.mtnn_nt(A, B, C)
    torch.cuda.synchronize()
    del A, B, C

    report = {"device": torch.cuda.get_device_name(0), "peak_tflops": PEAK_TFLOPS, "peak_gbs": PEAK_GBS, "shapes": []}
    named = []
    for cfg_name, cfg in (("config1", inputs.CONFIG1), ("config2", inputs.CONFIG2), ("config4", inputs.CONFIG4)):
        for shape, seed in zip(cfg["shapes"], cfg["seeds"]):
            named.append((cfg_name, shape, seed, cfg["dist"]))
    for shape in [(8192, 8192, 8192), (4096, 4096, 4096), (2048, 2048, 2048), (1024, 1024, 1024), (512, 512, 512),
                  (64, 64, 64), (1000, 1000, 1000), (8192, 8192, 32), (8192, 8192, 64), (8192, 8192, 128), (64, 8192, 8192),
                  (8192, 64, 8192), (8192, 8192, 1024)]:
        named.append(("config3", shape, 10000, "uniform"))
    for cfg_name, shape, seed, dist in named:
        row = time_shape(*shape, seed, dist, args.samples)
        row["config"] = cfg_name
        report["shapes"].append(row)
        print(f"[report] {cfg_name} {shape}: NT {row['nt_gflops'] / 1e3:.1f} TNN {row['tnn_gflops'] / 1e3:.1f} "
              f"MTNN {row['mtnn_gflops'] / 1e3:.1f} TFLOP/s  roofline {row['nt_roofline_frac']:.2f}", flush=True)

    # transposes: timed on one buffer pair (small shapes then live in the 256 MB memory-side cache and
    # the L2s) and again rotating over enough pairs that the footprint passes 1 GiB, so every call
    # reads from and writes to HBM
    report["transposes"] = []
    for rows, cols in TRANSPOSES:
        pair_bytes = 8.0 * rows * cols
        nsets = int(max(1, min(64, -(-(1 << 30) // int(pair_bytes)))))
        Xs = [torch.rand((rows, cols), device="cuda") for _ in range(nsets)]
        Ys = [torch.empty((cols, rows), device="cuda") for _ in range(nsets)]
        calls = [mt.prepare_transpose(x, y) for x, y in zip(Xs, Ys)]
        t, tmin = _time_batches(calls[0], stream, args.samples, 2000.0)
        turn = [0]

        def rotating():
            i = turn[0]
            turn[0] = (i + 1) % nsets
            calls[i]()

        t_rot, _ = _time_batches(rotating, stream, args.samples, 2000.0)
        report["transposes"].append({"rows": rows, "cols": cols, "t_us": t * 1e6, "gbs": pair_bytes / t / 1e9,
                                     "frac_of_peak": pair_bytes / t / 1e9 / PEAK_GBS,
                                     "buffer_pairs_rotated": nsets, "footprint_mib": nsets * pair_bytes / 2 ** 20,
                                     "cache_resident_when_repeated": pair_bytes <= 256e6,
                                     "t_rotating_us": t_rot * 1e6, "gbs_rotating": pair_bytes / t_rot / 1e9,
                                     "frac_of_peak_rotating": pair_bytes / t_rot / 1e9 / PEAK_GBS})
        print(f"[report] transpose {rows}x{cols}: {pair_bytes / t / 1e9:.0f} GB/s on one buffer pair, "
              f"{pair_bytes / t_rot / 1e9:.0f} GB/s rotating over {nsets}", flush=True)
        del Xs, Ys, calls
    # in-place transposes (square: tile-pair swaps; rectangular: two or three passes): one buffer each,
    # sized like the B operands they would serve; GB/s counts each word read once and written once
    report["inplace_transposes"] = []
    for rows, cols in INPLACE_TRANSPOSES:
        X = torch.rand(rows * cols, device="cuda")
        dims = [rows, cols]

        def flip():
            if dims[0] == dims[1]:
                mt.mtnn_transpose_inplace(X.view(rows, cols))
            else:
                mt.mtnn_transpose_inplace_rect(X, dims[0], dims[1])
                dims.reverse()

        t, _ = _time_batches(flip, stream, max(6, args.samples // 2), 2000.0)
        report["inplace_transposes"].append({"rows": rows, "cols": cols, "t_us": t * 1e6, "gbs": 8.0 * rows * cols / t / 1e9})
        print(f"[report] in-place transpose {rows}x{cols}: {t * 1e6:.1f} us, {8.0 * rows * cols / t / 1e9:.0f} GB/s", flush=True)
        del X
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    t, _ = _time_batches(lambda: mt.mtnn_copy_bytes(src, dst), stream, args.samples, 2000.0)
    report["copy_1gib_gbs"] = 2.0 * src.numel() / t / 1e9
    del src, dst

    # config 5: one training step, three forward modes
    cfg = inputs.CONFIG5
    dims, batch = cfg["dims"], cfg["batch"]
    L = len(dims) - 1
    gen.manual_seed(cfg["seed"])
    X = torch.randn((batch, dims[0]), generator=gen, device="cuda")
    labels = torch.randint(0, dims[-1], (batch,), generator=gen, device="cuda", dtype=torch.int32)
    W = [torch.from_numpy(inputs.xavier_uniform(cfg["seed"] + 1 + l, 2, dims[l + 1], dims[l])).cuda() for l in range(L)]
    b = [torch.zeros(dims[l + 1], device="cuda") for l in range(L)]
    gW = [torch.empty_like(w) for w in W]
    gb = [torch.empty_like(v) for v in b]
    loss = torch.empty(1, device="cuda")
    ws = torch.empty(mt.mtnn_fc_workspace_bytes(dims, batch), dtype=torch.uint8, device="cuda")
    flops = sum(2.0 * batch * dims[l] * dims[l + 1] * (3 if l > 0 else 2) for l in range(L))
    report["fc_step"] = {"dims": dims, "batch": batch, "gemm_flop": flops}
    for mode, name in ((1, "nt"), (-1, "tnn"), (0, "auto")):
        desc, keep = mt.make_fc_desc(dims, batch, X, labels, W, b, gW, gb, loss, ws, 0.0, mode)
        t, _ = _time_batches(lambda: mt.mtnn_fc_train_step(desc), stream, args.samples, 2000.0)
        report["fc_step"][name + "_ms"] = t * 1e3
        report["fc_step"][name + "_gemm_tflops"] = flops / t / 1e12
        print(f"[report] fc step {name}: {t * 1e3:.3f} ms ({flops / t / 1e12:.1f} TFLOP/s of GEMM work)", flush=True)

    if args.grid_verify:
        rows = []
        worse = worse_1pct = worse_strict = 0
        for (m, n, k, seed) in inputs.sweep_shapes():
            r = time_shape(m, n, k, seed, "uniform", max(8, args.samples // 2))
            rows.append(r)
            slowest = max(r["t_nt_us"], r["t_tnn_us"])
            worse += r["t_auto_us"] > slowest * 1.03
            worse_1pct += r["t_auto_us"] > slowest * 1.01
            worse_strict += r["t_auto_us"] > slowest
        p_nt = [r["nt_gflops"] for r in rows]
        p_tnn = [r["tnn_gflops"] for r in rows]
        p_m = [r["mtnn_gflops"] for r in rows]
        gow = [(pm - min(a, b)) / min(a, b) for pm, a, b in zip(p_m, p_nt, p_tnn)]
        lub = [(pm - max(a, b)) / max(a, b) for pm, a, b in zip(p_m, p_nt, p_tnn)]
        report["grid_verify"] = {
            "shapes": len(rows), "auto_slower_than_worse_strict": worse_strict,
            "auto_slower_than_worse_by_1pct": worse_1pct, "auto_slower_than_worse_by_3pct": worse,
            "measured_gow_avg": statistics.mean(gow), "measured_gow_max": max(gow),
            "measured_lub_avg": statistics.mean(lub), "measured_lub_min": min(lub),
            "mtnn_vs_nt_avg": statistics.mean((pm - a) / a for pm, a in zip(p_m, p_nt)),
            "mtnn_vs_tnn_avg": statistics.mean((pm - b) / b for pm, b in zip(p_m, p_tnn)),
            # (calls shorter than ~20 us are bound by the launch path)
            "mtnn_vs_nt_avg_calls_over_20us": statistics.mean((r["mtnn_gflops"] - r["nt_gflops"]) / r["nt_gflops"]
                                                              for r in rows if r["t_nt_us"] >= 20.0),
            "labels_nt": sum(1 for r in rows if r["label"] == 1), "labels_tnn": sum(1 for r in rows if r["label"] == -1),
        }
        print("[report] grid verify:", json.dumps(report["grid_verify"]), flush=True)

    with open(args.out, "w") as f:
        json.dump(report, f, indent=1)
    if args.md:
        with open(args.md, "w") as f:
            f.write("| config | m | n | k | bound | NT TFLOP/s | TNN TFLOP/s | MTNN TFLOP/s | label | NT / roofline | NT config | split-k |\n")
            f.write("|---|---|---|---|---|---|---|---|---|---|---|---|\n")
            for r in report["shapes"]:
                f.write(f"| {r['config']} | {r['m']} | {r['n']} | {r['k']} | {r['bound']} | {r['nt_gflops'] / 1e3:.1f} | "
                        f"{r['tnn_gflops'] / 1e3:.1f} | {r['mtnn_gflops'] / 1e3:.1f} | {r['label']:+d} | "
                        f"{r['nt_roofline_frac']:.2f} | {r['nt_cfg']} | {'even cut' if r['nt_splits'] == mt.EVEN_CUT else r['nt_splits']} |\n")
            f.write("\n| transpose rows x cols | us | GB/s | of 8 TB/s | fits the 256 MB cache | rotating pairs | us | GB/s | of 8 TB/s |\n")
            f.write("|---|---|---|---|---|---|---|---|---|\n")
            for r in report["transposes"]:
                f.write(f"| {r['rows']} x {r['cols']} | {r['t_us']:.1f} | {r['gbs']:.0f} | {r['frac_of_peak']:.2f} | "
                        f"{'yes' if r['cache_resident_when_repeated'] else 'no'} | {r['buffer_pairs_rotated']} | "
                        f"{r['t_rotating_us']:.1f} | {r['gbs_rotating']:.0f} | {r['frac_of_peak_rotating']:.2f} |\n")
            f.write("\n| in-place transpose rows x cols | us | GB/s (8 bytes per word) |\n|---|---|---|\n")
            for r in report["inplace_transposes"]:
                f.write(f"| {r['rows']} x {r['cols']} | {r['t_us']:.1f} | {r['gbs']:.0f} |\n")
            f.write(f"\ncopy kernel, 1 GiB: {report['copy_1gib_gbs']:.0f} GB/s\n\n")
            fc = report["fc_step"]
            f.write(f"FC step {fc['dims']} batch {fc['batch']} ({fc['gemm_flop'] / 1e9:.1f} GFLOP of GEMM work): "
                    f"NT {fc['nt_ms']:.3f} ms, TNN {fc['tnn_ms']:.3f} ms, auto {fc['auto_ms']:.3f} ms\n")
            if "grid_verify" in report:
                f.write("\ngrid verification (512 shapes, NT / TNN / auto timed in one session): "
                        + json.dumps(report["grid_verify"]) + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
