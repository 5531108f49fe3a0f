"""Data collection and model fitting for the selector (Section IV-A / IV-B of the MTNN paper).

  python -m paper_1702_03192_amd.sweep collect --out <dir>/sweep_gfx950.csv          (needs the GPU)
  python -m paper_1702_03192_amd.sweep train   --csv <table> [<table> ...] --model <file>   (host only)

collect: for every (m, n, k) of the grid {64, ..., 8192}^3 it times the direct NT kernel and TNN
(transpose + NN through mtnn_tnn, workspace allocated beforehand) and writes one CSV row per
shape, appended as it goes, so an interrupted sweep resumes where it stopped.  The paper states
no timing protocol; here each path gets 3 warm-up calls, then `samples` event-timed batches of
back-to-back calls sized to last at least `min_batch_us` (2 ms by default), and the table keeps median and
minimum per call.  TNN is also timed with a per-call allocation of the B^T buffer through
PyTorch's caching allocator, because the paper counts allocation and release in T_transpose
(Section III); labels use the pre-allocated figure.

train: evaluates the paper's protocol (80/20 split, 5-fold CV), fits the final model on all
rows inside libmtnn and saves it.
"""
from __future__ import annotations

import argparse
import csv
import json
import os
import statistics
import sys

FIELDS = ["m", "n", "k", "seed", "t_nt", "t_nt_min", "t_tnn", "t_tnn_min", "t_transpose", "t_nn",
          "t_tnn_alloc", "nt_cfg", "nn_cfg"]


def _time_batches(fn, stream, samples, min_batch_us, budget_s=None):
    """Median and minimum seconds per call.  budget_s (optional) caps the time spent on one path:
    long-running calls get fewer warm-ups and samples (never fewer than 2 samples)."""
    import torch
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    fn()                                                     # first warm-up, timed to size the rest
    b.record(stream)
    torch.cuda.synchronize()
    first = a.elapsed_time(b) * 1e-3                         # s
    if budget_s is None or first * 4 < budget_s:
        for _ in range(2):
            fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    fn()
    b.record(stream)
    torch.cuda.synchronize()
    once = max(a.elapsed_time(b) * 1e3, 1.0)                 # us
    reps = max(1, min(1000, int(min_batch_us / once + 0.999)))
    if budget_s is not None:
        samples = max(2, min(samples, int(budget_s / (once * 1e-6 * reps))))
    per_call = []
    for _ in range(samples):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(reps):
            fn()
        b.record(stream)
        b.synchronize()
        per_call.append(a.elapsed_time(b) * 1e-3 / reps)
    return statistics.median(per_call), min(per_call)


PAPER_SIZES = tuple(2 ** i for i in range(7, 17))            # Section IV-A: S = {2^7, ..., 2^16}


def paper_shapes():
    """The paper's 1000 shapes, smallest first, with a per-shape seed."""
    out = []
    for im, m in enumerate(PAPER_SIZES):
        for in_, n in enumerate(PAPER_SIZES):
            for ik, k in enumerate(PAPER_SIZES):
                out.append((m, n, k, 20000 + 100 * im + 10 * in_ + ik))
    out.sort(key=lambda s: (s[0] * s[1] * s[2], s))
    return out


def irregular_shapes(count=384):
    """Seeded shapes off the power-of-two grids: every dimension log-uniform on [64, 8192]; half of
    the dimensions are rounded to a multiple of 4 (rows stay 16-byte aligned when ld = width), the
    other half are left as drawn, so the table also holds shapes only the guarded kernels serve."""
    from . import inputs
    e = inputs.uniform_ints(30000, 0, 3 * count, 0, 7 * 1024 - 1).reshape(count, 3)
    r = inputs.uniform_ints(30000, 1, 3 * count, 0, 1).reshape(count, 3)
    out = []
    for i in range(count):
        dims = []
        for j in range(3):
            v = int(64.0 * 2.0 ** (int(e[i, j]) / 1024.0))
            if r[i, j]:
                v = max(64, (v // 4) * 4)
            dims.append(v)
        out.append((dims[0], dims[1], dims[2], 30000 + i))
    out.sort(key=lambda s: (s[0] * s[1] * s[2], s))
    return out


def collect(out_path, samples, min_batch_us, limit=None, grid="bench", budget_s=None, mem_limit_gib=None):
    import torch
    from . import binding as mt
    from . import inputs
    torch.cuda.set_device(0)
    mt.lib()
    stream = torch.cuda.current_stream()
    done = set()
    if os.path.exists(out_path):
        with open(out_path, newline="") as f:
            for rec in csv.DictReader(f):
                done.add((int(rec["m"]), int(rec["n"]), int(rec["k"])))
    new_file = not os.path.exists(out_path)
    os.makedirs(os.path.dirname(os.path.abspath(out_path)), exist_ok=True)
    shapes = {"paper": paper_shapes, "irregular": irregular_shapes}.get(grid, inputs.sweep_shapes)()
    if limit:
        shapes = shapes[:limit]
    free_b, total_b = torch.cuda.mem_get_info()
    mem_limit = (mem_limit_gib * (1 << 30)) if mem_limit_gib else 0.9 * total_b
    cfgs = mt.gemm_configs()
    gen = torch.Generator(device="cuda")
    with open(out_path, "a", newline="") as f:
        wr = csv.DictWriter(f, fieldnames=FIELDS)
        if new_file:
            wr.writeheader()
        for idx, (m, n, k, seed) in enumerate(shapes):
            if (m, n, k) in done:
                continue
            # Section IV-A drops the samples that do not fit in memory: A, B, C, the B^T workspace
            # and the second B^T buffer of the separate transpose / NN timings
            need = 4.0 * (m * k + 3.0 * n * k + m * n)
            if need > mem_limit:
                print(f"[sweep] skip ({m},{n},{k}): needs {need / 2 ** 30:.1f} GiB", flush=True)
                continue
            big = need > 8 * (1 << 30)
            if big:
                torch.cuda.empty_cache()
            gen.manual_seed(seed)                             # uniform[-1, 1) operands, seeded per shape
            A = torch.rand((m, k), generator=gen, device="cuda").mul_(2).sub_(1)
            B = torch.rand((n, k), generator=gen, device="cuda").mul_(2).sub_(1)
            C = torch.empty((m, n), dtype=torch.float32, device="cuda")
            Bt = torch.empty((k, n), dtype=torch.float32, device="cuda")
            ws = torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda")
            nbytes = mt.mtnn_tnn_workspace_bytes(n, k)

            def tnn_alloc():
                w = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
                mt.mtnn_tnn(A, B, C, w)
                del w

            # (prepared calls: arguments resolved once, one ctypes call per launch)
            t_nt, t_nt_min = _time_batches(mt.prepare_nt(A, B, C), stream, samples, min_batch_us, budget_s)
            t_tnn, t_tnn_min = _time_batches(mt.prepare_tnn(A, B, C, ws), stream, samples, min_batch_us, budget_s)
            t_tr, _ = _time_batches(mt.prepare_transpose(B, Bt), stream, samples, min_batch_us, budget_s)
            if budget_s is not None and t_nt > budget_s / 8:
                t_nn = t_tnn - t_tr                           # long shapes: the difference stands in
                t_al = float("nan")
            else:
                t_nn, _ = _time_batches(mt.prepare_nn(A, Bt, C), stream, samples, min_batch_us, budget_s)
                t_al, _ = _time_batches(tnn_alloc, stream, max(5, samples // 4), min_batch_us, budget_s)
            wr.writerow({"m": m, "n": n, "k": k, "seed": seed, "t_nt": "%.9g" % t_nt, "t_nt_min": "%.9g" % t_nt_min,
                         "t_tnn": "%.9g" % t_tnn, "t_tnn_min": "%.9g" % t_tnn_min, "t_transpose": "%.9g" % t_tr,
                         "t_nn": "%.9g" % t_nn, "t_tnn_alloc": "%.9g" % t_al,
                         "nt_cfg": cfgs[mt.mtnn_gemm_default_config(mt.OP_NT, m, n, k)],
                         "nn_cfg": cfgs[mt.mtnn_gemm_default_config(mt.OP_NN, m, n, k)]})
            f.flush()
            if idx % 16 == 0 or t_nt > 0.05:
                print(f"[sweep] {idx + 1}/{len(shapes)} ({m},{n},{k}) nt {t_nt * 1e6:.1f} us tnn {t_tnn * 1e6:.1f} us",
                      flush=True)
            del A, B, C, Bt, ws
    print(f"[sweep] wrote {out_path}", flush=True)


def train(csv_paths, model_path, report_path=None):
    """Fit and evaluate on the union of the given timing tables (a shape listed twice keeps its first row)."""
    from . import binding as mt
    from . import selector_data as sd
    if isinstance(csv_paths, str):
        csv_paths = [csv_paths]
    rows = sd.load_training_rows(csv_paths)
    report = sd.evaluate(rows)                                   # leaves the all-rows model installed
    mt.mtnn_save_model(model_path)
    report["model"] = model_path
    report["tables"] = list(csv_paths) if csv_paths else [os.path.basename(p) for p in sd.TRAINING_TABLES if os.path.exists(p)]
    report["trees"] = mt.lib().mtnn_model_num_trees()
    text = json.dumps(report, indent=1, sort_keys=True)
    print(text)
    if report_path:
        with open(report_path, "w") as f:
            f.write(text + "\n")
    return report


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    c = sub.add_parser("collect")
    c.add_argument("--out", required=True)
    c.add_argument("--samples", type=int, default=20)
    c.add_argument("--min-batch-us", type=float, default=2000.0)
    c.add_argument("--limit", type=int, default=None)
    c.add_argument("--grid", choices=["bench", "paper", "irregular"], default="bench",
                   help="bench: {64..8192}^3 (512 shapes); paper: {2^7..2^16}^3 (1000 shapes, Section IV-A); "
                        "irregular: 384 seeded shapes off the power-of-two grids")
    c.add_argument("--budget-s", type=float, default=None, help="cap on the time spent timing one path of one shape")
    c.add_argument("--mem-limit-gib", type=float, default=None, help="drop shapes needing more device memory")
    t = sub.add_parser("train")
    t.add_argument("--csv", nargs="+", default=None,
                   help="one or more timing tables; the model is fitted on their union (default: the shipped tables)")
    t.add_argument("--model", required=True)
    t.add_argument("--report", default=None)
    st = sub.add_parser("stats", help="the case counts of the paper's Sections II / III and Eq. 4 on stored tables (host only)")
    st.add_argument("--csv", nargs="+", default=None, help="timing tables (default: the shipped ones, one report each)")
    args = ap.parse_args(argv)
    if args.cmd == "stats":
        from . import selector_data as sd
        for path in (args.csv or sd.TRAINING_TABLES):
            print(os.path.basename(path), json.dumps(sd.nt_tnn_statistics(sd.load_sweep(path))))
        return 0
    if args.cmd == "collect":
        collect(args.out, args.samples, args.min_batch_us, args.limit, args.grid, args.budget_s, args.mem_limit_gib)
    else:
        train(args.csv, args.model, args.report)
    return 0


if __name__ == "__main__":
    sys.exit(main())
