"""Where the cost model's numbers come from (gemm_cost.cpp: eff / round_s per configuration and operation).

  python -m paper_1702_03192_amd.tune collect --out <dir>/gemm_table.csv [--odd-ld]      (needs the GPU)
  python -m paper_1702_03192_amd.tune fit     --table <dir>/gemm_table.csv                (host only)
  python -m paper_1702_03192_amd.tune extract --table <dir>/gemm_table.csv --out data/gemm_fit_rows_gfx950.csv   (host only)
  python -m paper_1702_03192_amd.tune even-cut --out <dir>/even_cut.csv                   (needs the GPU)

collect: for every (m, n, k) of the grid {64, ..., 8192}^3, both operations, every tile configuration
and every split count the library would consider (1, 2, 4, ..., 32 while k / splits >= 128 and the
partial products fit the 64 MiB scratch), the time of mtnn_gemm_ex: 2 warm-up calls, then the median
of `samples` event-timed batches of back-to-back calls lasting at least `min_batch_us`.  --odd-ld pads
every leading dimension by one element, which forces the guarded kernel (its numbers are fitted from
that table).

fit: per configuration and operation, a least-squares fit (in relative error) of
    time = tile_units x 2 bm bn k / (eff x peak_per_CU) + rounds x round_s + 3 us
(tile_units = tiles per CU, with a workgroup left alone at the end of a CU's share counted at its slower rate)
over the shapes whose tiles fill all 256 CUs at the configuration's occupancy with no partial tiles
and no split; prints the fitted (eff, round_s) in the order of the table in gemm_cost.cpp, and how far the
library's compiled-in choice (mtnn_gemm_default_config / _splits) is from the best measured
(configuration, split) pair of each shape.

even-cut: on seeded shapes off the power-of-two grids (k % 4 = 0, at least 2^30 multiply-adds) and a few
cubes, the NT time of the best unsplit or split ordinary launch among all configurations against the
even cut (splits = EVEN_CUT) with the 64 x 128 and 128 x 128 two-per-CU configurations; fits the four
weights of predicted_seconds_even_cut (gemm_cost.cpp) by least squares in relative error and reports where
the even cut wins and what the library's rule decides.
"""
from __future__ import annotations

import argparse
import csv
import re
import sys

PEAK_PER_CU = 157.3e12 / 256.0
SIZES = (64, 128, 256, 512, 1024, 2048, 4096, 8192)
SCRATCH_BYTES = 64 << 20


def collect(out_path, samples, min_batch_us, odd_ld):
    import torch
    from . import binding as mt
    from .sweep import _time_batches
    torch.cuda.set_device(0)
    mt.lib()
    stream = torch.cuda.current_stream()
    ncfg = len(mt.gemm_configs())
    pad = 1 if odd_ld else 0
    big = 8192
    bufA = torch.rand(big * (big + pad), device="cuda").mul_(2).sub_(1)
    bufB = torch.rand(big * (big + pad), device="cuda").mul_(2).sub_(1)
    bufC = torch.empty(big * big, device="cuda")
    for _ in range(40):                                           # clocks up
        mt.mtnn_gemm_ex(mt.OP_NT, 0, bufA[: 4096 * 4096].view(4096, 4096), bufB[: 4096 * 4096].view(4096, 4096),
                        bufC[: 4096 * 4096].view(4096, 4096))
    torch.cuda.synchronize()
    with open(out_path, "w", newline="") as f:
        wr = csv.writer(f)
        wr.writerow(["op", "m", "n", "k", "cfg", "splits", "seconds"])
        for m in SIZES:
            for n in SIZES:
                for k in SIZES:
                    for op in (mt.OP_NT, mt.OP_NN):
                        A = bufA[: m * (k + pad)].view(m, k + pad)[:, :k]
                        if op == mt.OP_NT:
                            B = bufB[: n * (k + pad)].view(n, k + pad)[:, :k]
                        else:
                            B = bufB[: k * (n + pad)].view(k, n + pad)[:, :n]
                        C = bufC[: m * n].view(m, n)
                        for cfg in range(ncfg):
                            splits = 1
                            while splits <= 32:
                                if splits > 1 and (k // splits < 128 or m * n * splits * 4 > SCRATCH_BYTES):
                                    break
                                t, _ = _time_batches(mt.prepare_gemm_ex(op, cfg, A, B, C, splits=splits),
                                                     stream, samples, min_batch_us)
                                wr.writerow([op, m, n, k, cfg, splits, "%.9g" % t])
                                splits *= 2
            f.flush()
            print(f"[tune] m = {m} done", flush=True)


def tile_units(per_cu, occ, waves):
    """A CU's share in tile times, as gemm_cost.cpp's cost model counts it: `per_cu` tiles worked through `occ`
    at a time; one 4-wave workgroup left over at the end runs alone, at 0.85 of the rate (0.92 after rounds
    of three)."""
    if waves >= 8 or per_cu % occ != 1:
        return float(per_cu)
    rate = 0.92 if (occ >= 3 and per_cu > 1) else 0.85
    return per_cu - 1 + 1.0 / rate


def _config_waves(name):
    g = re.match(r"\d+x\d+x\d+_w(\d+)x(\d+)(?:k(\d+))?_", name)          # (k2: two sets of waves per workgroup)
    return int(g.group(1)) * int(g.group(2)) * int(g.group(3) or 1)


def _config_geometry(name):
    """(bm, bn, workgroups per CU the launch allows, LDS bytes of the pipelined kernel) from a configuration name."""
    g = re.match(r"(\d+)x(\d+)x(\d+)_w(\d+)x(\d+)(?:k(\d+))?_dma(\d+)_x(\d+)", name)
    bm, bn, bk, wm, wn, ks, ns, max_wg = (int(v or 1) for v in g.groups())
    ring = ns * (bm + bn) * bk * 4
    patches = ks * wm * wn * 16 * (bn // wn + 8) * 4
    occ = max(1, min((160 * 1024) // max(ring, patches), max_wg))
    return bm, bn, occ


def load_table(table_path):
    table = {}
    with open(table_path, newline="") as f:
        for r in csv.DictReader(f):
            key = (int(r["op"]), int(r["m"]), int(r["n"]), int(r["k"]))
            table.setdefault(key, {})[(int(r["cfg"]), int(r["splits"]))] = float(r["seconds"])
    return table


def fit_table(table, names):
    """{(cfg, op): (eff, round_s, shapes used, mean relative error, max relative error)} -- None where a
    configuration has fewer than four usable shapes."""
    import numpy as np
    out = {}
    for c, nm in enumerate(names):
        bm, bn, occ = _config_geometry(nm)
        for op in (0, 1):
            X, y = [], []
            for (o, m, n, k), tab in table.items():
                if o != op or (c, 1) not in tab or m % bm or n % bn:
                    continue
                tiles = (m // bm) * (n // bn)
                if tiles < 256 * occ:
                    continue
                per_cu = -(-tiles // 256)
                X.append([tile_units(per_cu, occ, _config_waves(nm)) * 2.0 * bm * bn * k / PEAK_PER_CU, -(-per_cu // occ)])
                y.append(tab[(c, 1)] - 3e-6)
            if len(y) < 4:
                out[(c, op)] = None
                continue
            X, y = np.array(X), np.array(y)
            w = 1.0 / y
            co = np.linalg.lstsq(X * w[:, None], y * w, rcond=None)[0]
            err = np.abs(X @ co / y - 1.0)
            out[(c, op)] = (1.0 / co[0], co[1], len(y), float(err.mean()), float(err.max()))
    return out


def fit(table_path):
    import numpy as np
    from . import binding as mt
    names = mt.gemm_configs()
    table = load_table(table_path)
    fitted = fit_table(table, names)
    print("configuration: NN eff, round_s | NT eff, round_s   (shapes used, mean / max relative error of the fit)")
    for c, nm in enumerate(names):
        parts = []
        for op in (mt.OP_NN, mt.OP_NT):
            r = fitted[(c, op)]
            parts.append("(too few shapes)" if r is None else
                         f"{r[0]:.3f}, {r[1] * 1e6:.1f}e-6  (n={r[2]}, {r[3] * 100:.1f} % / {r[4] * 100:.1f} %)")
        print(f"  {c:2d} {nm}: " + " | ".join(parts))
    regrets = []
    for (op, m, n, k), tab in table.items():
        cfg = mt.mtnn_gemm_default_config(op, m, n, k)
        splits = mt.mtnn_gemm_default_splits(op, m, n, k)
        if (cfg, splits) not in tab:
            continue                                              # e.g. the even cut: not in this table
        regrets.append(tab[(cfg, splits)] / min(tab.values()) - 1.0)
    regrets = np.array(regrets)
    print(f"compiled-in choice against the best measured pair, {len(regrets)} (op, shape) cases: mean "
          f"{regrets.mean() * 100:.2f} %, worst {regrets.max() * 100:.1f} %, above 5 %: {(regrets > 0.05).sum()}")
    print("(the compiled-in choice assumes operands the pipelined kernel can take: compare it with a table "
          "collected without --odd-ld)")


def extract(table_path, out_path):
    """The part of a collected table that the numbers in the library rest on, small enough to keep under
    version control: the rows `fit` uses (unsplit launches on shapes whose tiles fill every CU with no
    partial tile), and per (operation, shape) the best measured (configuration, split) pair and the pair
    the compiled-in rule chooses, from which `fit` recomputes how far the rule is from the best."""
    from . import binding as mt
    names = mt.gemm_configs()
    table = load_table(table_path)
    keep = set()
    for (op, m, n, k), tab in table.items():
        for c, nm in enumerate(names):
            bm, bn, occ = _config_geometry(nm)
            if (c, 1) in tab and m % bm == 0 and n % bn == 0 and (m // bm) * (n // bn) >= 256 * occ:
                keep.add((op, m, n, k, c, 1))
        best = min(tab, key=tab.get)
        keep.add((op, m, n, k) + best)
        chosen = (mt.mtnn_gemm_default_config(op, m, n, k), mt.mtnn_gemm_default_splits(op, m, n, k))
        if chosen in tab:
            keep.add((op, m, n, k) + chosen)
    with open(out_path, "w", newline="") as f:
        wr = csv.writer(f)
        wr.writerow(["op", "m", "n", "k", "cfg", "splits", "seconds"])
        for key in sorted(keep):
            wr.writerow(list(key) + ["%.5g" % table[key[:4]][key[4:]]])
    print(f"[tune] kept {len(keep)} of {sum(len(v) for v in table.values())} rows in {out_path}")


def even_cut(out_path, samples, min_batch_us, count):
    import numpy as np
    import torch
    from . import binding as mt
    from .sweep import _time_batches, irregular_shapes
    torch.cuda.set_device(0)
    mt.lib()
    stream = torch.cuda.current_stream()
    names = mt.gemm_configs()
    even_cfgs = [c for c, nm in enumerate(names) if nm.startswith(("64x128x32_w2x2_dma2_x2", "128x128x32_w2x2_dma2_x2"))]
    shapes = [(m, n, k) for (m, n, k, _s) in irregular_shapes() if k % 4 == 0 and m * n * k >= 2 ** 30][:count]
    shapes += [(1536, 1536, 1536), (2560, 2560, 2560), (3072, 3072, 3072), (5120, 5120, 5120), (3000, 1500, 4500)]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(40000)
    rows = []
    for (m, n, k) in shapes:
        A = torch.rand((m, k), generator=gen, device="cuda").mul_(2).sub_(1)
        B = torch.rand((n, k), generator=gen, device="cuda").mul_(2).sub_(1)
        C = torch.empty((m, n), device="cuda")
        best = None
        for cfg in range(len(names)):
            splits = 1
            while splits <= 8:
                if splits > 1 and (k // splits < 128 or m * n * splits * 4 > SCRATCH_BYTES):
                    break
                t, _ = _time_batches(lambda: mt.mtnn_gemm_ex(mt.OP_NT, cfg, A, B, C, splits=splits), stream, samples, min_batch_us)
                if best is None or t < best[0]:
                    best = (t, cfg, splits)
                splits *= 2
        rec = {"m": m, "n": n, "k": k, "t_ordinary": best[0], "cfg_ordinary": names[best[1]], "splits_ordinary": best[2],
               "rule": mt.mtnn_gemm_default_splits(mt.OP_NT, m, n, k)}
        for cfg in even_cfgs:
            before = mt.mtnn_gemm_even_cut_launches()
            mt.mtnn_gemm_ex(mt.OP_NT, cfg, A, B, C, splits=mt.EVEN_CUT)
            if mt.mtnn_gemm_even_cut_launches() == before:
                rec[f"t_even_{cfg}"] = float("nan")                 # the even cut cannot run on this shape
                continue
            t, _ = _time_batches(lambda: mt.mtnn_gemm_ex(mt.OP_NT, cfg, A, B, C, splits=mt.EVEN_CUT), stream, samples, min_batch_us)
            rec[f"t_even_{cfg}"] = t
        rows.append(rec)
        print(f"[tune] {m}x{n}x{k}: ordinary {best[0] * 1e6:.1f} us ({names[best[1]]} x{best[2]}), even cut "
              + ", ".join(f"{rec[f't_even_{c}'] * 1e6:.1f}" for c in even_cfgs) + f" us, rule {rec['rule']}", flush=True)
        del A, B, C
    with open(out_path, "w", newline="") as f:
        wr = csv.DictWriter(f, fieldnames=list(rows[0].keys()))
        wr.writeheader()
        wr.writerows(rows)
    # the four weights: time = a x k-loop + b x segments x round_s + c x fix-up bytes / 4e12 + d,
    # with the NT k-loop rate and per-round time of the two configurations as compiled into gemm_cost.cpp
    compiled = {"64x128x32_w2x2_dma2_x2": (0.913, 2.7e-6), "128x128x32_w2x2_dma2_x2": (0.933, 5.3e-6)}
    X, y = [], []
    for r in rows:
        for cfg in even_cfgs:
            t = r[f"t_even_{cfg}"]
            if t != t:
                continue
            bm, bn, occ = _config_geometry(names[cfg])
            tiles = -(-r["m"] // bm) * -(-r["n"] // bn)
            upt = -(-r["k"] // 64)
            groups = 256 * occ
            upw = tiles * upt / groups
            eff, round_s = compiled[names[cfg]]
            main_s = upw * occ * 2.0 * bm * bn * 64 / (PEAK_PER_CU * eff)
            segments = upw / upt + 1.0
            pieces = max(2.0, groups / tiles + 1.0) if tiles < groups else 2.0
            fix_bytes = min(tiles, groups) * (pieces + 1.0) * bm * bn * 4.0
            X.append([main_s, segments * round_s, fix_bytes / 4.0e12, 1.0])
            y.append(t)
    X, y = np.array(X), np.array(y)
    w = 1.0 / y
    co = np.linalg.lstsq(X * w[:, None], y * w, rcond=None)[0]
    err = np.abs(X @ co / y - 1.0)
    print(f"weights (k loop, segments x round_s, fix-up bytes at 4 TB/s, constant; single-call timing adds ~3 us "
          f"to the constant that the model carries separately): "
          f"{co[0]:.2f}, {co[1]:.2f}, {co[2]:.2f}, {co[3] * 1e6:.1f} us; mean error {err.mean() * 100:.1f} %")
    wins = [r for r in rows if min(r[f"t_even_{c}"] for c in even_cfgs) < r["t_ordinary"]]
    taken = [r for r in rows if r["rule"] == mt.EVEN_CUT]
    wrong = [r for r in taken if min(r[f"t_even_{c}"] for c in even_cfgs) > 1.02 * r["t_ordinary"]]
    print(f"even cut faster than the best ordinary launch on {len(wins)} of {len(rows)} shapes; the rule takes it on "
          f"{len(taken)}, wrongly (2 % slower or more) on {len(wrong)}")


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    c = sub.add_parser("collect")
    c.add_argument("--out", required=True)
    c.add_argument("--samples", type=int, default=5)
    c.add_argument("--min-batch-us", type=float, default=300.0)
    c.add_argument("--odd-ld", action="store_true")
    f = sub.add_parser("fit")
    f.add_argument("--table", required=True)
    x = sub.add_parser("extract")
    x.add_argument("--table", required=True)
    x.add_argument("--out", required=True)
    e = sub.add_parser("even-cut")
    e.add_argument("--out", required=True)
    e.add_argument("--samples", type=int, default=7)
    e.add_argument("--min-batch-us", type=float, default=1000.0)
    e.add_argument("--count", type=int, default=60)
    args = ap.parse_args(argv)
    if args.cmd == "collect":
        collect(args.out, args.samples, args.min_batch_us, args.odd_ld)
    elif args.cmd == "extract":
        extract(args.table, args.out)
    elif args.cmd == "even-cut":
        even_cut(args.out, args.samples, args.min_batch_us, args.count)
    else:
        fit(args.table)
    return 0


if __name__ == "__main__":
    sys.exit(main())
