"""Offline side of the selector (Section IV of the MTNN paper): the timing table of the shape
sweep, labels, train/test protocol and the report of Section V.

The boosted trees themselves are fitted and evaluated inside libmtnn (``mtnn_train_selector`` /
``mtnn_select``); this module only moves rows in and out and does the bookkeeping around them:

  * label rule (Section IV-A): +1 when P_NT >= P_TNN (ties to NT), else -1; for one shape
    that is t_NT <= t_TNN;
  * protocol (Section IV-B): seeded 80/20 split, 5-fold cross-validation, final model trained
    on every row.  The paper stratifies its split by GPU; with one GPU the split is stratified
    by class;
  * metrics (Section V-B): GOW, LUB, average gain over always-NT / always-TNN, accuracy.
"""
from __future__ import annotations

import csv
import json
import os
from typing import Dict, List, Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
DATA = os.path.join(HERE, "data")
SWEEP_CSV = os.path.join(DATA, "sweep_gfx950.csv")
MODEL_FILE = os.path.join(DATA, "selector_gfx950.model")
# the shipped model is fitted on the union of the three measured tables: the benchmark grid
# {64..8192}^3, the paper's range {2^7..2^16}^3 and the seeded shapes off the power-of-two grids
TRAINING_TABLES = (SWEEP_CSV, os.path.join(DATA, "sweep_irregular_gfx950.csv"),
                   os.path.join(DATA, "sweep_paper_range_gfx950.csv"))
TRAFFIC_JSON = os.path.join(DATA, "measured_traffic_gfx950.json")


def load_sweep(path: str = SWEEP_CSV) -> List[Dict[str, float]]:
    """Rows of the timing table: m, n, k (ints) and t_nt, t_tnn in seconds (medians), plus extras."""
    rows = []
    with open(path, newline="") as f:
        for rec in csv.DictReader(f):
            row = {}
            for key, val in rec.items():
                if key in ("m", "n", "k", "seed"):
                    row[key] = int(val)
                elif key in ("nt_cfg", "nn_cfg"):
                    row[key] = val
                else:
                    row[key] = float(val)
            rows.append(row)
    return rows


def load_training_rows(paths: Optional[Sequence[str]] = None) -> List[Dict[str, float]]:
    """Union of the given timing tables (default: the shipped ones that exist); a shape listed in
    more than one table keeps its first row."""
    rows, seen = [], set()
    for path in (TRAINING_TABLES if paths is None else paths):
        if paths is None and not os.path.exists(path):
            continue
        for row in load_sweep(path):
            key = (row["m"], row["n"], row["k"])
            if key not in seen:
                seen.add(key)
                rows.append(row)
    return rows


def label_of(t_nt: float, t_tnn: float) -> int:
    return 1 if t_nt <= t_tnn else -1


def stratified_split(labels: Sequence[int], seed: int, test_fraction: float = 0.2) -> Tuple[List[int], List[int]]:
    """Seeded split that keeps the class proportions; returns (train indices, test indices)."""
    import numpy as np
    rng = np.random.default_rng(seed)
    train: List[int] = []
    test: List[int] = []
    for cls in (-1, 1):
        members = [i for i, l in enumerate(labels) if l == cls]
        order = rng.permutation(len(members))
        cut = int(round(test_fraction * len(members)))
        test += [members[j] for j in order[:cut]]
        train += [members[j] for j in order[cut:]]
    return sorted(train), sorted(test)


def kfold(labels: Sequence[int], folds: int, seed: int) -> List[Tuple[List[int], List[int]]]:
    """Class-stratified k folds; returns (train, test) index lists per fold."""
    import numpy as np
    rng = np.random.default_rng(seed)
    buckets: List[List[int]] = [[] for _ in range(folds)]
    for cls in (-1, 1):
        members = [i for i, l in enumerate(labels) if l == cls]
        order = rng.permutation(len(members))
        for pos, j in enumerate(order):
            buckets[pos % folds].append(members[j])
    out = []
    for f in range(folds):
        test = sorted(buckets[f])
        train = sorted(i for g in range(folds) if g != f for i in buckets[g])
        out.append((train, test))
    return out


def selection_metrics(t_nt: Sequence[float], t_tnn: Sequence[float], shapes, predicted: Sequence[int]) -> Dict[str, float]:
    """Table VII on measured times.  P = 2mnk / t; P_MTNN is the P of the predicted algorithm."""
    n = len(predicted)
    gows, lubs, vs_nt, vs_tnn = [], [], [], []
    correct = 0
    for i in range(n):
        m, nn, k = shapes[i]
        flop = 2.0 * m * nn * k
        p_nt, p_tnn = flop / t_nt[i], flop / t_tnn[i]
        p_m = p_nt if predicted[i] == 1 else p_tnn
        lo, hi = min(p_nt, p_tnn), max(p_nt, p_tnn)
        gows.append((p_m - lo) / lo)
        lubs.append((p_m - hi) / hi)
        vs_nt.append((p_m - p_nt) / p_nt)
        vs_tnn.append((p_m - p_tnn) / p_tnn)
        correct += int(predicted[i] == label_of(t_nt[i], t_tnn[i]))
    return {"mtnn_vs_nt": sum(vs_nt) / n, "mtnn_vs_tnn": sum(vs_tnn) / n,
            "gow_avg": sum(gows) / n, "gow_max": max(gows), "lub_avg": sum(lubs) / n, "lub_min": min(lubs),
            "accuracy": correct / n}


def nt_tnn_statistics(rows) -> Dict[str, object]:
    """What Sections II and III of the paper read off their figures, on one of our timing tables (rows
    with t_nt, t_nn, t_transpose and t_tnn, the last timed as one mtnn_tnn call):

      * Fig. 1 / 2: the share of shapes on which the NN kernel beats the NT kernel, and by 2x or more;
      * Fig. 3: the share of shapes with P_TNN / P_NT below 1, the largest ratio either way, and the
        distribution of log2(P_TNN / P_NT) in bins of a quarter;
      * Eq. 4: on how many shapes T_transpose < T_NT - T_NN holds for the separately timed parts, and on
        how many that agrees with the label of the directly timed pair (t_tnn < t_nt) -- i.e. whether
        TNN's time is the sum of its two parts.
    """
    import math
    n = len(rows)
    nn_faster = sum(1 for r in rows if r["t_nn"] < r["t_nt"])
    nn_twice = sum(1 for r in rows if r["t_nt"] >= 2.0 * r["t_nn"])
    below = sum(1 for r in rows if r["t_nt"] < r["t_tnn"])
    best_tnn = max(rows, key=lambda r: r["t_nt"] / r["t_tnn"])
    best_nt = max(rows, key=lambda r: r["t_tnn"] / r["t_nt"])
    eq4 = [r["t_transpose"] < r["t_nt"] - r["t_nn"] for r in rows]
    direct = [r["t_tnn"] < r["t_nt"] for r in rows]
    hist: Dict[str, int] = {}
    for r in rows:
        b = math.floor(math.log2(r["t_nt"] / r["t_tnn"]) * 4.0) / 4.0
        key = "%+.2f" % b
        hist[key] = hist.get(key, 0) + 1
    additivity = [(r["t_transpose"] + r["t_nn"]) / r["t_tnn"] for r in rows]
    return {"shapes": n,
            "nn_faster_than_nt": nn_faster / n, "nn_twice_nt": nn_twice / n,
            "tnn_over_nt_below_1": below / n,
            "max_tnn_over_nt": best_tnn["t_nt"] / best_tnn["t_tnn"],
            "max_tnn_over_nt_shape": (best_tnn["m"], best_tnn["n"], best_tnn["k"]),
            "max_nt_over_tnn": best_nt["t_tnn"] / best_nt["t_nt"],
            "max_nt_over_tnn_shape": (best_nt["m"], best_nt["n"], best_nt["k"]),
            "eq4_holds": sum(eq4), "eq4_agrees_with_direct_label": sum(int(a == b) for a, b in zip(eq4, direct)),
            "parts_over_whole_median": sorted(additivity)[n // 2],
            "log2_tnn_over_nt_histogram": dict(sorted(hist.items(), key=lambda kv: float(kv[0])))}


def _fit_predict(train_shapes, train_labels, test_shapes) -> List[int]:
    from . import binding as mt
    mt.mtnn_train_selector(train_shapes, train_labels)
    return [mt.mtnn_select(*s) for s in test_shapes]


def evaluate(rows, split_seeds=(1, 2, 3, 4, 5), cv_seed=0) -> Dict[str, object]:
    """The paper's evaluation protocol on a timing table; trains through the library.
    Leaves the library's current predictor trained on all rows."""
    shapes = [(r["m"], r["n"], r["k"]) for r in rows]
    t_nt = [r["t_nt"] for r in rows]
    t_tnn = [r["t_tnn"] for r in rows]
    labels = [label_of(a, b) for a, b in zip(t_nt, t_tnn)]
    n_pos = sum(1 for l in labels if l == 1)
    n_neg = len(labels) - n_pos
    report: Dict[str, object] = {"samples": len(rows), "n_label_nt": n_pos, "n_label_tnn": n_neg,
                                 "majority_class_accuracy": max(n_pos, n_neg) / len(rows)}
    if n_pos == 0 or n_neg == 0:
        report["note"] = "one class only: every predictor is the majority rule"
    held = []
    for seed in split_seeds:
        tr, te = stratified_split(labels, seed)
        pred = _fit_predict([shapes[i] for i in tr], [labels[i] for i in tr], [shapes[i] for i in te])
        held.append(sum(int(p == labels[i]) for p, i in zip(pred, te)) / max(len(te), 1))
    report["held_out_accuracy_mean"] = sum(held) / len(held)
    report["held_out_accuracy_min"] = min(held)
    report["held_out_accuracy_max"] = max(held)
    cv = []
    cv_neg, cv_pos = [], []
    for tr, te in kfold(labels, 5, cv_seed):
        pred = _fit_predict([shapes[i] for i in tr], [labels[i] for i in tr], [shapes[i] for i in te])
        cv.append(sum(int(p == labels[i]) for p, i in zip(pred, te)) / max(len(te), 1))
        neg = [(p, i) for p, i in zip(pred, te) if labels[i] == -1]
        pos = [(p, i) for p, i in zip(pred, te) if labels[i] == 1]
        if neg:
            cv_neg.append(sum(int(p == -1) for p, _ in neg) / len(neg))
        if pos:
            cv_pos.append(sum(int(p == 1) for p, _ in pos) / len(pos))
    report["cv5_accuracy_mean"] = sum(cv) / len(cv)
    report["cv5_accuracy_min"] = min(cv)
    report["cv5_accuracy_max"] = max(cv)
    report["cv5_accuracy_tnn_class"] = sum(cv_neg) / len(cv_neg) if cv_neg else None
    report["cv5_accuracy_nt_class"] = sum(cv_pos) / len(cv_pos) if cv_pos else None
    # margin-aware accuracy: shapes whose two times differ by more than 3 %
    pred_all = _fit_predict(shapes, labels, shapes)            # final model: all rows
    report["train_on_all_accuracy"] = sum(int(p == l) for p, l in zip(pred_all, labels)) / len(labels)
    clear = [i for i in range(len(rows)) if abs(t_nt[i] - t_tnn[i]) / min(t_nt[i], t_tnn[i]) > 0.03]
    report["clear_margin_samples"] = len(clear)
    report["train_on_all_accuracy_clear_margin"] = (
        sum(int(pred_all[i] == labels[i]) for i in clear) / len(clear) if clear else None)
    report.update({"all_" + k: v for k, v in selection_metrics(t_nt, t_tnn, shapes, pred_all).items()})
    # held-out selection quality with the first split (what a deployed model faces on unseen shapes)
    tr, te = stratified_split(labels, split_seeds[0])
    pred = _fit_predict([shapes[i] for i in tr], [labels[i] for i in tr], [shapes[i] for i in te])
    held_m = selection_metrics([t_nt[i] for i in te], [t_tnn[i] for i in te], [shapes[i] for i in te], pred)
    report.update({"held_out_" + k: v for k, v in held_m.items()})
    _fit_predict(shapes, labels, shapes[:1])                    # leave the all-rows model installed
    return report


def selector_report() -> Dict[str, object]:
    """Evaluation of the selector on the stored sweep, if there is one; restores the shipped model."""
    from . import binding as mt
    if not os.path.exists(SWEEP_CSV):
        return {"sweep": None, "note": "no stored sweep table: selector untrained, mtnn_select answers NT"}
    rows = load_sweep()
    rep = evaluate(rows)
    rep["sweep"] = os.path.relpath(SWEEP_CSV, os.path.dirname(HERE))
    if os.path.exists(MODEL_FILE):
        mt.mtnn_load_model(MODEL_FILE)
    return rep


def measured_traffic_bytes(kernel_name: str) -> Optional[float]:
    """HBM bytes per launch of a kernel as measured with hardware counters (stored with the
    profiles' summaries); None when there is no measurement for that kernel."""
    if not os.path.exists(TRAFFIC_JSON):
        return None
    with open(TRAFFIC_JSON) as f:
        table = json.load(f)
    entry = table.get(kernel_name)
    return float(entry["bytes_per_launch"]) if entry else None
