"""Classifier comparison and training-size curve on a timing table (Section V-A of the MTNN paper:
Table VI and the convergence figure).  Host only.

  python -m paper_1702_03192_amd.classifier_study --csv <table> --out <report.json>

Compared: the boosted trees of the paper (8 trees, depth 8), a single decision tree (one tree, depth 8:
the paper's "DT"), the two support vector machines of Table VI (radial basis function and polynomial
kernels with the paper's C = 1000 and gamma = 0.01, features scaled to (0, 1) on the training rows;
our own solver, svm.py) and the majority rule.  Accuracy is 5-fold cross-validated; train time is
one fit on all rows; predict time is per prediction (trees: inside the library, mtnn_select_batch
over 10^6 shapes; SVMs: the decision function over 20000 shapes).  The training-size curve trains on x % of the rows (stratified, seeded) and tests on all
rows, x = 10, 15, ..., 100, as in the paper.
"""
from __future__ import annotations

import argparse
import json
import sys
import time


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--csv", required=True)
    ap.add_argument("--out", required=True)
    args = ap.parse_args(argv)

    import numpy as np
    from . import binding as mt
    from . import selector_data as sd

    rows = sd.load_sweep(args.csv)
    shapes = np.array([(r["m"], r["n"], r["k"]) for r in rows], dtype=np.int32)
    labels = np.array([sd.label_of(r["t_nt"], r["t_tnn"]) for r in rows], dtype=np.int32)
    L = mt.lib()
    X = np.array([mt.mtnn_features(*map(int, s)) for s in shapes])
    rng = np.random.default_rng(0)
    probe = rng.integers(64, 65536, size=(1000000, 3)).astype(np.int32)

    def fit(idx, trees):
        mt.mtnn_gbdt_train(X[idx], labels[idx], num_trees=trees, max_depth=8)

    report = {"table": args.csv, "samples": int(len(rows)), "n_label_nt": int((labels == 1).sum()),
              "n_label_tnn": int((labels == -1).sum()), "classifiers": {}}
    folds = sd.kfold(list(labels), 5, 0)
    for name, trees in (("GBDT (8 trees, depth 8)", 8), ("DT (1 tree, depth 8)", 1)):
        accs = []
        for tr, te in folds:
            fit(np.array(tr), trees)
            pred = mt.mtnn_select_batch(shapes[te])
            accs.append(float((pred == labels[te]).mean()))
        times = []
        for _ in range(5):
            t0 = time.perf_counter()
            fit(np.arange(len(rows)), trees)
            times.append(time.perf_counter() - t0)
        t0 = time.perf_counter()
        mt.mtnn_select_batch(probe)
        per_pred = (time.perf_counter() - t0) / len(probe)
        train_acc = float((mt.mtnn_select_batch(shapes) == labels).mean())
        report["classifiers"][name] = {"cv5_accuracy": float(np.mean(accs)), "cv5_min": min(accs), "cv5_max": max(accs),
                                       "train_on_all_accuracy": train_acc, "train_ms": float(np.median(times) * 1e3),
                                       "predict_us": per_pred * 1e6, "nodes": sum(L.mtnn_model_tree_size(t) for t in range(L.mtnn_model_num_trees()))}
    from . import svm
    probe_x = np.array([mt.mtnn_features(*map(int, s)) for s in probe[:20000]])
    for name, kind in (("SVM-RBF (C 1000, gamma 0.01)", "rbf"), ("SVM-Poly (C 1000, gamma 0.01, degree 3)", "poly")):
        accs, acc_nt, acc_tnn = [], [], []
        for tr, te in folds:
            tr, te = np.array(tr), np.array(te)
            if len(set(labels[tr])) < 2:
                pred = np.full(len(te), labels[tr][0])
            else:
                xs, lo, hi = svm.scale01(X[tr])
                model = svm.train(xs, labels[tr], kind)
                pred = model.predict(svm.scale01(X[te], lo, hi)[0])
            accs.append(float((pred == labels[te]).mean()))
            if (labels[te] == 1).any():
                acc_nt.append(float((pred[labels[te] == 1] == 1).mean()))
            if (labels[te] == -1).any():
                acc_tnn.append(float((pred[labels[te] == -1] == -1).mean()))
        entry = {"cv5_accuracy": float(np.mean(accs)), "cv5_min": min(accs), "cv5_max": max(accs),
                 "cv5_accuracy_nt_class": float(np.mean(acc_nt)) if acc_nt else None,
                 "cv5_accuracy_tnn_class": float(np.mean(acc_tnn)) if acc_tnn else None}
        if len(set(labels)) >= 2:
            xs, lo, hi = svm.scale01(X)
            t0 = time.perf_counter()
            model = svm.train(xs, labels, kind)
            entry["train_ms"] = (time.perf_counter() - t0) * 1e3
            entry["train_on_all_accuracy"] = float((model.predict(xs) == labels).mean())
            entry["support_vectors"] = int(model.sv.shape[0])
            entry["solver_steps"], entry["solver_converged"] = int(model.steps), bool(model.converged)
            ps = svm.scale01(probe_x, lo, hi)[0]
            t0 = time.perf_counter()
            model.predict(ps)
            entry["predict_us"] = (time.perf_counter() - t0) / len(ps) * 1e6
        report["classifiers"][name] = entry
    maj = 1 if (labels == 1).sum() >= (labels == -1).sum() else -1
    report["classifiers"]["majority rule"] = {"cv5_accuracy": float(np.mean([(labels[te] == maj).mean() for _, te in folds])),
                                              "train_ms": 0.0, "predict_us": 0.0}
    curve = []
    for pct in range(10, 101, 5):
        accs = []
        for seed in range(3):
            if pct == 100:
                idx = np.arange(len(rows))
            else:
                tr, te = sd.stratified_split(list(labels), 100 + seed, test_fraction=1.0 - pct / 100.0)
                idx = np.array(tr)
            if len(set(labels[idx])) < 2:
                accs.append(float((labels == labels[idx][0]).mean()))
                continue
            fit(idx, 8)
            accs.append(float((mt.mtnn_select_batch(shapes) == labels).mean()))
        curve.append({"train_percent": pct, "accuracy_on_all": float(np.mean(accs))})
    report["training_size_curve"] = curve
    mt.mtnn_unload_model()
    if sd.os.path.exists(sd.MODEL_FILE):
        mt.mtnn_load_model(sd.MODEL_FILE)
    text = json.dumps(report, indent=1)
    with open(args.out, "w") as f:
        f.write(text + "\n")
    print(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
