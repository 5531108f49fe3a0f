"""The library's boosted-tree trainer and evaluator against the CPU oracle (host only)."""
import os

import numpy as np
import pytest

from oracle import selection as S
from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import inputs as I


@pytest.fixture(autouse=True)
def _fresh_model():
    mt.lib()
    yield
    mt.mtnn_unload_model()
    if os.path.exists(mt.DEFAULT_MODEL):
        mt.mtnn_load_model(mt.DEFAULT_MODEL)


def same_trees(ours, ref, rel=1e-12):
    assert len(ours) == len(ref)
    for a, b in zip(ours, ref):
        assert len(a) == len(b)
        for (f1, t1, l1, r1, v1), (f2, t2, l2, r2, v2) in zip(a, b):
            assert (f1, l1, r1) == (f2, l2, r2)
            assert t1 == t2
            assert v1 == pytest.approx(v2, rel=rel, abs=1e-15)


def synthetic_table(rule_seed=0):
    """(m, n, k, label) over the sweep grid from a made-up timing model with noise (host only)."""
    rng = np.random.RandomState(rule_seed)
    rows, lab = [], []
    for (m, n, k, _seed) in I.sweep_shapes():
        t_nt = m * n * k / 100e3 * (1.0 + 0.3 * (k >= 2048)) + 5.0
        t_tnn = m * n * k / 100e3 + n * k / 2e3 + 9.0
        t_nt *= 1.0 + 0.05 * rng.standard_normal()
        t_tnn *= 1.0 + 0.05 * rng.standard_normal()
        rows.append((m, n, k))
        lab.append(S.label_from_times(t_nt, t_tnn))
    return rows, lab


def test_features_match_the_oracle():
    assert mt.lib().mtnn_num_features() == len(S.FEATURE_NAMES)
    for shape in [(1, 1, 1), (64, 128, 8192), (8192, 8192, 8192), (65536, 65536, 65536), (3000, 1500, 4500)]:
        assert mt.mtnn_features(*shape) == S.features(*shape)


def test_no_model_means_nt_and_bad_shapes_give_zero():
    mt.mtnn_unload_model()
    assert mt.mtnn_select(4096, 4096, 4096) == 1
    assert mt.mtnn_select(0, 4, 4) == 0 and mt.mtnn_select(4, -1, 4) == 0


def test_trainer_first_round_closed_form():
    X = np.arange(1, 9, dtype=np.float64).reshape(-1, 1)
    mt.mtnn_gbdt_train(X, [-1] * 4 + [1] * 4, num_trees=1)
    assert mt.model_trees() == [[(0, 4.5, 1, 2, 0.0), (-1, 0.0, -1, -1, -1.0), (-1, 0.0, -1, -1, 1.0)]]


def test_trainer_matches_oracle_on_toy_sets():
    rng = np.random.RandomState(5)
    X = rng.uniform(0, 1, size=(300, 4))
    y = [1 if (a * 2 - b + 0.3 * np.sin(6 * c) + 0.1 * rng.standard_normal()) > 0.5 else -1 for a, b, c, _ in X]
    mt.mtnn_gbdt_train(X, y)
    same_trees(mt.model_trees(), S.flatten(S.train_gbdt(X, y)))


def test_trainer_matches_oracle_on_a_sweep_shaped_table():
    rows, lab = synthetic_table()
    assert 50 < sum(1 for l in lab if l == -1) < 462      # both classes present
    mt.mtnn_train_selector(rows, lab)
    ref = S.train_gbdt(np.array([S.features(*r) for r in rows]), lab)
    same_trees(mt.model_trees(), S.flatten(ref))
    assert len(mt.model_trees()) == 8
    # evaluator parity: every grid shape and 10^4 random shapes, exact label equality
    for r in rows:
        assert mt.mtnn_select(*r) == S.select(ref, *r)
    dims = I.uniform_ints(77, 0, 30000, 1, 20000).reshape(-1, 3)
    for m, n, k in dims:
        assert mt.mtnn_select(int(m), int(n), int(k)) == S.select(ref, int(m), int(n), int(k))
        x = S.features(int(m), int(n), int(k))
        assert mt.mtnn_model_margin(x) == pytest.approx(S.margin(ref, x), rel=1e-12, abs=1e-15)


def test_held_out_accuracy_equals_the_oracles():
    rows, lab = synthetic_table(rule_seed=3)
    tr, te = S.stratified_split(lab, seed=11)
    mt.mtnn_train_selector([rows[i] for i in tr], [lab[i] for i in tr])
    ref = S.train_gbdt(np.array([S.features(*rows[i]) for i in tr]), [lab[i] for i in tr])
    ours = [mt.mtnn_select(*rows[i]) for i in te]
    theirs = [S.select(ref, *rows[i]) for i in te]
    assert ours == theirs
    acc = np.mean([o == lab[i] for o, i in zip(ours, te)])
    assert acc > 0.8


def test_model_file_round_trip_and_rejection(tmp_path):
    rows, lab = synthetic_table()
    mt.mtnn_train_selector(rows, lab)
    before = mt.model_trees()
    path = str(tmp_path / "m.model")
    mt.mtnn_save_model(path)
    mt.mtnn_unload_model()
    assert mt.lib().mtnn_model_num_trees() == 0
    mt.mtnn_load_model(path)
    assert mt.model_trees() == before                      # hex floats round-trip exactly
    # corrupt files leave the current model in place
    text = open(path).read()
    for bad in [text.replace("mtnn-gbdt 1", "mtnn-gbdt 9"), text[: len(text) // 2], "garbage",
                text.replace("features 7", "features 0")]:
        p = str(tmp_path / "bad.model")
        open(p, "w").write(bad)
        with pytest.raises(mt.MtnnError) as e:
            mt.mtnn_load_model(p)
        assert e.value.status == 7
        assert mt.model_trees() == before
    with pytest.raises(mt.MtnnError):
        mt.mtnn_load_model(str(tmp_path / "missing.model"))
    # a child index pointing backwards would loop forever: rejected
    lines = text.splitlines()
    idx = next(i for i, l in enumerate(lines) if l.startswith("tree 0")) + 1
    f = lines[idx].split()
    f[2] = "0"
    lines[idx] = " ".join(f)
    p = str(tmp_path / "loop.model")
    open(p, "w").write("\n".join(lines) + "\n")
    with pytest.raises(mt.MtnnError):
        mt.mtnn_load_model(p)


def test_trainer_argument_checks():
    L = mt.lib()
    X = np.zeros((4, 2))
    y = np.array([1, -1, 1, 0], dtype=np.int32)
    assert L.mtnn_gbdt_train(4, 2, X.ctypes.data, y.ctypes.data, 8, 8, 1.0, 0.0, 1.0, 1.0) == 8   # label 0
    y[3] = 1
    assert L.mtnn_gbdt_train(0, 2, X.ctypes.data, y.ctypes.data, 8, 8, 1.0, 0.0, 1.0, 1.0) == 8
    assert L.mtnn_gbdt_train(4, 2, None, y.ctypes.data, 8, 8, 1.0, 0.0, 1.0, 1.0) == 2
    X[0, 0] = np.nan
    assert L.mtnn_gbdt_train(4, 2, X.ctypes.data, y.ctypes.data, 8, 8, 1.0, 0.0, 1.0, 1.0) == 8


def parse_model_file(path):
    """Independent reader of the model text format (C99 hex floats), for the oracle's evaluator."""
    lines = [l.split() for l in open(path).read().splitlines() if l.strip()]
    assert lines[0] == ["mtnn-gbdt", "1"]
    nfeat = int(lines[1][1])
    ntrees = int(lines[2][1])
    pos = 3
    trees = []
    for t in range(ntrees):
        assert lines[pos][0] == "tree" and int(lines[pos][1]) == t
        n = int(lines[pos][3])
        pos += 1
        rows = []
        for _ in range(n):
            f, thr, l, r, v = lines[pos]
            rows.append((int(f), float.fromhex(thr), int(l), int(r), float.fromhex(v)))
            pos += 1
        trees.append(rows)
    return nfeat, trees


def flat_margin(trees, x):
    total = 0.0
    for rows in trees:
        at = 0
        while rows[at][0] >= 0:
            at = rows[at][2] if x[rows[at][0]] < rows[at][1] else rows[at][3]
        total += rows[at][4]
    return total


def test_shipped_model_agrees_with_an_independent_evaluator_on_grid_and_random_shapes():
    if not os.path.exists(mt.DEFAULT_MODEL):
        pytest.skip("no shipped model")
    mt.mtnn_load_model(mt.DEFAULT_MODEL)
    nfeat, trees = parse_model_file(mt.DEFAULT_MODEL)
    assert nfeat == 7 and len(trees) <= 8
    assert mt.model_trees() == trees
    shapes = [(m, n, k) for (m, n, k, _s) in I.sweep_shapes()]
    shapes += [tuple(int(v) for v in row) for row in I.uniform_ints(78, 0, 30000, 1, 70000).reshape(-1, 3)]
    for s in shapes:
        want = 1 if flat_margin(trees, S.features(*s)) >= 0.0 else -1
        assert mt.mtnn_select(*s) == want


def test_trained_on_the_shipped_sweep_table_trainer_parity():
    """The library's trainer and the oracle's, on the real MI355X timing tables (the union the shipped
    model is fitted on)."""
    from paper_1702_03192_amd import selector_data as sd
    if not os.path.exists(sd.SWEEP_CSV):
        pytest.skip("no shipped sweep table")
    rows = sd.load_training_rows()
    shapes = [(r["m"], r["n"], r["k"]) for r in rows]
    labels = [S.label_from_times(r["t_nt"], r["t_tnn"]) for r in rows]
    assert labels == [sd.label_of(r["t_nt"], r["t_tnn"]) for r in rows]
    if len(set(labels)) < 2:
        pytest.skip("single-class table")
    mt.mtnn_train_selector(shapes, labels)
    ref = S.train_gbdt(np.array([S.features(*s) for s in shapes]), labels)
    same_trees(mt.model_trees(), S.flatten(ref))
    # and the shipped model file is this model
    if os.path.exists(mt.DEFAULT_MODEL):
        assert parse_model_file(mt.DEFAULT_MODEL)[1] == mt.model_trees()


def test_env_model_is_loaded_on_first_use(tmp_path):
    import subprocess
    import sys
    rows, lab = synthetic_table()
    mt.mtnn_train_selector(rows, lab)
    path = str(tmp_path / "env.model")
    mt.mtnn_save_model(path)
    want = [mt.mtnn_select(*r) for r in rows[:64]]
    code = ("import ctypes, torch; L = ctypes.CDLL(%r); "
            "print([L.mtnn_select(*r) for r in %r])" % (mt.LIB_PATH, rows[:64]))
    out = subprocess.run([sys.executable, "-c", code], env=dict(os.environ, MTNN_MODEL=path),
                         capture_output=True, text=True, check=True).stdout
    assert eval(out.strip().splitlines()[-1]) == want
    out = subprocess.run([sys.executable, "-c", code], env=dict(os.environ, MTNN_MODEL=str(tmp_path / "none")),
                         capture_output=True, text=True, check=True).stdout
    assert eval(out.strip().splitlines()[-1]) == [1] * 64


def test_select_batch_equals_select():
    rows, lab = synthetic_table()
    mt.mtnn_train_selector(rows, lab)
    shapes = [tuple(int(v) for v in row) for row in I.uniform_ints(79, 0, 3000, -2, 9000).reshape(-1, 3)]
    shapes += [(0, 5, 5), (7, -1, 3)]
    got = mt.mtnn_select_batch(shapes)
    assert list(got) == [mt.mtnn_select(*s) for s in shapes]
    assert 0 in got                                         # non-positive sizes answer 0
    mt.mtnn_unload_model()
    assert set(mt.mtnn_select_batch([(5, 5, 5), (0, 1, 1)])) == {1, 0}
    assert mt.lib().mtnn_select_batch(-1, None, None) == 1
    assert mt.lib().mtnn_select_batch(2, None, None) == 2


def test_classifier_study_runs_on_a_synthetic_table(tmp_path):
    import csv
    import json
    from paper_1702_03192_amd import classifier_study, sweep
    rows, lab = synthetic_table()
    p = tmp_path / "t.csv"
    with open(p, "w", newline="") as f:
        wr = csv.DictWriter(f, fieldnames=sweep.FIELDS)
        wr.writeheader()
        for (m, n, k), l in zip(rows, lab):
            wr.writerow({"m": m, "n": n, "k": k, "seed": 0, "t_nt": 1.0 if l == 1 else 2.0, "t_nt_min": 1.0,
                         "t_tnn": 1.5, "t_tnn_min": 1.5, "t_transpose": 0.1, "t_nn": 1.4, "t_tnn_alloc": 1.6,
                         "nt_cfg": "a", "nn_cfg": "b"})
    out = tmp_path / "r.json"
    classifier_study.main(["--csv", str(p), "--out", str(out)])
    rep = json.load(open(out))
    assert rep["samples"] == 512 and len(rep["training_size_curve"]) == 19
    g = rep["classifiers"]["GBDT (8 trees, depth 8)"]
    assert g["cv5_accuracy"] >= rep["classifiers"]["majority rule"]["cv5_accuracy"] - 0.02
    assert rep["training_size_curve"][-1]["accuracy_on_all"] >= rep["training_size_curve"][0]["accuracy_on_all"] - 0.01


def test_memo_follows_the_model_through_retraining():
    """mtnn_select memoises its last answer; the memo must die with the model it came from, also when a
    later model happens to be allocated where an earlier one was (train A, train B, train C, querying
    one shape under A and C only)."""
    shapes = np.array([[m, n, k] for m in (64, 256, 1024, 4096) for n in (64, 256, 1024, 4096) for k in (64, 256, 1024, 4096)],
                      dtype=np.int32)
    probe = (1024, 1024, 1024)
    all_nt = np.ones(len(shapes), dtype=np.int32)
    all_tnn = -all_nt
    try:
        for round_ in range(6):
            mt.mtnn_train_selector(shapes, all_nt)
            assert mt.mtnn_select(*probe) == 1
            mt.mtnn_train_selector(shapes, all_tnn)          # not queried with the probe shape
            mt.mtnn_train_selector(shapes, all_tnn if round_ % 2 else all_nt)
            mt.mtnn_train_selector(shapes, all_tnn)
            assert mt.mtnn_select(*probe) == -1
            mt.mtnn_unload_model()
            assert mt.mtnn_select(*probe) == 1               # no model: NT
    finally:
        mt.mtnn_unload_model()
        if os.path.exists(mt.DEFAULT_MODEL):
            mt.mtnn_load_model(mt.DEFAULT_MODEL)
