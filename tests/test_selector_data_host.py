"""The product's offline bookkeeping (labels, metrics, protocol) against the oracle's formulas (host only)."""
import numpy as np
import pytest

from oracle import selection as S
from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import inputs as I
from paper_1702_03192_amd import selector_data as sd


def fake_rows(seed=0):
    rng = np.random.RandomState(seed)
    rows = []
    for (m, n, k, s) in I.sweep_shapes():
        t_nt = (m * n * k / 100e12 * (1.0 + 0.25 * (k >= 1024)) + 6e-6) * (1 + 0.03 * rng.standard_normal())
        t_tnn = (m * n * k / 100e12 + n * k * 8 / 4e12 + 11e-6) * (1 + 0.03 * rng.standard_normal())
        rows.append({"m": m, "n": n, "k": k, "seed": s, "t_nt": t_nt, "t_tnn": t_tnn})
    return rows


def test_label_rule_matches_oracle():
    for a, b in [(1.0, 2.0), (2.0, 1.0), (1.5, 1.5), (1e-6, 1.0000001e-6)]:
        assert sd.label_of(a, b) == S.label_from_times(a, b)
        assert sd.label_of(a, b) == S.label_from_perf(S.gflops(64, 64, 64, a), S.gflops(64, 64, 64, b))


def test_metrics_match_oracle_formulas():
    rows = fake_rows()
    shapes = [(r["m"], r["n"], r["k"]) for r in rows]
    t_nt = [r["t_nt"] for r in rows]
    t_tnn = [r["t_tnn"] for r in rows]
    rng = np.random.RandomState(1)
    pred = [int(x) for x in rng.choice([-1, 1], size=len(rows))]
    ours = sd.selection_metrics(t_nt, t_tnn, shapes, pred)
    p_nt = [S.gflops(*s, t) for s, t in zip(shapes, t_nt)]
    p_tnn = [S.gflops(*s, t) for s, t in zip(shapes, t_tnn)]
    ref = S.selection_metrics(p_nt, p_tnn, pred)
    for key, val in ref.items():
        assert ours[key] == pytest.approx(val, rel=1e-12, abs=1e-15), key
    assert ours["gow_avg"] >= 0 and ours["lub_avg"] <= 0


def test_splits_are_seeded_disjoint_and_stratified():
    labels = [1] * 150 + [-1] * 362
    tr, te = sd.stratified_split(labels, 4)
    assert not set(tr) & set(te) and len(tr) + len(te) == 512
    assert sum(1 for i in te if labels[i] == 1) == 30 and len(te) == 30 + 72
    assert sd.stratified_split(labels, 4) == (tr, te) and sd.stratified_split(labels, 5)[1] != te
    folds = sd.kfold(labels, 5, 0)
    seen = sorted(i for _, te_ in folds for i in te_)
    assert seen == list(range(512))
    for tr_, te_ in folds:
        assert not set(tr_) & set(te_)
        assert 29 <= sum(1 for i in te_ if labels[i] == 1) <= 31


def test_protocol_end_to_end_on_a_synthetic_table(tmp_path):
    rows = fake_rows(2)
    rep = sd.evaluate(rows, split_seeds=(1, 2))
    assert rep["samples"] == 512 and rep["n_label_nt"] + rep["n_label_tnn"] == 512
    assert rep["held_out_accuracy_mean"] > rep["majority_class_accuracy"] - 0.05
    assert rep["train_on_all_accuracy"] >= rep["held_out_accuracy_mean"] - 0.02
    assert rep["all_gow_avg"] >= 0 and rep["all_lub_avg"] <= 0 and rep["all_lub_min"] >= -1
    # the model left installed is the all-rows one and agrees with the oracle's trainer
    shapes = [(r["m"], r["n"], r["k"]) for r in rows]
    labels = [sd.label_of(r["t_nt"], r["t_tnn"]) for r in rows]
    ref = S.train_gbdt(np.array([S.features(*s) for s in shapes]), labels)
    assert [mt.mtnn_select(*s) for s in shapes] == [S.select(ref, *s) for s in shapes]
    mt.mtnn_unload_model()


def test_sweep_table_round_trip(tmp_path):
    import csv
    from paper_1702_03192_amd import sweep
    p = tmp_path / "t.csv"
    with open(p, "w", newline="") as f:
        wr = csv.DictWriter(f, fieldnames=sweep.FIELDS)
        wr.writeheader()
        wr.writerow({"m": 64, "n": 128, "k": 256, "seed": 10001, "t_nt": "1.5e-05", "t_nt_min": "1.4e-05",
                     "t_tnn": "2.5e-05", "t_tnn_min": "2.4e-05", "t_transpose": "5e-06", "t_nn": "1.6e-05",
                     "t_tnn_alloc": "3e-05", "nt_cfg": "a", "nn_cfg": "b"})
    rows = sd.load_sweep(str(p))
    assert rows[0]["m"] == 64 and rows[0]["t_tnn"] == 2.5e-05 and rows[0]["nt_cfg"] == "a"


def test_nt_tnn_statistics_match_the_oracle_and_a_hand_table():
    # the hand table of the oracle's own pin, with transposes that make t_tnn = t_transpose + t_nn on three rows
    rows = [{"m": 64, "n": 64, "k": 64, "t_nt": 10.0, "t_nn": 4.0, "t_tnn": 5.0, "t_transpose": 1.0},
            {"m": 128, "n": 64, "k": 64, "t_nt": 10.0, "t_nn": 8.0, "t_tnn": 12.0, "t_transpose": 4.0},
            {"m": 64, "n": 128, "k": 64, "t_nt": 6.0, "t_nn": 7.0, "t_tnn": 9.0, "t_transpose": 2.0},
            {"m": 64, "n": 64, "k": 128, "t_nt": 8.0, "t_nn": 8.0, "t_tnn": 8.0, "t_transpose": 1.0}]
    got = sd.nt_tnn_statistics(rows)
    ref = S.ratio_statistics([r["t_nt"] for r in rows], [r["t_nn"] for r in rows], [r["t_tnn"] for r in rows])
    for key, val in ref.items():
        assert got[key] == pytest.approx(val, rel=1e-12), key
    assert got["max_tnn_over_nt_shape"] == (64, 64, 64) and got["max_nt_over_tnn_shape"] == (64, 128, 64)
    # Eq. 4 holds on the first row only (1 < 10 - 4); the directly timed pair says TNN on the first row only: 4 of 4 agree
    eq4 = [S.tnn_pays(r["t_transpose"], r["t_nt"], r["t_nn"]) for r in rows]
    assert eq4 == [True, False, False, False]
    assert got["eq4_holds"] == 1 and got["eq4_agrees_with_direct_label"] == 4
    # log2(P_TNN / P_NT) = 1, -0.263, -0.585, 0 -> bins of a quarter, lower edge
    assert got["log2_tnn_over_nt_histogram"] == {"-0.75": 1, "-0.50": 1, "+0.00": 1, "+1.00": 1}
    # the shipped tables carry the columns the statistics need
    for path in sd.TRAINING_TABLES:
        st = sd.nt_tnn_statistics(sd.load_sweep(path))
        assert st["shapes"] >= 384 and 0.0 <= st["nn_faster_than_nt"] <= 1.0
        assert 0.9 < st["parts_over_whole_median"] < 1.1          # TNN's time is the sum of its two parts
