"""Algorithm 2 on the GPU with a predictor that really has two classes.

The shipped model answers +1 (NT) on almost every shape of this machine, so on its own it never sends
mtnn_auto down the -1 (TNN) branch.  Here a two-class model is trained through the library on a
made-up timing table, saved, and read back by an independent parser; for every tested shape the path
mtnn_auto takes must be the one the oracle's evaluator names on the parsed trees, both branches must
occur, and the result must match the fp64 oracle whichever branch ran."""
import os

import numpy as np
import pytest

import oracle
from oracle import selection as S
from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import inputs as I
from gpu_util import Guarded, check_gemm, dev_matrix
from test_selector_host import flat_margin, parse_model_file, synthetic_table

pytestmark = pytest.mark.gpu

SHAPES = [(m, n, k) for m in (64, 256, 1024, 2048) for n in (64, 512) for k in (256, 2048, 4096)]


@pytest.fixture()
def two_class_model(tmp_path):
    rows, labels = synthetic_table()
    assert 1 in labels and -1 in labels
    mt.mtnn_train_selector(rows, labels)
    path = str(tmp_path / "two_class.model")
    mt.mtnn_save_model(path)
    nfeat, trees = parse_model_file(path)
    assert nfeat == 7
    try:
        yield trees
    finally:
        mt.mtnn_unload_model()
        if os.path.exists(mt.DEFAULT_MODEL):
            mt.mtnn_load_model(mt.DEFAULT_MODEL)


def expected_label(trees, m, n, k):
    return 1 if flat_margin(trees, S.features(m, n, k)) >= 0.0 else -1


def test_auto_takes_both_branches_and_matches_the_oracle(two_class_model):
    import torch
    trees = two_class_model
    taken = []
    for i, (m, n, k) in enumerate(SHAPES):
        want_label = expected_label(trees, m, n, k)
        A, B = I.nt_operands(m, n, k, 8100 + i, "uniform")
        C, Sb = oracle.nt_ref(A, B, with_bound=True)
        dA, dB = dev_matrix(A), dev_matrix(B)
        ws = torch.full((mt.mtnn_tnn_workspace_bytes(n, k) // 4,), float("nan"), device="cuda")
        out = Guarded(m, n, n + 4)
        chosen = mt.mtnn_auto(dA, dB, out.view, ws)
        torch.cuda.synchronize()
        assert chosen == want_label == mt.mtnn_select(m, n, k), (m, n, k)
        got, intact = out.host()
        assert intact
        check_gemm(got, C, Sb, k, f"auto -> {chosen} at {m}x{n}x{k}")
        bt = ws[: n * k].view(k, n).cpu().numpy()
        if chosen == -1:        # Algorithm 1 ran: B^T is in the workspace, bit-exact
            assert bt.tobytes() == np.ascontiguousarray(B.T).tobytes()
        else:                   # the NT kernel ran: the workspace was not touched
            assert np.isnan(bt).all()
        taken.append(chosen)
        # memory rule of Section II: no room for B^T -> NT whatever the predictor says
        out2 = Guarded(m, n)
        assert mt.mtnn_auto(dA, dB, out2.view, None) == 1
        short = ws[: max(n * k - 64, 1)]
        assert mt.mtnn_auto(dA, dB, out2.view, short) == (1 if n * k > 64 else want_label)
        torch.cuda.synchronize()
        got2, intact2 = out2.host()
        assert intact2
        check_gemm(got2, C, Sb, k, f"auto without room at {m}x{n}x{k}")
    assert len(taken) >= 20 and taken.count(-1) >= 4 and taken.count(1) >= 4, taken


def test_layer_forward_mode_0_takes_both_branches(two_class_model):
    """mtnn_fc_layer_forward(mode = 0) is Algorithm 2 with the bias and the clamp in the epilogue."""
    import torch
    trees = two_class_model
    taken = []
    for i, (m, n, k) in enumerate(SHAPES[::2]):
        want_label = expected_label(trees, m, n, k)
        X, W = I.nt_operands(m, n, k, 8200 + i, "normal")
        b = I.normal01(8300 + i, 0, 1, n)[0]
        Z, Sb = oracle.nt_ref(X, W, with_bound=True)
        want = np.maximum(Z + b.astype(np.float64), 0.0)
        dX, dW = dev_matrix(X), dev_matrix(W)
        db = torch.from_numpy(b).cuda()
        ws = torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda")
        out = Guarded(m, n)
        chosen = mt.mtnn_fc_layer_forward(dX, dW, db, out.view, relu=True, mode=0, workspace=ws)
        torch.cuda.synchronize()
        assert chosen == want_label, (m, n, k)
        got, intact = out.host()
        assert intact
        # the bias adds one rounding of a value of size |Z| + |b|: bound as for the product, against S + |b|
        bound = Sb + np.abs(b.astype(np.float64))
        err = np.abs(got.astype(np.float64) - want) / bound
        assert err.max() <= 1e-5 * np.sqrt(k), (m, n, k, err.max())
        taken.append(chosen)
    assert taken.count(-1) >= 2 and taken.count(1) >= 2, taken
