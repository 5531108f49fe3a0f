"""Seeded random cases through the GEMM, transpose and TNN entry points: shapes off every grid (log-uniform 1..1500 per
dimension, so tiny, ragged and multi-tile cases all occur), random leading-dimension padding and base
misalignment (NaN in the padding, canaries around the result), NT and NN, the rule's own choice or a random
tile configuration with a random division of the k range -- each compared element by element with the
fp64 oracle, and a second run bit for bit with the first."""
import numpy as np
import pytest

from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import inputs as I
import oracle
from gpu_util import check_gemm
from test_gpu_gemm import NCFG, operands, reference, run
from test_gpu_transpose import run_transpose

pytestmark = pytest.mark.gpu

N_CASES = 400


def case(i):
    r = I.uniform_ints(20260, i, 12, 0, 1 << 20)
    dim = lambda v: int(round(np.exp(np.log(1500.0) * (int(v) / float(1 << 20)))))      # log-uniform on [1, 1500]
    m, n, k = max(dim(r[0]), 1), max(dim(r[1]), 1), max(dim(r[2]), 1)
    if r[3] % 4 == 0:
        k = max(4, k // 4 * 4)                      # a quarter of the cases: k a multiple of 4 (pipelined kernel)
    op = mt.OP_NT if r[4] % 2 else mt.OP_NN
    if r[3] % 4 == 0 and op == mt.OP_NN:
        n = max(4, n // 4 * 4)
    pad = [0, 0, 0] if r[5] % 3 == 0 else [int(r[6] % 2) * 4, int(r[7] % 5), int(r[8] % 4)]
    if r[5] % 3 == 1:
        pad = [4 * int(r[6] % 3), 4 * int(r[7] % 3), int(r[8] % 4)]      # padded but still 16-byte aligned rows
    mis = 1 if r[5] % 7 == 0 else 0
    cfg = -1 if r[9] % 2 else int(r[9] // 2 % NCFG)
    splits = [0, 0, 2, 3, 5, mt.EVEN_CUT][int(r[10] % 6)]
    dist = ["uniform", "normal", "int"][int(r[11] % 3)]
    return m, n, k, op, pad, mis, cfg, splits, dist


@pytest.mark.parametrize("i", range(N_CASES))
def test_random_case_against_oracle(i):
    m, n, k, op, pad, mis, cfg, splits, dist = case(i)
    what = f"case {i}: op{op} {m}x{n}x{k} pad{pad} mis{mis} cfg{cfg} splits{splits} {dist}"
    print(what, flush=True)
    A, B = operands(op, m, n, k, 7000 + i, dist=dist)
    C, S = reference(op, A, B)
    bcols = B.shape[1]
    got = run(op, cfg, A, B, lda=k + pad[0], ldb=bcols + pad[1], ldc=n + pad[2], misalign=mis, splits=splits)
    if dist == "int":
        assert np.array_equal(got, C.astype(np.float32)), what
    else:
        check_gemm(got, C, S, k, what)
    again = run(op, cfg, A, B, lda=k + pad[0], ldb=bcols + pad[1], ldc=n + pad[2], misalign=mis, splits=splits)
    assert again.tobytes() == got.tobytes(), what + ": a second run differs"


def test_the_cases_cover_what_they_claim():
    cs = [case(i) for i in range(N_CASES)]
    assert {c[3] for c in cs} == {mt.OP_NT, mt.OP_NN}
    assert sum(1 for c in cs if c[2] % 4 == 0) >= N_CASES // 5 and sum(1 for c in cs if c[2] % 4) >= N_CASES // 3
    assert sum(1 for c in cs if min(c[0], c[1]) <= 8) >= 10 and sum(1 for c in cs if min(c[0], c[1]) > 128) >= 10
    assert len({c[6] for c in cs}) >= NCFG // 2 and {c[7] for c in cs} >= {0, 2, 3, 5, mt.EVEN_CUT}
    assert any(c[5] for c in cs) and any(sum(c[4]) == 0 for c in cs) and any(c[4][1] % 4 for c in cs)


def _dims(stream, i, hi, count=2):
    r = I.uniform_ints(20261 + stream, i, count + 4, 0, 1 << 20)
    d = [max(1, int(round(np.exp(np.log(float(hi)) * (int(v) / float(1 << 20)))))) for v in r[:count]]
    return d, r[count:]


@pytest.mark.parametrize("i", range(200))
def test_random_transpose_is_bit_exact(i):
    """rows, cols log-uniform on [1, 3000]; a third dense, a third with padded but aligned rows, a third with
    arbitrary padding; every seventh case off the 16-byte alignment; arbitrary bit patterns as data."""
    (rows, cols), r = _dims(0, i, 3000)
    pads = {0: (0, 0), 1: (4 * int(r[1] % 4), 4 * int(r[2] % 4)), 2: (int(r[1] % 7), int(r[2] % 5))}[int(r[0] % 3)]
    mis = int(r[3] % 3) + 1 if i % 7 == 0 else 0
    print(f"case {i}: {rows}x{cols} pads{pads} mis{mis}", flush=True)
    bits = (I._bits(6100 + i, 0, rows, cols) >> np.uint64(32)).astype(np.uint32)
    x = bits.view(np.float32)
    got = run_transpose(x, cols + pads[0], rows + pads[1], misalign=mis)
    assert np.array_equal(got.view(np.uint32), bits.T)


@pytest.mark.parametrize("i", range(80))
def test_random_rectangular_inplace_transpose_is_bit_exact(i):
    import torch
    (rows, cols), _ = _dims(1, i, 1500)
    print(f"case {i}: {rows}x{cols}", flush=True)
    x = np.arange(rows * cols, dtype=np.float32).reshape(rows, cols)       # word e holds the value e (< 2^24: exact)
    guard = 32
    host = np.full(guard + rows * cols + guard, np.float32(-1.0), dtype=np.float32)
    host[guard:guard + rows * cols] = x.reshape(-1)
    buf = torch.from_numpy(host).cuda()
    mt.mtnn_transpose_inplace_rect(buf[guard:guard + rows * cols], rows, cols)
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    assert got[guard:guard + rows * cols].tobytes() == np.ascontiguousarray(oracle.transpose_ref(x)).tobytes()
    assert (got[:guard] == -1.0).all() and (got[guard + rows * cols:] == -1.0).all()


@pytest.mark.parametrize("i", range(60))
def test_random_tnn_and_auto_against_oracle(i):
    """Algorithm 1 and Algorithm 2 on random shapes: C within the tolerance, B^T in the workspace bit for bit."""
    import torch
    (m, n, k), r = _dims(2, i, 600, count=3)
    print(f"case {i}: {m}x{n}x{k}", flush=True)
    A, B = I.nt_operands(m, n, k, 7500 + i, "normal" if r[0] % 2 else "uniform")
    C, S = oracle.nt_ref(A, B, with_bound=True)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    ws = torch.full((mt.mtnn_tnn_workspace_bytes(n, k),), 0xAB, dtype=torch.uint8, device="cuda")
    out = torch.empty((2, m, n), dtype=torch.float32, device="cuda")
    mt.mtnn_tnn(dA, dB, out[0], ws)
    torch.cuda.synchronize()
    bt = ws[: n * k * 4].view(torch.float32).view(k, n).cpu().numpy()
    assert bt.tobytes() == np.ascontiguousarray(oracle.transpose_ref(B)).tobytes()
    label = mt.mtnn_auto(dA, dB, out[1], ws)
    torch.cuda.synchronize()
    assert label in (1, -1)
    got = out.cpu().numpy()
    check_gemm(got[0], C, S, k, f"tnn {m}x{n}x{k}")
    check_gemm(got[1], C, S, k, f"auto {m}x{n}x{k}")


@pytest.mark.parametrize("i", range(60))
def test_random_layer_products_with_fused_epilogues(i):
    """The two layer products of the training step on random shapes and paddings: Y = act(X W^T + b) through
    every forward mode, and dW = A B with W = fma(-lr, dW, W), against the fp64 oracle products with the bias,
    clamp and update applied in float64."""
    import torch
    from gpu_util import Guarded, dev_matrix, tol
    (m, n, k), r = _dims(3, i, 700, count=3)
    pads = (0, 0, 0) if r[0] % 2 else (4 * int(r[1] % 3), int(r[2] % 5), 4 * int(r[3] % 2))
    relu = bool(r[1] % 2)
    mode = (1, -1, 0)[int(r[2] % 3)]
    print(f"case {i}: {m}x{n}x{k} pads{pads} relu{relu} mode{mode}", flush=True)
    X, W = I.nt_operands(m, n, k, 7700 + i, "normal")
    b = (I.uniform_pm1(7700 + i, 2, 1, n)[0] * np.float32(np.sqrt(k))).astype(np.float32)
    C, S = oracle.nt_ref(X, W, with_bound=True)
    want = C + b.astype(np.float64)[None, :]
    if relu:
        want = np.maximum(want, 0.0)
    dX, dW_ = dev_matrix(X, k + pads[0]), dev_matrix(W, k + pads[1])
    db = torch.from_numpy(b).cuda()
    ws = torch.empty(max(mt.mtnn_tnn_workspace_bytes(n, k), 256), dtype=torch.uint8, device="cuda")
    out = Guarded(m, n, n + pads[2])
    chosen = mt.mtnn_fc_layer_forward(dX, dW_, db, out.view, relu, mode, ws)
    torch.cuda.synchronize()
    assert chosen in (1, -1) and (mode == 0 or chosen == mode)
    got, intact = out.host()
    assert intact
    # the clamp is 1-Lipschitz and the bias one more rounding: the product's bound plus an ulp of the sum
    bound = tol(k) * S + 2.0 ** -23 * (np.abs(C) + np.abs(b)[None, :])
    assert float((np.abs(got.astype(np.float64) - want) - bound).max()) <= 0

    # the weight gradient of the same layer: dW = dY^T X (an NN product: (n x m) x (m x k)), W updated in its epilogue
    lr = np.float32(0.03)
    A = np.ascontiguousarray(I.normal01(7800 + i, 0, n, m))          # dY^T
    Bm = X                                                            # m x k
    G, Sg = oracle.nn_ref(A, Bm, with_bound=True)
    W0 = W.copy()
    dA, dB = dev_matrix(A, m + pads[0]), dev_matrix(Bm, k + pads[0])
    g_out = Guarded(n, k, k + pads[2])
    w_dev = torch.from_numpy(W0.copy()).cuda()
    mt.mtnn_fc_weight_grad_sgd(dA, dB, g_out.view, w_dev, float(lr))
    torch.cuda.synchronize()
    g, g_ok = g_out.host()
    assert g_ok
    assert float((np.abs(g.astype(np.float64) - G) - tol(m) * Sg).max()) <= 0
    w_want = W0.astype(np.float64) - float(lr) * G
    w_bound = float(lr) * tol(m) * Sg + 2.0 ** -23 * (np.abs(W0) + float(lr) * np.abs(G))
    assert float((np.abs(w_dev.cpu().numpy().astype(np.float64) - w_want) - w_bound).max()) <= 0
